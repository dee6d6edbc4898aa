// Device-side pieces of the byte walk shared by cfgzip_signatures and by the
// class builder's re-walk verification (paper Section 3.2.1 / Algorithm 1
// restricted to a deterministic byte automaton:  sig[t][q] = delta*(q, bytes(t))).
//
// Image walk.  After its first byte b a token can only be in one of the
// distinct states of column b of the automaton, whatever state it started in.
// So a token is not walked from all S states: only the nimg[b] distinct states
// of its first byte's column are walked through the remaining bytes, giving a
// short vector w, and
//     sig[t][q] = w[idx[b][q]],
//     H(t)      = sum_j wsum[b][j] * w[j]      (the hash is linear, so this is
//                                               bit-identical to the sum over q).
// Lexer-like automata send most (state, byte) pairs to the reject state, so
// nimg[b] is typically a few percent of S; a random automaton gives no gain
// (nimg[b] ~ 0.63 S) and costs one extra indirection.
//
// Tables kept in the signature workspace (built per call by prepare_tables):
//   Tt[b][q]   = table[q][b]            one byte selects one contiguous column
//   per image row b (0..255 = first byte; 256 = "no byte", the identity map of
//   the empty token):
//   nimg[b]    = number of distinct states in column b
//   img[b][j]  = j-th distinct state of column b, ascending           (j < nimg[b])
//   idx[b][q]  = position of Tt[b][q] in img[b]
//   wsum[b][j] = sum of the hash multipliers a_q over all q with idx[b][q] == j
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cfgzip {

// Tt is over-allocated by this many entries so that a table entry >= S (a
// caller error) still indexes inside the workspace.
constexpr int kTablePad = 65536;
constexpr int kImageRows = 257;     // 256 first bytes + the "empty token" row
constexpr int kBatchTokens = 64;    // tokens a workgroup walks together (one per lane of a wave)
constexpr int kByteCap = 4096;      // token bytes staged in LDS per batch
constexpr int kMinWalkCap = 8192;   // walks (entries of w) held in LDS per batch, at least
// Walks of one token that a thread carries together.  Fewer walks per thread put more lanes on one
// token, so a wave's table reads fall into fewer columns (measured on 4,096 states: 8 -> 147 us,
// 4 -> 130 us, 2 -> 130 us, 1 -> 153 us per signature call).
constexpr int kWalkGroup = 4;

struct Tables {
    const uint16_t *Tt;
    const int32_t *nimg;
    const uint16_t *img;
    const uint16_t *idx;
    const uint64_t *wsum;  // null when no hash is wanted
};

// Walk vectors kept in the signature workspace after cfgzip_signatures, so that the class
// builder can compare signatures without walking again: token t has image row wrow[t] and its
// vector is wvec[t * stride .. t * stride + nimg[wrow[t]]), padded with zeros to a multiple of
// 8 entries (16-byte compares).  A token whose vector is longer than the stride does not fit;
// then `overflow` is set and the store is unusable.
struct WalkStore {
    uint32_t magic;     // kWalkStoreMagic once the header is written for this (V, S)
    int32_t V, S;
    uint32_t stride;    // entries per token, a multiple of 8
    uint32_t overflow;  // 1: some vector did not fit
    uint32_t pad[3];
};
constexpr uint32_t kWalkStoreMagic = 0xCF621A1Cu;
constexpr int kWalkStoreMaxStride = 256;  // entries kept per token at most (512 bytes)
__host__ __device__ inline uint32_t walk_store_stride(int32_t S) {
    const uint32_t s8 = ((uint32_t)S + 7u) & ~7u;
    return s8 < (uint32_t)kWalkStoreMaxStride ? s8 : (uint32_t)kWalkStoreMaxStride;
}

struct WalkStoreView {
    WalkStore *header;  // null: nothing is kept
    uint16_t *wrow;     // [V]: image row (9 bits) and, above it, how many 16-byte units of the vector are in use
    uint16_t *wvec;     // [V][stride]
};
// wrow entry: the comparison of two kept vectors then needs no look-up of the row's image size
__host__ __device__ inline uint16_t pack_walk_row(uint32_t row, uint32_t count, uint32_t stride) {
    const uint32_t kept = row >= 256u ? 0u : (count < stride ? count : stride);  // the empty token keeps nothing
    return (uint16_t)((row < 256u ? row : 256u) | (((kept + 7u) / 8u) << 9));
}
__host__ __device__ inline uint32_t walk_row_of(uint16_t packed) { return packed & 0x1FFu; }
__host__ __device__ inline uint32_t walk_units_of(uint16_t packed) { return packed >> 9; }

// Builds all tables in the signature workspace.  Host functions, defined in walk.hip.
// V > 0 also lays out (and resets) the walk store for V tokens.
int prepare_tables(const uint16_t *table, int32_t S, uint64_t hash_seed, bool want_wsum, int32_t V,
                   void *ws, Tables *out, WalkStoreView *store, hipStream_t stream);
size_t sig_workspace_bytes(int32_t V, int32_t S);
// Views of a workspace that a finished cfgzip_signatures(V, S) call left behind.
void view_signature_workspace(void *ws, int32_t V, int32_t S, Tables *tables, WalkStoreView *store);
// Entries of w a batch may hold for an automaton of S states: room for any two tokens, each
// padded to a whole number of walk groups.
inline int walk_cap_for(int32_t S) {
    const int two = 2 * ((S + kWalkGroup - 1) / kWalkGroup * kWalkGroup);
    return two > kMinWalkCap ? two : kMinWalkCap;
}

__device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint32_t index) {
    // index-th output (0-based) of the SplitMix64 generator seeded with `seed`
    uint64_t z = seed + (uint64_t)(index + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ int wave_inclusive_sum(int v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    return v;
}

// A batch of up to kBatchTokens byte strings that a workgroup walks together.
// Slot m has cnt[m] walks; they are carried in groups of kWalkGroup (the last group padded),
// groups [gstart[m], gstart[m+1]), and their end states land in w[wstart[m] ..], a region
// padded to whole groups whose padding reads 0.  Staged bytes: [boff[m], boff[m+1]).
// A slot with no walks (an unused lane) has no groups.
struct Batch {
    int32_t k;             // slots in use
    int32_t wtotal;        // walks of the batch
    int32_t btotal;        // staged bytes of the batch
    int32_t bytes_in_lds;  // 0: a single over-long token, its bytes are read from global memory
    int32_t gtotal;        // walk groups of the batch
    int32_t wstart[kBatchTokens + 1];
    int32_t gstart[kBatchTokens + 1];
    int32_t cnt[kBatchTokens];
    int32_t boff[kBatchTokens + 1];
    int32_t len[kBatchTokens];
    int32_t row[kBatchTokens];  // image row: first byte, or 256 for an empty byte string
    int32_t aux[kBatchTokens];  // free for the kernel that fills the batch
    // composition (sig(tu) = sig(u) o sig(t)): a slot may start from the kept walk vector of a
    // token that is a proper prefix of its own byte string instead of from the image states
    int32_t parent[kBatchTokens];  // that token's id, or -1
    int32_t skip[kBatchTokens];    // bytes the start vector has already read: the prefix's length, else 1
    int64_t beg[kBatchTokens];  // offset of the first byte in tok_bytes
    unsigned long long hash[kBatchTokens];
};

// Largest m < k with starts[m] <= i (starts non-decreasing, starts[0] <= i).
__device__ __forceinline__ int batch_find(const int32_t *starts, int k, int i) {
    int lo = 0;
#pragma unroll
    for (int step = kBatchTokens / 2; step >= 1; step >>= 1) {
        const int c = lo + step;
        if (c < k && starts[c] <= i) lo = c;
    }
    return lo;
}

// Filled by the 64 lanes of one wave: lane l proposes byte string (beg, len) (len < 0: lane
// unused).  Slots are accepted in lane order while the walks fit in `wcap` entries and the
// bytes in kByteCap; at least `min_lanes` lanes are accepted (their walks always fit, see
// walk_cap_for; if their bytes do not, the batch reads bytes from global memory).  Returns
// the number of accepted lanes, rounded down to a multiple of `group` (wave-uniform).
// `parent` / `parent_len`: see Batch::parent (pass -1 / 0 for a plain walk).
__device__ __forceinline__ int batch_fill(Batch &B, const Tables &T, const uint8_t *tok_bytes,
                                          int64_t beg, int64_t len64, int wcap, int min_lanes,
                                          int group, int32_t parent = -1, int32_t parent_len = 0) {
    const int lane = threadIdx.x & 63;
    const bool used = len64 >= 0;
    const int len = !used ? 0 : (len64 > 0x7FFFFFFF ? 0x7FFFFFFF : (int)len64);
    const int row = len > 0 ? (int)tok_bytes[beg] : 256;
    const int n = used ? T.nimg[row] : 0;
    const int groups = (n + kWalkGroup - 1) / kWalkGroup;
    const int npad = groups * kWalkGroup;
    const int lenc = len > kByteCap ? kByteCap + 1 : len;
    const int incl_n = wave_inclusive_sum(npad);
    const int incl_g = wave_inclusive_sum(groups);
    const int incl_b = wave_inclusive_sum(lenc);
    const bool fits = lane < min_lanes || (incl_n <= wcap && incl_b <= kByteCap);
    const uint64_t mask = __ballot(fits);
    // accepted lanes form a prefix: the sums are non-decreasing
    int k = mask == ~0ull ? 64 : __ffsll((unsigned long long)~mask) - 1;
    k -= k % group;
    if (lane < k) {
        B.wstart[lane] = incl_n - npad;
        B.gstart[lane] = incl_g - groups;
        B.cnt[lane] = n;
        B.boff[lane] = incl_b - lenc;
        B.len[lane] = len;
        B.row[lane] = row;
        B.beg[lane] = beg;
        B.hash[lane] = 0ull;
        const bool composed = parent >= 0 && parent_len >= 1 && parent_len < len;
        B.parent[lane] = composed ? parent : -1;
        B.skip[lane] = composed ? parent_len : 1;
    }
    if (lane == k - 1) {
        B.wstart[k] = incl_n;
        B.gstart[k] = incl_g;
        B.boff[k] = incl_b;
        B.k = k;
        B.wtotal = incl_n;
        B.gtotal = incl_g;
        B.btotal = incl_b;
        B.bytes_in_lds = incl_b <= kByteCap ? 1 : 0;
    }
    return k;
}

// Copies the batch's bytes into LDS (all threads of the workgroup).
__device__ __forceinline__ void batch_stage_bytes(const Batch &B, const uint8_t *__restrict__ tok_bytes,
                                                  uint8_t *ldsb) {
    if (!B.bytes_in_lds) return;
    const int total = B.btotal, k = B.k;
    for (int x = threadIdx.x; x < total; x += blockDim.x) {
        const int m = batch_find(B.boff, k, x);
        ldsb[x] = tok_bytes[B.beg[m] + (x - B.boff[m])];
    }
}

// Walks every (slot, image state) pair of the batch: w[wstart[m] + j] = state reached from
// img[row][j] on bytes 1.. of slot m (0 in the padding).  A walk is a chain of dependent table
// reads, so a thread carries a group of kWalkGroup walks of ONE slot: they share the bytes,
// have the same length, and give kWalkGroup independent reads per step; the next byte is fetched
// while the current reads are outstanding.  With HASH, adds the group's part of
// sum_j wsum[row][j] * w[j] to B.hash[m] (order-free).  `keep` (or null) is where slot 0's
// walk vector is kept, slot m's follows keep_stride entries on (keep_stride a multiple of
// kWalkGroup; a vector longer than that is cut off).
// `kept` (or null): kept walk vectors of finished tokens, kept_stride entries apart, from which
// the slots with a parent start.
template <bool LDS_BYTES, bool HASH>
__device__ __forceinline__ void batch_walk_impl(const Tables &T, const uint16_t *tab, int S,
                                                const uint8_t *__restrict__ tok_bytes, Batch &B,
                                                const uint8_t *ldsb, uint16_t *w, uint16_t *keep,
                                                uint32_t keep_stride, const uint16_t *kept = nullptr) {
    // every table index fits 32 bits: 257 rows of at most 65536 entries
    const uint32_t nt = blockDim.x, k = B.k, gtotal = B.gtotal, Su = (uint32_t)S;
    const bool vec4 = (S % 4) == 0;
    for (uint32_t g = threadIdx.x; g < gtotal; g += nt) {
        const uint32_t m = (uint32_t)batch_find(B.gstart, (int)k, (int)g);
        const uint32_t j0 = (g - (uint32_t)B.gstart[m]) * kWalkGroup;
        const uint32_t n = (uint32_t)B.cnt[m];
        const uint32_t e0 = (uint32_t)B.row[m] * Su + j0;
        uint32_t cur[kWalkGroup];
        // (a vector longer than what is kept of it cannot be started from)
        const int32_t par = (kept && n <= keep_stride) ? B.parent[m] : -1;
        const uint32_t skip = par >= 0 ? (uint32_t)B.skip[m] : 1u;
        // A group's four start states (and its four hash multipliers) lie next to each other: with
        // S a multiple of 4 they are 8-byte (32-byte) aligned and come in one (two) loads.
        static_assert(kWalkGroup == 4, "the vector forms below are written for groups of four");
        if (par >= 0) {  // the prefix's end states are this token's start states
            const uint2 v = *reinterpret_cast<const uint2 *>(kept + (size_t)par * keep_stride + j0);
            cur[0] = v.x & 0xFFFFu, cur[1] = v.x >> 16, cur[2] = v.y & 0xFFFFu, cur[3] = v.y >> 16;
        } else if (vec4) {
            const uint2 v = *reinterpret_cast<const uint2 *>(T.img + e0);
            cur[0] = v.x & 0xFFFFu, cur[1] = v.x >> 16, cur[2] = v.y & 0xFFFFu, cur[3] = v.y >> 16;
        } else {
#pragma unroll
            for (int u = 0; u < kWalkGroup; ++u) cur[u] = j0 + u < n ? (uint32_t)T.img[e0 + u] : 0u;
        }
#pragma unroll
        for (int u = 0; u < kWalkGroup; ++u)
            if (j0 + u >= n) cur[u] = 0u;  // padding of the token's last group
        // the hash multipliers are asked for now and used after the walk: off the critical path
        uint64_t mult[kWalkGroup];
        if (HASH) {
            if (vec4) {
                const uint4 lo = *reinterpret_cast<const uint4 *>(T.wsum + e0);
                const uint4 hi = *reinterpret_cast<const uint4 *>(T.wsum + e0 + 2);
                mult[0] = lo.x | ((uint64_t)lo.y << 32), mult[1] = lo.z | ((uint64_t)lo.w << 32);
                mult[2] = hi.x | ((uint64_t)hi.y << 32), mult[3] = hi.z | ((uint64_t)hi.w << 32);
            } else {
#pragma unroll
                for (int u = 0; u < kWalkGroup; ++u) mult[u] = j0 + u < n ? T.wsum[e0 + u] : 0ull;
            }
        }
        const uint32_t rem = B.len[m] > 0 ? (uint32_t)B.len[m] - skip : 0u;
        const uint32_t lsrc = (uint32_t)B.boff[m] + skip;                             // first byte to read, in ldsb
        const uint8_t *gsrc = LDS_BYTES ? tok_bytes : tok_bytes + B.beg[m] + skip;    // or in memory
        uint32_t nextb = 0;
        if (rem > 0) nextb = LDS_BYTES ? ldsb[lsrc] : gsrc[0];
        for (uint32_t p = 0; p < rem; ++p) {
            const uint32_t b = nextb;
            if (p + 1 < rem) nextb = LDS_BYTES ? ldsb[lsrc + p + 1] : gsrc[(size_t)p + 1];
            const uint16_t *col = tab + b * Su;
#pragma unroll
            for (int u = 0; u < kWalkGroup; ++u) cur[u] = col[cur[u]];
        }
        uint64_t term = 0;
#pragma unroll
        for (int u = 0; u < kWalkGroup; ++u) {
            if (j0 + u >= n) cur[u] = 0;  // padding
            else if (HASH) term += mult[u] * (uint64_t)cur[u];
        }
        // the four end states as one 8-byte store each way (both regions are 8-byte aligned: a slot's
        // region in w starts at a multiple of the group size, a kept vector at a multiple of 8 entries)
        const uint2 packed = make_uint2(cur[0] | (cur[1] << 16), cur[2] | (cur[3] << 16));
        if (w) *reinterpret_cast<uint2 *>(w + (uint32_t)B.wstart[m] + j0) = packed;  // null: only hash and `keep` are wanted
        if (keep && j0 < keep_stride) {
            uint16_t *kd = keep + (size_t)m * keep_stride + j0;
            *reinterpret_cast<uint2 *>(kd) = packed;
            // a kept vector is compared 8 entries at a time: the token's last group also zeroes
            // what lies between its own end and the next multiple of 8 (keep_stride is one)
            if (j0 + kWalkGroup >= n && j0 + kWalkGroup < ((n + 7u) & ~7u) && j0 + kWalkGroup < keep_stride)
                *reinterpret_cast<uint2 *>(kd + kWalkGroup) = make_uint2(0u, 0u);
        }
        if (HASH) atomicAdd(&B.hash[m], (unsigned long long)term);
    }
}

template <bool HASH>
__device__ __forceinline__ void batch_walk(const Tables &T, const uint16_t *tab, int S,
                                           const uint8_t *__restrict__ tok_bytes, Batch &B,
                                           const uint8_t *ldsb, uint16_t *w, uint16_t *keep = nullptr,
                                           uint32_t keep_stride = 0, const uint16_t *kept = nullptr) {
    if (B.bytes_in_lds) batch_walk_impl<true, HASH>(T, tab, S, tok_bytes, B, ldsb, w, keep, keep_stride, kept);
    else batch_walk_impl<false, HASH>(T, tab, S, tok_bytes, B, ldsb, w, keep, keep_stride, kept);
}

}  // namespace cfgzip
