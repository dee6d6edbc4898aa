// cfgzip_build_classes: group tokens with equal signature, number the classes
// and pick representatives (paper Section 3.1 "Pre-Computation").
//
// Pipeline (all on the device):
//   1. stable LSD radix sort of the key (low 32 or 40 bits of the hash, first
//      byte of the token) with the token id as value, 8 bits per pass, two
//      kernels per pass: per-tile digit counts, then a scatter that ranks its
//      tile and adds over the counts of the earlier tiles itself;
//   2. equal-hash segments; inside a segment tokens with the same first byte are
//      neighbours.  Every member is compared with its left neighbour (a chain:
//      equality is transitive).  Three sources, in order of preference: the walk
//      vectors a preceding cfgzip_signatures call left in its workspace (compared
//      on the short vector w when both tokens share the first byte, through the
//      index tables otherwise - walk_device.hpp); stored signature rows; or, with
//      neither, both tokens are re-walked with the image walk;
//   3. if no link differs (no hash collision - the overwhelmingly common case),
//      the segments are the classes.  Otherwise every differing member starts a
//      new chain and the chain starts of a segment are matched against each
//      other in rounds (the first unmatched one becomes a class, the rest are
//      compared with it) - exact for any hash that is a function of the signature;
//   4. class id = rank of the class's smallest token id among all classes, by a
//      prefix sum over token ids;
//   5. representative = min over members of (byte length, token id).
// The host waits once, for the class count and the number of differing links.

#include <algorithm>

#include "common.hpp"
#include "walk_device.hpp"

namespace cfgzip {
namespace {

constexpr int kThreads = 256;
constexpr int kItems = 8;
constexpr int kTile = kThreads * kItems;  // keys per workgroup in sort and scan kernels
constexpr int kRadixBits = 8;
constexpr int kBins = 1 << kRadixBits;
// Hash bits that take part in the sort, above the 8 bits of the first byte.  Two classes that
// agree in these bits only cost a pass through the collision rounds (C classes: about
// C^2 / 2^(bits+1) such pairs), so small vocabularies sort 32 bits (5 passes) and large ones 40.
constexpr int32_t kLargeVocabulary = 1 << 18;
inline int hash_bits_for(int32_t V) { return V > kLargeVocabulary ? 40 : 32; }
static_assert(kThreads == kBins, "one thread per bin in the sort kernels");

struct Counters {
    int32_t unresolved;
    int32_t num_classes;
    int32_t store_unusable;  // the walk store did not match this call or had overflowed
    int32_t pad[5];
};

// ---------------------------------------------------------------- radix sort

// key of token t: hash bits above its first byte (0 for the empty token; a clash
// of that 0 with a real first byte only costs a slower comparison)
__device__ __forceinline__ uint64_t sort_key(const uint64_t *__restrict__ hash,
                                             const int64_t *__restrict__ tok_off,
                                             const uint8_t *__restrict__ tok_bytes, int t,
                                             uint64_t hash_mask) {
    const int64_t beg = tok_off[t];
    const uint32_t fb = tok_off[t + 1] > beg ? (uint32_t)tok_bytes[beg] : 0u;
    return ((hash[t] & hash_mask) << 8) | fb;
}

// Digit counts of one pass per tile: hist[tile][digit].  The first pass forms its keys from
// the hash and the first bytes; later passes read the keys the previous pass wrote.
template <bool FIRST>
__global__ __launch_bounds__(kThreads) void radix_hist_kernel(
    const uint64_t *__restrict__ hash, const int64_t *__restrict__ tok_off,
    const uint8_t *__restrict__ tok_bytes, const uint64_t *__restrict__ keys, int n, int shift,
    uint64_t hash_mask, uint32_t *hist) {
    __shared__ uint32_t bins[kBins];
    bins[threadIdx.x] = 0;
    __syncthreads();
    const int base = blockIdx.x * kTile;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int idx = base + j * kThreads + threadIdx.x;
        if (idx < n) {
            const uint64_t key = FIRST ? sort_key(hash, tok_off, tok_bytes, idx, hash_mask) : keys[idx];
            atomicAdd(&bins[(uint32_t)(key >> shift) & (kBins - 1)], 1u);
        }
    }
    __syncthreads();
    hist[(size_t)blockIdx.x * kBins + threadIdx.x] = bins[threadIdx.x];
}

struct ScatterArgs {
    const uint64_t *hash;  // first pass: keys are formed from the hash and the first bytes
    const int64_t *tok_off;
    const uint8_t *tok_bytes;
    const uint64_t *keys_in;  // later passes
    const int32_t *vals_in;
    uint64_t *keys_out;
    int32_t *vals_out;
    const uint32_t *hist;  // [nb][256] digit counts of this pass per input tile
    uint64_t hash_mask;
    int n, nb, shift;
};

// One stable pass.  A wave owns a contiguous chunk of the tile and visits it 64 keys at a
// time, so (wave, visit, lane) order is index order.
template <bool FIRST>
__global__ __launch_bounds__(kThreads) void radix_scatter_kernel(ScatterArgs a) {
    __shared__ uint32_t wave_count[kThreads / 64][kBins];
    __shared__ uint32_t wave_tot[kThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < (kThreads / 64) * kBins; i += kThreads)
        (&wave_count[0][0])[i] = 0;

    // first output position of this tile's keys with digit d:
    //   keys with a smaller digit anywhere + keys with digit d in earlier tiles
    uint32_t bin_base;
    {
        const int d = threadIdx.x;
        uint32_t tot = 0, before = 0;
        constexpr int kAhead = 16;  // independent loads in flight: the loop is latency-bound
        for (int t0 = 0; t0 < a.nb; t0 += kAhead) {
            uint32_t c[kAhead];
#pragma unroll
            for (int u = 0; u < kAhead; ++u)
                c[u] = t0 + u < a.nb ? a.hist[(size_t)(t0 + u) * kBins + d] : 0u;
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                tot += c[u];
                if (t0 + u < (int)blockIdx.x) before += c[u];
            }
        }
        const int incl = wave_inclusive_sum((int)tot);
        if (lane == 63) wave_tot[wave] = (uint32_t)incl;
        __syncthreads();  // also orders the clearing of wave_count before its use
        uint32_t prefix = 0;
        for (int w = 0; w < wave; ++w) prefix += wave_tot[w];
        bin_base = prefix + (uint32_t)incl - tot + before;
    }

    volatile uint32_t *my_count = wave_count[wave];
    const int chunk = blockIdx.x * kTile + wave * (64 * kItems);
    uint64_t key[kItems];
    uint32_t rank[kItems];
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int idx = chunk + j * 64 + lane;
        const bool valid = idx < a.n;
        key[j] = !valid ? 0ull
                 : FIRST ? sort_key(a.hash, a.tok_off, a.tok_bytes, idx, a.hash_mask)
                         : a.keys_in[idx];
        const uint32_t d = (uint32_t)(key[j] >> a.shift) & (kBins - 1);
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < kRadixBits; ++bit) {
            const bool one = (d >> bit) & 1u;
            const uint64_t bm = __ballot(one);
            peers &= one ? bm : ~bm;
        }
        rank[j] = 0;
        if (valid) {
            const uint32_t before = my_count[d];
            const uint32_t r = (uint32_t)__popcll(peers & lt_mask);
            rank[j] = before + r;
            if (r == 0) my_count[d] = before + (uint32_t)__popcll(peers);
        }
    }
    __syncthreads();
    {
        const int d = threadIdx.x;
        uint32_t run = bin_base;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) {
            const uint32_t c = wave_count[w][d];
            wave_count[w][d] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int idx = chunk + j * 64 + lane;
        if (idx < a.n) {
            const uint32_t d = (uint32_t)(key[j] >> a.shift) & (kBins - 1);
            const uint32_t pos = wave_count[wave][d] + rank[j];
            if (pos >= (uint32_t)a.n) continue;  // cannot happen with consistent counts; stay in bounds
            a.keys_out[pos] = key[j];
            a.vals_out[pos] = FIRST ? idx : a.vals_in[idx];
        }
    }
}

// ---------------------------------------------------------------- scans over int32

template <bool MAX>
__device__ __forceinline__ int32_t scan_op(int32_t a, int32_t b) {
    return MAX ? max(a, b) : a + b;
}

// Per-tile totals.
template <bool MAX>
__global__ __launch_bounds__(kThreads) void scan_reduce_kernel(const int32_t *__restrict__ in, int n,
                                                               int32_t *tile_tot) {
    __shared__ int32_t wave_tot[kThreads / 64];
    const int base = blockIdx.x * kTile + threadIdx.x * kItems;
    int32_t acc = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j)
        if (base + j < n) acc = scan_op<MAX>(acc, in[base + j]);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) acc = scan_op<MAX>(acc, __shfl_xor(acc, off, 64));
    if ((threadIdx.x & 63) == 0) wave_tot[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t t = 0;
        for (int w = 0; w < kThreads / 64; ++w) t = scan_op<MAX>(t, wave_tot[w]);
        tile_tot[blockIdx.x] = t;
    }
}

// Scan inside each tile (values >= 0, identity 0), seeded with the combination of the totals
// of all earlier tiles, which every workgroup folds for itself.  The last tile also writes
// the grand total.
template <bool MAX, bool INCLUSIVE>
__global__ __launch_bounds__(kThreads) void scan_final_kernel(const int32_t *__restrict__ in, int n,
                                                              const int32_t *__restrict__ tile_tot,
                                                              int32_t *__restrict__ out,
                                                              int32_t *grand_total) {
    __shared__ int32_t wave_tot[kThreads / 64];
    __shared__ int32_t wave_pre[kThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t tp = 0;
    for (int t = threadIdx.x; t < (int)blockIdx.x; t += kThreads) tp = scan_op<MAX>(tp, tile_tot[t]);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) tp = scan_op<MAX>(tp, __shfl_xor(tp, off, 64));
    if (lane == 0) wave_pre[wave] = tp;

    const int base = blockIdx.x * kTile + threadIdx.x * kItems;
    int32_t v[kItems];
    int32_t acc = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        v[j] = base + j < n ? in[base + j] : 0;
        acc = scan_op<MAX>(acc, v[j]);
    }
    int32_t inc = acc;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int32_t o = __shfl_up(inc, off, 64);
        if (lane >= off) inc = scan_op<MAX>(inc, o);
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    int32_t prefix = 0;
    for (int w = 0; w < kThreads / 64; ++w) prefix = scan_op<MAX>(prefix, wave_pre[w]);
    for (int w = 0; w < wave; ++w) prefix = scan_op<MAX>(prefix, wave_tot[w]);
    int32_t before = __shfl_up(inc, 1, 64);
    if (lane == 0) before = 0;
    int32_t run = scan_op<MAX>(prefix, before);
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int32_t next = scan_op<MAX>(run, v[j]);
        if (base + j < n) out[base + j] = INCLUSIVE ? next : run;
        run = next;
    }
    if (grand_total && blockIdx.x == gridDim.x - 1 && threadIdx.x == kThreads - 1) *grand_total = run;
}

template <bool MAX, bool INCLUSIVE>
int device_scan(const int32_t *in, int32_t *out, int n, int32_t *tile_tmp, int32_t *grand_total,
                hipStream_t stream) {
    const int nt = (int)ceil_div(n, kTile);
    hipLaunchKernelGGL(scan_reduce_kernel<MAX>, dim3(nt), dim3(kThreads), 0, stream, in, n, tile_tmp);
    CFGZIP_TRY(check_launch());
    hipLaunchKernelGGL((scan_final_kernel<MAX, INCLUSIVE>), dim3(nt), dim3(kThreads), 0, stream, in,
                       n, tile_tmp, out, grand_total);
    return check_launch();
}

// ---------------------------------------------------------------- segments

__device__ __forceinline__ uint64_t hash_part(uint64_t key) { return key >> 8; }

// seg_head[i] = first sorted position with the same hash bits as position i.  Chain set-up:
// a segment start is its own head and settled; every other position is compared with its
// left neighbour.  Also clears the per-position and per-token arrays used later.
__global__ __launch_bounds__(kThreads) void segments_kernel(
    const uint64_t *__restrict__ keys, int n, int32_t *seg_head, int32_t *head_pos,
    int32_t *resolved, int32_t *mismatch, int32_t *min_id, uint64_t *rep_key,
    int32_t *is_head_token, Counters *ctr) {
    __shared__ int32_t wave_tot[kThreads / 64];
    __shared__ int32_t carry_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile0 = blockIdx.x * kTile;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ctr->unresolved = 0;
        ctr->num_classes = 0;
        ctr->store_unusable = 0;
    }
    // where the segment that reaches into this tile starts (64-ary search by the first wave)
    if (wave == 0) {
        int lo = tile0;
        if (tile0 > 0 && hash_part(keys[tile0]) == hash_part(keys[tile0 - 1])) {
            const uint64_t target = hash_part(keys[tile0]);
            lo = 0;
            int hi = tile0 - 1;  // the first position with hash bits >= target lies in [lo, hi]
            while (hi > lo) {
                const int step = (hi - lo + 63) / 64;
                const int x = lo + lane * step;
                const bool p = x >= hi || hash_part(keys[x]) >= target;
                const uint64_t m = __ballot(p);
                if (m == 0ull) {
                    lo = lo + 63 * step + 1;
                } else {
                    const int f = __ffsll((unsigned long long)m) - 1;
                    const int new_hi = min(hi, lo + f * step);
                    if (f > 0) lo = lo + (f - 1) * step + 1;
                    hi = new_hi;
                }
            }
        }
        if (lane == 0) carry_s = lo;
    }
    const int base = tile0 + threadIdx.x * kItems;
    int32_t v[kItems];
    int32_t acc = -1;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int i = base + j;
        v[j] = -1;
        if (i < n && (i == 0 || hash_part(keys[i]) != hash_part(keys[i - 1]))) v[j] = i;
        acc = max(acc, v[j]);
    }
    int32_t inc = acc;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int32_t o = __shfl_up(inc, off, 64);
        if (lane >= off) inc = max(inc, o);
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    int32_t run = carry_s;
    for (int w = 0; w < wave; ++w) run = max(run, wave_tot[w]);
    int32_t before = __shfl_up(inc, 1, 64);
    if (lane == 0) before = -1;
    run = max(run, before);
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int i = base + j;
        run = max(run, v[j]);
        if (i < n) {
            const bool start = v[j] == i;
            seg_head[i] = run;
            head_pos[i] = start ? i : i - 1;
            resolved[i] = start ? 1 : 0;
            mismatch[i] = 0;
            min_id[i] = 0x7FFFFFFF;
            rep_key[i] = ~0ull;
            is_head_token[i] = 0;
        }
    }
}

// ---------------------------------------------------------------- verification

__device__ __forceinline__ void settle(bool differs, int i, int32_t *resolved, int32_t *mismatch,
                                       Counters *ctr) {
    if ((threadIdx.x & 63) != 0) return;
    if (differs) {
        mismatch[i] = 1;
        atomicAdd(&ctr->unresolved, 1);
    } else {
        resolved[i] = 1;
    }
}

// One wave per sorted position: compares the stored signature rows of position i and of
// position head_pos[i].  Equal: the position is settled; different: it is flagged and counted.
__global__ __launch_bounds__(kThreads) void verify_stored_kernel(
    const uint16_t *__restrict__ sig, int S, const int32_t *__restrict__ vals,
    const int32_t *__restrict__ head_pos, int32_t *resolved, int n, int32_t *mismatch,
    Counters *ctr) {
    const int lane = threadIdx.x & 63;
    const int64_t gw = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    const int64_t total = (int64_t)gridDim.x * (kThreads / 64);
    const bool vec = (S % 8) == 0 && (reinterpret_cast<uintptr_t>(sig) % 16) == 0;
    for (int64_t i = gw; i < n; i += total) {
        if (resolved[i]) continue;  // wave-uniform
        const uint16_t *a = sig + (size_t)vals[i] * S;
        const uint16_t *b = sig + (size_t)vals[head_pos[i]] * S;
        bool diff = false;
        if (vec) {
            const uint4 *a4 = reinterpret_cast<const uint4 *>(a);
            const uint4 *b4 = reinterpret_cast<const uint4 *>(b);
            for (int j = lane; j < S / 8; j += 64) {
                const uint4 x = a4[j], y = b4[j];
                diff |= (x.x != y.x) | (x.y != y.y) | (x.z != y.z) | (x.w != y.w);
            }
        } else {
            for (int j = lane; j < S; j += 64) diff |= a[j] != b[j];
        }
        settle(__ballot(diff) != 0ull, (int)i, resolved, mismatch, ctr);
    }
}

// Compares the walk vectors that cfgzip_signatures kept for position i and for position
// head_pos[i], for the pairs whose tokens have the same image row: idx[row] is onto, so sig
// equal <=> w equal.  One thread per position, 16 bytes at a time (the padding behind a
// vector is zero on both sides).  A store that does not belong to this (V, S) or has
// overflowed is reported and nothing is compared.
struct StoreVerifyArgs {
    Tables T;
    WalkStoreView store;
    int32_t V, S, n;
    const int32_t *vals;
    const int32_t *head_pos;
    int32_t *resolved;
    int32_t *mismatch;
    Counters *ctr;
};

__device__ __forceinline__ bool walk_store_usable(const StoreVerifyArgs &a, uint32_t stride) {
    const WalkStore hdr = *a.store.header;
    return hdr.magic == kWalkStoreMagic && hdr.V == a.V && hdr.S == a.S && hdr.stride == stride &&
           !hdr.overflow;
}

__device__ __forceinline__ void verify_store_same_row(const StoreVerifyArgs &a, int block) {
    const uint32_t stride = walk_store_stride(a.S);
    if (!walk_store_usable(a, stride)) {
        if (block == 0 && threadIdx.x == 0) a.ctr->store_unusable = 1;
        return;
    }
    const int i = block * (int)blockDim.x + threadIdx.x;
    if (i >= a.n || a.resolved[i]) return;
    const int32_t ta = a.vals[i], tb = a.vals[a.head_pos[i]];
    const uint32_t ra = min((uint32_t)a.store.wrow[ta], 256u), rb = min((uint32_t)a.store.wrow[tb], 256u);
    if (ra != rb) return;  // left to verify_store_other_row
    const uint32_t cnt = min((uint32_t)a.T.nimg[ra], stride);
    const uint4 *wa = reinterpret_cast<const uint4 *>(a.store.wvec + (size_t)ta * stride);
    const uint4 *wb = reinterpret_cast<const uint4 *>(a.store.wvec + (size_t)tb * stride);
    const uint32_t n16 = (cnt + 7u) / 8u;
    bool diff = false;
    constexpr int kAhead = 4;  // independent 16-byte loads in flight per side
    for (uint32_t k0 = 0; k0 < n16; k0 += kAhead) {
        uint4 x[kAhead], y[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const uint32_t k = min(k0 + u, n16 - 1);  // repeats the last one past the end
            x[u] = wa[k];
            y[u] = wb[k];
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u)
            diff |= (x[u].x != y[u].x) | (x[u].y != y[u].y) | (x[u].z != y[u].z) | (x[u].w != y[u].w);
    }
    if (diff) {
        a.mismatch[i] = 1;
        atomicAdd(&a.ctr->unresolved, 1);
    } else {
        a.resolved[i] = 1;
    }
}

// The pairs whose tokens have different image rows (neighbours at the border between two
// first bytes inside a segment): sig[q] = w[idx[row][q]] has to be compared for every q.  A
// workgroup of 16 waves looks at 64 consecutive positions; every wave finds the same list of
// such pairs and takes every 16th of it, staging the two vectors in LDS.
constexpr int kStoreVerifyThreads = 1024;
__device__ __forceinline__ void verify_store_other_row(
    const StoreVerifyArgs &a, int block, uint16_t (*staged)[2][kWalkStoreMaxStride]) {
    const uint32_t stride = walk_store_stride(a.S);
    if (!walk_store_usable(a, stride)) return;  // reported by the same-row part
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int S = a.S;
    const int i = block * 64 + lane;
    const bool todo = i < a.n && !a.resolved[i];
    int32_t ta = 0, tb = 0;
    uint32_t ra = 256, rb = 256;
    if (todo) {
        ta = a.vals[i];
        tb = a.vals[a.head_pos[i]];
        ra = min((uint32_t)a.store.wrow[ta], 256u);
        rb = min((uint32_t)a.store.wrow[tb], 256u);
    }
    uint64_t list = __ballot(todo && ra != rb);  // same-row pairs settle in the other kernel
    uint16_t *la = staged[wave][0], *lb = staged[wave][1];
    for (int ordinal = 0; list; ++ordinal) {
        const int l = __ffsll((unsigned long long)list) - 1;
        list &= list - 1;
        if (ordinal % (kStoreVerifyThreads / 64) != wave) continue;  // wave-uniform
        const int32_t sa = __shfl(ta, l, 64), sb = __shfl(tb, l, 64);
        const uint32_t qa = __shfl(ra, l, 64), qb = __shfl(rb, l, 64);
        const uint32_t na = min((uint32_t)a.T.nimg[qa], stride), nb = min((uint32_t)a.T.nimg[qb], stride);
        {
            // lanes 0..31 copy vector a, lanes 32..63 vector b, 16 bytes each (stride <= 256 entries)
            const uint32_t half = lane & 31;
            const uint16_t *src = a.store.wvec + (size_t)(lane < 32 ? sa : sb) * stride;
            if (half * 8 < stride)
                reinterpret_cast<uint4 *>(lane < 32 ? la : lb)[half] =
                    reinterpret_cast<const uint4 *>(src)[half];
        }
        const uint16_t *ia = a.T.idx + (size_t)qa * S, *ib = a.T.idx + (size_t)qb * S;
        bool d = false;
        if ((S % 8) == 0) {
            for (int q0 = lane * 8; q0 < S; q0 += 512) {
                const uint4 xa = *reinterpret_cast<const uint4 *>(ia + q0);
                const uint4 xb = *reinterpret_cast<const uint4 *>(ib + q0);
                const uint32_t ja[8] = {xa.x & 0xFFFFu, xa.x >> 16, xa.y & 0xFFFFu, xa.y >> 16,
                                        xa.z & 0xFFFFu, xa.z >> 16, xa.w & 0xFFFFu, xa.w >> 16};
                const uint32_t jb[8] = {xb.x & 0xFFFFu, xb.x >> 16, xb.y & 0xFFFFu, xb.y >> 16,
                                        xb.z & 0xFFFFu, xb.z >> 16, xb.w & 0xFFFFu, xb.w >> 16};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    d |= (ja[e] < na ? la[ja[e]] : 0xFFFFu) != (jb[e] < nb ? lb[jb[e]] : 0xFFFFu);
            }
        } else {
            for (int q = lane; q < S; q += 64) {
                const uint32_t ja = ia[q], jb = ib[q];
                d |= (ja < na ? la[ja] : 0xFFFFu) != (jb < nb ? lb[jb] : 0xFFFFu);
            }
        }
        settle(__ballot(d) != 0ull, block * 64 + l, a.resolved, a.mismatch, a.ctr);
    }
}

// Both parts in one launch (they settle disjoint positions): the first `same_row_blocks`
// workgroups take one position per thread, the rest 64 positions per workgroup.
__global__ __launch_bounds__(kStoreVerifyThreads) void verify_store_kernel(StoreVerifyArgs a,
                                                                           int same_row_blocks) {
    __shared__ uint16_t staged[kStoreVerifyThreads / 64][2][kWalkStoreMaxStride];
    if ((int)blockIdx.x < same_row_blocks) verify_store_same_row(a, blockIdx.x);
    else verify_store_other_row(a, blockIdx.x - same_row_blocks, staged);
}

// Signatures of two walked batch slots, compared without materialising either: directly on w
// when both byte strings start with the same byte (idx[row] is onto, so sig equal <=> w
// equal), else through sig[q] = w[idx[row][q]] for every q.  One wave; returns whether any
// entry differs (wave-uniform).
__device__ __forceinline__ bool slots_differ(const Batch &B, const Tables &T, int S,
                                             const uint16_t *w, int sm, int sh) {
    const int lane = threadIdx.x & 63;
    const int rm = B.row[sm], rh = B.row[sh];
    const uint16_t *wm = w + B.wstart[sm], *wh = w + B.wstart[sh];
    bool diff = false;
    if (rm == rh) {
        const int cnt = B.cnt[sm];
        for (int j = lane; j < cnt; j += 64) diff |= wm[j] != wh[j];
    } else if ((S % 8) == 0) {
        const uint4 *im = reinterpret_cast<const uint4 *>(T.idx + (size_t)rm * S);
        const uint4 *ih = reinterpret_cast<const uint4 *>(T.idx + (size_t)rh * S);
        for (int v = lane; v < S / 8; v += 64) {
            const uint4 x = im[v], y = ih[v];
            diff |= wm[x.x & 0xFFFFu] != wh[y.x & 0xFFFFu];
            diff |= wm[x.x >> 16] != wh[y.x >> 16];
            diff |= wm[x.y & 0xFFFFu] != wh[y.y & 0xFFFFu];
            diff |= wm[x.y >> 16] != wh[y.y >> 16];
            diff |= wm[x.z & 0xFFFFu] != wh[y.z & 0xFFFFu];
            diff |= wm[x.z >> 16] != wh[y.z >> 16];
            diff |= wm[x.w & 0xFFFFu] != wh[y.w & 0xFFFFu];
            diff |= wm[x.w >> 16] != wh[y.w >> 16];
        }
    } else {
        const uint16_t *im = T.idx + (size_t)rm * S, *ih = T.idx + (size_t)rh * S;
        for (int q = lane; q < S; q += 64) diff |= wm[im[q]] != wh[ih[q]];
    }
    return __ballot(diff) != 0ull;
}

constexpr int kMaxLdsWalkEntries = 72 * 1024;  // 144 KB of uint16; beyond that w lives in global memory
constexpr int kGlobalWalkGrid = 256;

struct RewalkArgs {
    Tables T;
    int32_t S, wcap, n;
    uint16_t *w_global;
    const uint8_t *tok_bytes;
    const int64_t *tok_off;
    const int32_t *vals;
    const int32_t *head_pos;
    int32_t *resolved;
    int32_t *mismatch;
    Counters *ctr;
};

// Chain links without stored signatures: a workgroup takes 63 consecutive sorted positions
// (plus the left neighbour of the first) at a time, walks every token that takes part in a
// link once, and compares neighbours.  Requires head_pos[i] == i - 1 for every unsettled i.
template <bool W_GLOBAL>
__global__ __launch_bounds__(kThreads) void verify_chain_rewalk_kernel(RewalkArgs a) {
    extern __shared__ __align__(16) uint16_t dyn_lds[];
    __shared__ Batch B;
    __shared__ uint8_t ldsb[kByteCap];
    uint16_t *w = W_GLOBAL ? a.w_global + (size_t)blockIdx.x * a.wcap : dyn_lds;
    constexpr int kPositions = kBatchTokens - 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = a.n;
    const int n_chunks = (n + kPositions - 1) / kPositions;
    for (int chunk = blockIdx.x; chunk < n_chunks; chunk += gridDim.x) {
        const int i_end = min(n, (chunk + 1) * kPositions);
        int icur = chunk * kPositions;
        while (icur < i_end) {  // workgroup-uniform
            __syncthreads();
            if (threadIdx.x < 64) {
                // lane l holds sorted position icur - 1 + l
                const int i = icur - 1 + lane;
                const bool in_range = i >= 0 && i < i_end;
                const bool member = in_range && lane >= 1 && !a.resolved[i];
                const bool pred = in_range && i + 1 < i_end && lane < 63 && !a.resolved[i + 1];
                int64_t beg = 0, len = -1;
                if (member || pred) {
                    const int32_t tok = a.vals[i];
                    beg = a.tok_off[tok];
                    len = a.tok_off[tok + 1] - beg;
                    if (len < 0) len = 0;
                }
                const int k = batch_fill(B, a.T, a.tok_bytes, beg, len, a.wcap, 2, 1);
                if (lane < k) B.aux[lane] = member ? 1 : 0;
            }
            __syncthreads();
            const int links = min(B.k - 1, i_end - icur);
            batch_stage_bytes(B, a.tok_bytes, ldsb);
            __syncthreads();
            batch_walk<false>(a.T, a.T.Tt, a.S, a.tok_bytes, B, ldsb, w);
            __syncthreads();
            for (int l = 1 + wave; l <= links; l += kThreads / 64) {
                if (!B.aux[l]) continue;  // wave-uniform
                settle(slots_differ(B, a.T, a.S, w, l, l - 1), icur + l - 1, a.resolved, a.mismatch,
                       a.ctr);
            }
            icur += links;
        }
    }
}

// Arbitrary pairs without stored signatures (collision rounds): a workgroup takes 32 sorted
// positions at a time; every unsettled position i and position head_pos[i] are walked and
// compared.
template <bool W_GLOBAL>
__global__ __launch_bounds__(kThreads) void verify_pairs_rewalk_kernel(RewalkArgs a) {
    extern __shared__ __align__(16) uint16_t dyn_lds[];
    __shared__ Batch B;
    __shared__ uint8_t ldsb[kByteCap];
    uint16_t *w = W_GLOBAL ? a.w_global + (size_t)blockIdx.x * a.wcap : dyn_lds;
    constexpr int kPairs = kBatchTokens / 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = a.n;
    const int n_chunks = (n + kPairs - 1) / kPairs;
    for (int chunk = blockIdx.x; chunk < n_chunks; chunk += gridDim.x) {
        const int i_end = min(n, (chunk + 1) * kPairs);
        int icur = chunk * kPairs;
        while (icur < i_end) {  // workgroup-uniform
            __syncthreads();
            if (threadIdx.x < 64) {
                // lanes 2p, 2p+1: sorted position icur + p and its candidate head
                const int i = icur + (lane >> 1);
                int64_t beg = 0, len = -1;
                if (i < i_end && !a.resolved[i]) {
                    const int32_t tok = (lane & 1) ? a.vals[a.head_pos[i]] : a.vals[i];
                    beg = a.tok_off[tok];
                    len = a.tok_off[tok + 1] - beg;
                    if (len < 0) len = 0;
                }
                const int k = batch_fill(B, a.T, a.tok_bytes, beg, len, a.wcap, 2, 2);
                if (lane < k) B.aux[lane] = len >= 0 ? 1 : 0;
            }
            __syncthreads();
            const int pairs = min(B.k / 2, i_end - icur);
            batch_stage_bytes(B, a.tok_bytes, ldsb);
            __syncthreads();
            batch_walk<false>(a.T, a.T.Tt, a.S, a.tok_bytes, B, ldsb, w);
            __syncthreads();
            for (int p = wave; p < pairs; p += kThreads / 64) {
                if (!B.aux[2 * p]) continue;  // wave-uniform
                settle(slots_differ(B, a.T, a.S, w, 2 * p, 2 * p + 1), icur + p, a.resolved,
                       a.mismatch, a.ctr);
            }
            icur += pairs;
        }
    }
}

// ---------------------------------------------------------------- collision rounds (rare)

// cand[i] = i if position i starts a chain (a segment start or a member that differs from
// its left neighbour), else 0 (max-scan input).
__global__ void chain_start_kernel(int n, const int32_t *__restrict__ seg_head,
                                   const int32_t *__restrict__ mismatch, int32_t *cand) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) cand[i] = (seg_head[i] == i || mismatch[i]) ? i : 0;
}

// Only chain starts take part in the rounds: the ones that are not segment starts are
// unsettled and first compared with their segment's start.
__global__ void rounds_init_kernel(int n, const int32_t *__restrict__ seg_head,
                                   const int32_t *__restrict__ mismatch, int32_t *head_pos,
                                   int32_t *resolved, Counters *ctr) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) ctr->unresolved = 0;
    if (i >= n) return;
    if (mismatch[i]) {
        resolved[i] = 0;
        head_pos[i] = seg_head[i];
    } else {
        resolved[i] = 1;
        if (seg_head[i] == i) head_pos[i] = i;
    }
}

__global__ void round_reset_kernel(int n, int32_t *next_head, Counters *ctr) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) ctr->unresolved = 0;
    if (i < n) next_head[i] = 0x7FFFFFFF;
}

__global__ void round_propose_kernel(int n, const int32_t *__restrict__ resolved,
                                     const int32_t *__restrict__ seg_head, int32_t *next_head) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && !resolved[i]) atomicMin(&next_head[seg_head[i]], i);
}

__global__ void round_assign_kernel(int n, int32_t *resolved, const int32_t *__restrict__ seg_head,
                                    const int32_t *__restrict__ next_head, int32_t *head_pos) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n || resolved[i]) return;
    const int32_t h = next_head[seg_head[i]];
    head_pos[i] = h;
    if (h == i) resolved[i] = 1;  // first unsettled chain start of its segment: a new class
}

// anchor[i] = sorted position that stands for the class of position i: the class of its
// chain start.  Also clears what the numbering kernels accumulate into.
__global__ void anchors_kernel(int n, const int32_t *__restrict__ chain_start,
                               const int32_t *__restrict__ head_pos, int32_t *anchor,
                               int32_t *min_id, uint64_t *rep_key, int32_t *is_head_token) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    anchor[i] = head_pos[chain_start[i]];
    min_id[i] = 0x7FFFFFFF;
    rep_key[i] = ~0ull;
    is_head_token[i] = 0;
}

// ---------------------------------------------------------------- numbering and representatives

// Per class (keyed by its anchor position): smallest token id and smallest (length, id).
// Sorted neighbours mostly share a class, so a wave first reduces over its lanes of equal
// anchor and issues one pair of atomics per distinct anchor.
__global__ __launch_bounds__(kThreads) void class_minima_kernel(
    int n, const int32_t *__restrict__ anchor, const int32_t *__restrict__ vals,
    const int64_t *__restrict__ tok_off, int32_t *min_id, uint64_t *rep_key) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool valid = i < n;
    int32_t a = -1;
    uint64_t packed = ~0ull;
    if (valid) {
        const int32_t tok = vals[i];
        a = anchor[i];
        int64_t len = tok_off[tok + 1] - tok_off[tok];
        if (len > 0x7FFFFFFF) len = 0x7FFFFFFF;
        if (len < 0) len = 0;
        packed = ((uint64_t)len << 32) | (uint32_t)tok;
    }
    uint64_t todo = __ballot(valid);
    const int lane = threadIdx.x & 63;
    while (todo) {
        const int leader = __ffsll((unsigned long long)todo) - 1;
        const int32_t a0 = __shfl(a, leader, 64);
        const bool mine = valid && a == a0;
        uint64_t m = mine ? packed : ~0ull;
        int32_t id = mine ? (int32_t)(packed & 0x7FFFFFFFull) : 0x7FFFFFFF;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint64_t o = __shfl_xor(m, off, 64);
            m = o < m ? o : m;
            id = min(id, __shfl_xor(id, off, 64));
        }
        if (lane == leader) {
            atomicMin(reinterpret_cast<unsigned long long *>(rep_key + a0), (unsigned long long)m);
            atomicMin(min_id + a0, id);
        }
        todo &= ~__ballot(mine);
    }
}

__global__ void mark_heads_kernel(int n, const int32_t *__restrict__ anchor,
                                  const int32_t *__restrict__ min_id, int32_t *is_head_token) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && anchor[i] == i) is_head_token[min_id[i]] = 1;
}

__global__ void assign_classes_kernel(int n, const int32_t *__restrict__ anchor,
                                      const int32_t *__restrict__ vals,
                                      const int32_t *__restrict__ min_id,
                                      const int32_t *__restrict__ id_of_head_token,
                                      const uint64_t *__restrict__ rep_key, const Counters *ctr,
                                      int32_t *class_of_token, int32_t *rep_of_class,
                                      int32_t *num_classes_dev) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0 && num_classes_dev) *num_classes_dev = ctr->num_classes;
    if (i >= n) return;
    const int32_t a = anchor[i];
    const int32_t k = id_of_head_token[min_id[a]];
    class_of_token[vals[i]] = k;
    if (a == i) rep_of_class[k] = (int32_t)(rep_key[i] & 0xFFFFFFFFull);
}

struct BuildWorkspace {
    void *sig_ws;
    uint64_t *keys[2];
    int32_t *vals[2];
    uint32_t *hist;
    int32_t *seg_head, *head_pos, *resolved, *mismatch, *next_head, *cand, *chain_start, *anchor;
    int32_t *min_id, *is_head_token, *id_of_head_token, *tile_tmp;
    uint64_t *rep_key;
    uint16_t *verify_w;  // walk vectors of the re-walk verification when they do not fit in LDS
    Counters *ctr;
    size_t bytes;
};

BuildWorkspace carve_build_ws(void *ws, int32_t V, int32_t S) {
    Carver c(ws);
    BuildWorkspace w;
    const size_t n = (size_t)V;
    const size_t nt = (size_t)ceil_div(V, kTile);
    w.sig_ws = c.take<char>(sig_workspace_bytes(0, S));
    w.keys[0] = c.take<uint64_t>(n);
    w.keys[1] = c.take<uint64_t>(n);
    w.vals[0] = c.take<int32_t>(n);
    w.vals[1] = c.take<int32_t>(n);
    w.hist = c.take<uint32_t>(nt * kBins);
    w.seg_head = c.take<int32_t>(n);
    w.head_pos = c.take<int32_t>(n);
    w.resolved = c.take<int32_t>(n);
    w.mismatch = c.take<int32_t>(n);
    w.next_head = c.take<int32_t>(n);
    w.cand = c.take<int32_t>(n);
    w.chain_start = c.take<int32_t>(n);
    w.anchor = c.take<int32_t>(n);
    w.min_id = c.take<int32_t>(n);
    w.is_head_token = c.take<int32_t>(n);
    w.id_of_head_token = c.take<int32_t>(n);
    w.tile_tmp = c.take<int32_t>(nt);
    w.rep_key = c.take<uint64_t>(n);
    w.verify_w = walk_cap_for(S) > kMaxLdsWalkEntries
                     ? c.take<uint16_t>((size_t)kGlobalWalkGrid * walk_cap_for(S))
                     : nullptr;
    w.ctr = c.take<Counters>(1);
    w.bytes = c.used;
    return w;
}

inline dim3 grid_for(int n) { return dim3((unsigned)ceil_div(n, kThreads)); }

template <typename Kern>
int launch_rewalk(Kern kern_lds, Kern kern_global, const RewalkArgs &a, int n_chunks,
                  hipStream_t stream) {
    if (a.wcap > kMaxLdsWalkEntries) {
        hipLaunchKernelGGL(kern_global, dim3((unsigned)std::min(n_chunks, kGlobalWalkGrid)),
                           dim3(kThreads), 0, stream, a);
    } else {
        const size_t dyn = (size_t)a.wcap * 2;
        if (dyn > 48 * 1024)
            CFGZIP_TRY(check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(kern_lds),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     (int)dyn)));
        hipLaunchKernelGGL(kern_lds, dim3((unsigned)n_chunks), dim3(kThreads), dyn, stream, a);
    }
    return check_launch();
}

}  // namespace
}  // namespace cfgzip

using namespace cfgzip;

extern "C" size_t cfgzip_build_classes_workspace_bytes(int32_t V, int32_t S) {
    if (V <= 0 || S <= 0 || S > 65536) return 0;
    return carve_build_ws(nullptr, V, S).bytes;
}

extern "C" int cfgzip_build_classes(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                                    const uint16_t *table, int32_t S, const uint16_t *sig,
                                    const uint64_t *hash, void *signatures_ws,
                                    int32_t *class_of_token,
                                    int32_t *rep_of_class, int32_t *num_classes_dev,
                                    int32_t *num_classes_host, int32_t *collisions_host, void *ws,
                                    size_t ws_bytes, void *stream_) {
    if (!tok_off || !hash || !class_of_token || !rep_of_class) return CFGZIP_E_INVALID;
    // without an automaton there is nothing to walk: the rows of `sig` are all there is
    if (!table && (!sig || signatures_ws)) return CFGZIP_E_INVALID;
    if (V <= 0 || S <= 0 || S > 65536) return CFGZIP_E_INVALID;
    if (!aligned_to(tok_off, 8) || !aligned_to(hash, 8) || !aligned_to(sig, 2) ||
        !aligned_to(table, 2) || !aligned_to(class_of_token, 4) || !aligned_to(rep_of_class, 4))
        return CFGZIP_E_INVALID;
    if (!ws || !aligned_to(ws, 256) || !aligned_to(signatures_ws, 256)) return CFGZIP_E_WORKSPACE;
    BuildWorkspace w = carve_build_ws(ws, V, S);
    if (ws_bytes < w.bytes) return CFGZIP_E_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int n = V;
    const int nb = (int)ceil_div(n, kTile);
    int n_cu = 256;
    {
        int dev = 0;
        CFGZIP_TRY(check_hip(hipGetDevice(&dev)));
        CFGZIP_TRY(check_hip(
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev)));
        if (n_cu <= 0) n_cu = 256;
    }

    // where the comparisons read signatures from
    enum { FROM_STORE, FROM_ROWS, FROM_REWALK } source =
        signatures_ws ? FROM_STORE : (sig ? FROM_ROWS : FROM_REWALK);
    Tables store_tables{};
    WalkStoreView store{};
    if (source == FROM_STORE) view_signature_workspace(signatures_ws, V, S, &store_tables, &store);
    RewalkArgs ra{};
    auto prepare_rewalk = [&]() -> int {
        CFGZIP_TRY(prepare_tables(table, S, 0, false, 0, w.sig_ws, &ra.T, nullptr, stream));
        ra.S = S;
        ra.wcap = walk_cap_for(S);
        ra.n = n;
        ra.w_global = w.verify_w;
        ra.tok_bytes = tok_bytes;
        ra.tok_off = tok_off;
        ra.resolved = w.resolved;
        ra.mismatch = w.mismatch;
        ra.ctr = w.ctr;
        return CFGZIP_OK;
    };
    // re-walking needs its own tables: enqueue them first (independent of the sort)
    if (source == FROM_REWALK) CFGZIP_TRY(prepare_rewalk());

    // 1. sort (hash bits, first byte) with the token id as value
    const int hash_bits = hash_bits_for(V);
    const uint64_t hash_mask = (1ull << hash_bits) - 1ull;
    const int passes = (hash_bits + 8) / kRadixBits;
    int cur = 0;
    for (int pass = 0; pass < passes; ++pass) {
        ScatterArgs sa{};
        sa.hash = hash;
        sa.tok_off = tok_off;
        sa.tok_bytes = tok_bytes;
        sa.keys_in = pass ? w.keys[cur ^ 1] : nullptr;
        sa.vals_in = pass ? w.vals[cur ^ 1] : nullptr;
        sa.keys_out = w.keys[cur];
        sa.vals_out = w.vals[cur];
        sa.hist = w.hist;
        sa.hash_mask = hash_mask;
        sa.n = n;
        sa.nb = nb;
        sa.shift = pass * kRadixBits;
        if (pass == 0) {
            hipLaunchKernelGGL(radix_hist_kernel<true>, dim3(nb), dim3(kThreads), 0, stream, hash,
                               tok_off, tok_bytes, nullptr, n, sa.shift, hash_mask, w.hist);
            CFGZIP_TRY(check_launch());
            hipLaunchKernelGGL(radix_scatter_kernel<true>, dim3(nb), dim3(kThreads), 0, stream, sa);
        } else {
            hipLaunchKernelGGL(radix_hist_kernel<false>, dim3(nb), dim3(kThreads), 0, stream, hash,
                               tok_off, tok_bytes, sa.keys_in, n, sa.shift, hash_mask, w.hist);
            CFGZIP_TRY(check_launch());
            hipLaunchKernelGGL(radix_scatter_kernel<false>, dim3(nb), dim3(kThreads), 0, stream, sa);
        }
        CFGZIP_TRY(check_launch());
        cur ^= 1;
    }
    const uint64_t *keys = w.keys[cur ^ 1];
    const int32_t *vals = w.vals[cur ^ 1];
    ra.vals = vals;
    ra.head_pos = w.head_pos;

    // 2. equal-hash segments, chain set-up
    auto set_up_chains = [&]() -> int {
        hipLaunchKernelGGL(segments_kernel, dim3(nb), dim3(kThreads), 0, stream, keys, n, w.seg_head,
                           w.head_pos, w.resolved, w.mismatch, w.min_id, w.rep_key, w.is_head_token,
                           w.ctr);
        return check_launch();
    };
    CFGZIP_TRY(set_up_chains());

    const int64_t wave_grid = ceil_div(std::min<int64_t>(n, (int64_t)n_cu * 32), kThreads / 64);
    StoreVerifyArgs sva{};
    sva.T = store_tables;
    sva.store = store;
    sva.V = V;
    sva.S = S;
    sva.n = n;
    sva.vals = vals;
    sva.head_pos = w.head_pos;
    sva.resolved = w.resolved;
    sva.mismatch = w.mismatch;
    sva.ctr = w.ctr;
    // compares every unsettled position i with position head_pos[i]
    auto verify_pairs = [&]() -> int {
        if (source == FROM_STORE) {
            const int same_row_blocks = (int)ceil_div(n, kStoreVerifyThreads);
            hipLaunchKernelGGL(verify_store_kernel,
                               dim3((unsigned)(same_row_blocks + ceil_div(n, 64))),
                               dim3(kStoreVerifyThreads), 0, stream, sva, same_row_blocks);
            return check_launch();
        }
        if (source == FROM_ROWS) {
            hipLaunchKernelGGL(verify_stored_kernel, dim3((unsigned)wave_grid), dim3(kThreads), 0,
                               stream, sig, S, vals, w.head_pos, w.resolved, n, w.mismatch, w.ctr);
            return check_launch();
        }
        return launch_rewalk(verify_pairs_rewalk_kernel<false>, verify_pairs_rewalk_kernel<true>, ra,
                             (int)ceil_div(n, kBatchTokens / 2), stream);
    };
    // the chain links: head_pos[i] == i - 1 for every unsettled i
    auto verify_links = [&]() -> int {
        if (source != FROM_REWALK) return verify_pairs();
        return launch_rewalk(verify_chain_rewalk_kernel<false>, verify_chain_rewalk_kernel<true>, ra,
                             (int)ceil_div(n, kBatchTokens - 1), stream);
    };
    // 4./5. class ids by ascending smallest member id, representatives
    auto number_classes = [&](const int32_t *anchor) -> int {
        hipLaunchKernelGGL(class_minima_kernel, grid_for(n), dim3(kThreads), 0, stream, n, anchor,
                           vals, tok_off, w.min_id, w.rep_key);
        CFGZIP_TRY(check_launch());
        hipLaunchKernelGGL(mark_heads_kernel, grid_for(n), dim3(kThreads), 0, stream, n, anchor,
                           w.min_id, w.is_head_token);
        CFGZIP_TRY(check_launch());
        CFGZIP_TRY((device_scan<false, false>(w.is_head_token, w.id_of_head_token, n, w.tile_tmp,
                                              &w.ctr->num_classes, stream)));
        hipLaunchKernelGGL(assign_classes_kernel, grid_for(n), dim3(kThreads), 0, stream, n, anchor,
                           vals, w.min_id, w.id_of_head_token, w.rep_key, w.ctr, class_of_token,
                           rep_of_class, num_classes_dev);
        return check_launch();
    };
    Counters host_ctr{};
    auto read_counters = [&]() -> int {
        CFGZIP_TRY(check_hip(hipMemcpyAsync(&host_ctr, w.ctr, sizeof(Counters),
                                            hipMemcpyDeviceToHost, stream)));
        return check_hip(hipStreamSynchronize(stream));
    };

    // 3. chain links; the numbering is enqueued right behind them on the assumption that no
    //    link differs (then the segments are the classes), and redone in the rare other case
    CFGZIP_TRY(verify_links());
    CFGZIP_TRY(number_classes(w.seg_head));
    CFGZIP_TRY(read_counters());
    if (source == FROM_STORE && host_ctr.store_unusable) {
        // the workspace did not hold this call's walk vectors (or they had overflowed): start
        // over from the chain set-up with the next source
        source = sig ? FROM_ROWS : FROM_REWALK;
        if (source == FROM_REWALK) CFGZIP_TRY(prepare_rewalk());
        CFGZIP_TRY(set_up_chains());
        CFGZIP_TRY(verify_links());
        CFGZIP_TRY(number_classes(w.seg_head));
        CFGZIP_TRY(read_counters());
    }
    const int32_t collisions = host_ctr.unresolved;

    if (collisions > 0) {
        hipLaunchKernelGGL(chain_start_kernel, grid_for(n), dim3(kThreads), 0, stream, n, w.seg_head,
                           w.mismatch, w.cand);
        CFGZIP_TRY(check_launch());
        CFGZIP_TRY((device_scan<true, true>(w.cand, w.chain_start, n, w.tile_tmp, nullptr, stream)));
        hipLaunchKernelGGL(rounds_init_kernel, grid_for(n), dim3(kThreads), 0, stream, n, w.seg_head,
                           w.mismatch, w.head_pos, w.resolved, w.ctr);
        CFGZIP_TRY(check_launch());
        CFGZIP_TRY(verify_pairs());
        CFGZIP_TRY(read_counters());
        int64_t rounds = 0;
        while (host_ctr.unresolved > 0) {
            if (++rounds > (int64_t)V) return CFGZIP_E_COLLISION;  // cannot happen: a round settles >= 1
            hipLaunchKernelGGL(round_reset_kernel, grid_for(n), dim3(kThreads), 0, stream, n,
                               w.next_head, w.ctr);
            CFGZIP_TRY(check_launch());
            hipLaunchKernelGGL(round_propose_kernel, grid_for(n), dim3(kThreads), 0, stream, n,
                               w.resolved, w.seg_head, w.next_head);
            CFGZIP_TRY(check_launch());
            hipLaunchKernelGGL(round_assign_kernel, grid_for(n), dim3(kThreads), 0, stream, n,
                               w.resolved, w.seg_head, w.next_head, w.head_pos);
            CFGZIP_TRY(check_launch());
            CFGZIP_TRY(verify_pairs());
            CFGZIP_TRY(read_counters());
        }
        hipLaunchKernelGGL(anchors_kernel, grid_for(n), dim3(kThreads), 0, stream, n, w.chain_start,
                           w.head_pos, w.anchor, w.min_id, w.rep_key, w.is_head_token);
        CFGZIP_TRY(check_launch());
        CFGZIP_TRY(number_classes(w.anchor));
        CFGZIP_TRY(read_counters());
    }
    if (num_classes_host) *num_classes_host = host_ctr.num_classes;
    if (collisions_host) *collisions_host = collisions;
    return CFGZIP_OK;
}
