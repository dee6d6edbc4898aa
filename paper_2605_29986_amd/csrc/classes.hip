// cfgzip_build_classes: group tokens with equal signature, number the classes
// and pick representatives (paper Section 3.1 "Pre-Computation").
//
// Pipeline (all on the device, eight launches when no hash collides):
//   1. keys: (low 32 or 40 bits of the hash, first byte of the token), and the digit counts of
//      the first sort pass per tile;
//   2. stable LSD radix sort of the keys with the token id as value, 10 bits per pass, one
//      launch per pass: a workgroup sums the counts of the earlier tiles itself, ranks its
//      tile by wave-level match-by-ballot, writes, and counts the next pass's digits per
//      destination tile on the way;
//   3. links: equal-hash segments; inside a segment tokens with the same first byte are
//      neighbours.  Every member is compared with its left neighbour (a chain: equality is
//      transitive).  Three sources, in order of preference: the walk vectors a preceding
//      cfgzip_signatures call left in its workspace (compared on the short vector w when both
//      tokens share the first byte, through the index tables otherwise - walk_device.hpp);
//      stored signature rows; or, with neither, both tokens are re-walked with the image walk
//      (a kernel of its own).  The same launch reduces, per segment, the smallest token id and
//      the smallest (byte length, token id);
//   4. if no link differs (no hash collision - the overwhelmingly common case), the segments
//      are the classes.  Otherwise every differing member starts a new chain and the chain
//      starts of a segment are matched against each other in rounds (the first unmatched one
//      becomes a class, the rest are compared with it) - exact for any hash that is a function
//      of the signature;
//   5. class id = rank of the class's smallest token id among all classes: the smallest ids
//      are marked in a bit vector over token ids, and every workgroup of the last kernel
//      ranks by prefix popcounts of that vector held in LDS;
//   6. representative = min over members of (byte length, token id).
// The host waits once, for the class count and the number of differing links.

#include <algorithm>

#include "common.hpp"
#include "walk_device.hpp"

namespace cfgzip {
namespace {

constexpr int kThreads = 256;             // link, minima and marking kernels: one position per thread
constexpr int kItems = 8;
constexpr int kTile = kThreads * kItems;  // items per workgroup in the scan kernels
constexpr int kSortThreads = 1024;
constexpr int kSortItems = 2;  // measured: 8 -> 156 us, 4 -> 133, 3 -> 128, 2 -> 130, 1 -> 151 per build of 152 K tokens (2 is best on the smaller ones)
constexpr int kSortTile = kSortThreads * kSortItems;  // keys per workgroup in the sort
constexpr int kRadixBits = 10;
constexpr int kBins = 1 << kRadixBits;
static_assert(kSortThreads == kBins, "one thread per bin in the sort kernels");
constexpr int kAggBits = 12;
constexpr int kAggSlots = 1 << kAggBits;
constexpr uint32_t kAggEmpty = 0xFFFFFFFFu;
constexpr int kListedParts = 4;  // waves that share one listed cross-row link
constexpr int kAssignThreads = 512;
constexpr int kAssignItems = 4;
constexpr int kAssignTile = kAssignThreads * kAssignItems;
// token-id bit vector and its word prefix sums fit in LDS up to this many words (V <= 262,144)
constexpr int kRankLdsWords = 8192;
// Hash bits that take part in the sort, above the 8 bits of the first byte.  Two classes that
// agree in these bits only cost a pass through the collision rounds (C classes: about
// C^2 / 2^(bits+1) such pairs), so small vocabularies sort 32 bits (4 passes) and large ones 40.
constexpr int32_t kLargeVocabulary = 1 << 18;
inline int hash_bits_for(int32_t V) { return V > kLargeVocabulary ? 40 : 32; }

struct Counters {
    int32_t unresolved;
    int32_t num_classes;
    int32_t store_state;  // of the walk store handed in: 0 usable, 1 not this call's, 2 overflowed
    int32_t other_rows;   // links between tokens of different image rows, listed for the kernel after
    int32_t pad[4];
};
constexpr int kStoreForeign = 1, kStoreOverflowed = 2;

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

struct KeysArgs {
    const uint64_t *hash;
    const int64_t *tok_off;
    const uint8_t *tok_bytes;
    uint64_t *keys_out;
    uint32_t *hist;  // [passes][nb][kBins]
    uint64_t hash_mask;
    int n, nb, passes;
    // what the later kernels accumulate into, reset here
    int32_t *min_id;
    uint64_t *rep_key;
    uint32_t *head_bits;
    int n_words;
    Counters *ctr;
};

// Forms the keys, counts the first pass's digits per tile, clears the later passes' counts and
// everything the numbering accumulates into.
__global__ __launch_bounds__(kSortThreads) void keys_kernel(KeysArgs a) {
    __shared__ uint32_t bins[kBins];
    bins[threadIdx.x] = 0;
    for (int p = 1; p < a.passes; ++p)
        a.hist[((size_t)p * a.nb + blockIdx.x) * kBins + threadIdx.x] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        a.ctr->unresolved = 0;
        a.ctr->num_classes = 0;
        a.ctr->store_state = 0;
        a.ctr->other_rows = 0;
    }
    __syncthreads();
    const int base = blockIdx.x * kSortTile;
#pragma unroll
    for (int j = 0; j < kSortItems; ++j) {
        const int idx = base + j * kSortThreads + threadIdx.x;
        if (idx < a.n) {
            const uint64_t key = sort_key(a.hash, a.tok_off, a.tok_bytes, idx, a.hash_mask);
            a.keys_out[idx] = key;
            atomicAdd(&bins[(uint32_t)key & (kBins - 1)], 1u);
            a.min_id[idx] = 0x7FFFFFFF;
            a.rep_key[idx] = ~0ull;
        }
    }
    if (threadIdx.x < kSortTile / 32) {
        const int w = base / 32 + threadIdx.x;
        if (w < a.n_words) a.head_bits[w] = 0;
    }
    __syncthreads();
    a.hist[(size_t)blockIdx.x * kBins + threadIdx.x] = bins[threadIdx.x];
}

struct PassArgs {
    const uint64_t *keys_in;
    const int32_t *vals_in;  // first pass: the value of position i is i
    uint64_t *keys_out;
    int32_t *vals_out;
    const uint32_t *hist;  // [nb][kBins] digit counts of this pass per input tile
    uint32_t *hist_next;   // the same for the next pass, counted here; null in the last pass
    int n, nb, shift;
};

// One stable pass.  A wave owns a contiguous chunk of the tile and visits it 64 keys at a
// time, so (wave, visit, lane) order is index order.
template <bool FIRST>
__global__ __launch_bounds__(kSortThreads) void radix_pass_kernel(PassArgs a) {
    constexpr int kWaves = kSortThreads / 64;
    __shared__ uint16_t wave_count[kWaves][kBins];  // a wave holds 512 keys: counts fit 16 bits
    __shared__ uint32_t bin_base[kBins];
    __shared__ uint32_t wave_tot[kWaves];
    // counts of the next pass's (destination tile, digit) pairs, gathered per workgroup before
    // they go to memory: a class with many members puts thousands of keys on one counter
    __shared__ uint32_t agg_tag[kAggSlots];
    __shared__ uint32_t agg_cnt[kAggSlots];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < kWaves * kBins / 2; i += kSortThreads)
        reinterpret_cast<uint32_t *>(&wave_count[0][0])[i] = 0;
    for (int i = threadIdx.x; i < kAggSlots; i += kSortThreads) {
        agg_tag[i] = kAggEmpty;
        agg_cnt[i] = 0;
    }

    // the keys first: their loads overlap the count sums below
    const int chunk = blockIdx.x * kSortTile + wave * (64 * kSortItems);
    uint64_t key[kSortItems];
    int32_t val[kSortItems];
#pragma unroll
    for (int j = 0; j < kSortItems; ++j) {
        const int idx = chunk + j * 64 + lane;
        key[j] = idx < a.n ? a.keys_in[idx] : 0ull;
        val[j] = FIRST ? idx : (idx < a.n ? a.vals_in[idx] : 0);
    }

    // first output position of this tile's keys with digit d:
    //   keys with a smaller digit anywhere + keys with digit d in earlier tiles
    {
        const int d = threadIdx.x;
        uint32_t tot = 0, before = 0;
        constexpr int kAhead = 8;  // independent loads in flight: the loop is latency-bound
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
        bin_base[d] = prefix + (uint32_t)incl - tot + before;
    }

    volatile uint16_t *my_count = wave_count[wave];
    uint32_t rank[kSortItems];
    uint64_t peers[kSortItems];  // lanes of this visit with the same digit
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < kSortItems; ++j) {
        const bool valid = chunk + j * 64 + lane < a.n;
        const uint32_t d = (uint32_t)(key[j] >> a.shift) & (kBins - 1);
        uint64_t p = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < kRadixBits; ++bit) {
            const bool one = (d >> bit) & 1u;
            const uint64_t bm = __ballot(one);
            p &= one ? bm : ~bm;
        }
        peers[j] = p;
        rank[j] = 0;
        if (valid) {
            const uint32_t before = my_count[d];
            const uint32_t r = (uint32_t)__popcll(p & lt_mask);
            rank[j] = before + r;
            if (r == 0) my_count[d] = (uint16_t)(before + (uint32_t)__popcll(p));
        }
    }
    __syncthreads();
    {
        const int d = threadIdx.x;
        uint32_t run = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const uint32_t c = wave_count[w][d];
            wave_count[w][d] = (uint16_t)run;  // keys of this tile with digit d in earlier waves
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kSortItems; ++j) {
        const bool valid = chunk + j * 64 + lane < a.n;
        const uint32_t d = (uint32_t)(key[j] >> a.shift) & (kBins - 1);
        uint32_t pos = valid ? bin_base[d] + wave_count[wave][d] + rank[j] : 0u;
        const bool ok = valid && pos < (uint32_t)a.n;  // always, with consistent counts; stay in bounds
        if (ok) {
            a.keys_out[pos] = key[j];
            a.vals_out[pos] = val[j];
        }
        if (a.hist_next) {  // the same for the whole grid
            // which counter of the next pass this key adds to
            const uint32_t v = (pos / kSortTile) * kBins +
                               ((uint32_t)(key[j] >> (a.shift + kRadixBits)) & (kBins - 1));
            // lanes with the same digit sit at consecutive positions; those that also share the
            // first such lane's counter are counted by it
            const uint64_t p = peers[j];
            const int first = p ? __ffsll((unsigned long long)p) - 1 : lane;
            const uint32_t v_first = __shfl(v, first, 64);
            const bool with_first = ok && v == v_first;
            const uint64_t group = __ballot(with_first) & p;
            uint32_t add = 0;
            if (ok) add = lane == first ? (uint32_t)__popcll(group) : (with_first ? 0u : 1u);
            if (add) {
                const uint32_t s = (v * 2654435761u) >> (32 - kAggBits);
                const uint32_t old = atomicCAS(&agg_tag[s], kAggEmpty, v);
                if (old == kAggEmpty || old == v) atomicAdd(&agg_cnt[s], add);
                else atomicAdd(&a.hist_next[v], add);  // the slot belongs to another counter
            }
        }
    }
    if (a.hist_next) {
        __syncthreads();
        for (int s = threadIdx.x; s < kAggSlots; s += kSortThreads)
            if (agg_cnt[s]) atomicAdd(&a.hist_next[agg_tag[s]], agg_cnt[s]);
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

// ---------------------------------------------------------------- comparing two tokens' signatures

__device__ __forceinline__ uint64_t hash_part(uint64_t key) { return key >> 8; }

// What the comparisons read when the walk vectors of cfgzip_signatures are at hand.
struct StoreSource {
    Tables T;
    WalkStoreView store;
    int32_t V, S;
};

// 0 if the store holds this call's vectors, else why not.
__device__ __forceinline__ int walk_store_state(const StoreSource &s) {
    const WalkStore hdr = *s.store.header;
    if (hdr.magic != kWalkStoreMagic || hdr.V != s.V || hdr.S != s.S ||
        hdr.stride != walk_store_stride(s.S))
        return kStoreForeign;
    return hdr.overflow ? kStoreOverflowed : 0;
}

// Image row of a token as the store has it (256: the empty token, whose signature is the
// identity and whose vector is not kept).
__device__ __forceinline__ uint32_t store_row(const StoreSource &s, int32_t tok) {
    return min(walk_row_of(s.store.wrow[tok]), 256u);
}

// Two tokens with the same image row `row` < 256: idx[row] is onto, so their signatures are
// equal iff their walk vectors are.  One thread, 16 bytes at a time (the padding behind a
// vector is zero on both sides).
__device__ __forceinline__ bool store_same_row_differ(const StoreSource &s, int32_t ta, int32_t tb,
                                                      uint32_t row) {
    const uint32_t stride = walk_store_stride(s.S);
    const uint4 *wa = reinterpret_cast<const uint4 *>(s.store.wvec + (size_t)ta * stride);
    const uint4 *wb = reinterpret_cast<const uint4 *>(s.store.wvec + (size_t)tb * stride);
    const uint32_t n16 = min(walk_units_of(s.store.wrow[ta]), stride / 8u);  // the same for both: one row
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
    return diff;
}

// Two tokens with different image rows (neighbours at the border between two first bytes inside
// a segment, or an empty token): sig[q] = w[idx[row][q]] has to be compared for every q; the
// empty token's signature is sig[q] = q.  One wave; both vectors are staged in the wave's LDS
// buffers la, lb (kWalkStoreMaxStride entries each).  Returns whether any entry differs
// (wave-uniform).  `part` of `parts`: the wave looks only at every parts-th stretch of 512 states,
// starting with stretch `part` (several waves then share one pair; S a multiple of 8 only).
__device__ __forceinline__ bool store_other_row_differ(const StoreSource &s, int32_t ta, int32_t tb,
                                                       uint32_t ra, uint32_t rb, uint16_t *la,
                                                       uint16_t *lb, int part = 0, int parts = 1) {
    const int lane = threadIdx.x & 63;
    const int S = s.S;
    const uint32_t stride = walk_store_stride(S);
    const bool ida = ra == 256u, idb = rb == 256u;
    if (ida && idb) return false;
    if (part * 512 >= S) return false;  // nothing of this pair falls to this wave
    // positions in a kept vector are below the row's image size, which is at most the stride in a
    // store that has not overflowed; the bound keeps a corrupt index inside the staged vector
    const uint32_t na = stride, nb = stride;
    {
        // lanes 0..31 copy vector a, lanes 32..63 vector b, 16 bytes each (stride <= 256 entries)
        const uint32_t half = lane & 31;
        const bool second = lane >= 32;
        const uint16_t *src = s.store.wvec + (size_t)(second ? tb : ta) * stride;
        if (half * 8 < stride && !(second ? idb : ida))
            reinterpret_cast<uint4 *>(second ? lb : la)[half] = reinterpret_cast<const uint4 *>(src)[half];
    }
    // the staged vectors are read below as 16-bit entries by other lanes of this wave
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint16_t *ia = s.T.idx + (size_t)ra * S, *ib = s.T.idx + (size_t)rb * S;
    bool d = false;
    auto entry_a = [&](uint32_t q, uint32_t j) -> uint32_t { return ida ? q : (j < na ? la[j] : 0xFFFFu); };
    auto entry_b = [&](uint32_t q, uint32_t j) -> uint32_t { return idb ? q : (j < nb ? lb[j] : 0xFFFFu); };
    if ((S % 8) == 0) {
        // 16 bytes of each index row per lane and step (the identity row is not read)
        const uint4 zero = make_uint4(0, 0, 0, 0);
        constexpr int kAhead = 2;
        for (int q0 = lane * 8 + 512 * part; q0 < S; q0 += 512 * parts * kAhead) {
            uint4 xa[kAhead], xb[kAhead];
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int q = q0 + 512 * parts * u;
                xa[u] = (!ida && q < S) ? *reinterpret_cast<const uint4 *>(ia + q) : zero;
                xb[u] = (!idb && q < S) ? *reinterpret_cast<const uint4 *>(ib + q) : zero;
            }
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int q = q0 + 512 * parts * u;
                if (q >= S) continue;
                const uint32_t ja[8] = {xa[u].x & 0xFFFFu, xa[u].x >> 16, xa[u].y & 0xFFFFu, xa[u].y >> 16,
                                        xa[u].z & 0xFFFFu, xa[u].z >> 16, xa[u].w & 0xFFFFu, xa[u].w >> 16};
                const uint32_t jb[8] = {xb[u].x & 0xFFFFu, xb[u].x >> 16, xb[u].y & 0xFFFFu, xb[u].y >> 16,
                                        xb[u].z & 0xFFFFu, xb[u].z >> 16, xb[u].w & 0xFFFFu, xb[u].w >> 16};
#pragma unroll
                for (int e = 0; e < 8; ++e) d |= entry_a(q + e, ja[e]) != entry_b(q + e, jb[e]);
            }
        }
    } else {
        for (int q = lane; q < S; q += 64)
            d |= entry_a(q, ida ? 0u : (uint32_t)ia[q]) != entry_b(q, idb ? 0u : (uint32_t)ib[q]);
    }
    const bool any = __ballot(d) != 0ull;
    __builtin_amdgcn_wave_barrier();  // the next pair restages la, lb
    return any;
}

// Stored signature rows of two tokens, one wave.
__device__ __forceinline__ bool rows_differ(const uint16_t *__restrict__ sig, int S, bool vec,
                                            int32_t ta, int32_t tb) {
    const int lane = threadIdx.x & 63;
    const uint16_t *a = sig + (size_t)ta * S;
    const uint16_t *b = sig + (size_t)tb * S;
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
    return __ballot(diff) != 0ull;
}

// ---------------------------------------------------------------- per-class minima

// Per class (keyed by its anchor position): smallest token id and smallest (length, id).
// Sorted neighbours mostly share a class, so a wave first reduces over its lanes of equal
// anchor and issues one pair of atomics per distinct anchor.  Called by whole waves.
// `ends` (or null): instead of issuing the atomics for the anchors of its first and of its last
// lane, the wave leaves them there (entries 2 * wave and 2 * wave + 1) for flush_wave_ends, which
// merges them over the workgroup: a class with many members spans whole workgroups, and thousands
// of atomics on one address are served one after the other.
struct WaveEnd {
    int32_t anchor;  // -1: nothing
    int32_t id;
    uint64_t packed;
};

__device__ __forceinline__ void wave_class_minima(bool valid, int32_t anchor, int32_t tok, int64_t len,
                                                  int32_t *min_id, uint64_t *rep_key,
                                                  WaveEnd *ends = nullptr) {
    if (len > 0x7FFFFFFF) len = 0x7FFFFFFF;
    if (len < 0) len = 0;
    const uint64_t packed = valid ? ((uint64_t)len << 32) | (uint32_t)tok : ~0ull;
    const int32_t a = valid ? anchor : -1;
    uint64_t todo = __ballot(valid);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // anchors do not decrease along the sorted positions: the first and the last valid lane hold
    // the two anchors that may continue in the neighbouring waves
    const int first_lane = todo ? __ffsll((unsigned long long)todo) - 1 : 0;
    const int last_lane = todo ? 63 - __clzll((unsigned long long)todo) : 0;
    const int32_t a_first = __shfl(a, first_lane, 64), a_last = __shfl(a, last_lane, 64);
    if (ends && lane < 2) ends[2 * wave + lane].anchor = -1;
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
            if (ends && (a0 == a_first || a0 == a_last)) {
                WaveEnd &e = ends[2 * wave + (a0 == a_first ? 0 : 1)];
                e.anchor = a0;
                e.id = id;
                e.packed = m;
            } else {
                atomicMin(reinterpret_cast<unsigned long long *>(rep_key + a0), (unsigned long long)m);
                atomicMin(min_id + a0, id);
            }
        }
        todo &= ~__ballot(mine);
    }
}

// After a __syncthreads(): one thread goes through the waves' end entries in order, merges
// neighbours with the same anchor and issues the atomics.
__device__ __forceinline__ void flush_wave_ends(const WaveEnd *ends, int n_entries, int32_t *min_id,
                                                uint64_t *rep_key) {
    if (threadIdx.x != 0) return;
    int32_t cur = -1, id = 0x7FFFFFFF;
    uint64_t m = ~0ull;
    for (int e = 0; e <= n_entries; ++e) {
        const int32_t an = e < n_entries ? ends[e].anchor : -2;
        if (e < n_entries && an == -1) continue;
        if (an != cur) {
            if (cur >= 0) {
                atomicMin(reinterpret_cast<unsigned long long *>(rep_key + cur), (unsigned long long)m);
                atomicMin(min_id + cur, id);
            }
            cur = an;
            id = 0x7FFFFFFF;
            m = ~0ull;
        }
        if (e < n_entries) {
            id = min(id, ends[e].id);
            m = ends[e].packed < m ? ends[e].packed : m;
        }
    }
}

// ---------------------------------------------------------------- links

enum : int { SRC_STORE = 0, SRC_ROWS = 1, SRC_NONE = 2 };

struct LinkArgs {
    const uint64_t *keys;  // sorted
    const int32_t *vals;
    int n;
    const int64_t *tok_off;
    int32_t *seg_head, *head_pos, *resolved, *mismatch, *min_id;
    uint64_t *rep_key;
    Counters *ctr;
    StoreSource store;    // SRC_STORE
    int4 *other_list;     // SRC_STORE: (sorted position, its token, its left neighbour's token, the two image rows) of the links that cross two image rows
    const uint16_t *sig;  // SRC_ROWS: [V][S]
    int S;
};

// One sorted position per thread.  seg_head[i] = first sorted position with the same hash bits
// as position i.  Chain set-up: a segment start is its own head and settled; every other
// position is compared with its left neighbour (SRC_NONE: left unsettled for the re-walk kernel
// that follows).  Also reduces the per-segment minima.
template <int SRC>
__global__ __launch_bounds__(kThreads) void link_kernel(LinkArgs a) {
    __shared__ int32_t wave_tot[kThreads / 64];
    __shared__ int32_t carry_s;
    __shared__ WaveEnd ends[2 * (kThreads / 64)];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile0 = blockIdx.x * kThreads;
    const int n = a.n;
    const uint64_t *keys = a.keys;
    const int i = tile0 + threadIdx.x;
    const bool in = i < n;
    bool start = false;
    int32_t ta = 0, tb = 0;
    int64_t len = 0;
    if (in) {
        start = i == 0 || hash_part(keys[i]) != hash_part(keys[i - 1]);
        ta = a.vals[i];
        tb = i > 0 ? a.vals[i - 1] : ta;
        len = a.tok_off[ta + 1] - a.tok_off[ta];
    }

    // SRC_STORE: is the store this call's?  The same answer in every workgroup.
    int store_state = 0;
    if (SRC == SRC_STORE) {
        store_state = walk_store_state(a.store);
        if (store_state && blockIdx.x == 0 && threadIdx.x == 0) a.ctr->store_state = store_state;
    }
    const bool verify = in && !start && SRC != SRC_NONE && store_state == 0;
    // Links inside one image row: the two walk vectors are compared by eight lanes together,
    // 16 bytes each per round, so that a wave's reads fall into whole cache lines; the wave takes
    // its 64 positions eight at a time and keeps all eight pairs' reads in flight.  The first
    // round is asked for before the rows are known (every token has a slot of `stride` entries;
    // what turns out not to be wanted is not looked at), so that it overlaps the row reads and
    // the search below.
    const uint32_t stride = SRC == SRC_STORE ? walk_store_stride(a.S) : 8u;
    const uint32_t sub = lane & 7, group = lane >> 3;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    uint16_t wa_row = 0, wb_row = 0;
    uint4 x0[8], y0[8];
    if (SRC == SRC_STORE) {
        if (verify) {
            wa_row = a.store.store.wrow[ta];
            wb_row = a.store.store.wrow[tb];
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int owner = k * 8 + (int)group;
            const bool want = __shfl((int)verify, owner, 64) != 0 && sub < stride / 8u;
            const int32_t pa = __shfl(ta, owner, 64), pb = __shfl(tb, owner, 64);
            x0[k] = want ? reinterpret_cast<const uint4 *>(a.store.store.wvec + (size_t)pa * stride)[sub] : zero;
            y0[k] = want ? reinterpret_cast<const uint4 *>(a.store.store.wvec + (size_t)pb * stride)[sub] : zero;
        }
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
    int32_t inc = start ? i : -1;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int32_t o = __shfl_up(inc, off, 64);
        if (lane >= off) inc = max(inc, o);
    }
    if (lane == 63) wave_tot[wave] = inc;

    __syncthreads();
    int32_t seg = carry_s;
    for (int w = 0; w < wave; ++w) seg = max(seg, wave_tot[w]);
    seg = max(seg, inc);

    // the per-segment minima go out now: their atomics are under way while the vectors are compared
    wave_class_minima(in, seg, ta, len, a.min_id, a.rep_key, ends);
    __syncthreads();
    flush_wave_ends(ends, 2 * (kThreads / 64), a.min_id, a.rep_key);

    bool differs = false;
    uint32_t ra = 0, rb = 0;
    if (SRC == SRC_STORE) {
        if (verify) {
            ra = min(walk_row_of(wa_row), 256u);
            rb = min(walk_row_of(wb_row), 256u);
        }
        const bool same = verify && ra == rb && ra != 256u;
        const uint32_t n16 = same ? min(walk_units_of(wa_row), stride / 8u) : 0u;
        uint32_t dmask = 0;  // bit k: this lane saw a difference in the pair of position 8 k + group
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const uint32_t pn = __shfl(n16, k * 8 + (int)group, 64);
            if (sub < pn && ((x0[k].x != y0[k].x) | (x0[k].y != y0[k].y) | (x0[k].z != y0[k].z) |
                             (x0[k].w != y0[k].w)))
                dmask |= 1u << k;
        }
        for (uint32_t r = 1; r < kWalkStoreMaxStride / 64; ++r) {
            if (__ballot(n16 > 8u * r) == 0ull) break;  // nobody's vector is that long
            uint4 x[8], y[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int owner = k * 8 + (int)group;
                const uint32_t pn = __shfl(n16, owner, 64);
                const int32_t pa = __shfl(ta, owner, 64), pb = __shfl(tb, owner, 64);
                const uint32_t u = sub + 8u * r;
                const bool ok = u < pn;
                x[k] = ok ? reinterpret_cast<const uint4 *>(a.store.store.wvec + (size_t)pa * stride)[u] : zero;
                y[k] = ok ? reinterpret_cast<const uint4 *>(a.store.store.wvec + (size_t)pb * stride)[u] : zero;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if ((x[k].x != y[k].x) | (x[k].y != y[k].y) | (x[k].z != y[k].z) | (x[k].w != y[k].w))
                    dmask |= 1u << k;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const uint64_t dm = __ballot((dmask >> k) & 1u);
            // position 8 k + j was looked at by the eight lanes of group j
            if ((lane >> 3) == k) differs = differs || ((dm >> (8 * (lane & 7))) & 0xFFull) != 0ull;
        }
    }
    bool listed = false;
    if (SRC == SRC_STORE) {
        // Links between different image rows cost a pass over all S states each and bunch up
        // where small classes sit: they are listed, and the next launch spreads them over the
        // chip, a wave per link.  One append per wave.
        listed = verify && ra != rb;  // two empty tokens (both rows 256) are equal as they are
        const uint64_t lm = __ballot(listed);
        if (lm) {
            int32_t at = 0;
            if (lane == 0) at = atomicAdd(&a.ctr->other_rows, (int)__popcll(lm));
            at = __shfl(at, 0, 64);
            if (listed)
                a.other_list[at + __popcll(lm & ((1ull << lane) - 1ull))] = make_int4(i, ta, tb, (int)(ra | (rb << 16)));
        }
    } else if (SRC == SRC_ROWS) {
        // a wave takes its own positions four at a time: more row reads in flight
        const bool vec = (a.S % 8) == 0 && (reinterpret_cast<uintptr_t>(a.sig) % 16) == 0;
        uint64_t todo = __ballot(verify);
        bool mine = false;
        while (todo) {
            int ls[4];
            int32_t xa[4], xb[4];
            int cnt = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (todo) {
                    ls[u] = __ffsll((unsigned long long)todo) - 1;
                    todo &= todo - 1;
                    ++cnt;
                } else {
                    ls[u] = ls[0];  // repeats the first pair
                }
                xa[u] = __shfl(ta, ls[u], 64);
                xb[u] = __shfl(tb, ls[u], 64);
            }
            bool d[4] = {false, false, false, false};
            if (vec) {
                for (int j = lane; j < a.S / 8; j += 64) {
                    uint4 x[4], y[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        x[u] = reinterpret_cast<const uint4 *>(a.sig + (size_t)xa[u] * a.S)[j];
                        y[u] = reinterpret_cast<const uint4 *>(a.sig + (size_t)xb[u] * a.S)[j];
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        d[u] |= (x[u].x != y[u].x) | (x[u].y != y[u].y) | (x[u].z != y[u].z) |
                                (x[u].w != y[u].w);
                }
            } else {
                for (int j = lane; j < a.S; j += 64)
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        d[u] |= a.sig[(size_t)xa[u] * a.S + j] != a.sig[(size_t)xb[u] * a.S + j];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool any = __ballot(d[u]) != 0ull;
                if (u < cnt && lane == ls[u]) mine = any;
            }
        }
        differs = mine;
    }

    if (in) {
        a.seg_head[i] = seg;
        a.head_pos[i] = start ? i : i - 1;
        // (a listed link counts as settled until a wave of the next launch finds a difference)
        a.resolved[i] = (start || (verify && !differs)) ? 1 : 0;
        a.mismatch[i] = differs ? 1 : 0;
    }
    const uint64_t dm = __ballot(differs);
    if (dm && lane == 0) atomicAdd(&a.ctr->unresolved, (int)__popcll(dm));
}

// ---------------------------------------------------------------- verification of arbitrary pairs
// (the collision rounds: position i against position head_pos[i], for every unsettled i)

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
    const int64_t gw = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    const int64_t total = (int64_t)gridDim.x * (kThreads / 64);
    const bool vec = (S % 8) == 0 && (reinterpret_cast<uintptr_t>(sig) % 16) == 0;
    for (int64_t i = gw; i < n; i += total) {
        if (resolved[i]) continue;  // wave-uniform
        settle(rows_differ(sig, S, vec, vals[i], vals[head_pos[i]]), (int)i, resolved, mismatch, ctr);
    }
}

struct StoreVerifyArgs {
    StoreSource src;
    int32_t n;
    const int32_t *vals;
    const int32_t *head_pos;
    int32_t *resolved;
    int32_t *mismatch;
    Counters *ctr;
};

// A workgroup looks at 256 positions.  Pairs with the same image row are compared by their own
// thread; for the others, wave w takes the positions of its own 64 lanes one after the other (so
// which wave settles a position never depends on what another wave has settled meanwhile).
__global__ __launch_bounds__(kThreads) void verify_store_kernel(StoreVerifyArgs a) {
    __shared__ __align__(16) uint16_t staged[kThreads / 64][2][kWalkStoreMaxStride];
    const int state = walk_store_state(a.src);
    if (state) {
        if (blockIdx.x == 0 && threadIdx.x == 0) a.ctr->store_state = state;
        return;
    }
    const int wave = threadIdx.x >> 6;
    const int i = blockIdx.x * kThreads + threadIdx.x;
    const bool todo = i < a.n && !a.resolved[i];
    int32_t ta = 0, tb = 0;
    uint32_t ra = 256, rb = 256;
    if (todo) {
        ta = a.vals[i];
        tb = a.vals[a.head_pos[i]];
        ra = store_row(a.src, ta);
        rb = store_row(a.src, tb);
    }
    const bool same = todo && ra == rb && ra != 256u;
    if (same) {
        if (store_same_row_differ(a.src, ta, tb, ra)) {
            a.mismatch[i] = 1;
            atomicAdd(&a.ctr->unresolved, 1);
        } else {
            a.resolved[i] = 1;
        }
    }
    uint64_t list = __ballot(todo && !same);
    while (list) {
        const int l = __ffsll((unsigned long long)list) - 1;
        list &= list - 1;
        const bool d = store_other_row_differ(a.src, __shfl(ta, l, 64), __shfl(tb, l, 64),
                                              __shfl(ra, l, 64), __shfl(rb, l, 64), staged[wave][0],
                                              staged[wave][1]);
        settle(d, blockIdx.x * kThreads + wave * 64 + l, a.resolved, a.mismatch, a.ctr);
    }
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
                               int32_t *min_id, uint64_t *rep_key, uint32_t *head_bits, int n_words) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_words) head_bits[i] = 0;
    if (i >= n) return;
    anchor[i] = head_pos[chain_start[i]];
    min_id[i] = 0x7FFFFFFF;
    rep_key[i] = ~0ull;
}

// The same clearing alone, before the links are taken again from another source.
__global__ void reset_numbering_kernel(int n, int32_t *min_id, uint64_t *rep_key, uint32_t *head_bits,
                                       int n_words, Counters *ctr) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        ctr->unresolved = 0;
        ctr->num_classes = 0;
        ctr->store_state = 0;
        ctr->other_rows = 0;
    }
    if (i < n_words) head_bits[i] = 0;
    if (i >= n) return;
    min_id[i] = 0x7FFFFFFF;
    rep_key[i] = ~0ull;
}

// ---------------------------------------------------------------- numbering and representatives

// The per-class minima over arbitrary anchors (after collision rounds; without collisions the
// link kernel has done it over the segments).
__global__ __launch_bounds__(kThreads) void class_minima_kernel(
    int n, const int32_t *__restrict__ anchor, const int32_t *__restrict__ vals,
    const int64_t *__restrict__ tok_off, int32_t *min_id, uint64_t *rep_key) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool valid = i < n;
    int32_t a = 0, tok = 0;
    int64_t len = 0;
    if (valid) {
        tok = vals[i];
        a = anchor[i];
        len = tok_off[tok + 1] - tok_off[tok];
    }
    wave_class_minima(valid, a, tok, len, min_id, rep_key);
}

// head_bits bit t = token t is the smallest member of its class (the first `mark_blocks`
// workgroups, a sorted position per thread).  The other workgroups settle the links that the
// link kernel listed: a wave per link, striding over the list.
struct MarkArgs {
    int n, mark_blocks;
    const int32_t *anchor;
    const int32_t *min_id;
    uint32_t *head_bits;
    // listed links (null list: none)
    const int4 *other_list;
    StoreSource store;
    int32_t *resolved, *mismatch;
    Counters *ctr;
};

__global__ __launch_bounds__(kThreads) void mark_heads_kernel(MarkArgs a) {
    __shared__ __align__(16) uint16_t staged[kThreads / 64][2][kWalkStoreMaxStride];
    if ((int)blockIdx.x < a.mark_blocks) {
        const int i = blockIdx.x * kThreads + threadIdx.x;
        if (i < a.n && a.anchor[i] == i) {
            const uint32_t m = (uint32_t)a.min_id[i];
            if (m < (uint32_t)a.n) atomicOr(&a.head_bits[m >> 5], 1u << (m & 31));  // always: a class has a member
        }
        return;
    }
    if (!a.other_list) return;
    // kListedParts waves share a link when the signatures are long (S a multiple of 8 only)
    const int wave = threadIdx.x >> 6;
    const int parts = (a.store.S % 8) == 0 ? kListedParts : 1;
    const int count = min(a.ctr->other_rows, a.n);
    const int waves = ((int)gridDim.x - a.mark_blocks) * (kThreads / 64);
    for (int64_t e = ((int)blockIdx.x - a.mark_blocks) * (kThreads / 64) + wave; e < (int64_t)count * parts;
         e += waves) {
        const int4 link = a.other_list[e / parts];
        const int i = link.x;
        if (i <= 0 || i >= a.n) continue;  // never listed; stay in bounds
        const bool d = store_other_row_differ(a.store, link.y, link.z, (uint32_t)link.w & 0xFFFFu,
                                              (uint32_t)link.w >> 16, staged[wave][0], staged[wave][1],
                                              (int)(e % parts), parts);
        if (d && (threadIdx.x & 63) == 0) {  // the first wave to find a difference counts it
            a.resolved[i] = 0;
            if (atomicExch(&a.mismatch[i], 1) == 0) atomicAdd(&a.ctr->unresolved, 1);
        }
    }
}

__global__ void popcount_words_kernel(const uint32_t *__restrict__ bits, int n_words, int32_t *out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_words) out[i] = __popc(bits[i]);
}

struct AssignArgs {
    int n, n_words;
    const int32_t *anchor;
    const int32_t *vals;
    const int32_t *min_id;
    const uint32_t *head_bits;
    const int32_t *word_prefix;  // !LDS_RANK: set bits before each word of head_bits
    const uint64_t *rep_key;
    Counters *ctr;
    Counters *host_ctr;  // pinned host memory: the counters as they stand when this kernel ends
    int32_t *class_of_token, *rep_of_class, *num_classes_dev;
};

// The host reads the counters from pinned memory after waiting for the stream: every kernel that
// counts has finished before this one starts, so one thread copies them over.
__device__ __forceinline__ void publish_counters(const AssignArgs &a, int32_t num_classes) {
    if (!a.host_ctr) return;
    a.host_ctr->unresolved = a.ctr->unresolved;
    a.host_ctr->store_state = a.ctr->store_state;
    a.host_ctr->other_rows = a.ctr->other_rows;
    a.host_ctr->num_classes = num_classes;
}

// Class id of a class = number of classes whose smallest token id is smaller = set bits of
// head_bits below its own.  LDS_RANK: every workgroup copies the bit vector into LDS and sums
// its words' popcounts there (a redundant scan per workgroup, no launch of its own).
template <bool LDS_RANK>
__global__ __launch_bounds__(kAssignThreads) void assign_classes_kernel(AssignArgs a) {
    extern __shared__ uint32_t rank_lds[];  // LDS_RANK: [n_words] bits, [n_words] prefix
    __shared__ uint32_t wave_tot[kAssignThreads / 64];
    uint32_t *bits = rank_lds, *prefix = rank_lds + a.n_words;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (LDS_RANK) {
        for (int w = threadIdx.x; w < a.n_words; w += kAssignThreads) bits[w] = a.head_bits[w];
        __syncthreads();
        // thread t owns the words [t * per, (t + 1) * per)
        const int per = (a.n_words + kAssignThreads - 1) / kAssignThreads;
        const int w0 = min(a.n_words, (int)threadIdx.x * per), w1 = min(a.n_words, w0 + per);
        uint32_t sum = 0;
        for (int w = w0; w < w1; ++w) sum += __popc(bits[w]);
        const uint32_t incl = (uint32_t)wave_inclusive_sum((int)sum);
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        uint32_t run = incl - sum;
        for (int w = 0; w < wave; ++w) run += wave_tot[w];
        for (int w = w0; w < w1; ++w) {
            prefix[w] = run;
            run += __popc(bits[w]);
        }
        if (blockIdx.x == 0 && threadIdx.x == kAssignThreads - 1) {
            a.ctr->num_classes = (int32_t)run;  // the last thread's running sum is the total
            if (a.num_classes_dev) *a.num_classes_dev = (int32_t)run;
            publish_counters(a, (int32_t)run);
        }
        __syncthreads();
    } else if (blockIdx.x == 0 && threadIdx.x == 0) {
        const int32_t total = a.ctr->num_classes;  // written by the scan before this launch
        if (a.num_classes_dev) *a.num_classes_dev = total;
        publish_counters(a, total);
    }
    const int base = blockIdx.x * kAssignTile;
    int32_t anc[kAssignItems], tok[kAssignItems];
#pragma unroll
    for (int j = 0; j < kAssignItems; ++j) {
        const int i = base + j * kAssignThreads + threadIdx.x;
        anc[j] = i < a.n ? a.anchor[i] : 0;
        tok[j] = i < a.n ? a.vals[i] : 0;
    }
    uint32_t m[kAssignItems];
#pragma unroll
    for (int j = 0; j < kAssignItems; ++j) m[j] = (uint32_t)a.min_id[anc[j]];
#pragma unroll
    for (int j = 0; j < kAssignItems; ++j) {
        const int i = base + j * kAssignThreads + threadIdx.x;
        if (i >= a.n) continue;
        if (m[j] >= (uint32_t)a.n) continue;  // cannot happen: every anchor has a member; stay in bounds
        const uint32_t w = m[j] >> 5, below = (1u << (m[j] & 31)) - 1u;
        const int32_t k = LDS_RANK ? (int32_t)(prefix[w] + __popc(bits[w] & below))
                                   : a.word_prefix[w] + __popc(a.head_bits[w] & below);
        a.class_of_token[tok[j]] = k;
        if (anc[j] == i) a.rep_of_class[k] = (int32_t)(a.rep_key[i] & 0xFFFFFFFFull);
    }
}

struct BuildWorkspace {
    void *sig_ws;
    uint64_t *keys[2];
    int32_t *vals[2];
    uint32_t *hist;
    int32_t *seg_head, *head_pos, *resolved, *mismatch, *next_head, *cand, *chain_start, *anchor;
    int32_t *min_id, *word_prefix, *tile_tmp;
    int4 *other_list;
    uint32_t *head_bits;
    uint64_t *rep_key;
    uint16_t *verify_w;  // walk vectors of the re-walk verification when they do not fit in LDS
    Counters *ctr;
    size_t bytes;
};

inline int sort_passes_for(int32_t V) { return (hash_bits_for(V) + 8 + kRadixBits - 1) / kRadixBits; }

BuildWorkspace carve_build_ws(void *ws, int32_t V, int32_t S) {
    Carver c(ws);
    BuildWorkspace w;
    const size_t n = (size_t)V;
    const size_t nb = (size_t)ceil_div(V, kSortTile);
    const size_t nt = (size_t)ceil_div(V, kTile);
    const size_t n_words = (size_t)words_for(V);
    w.sig_ws = c.take<char>(sig_workspace_bytes(0, S));
    w.keys[0] = c.take<uint64_t>(n);
    w.keys[1] = c.take<uint64_t>(n);
    w.vals[0] = c.take<int32_t>(n);
    w.vals[1] = c.take<int32_t>(n);
    w.hist = c.take<uint32_t>((size_t)sort_passes_for(V) * nb * kBins);
    w.seg_head = c.take<int32_t>(n);
    w.head_pos = c.take<int32_t>(n);
    w.resolved = c.take<int32_t>(n);
    w.mismatch = c.take<int32_t>(n);
    w.next_head = c.take<int32_t>(n);
    w.cand = c.take<int32_t>(n);
    w.chain_start = c.take<int32_t>(n);
    w.anchor = c.take<int32_t>(n);
    w.min_id = c.take<int32_t>(n);
    w.other_list = c.take<int4>(n);
    w.word_prefix = c.take<int32_t>(n_words);
    w.head_bits = c.take<uint32_t>(n_words);
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

// One small pinned host buffer per host thread (a thread runs one build at a time: the call
// waits for its stream), allocated at the thread's first build and kept until the thread ends.
struct PinnedCounters {
    Counters *ptr = nullptr;
    ~PinnedCounters() {
        if (ptr) (void)hipHostFree(ptr);
    }
};
int pinned_counters(Counters **out) {
    static thread_local PinnedCounters slot;
    if (!slot.ptr) {
        void *p = nullptr;
        CFGZIP_TRY(check_hip(hipHostMalloc(&p, sizeof(Counters), hipHostMallocDefault)));
        slot.ptr = static_cast<Counters *>(p);
    }
    *out = slot.ptr;
    return CFGZIP_OK;
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
    Counters *pinned = nullptr;
    CFGZIP_TRY(pinned_counters(&pinned));
    const int n = V;
    const int nb = (int)ceil_div(n, kSortTile);
    const int n_words = (int)words_for(n);

    // where the comparisons read signatures from
    enum { FROM_STORE, FROM_ROWS, FROM_REWALK } source =
        signatures_ws ? FROM_STORE : (sig ? FROM_ROWS : FROM_REWALK);
    StoreSource store_src{};
    store_src.V = V;
    store_src.S = S;
    if (source == FROM_STORE) view_signature_workspace(signatures_ws, V, S, &store_src.T, &store_src.store);
    RewalkArgs ra{};
    // tables_from_store: the signature call's tables are good although its walk vectors are not
    auto prepare_rewalk = [&](bool tables_from_store) -> int {
        if (tables_from_store) ra.T = store_src.T;
        else CFGZIP_TRY(prepare_tables(table, S, 0, false, 0, w.sig_ws, &ra.T, nullptr, stream));
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
    if (source == FROM_REWALK) CFGZIP_TRY(prepare_rewalk(false));

    // 1. keys and the first pass's digit counts
    const int hash_bits = hash_bits_for(V);
    const int passes = sort_passes_for(V);
    {
        KeysArgs ka{};
        ka.hash = hash;
        ka.tok_off = tok_off;
        ka.tok_bytes = tok_bytes;
        ka.keys_out = w.keys[0];
        ka.hist = w.hist;
        ka.hash_mask = (1ull << hash_bits) - 1ull;
        ka.n = n;
        ka.nb = nb;
        ka.passes = passes;
        ka.min_id = w.min_id;
        ka.rep_key = w.rep_key;
        ka.head_bits = w.head_bits;
        ka.n_words = n_words;
        ka.ctr = w.ctr;
        hipLaunchKernelGGL(keys_kernel, dim3(nb), dim3(kSortThreads), 0, stream, ka);
        CFGZIP_TRY(check_launch());
    }
    // 2. sort (hash bits, first byte) with the token id as value
    int cur = 0;
    for (int pass = 0; pass < passes; ++pass, cur ^= 1) {
        PassArgs pa{};
        pa.keys_in = w.keys[cur];
        pa.vals_in = w.vals[cur];
        pa.keys_out = w.keys[cur ^ 1];
        pa.vals_out = w.vals[cur ^ 1];
        pa.hist = w.hist + (size_t)pass * nb * kBins;
        pa.hist_next = pass + 1 < passes ? w.hist + (size_t)(pass + 1) * nb * kBins : nullptr;
        pa.n = n;
        pa.nb = nb;
        pa.shift = pass * kRadixBits;
        if (pass == 0) hipLaunchKernelGGL(radix_pass_kernel<true>, dim3(nb), dim3(kSortThreads), 0, stream, pa);
        else hipLaunchKernelGGL(radix_pass_kernel<false>, dim3(nb), dim3(kSortThreads), 0, stream, pa);
        CFGZIP_TRY(check_launch());
    }
    const uint64_t *keys = w.keys[cur];
    const int32_t *vals = w.vals[cur];
    ra.vals = vals;
    ra.head_pos = w.head_pos;

    // 3. equal-hash segments, chain links, per-segment minima
    auto link = [&]() -> int {
        LinkArgs la{};
        la.keys = keys;
        la.vals = vals;
        la.n = n;
        la.tok_off = tok_off;
        la.seg_head = w.seg_head;
        la.head_pos = w.head_pos;
        la.resolved = w.resolved;
        la.mismatch = w.mismatch;
        la.min_id = w.min_id;
        la.rep_key = w.rep_key;
        la.ctr = w.ctr;
        la.store = store_src;
        la.other_list = w.other_list;
        la.sig = sig;
        la.S = S;
        if (source == FROM_STORE) hipLaunchKernelGGL(link_kernel<SRC_STORE>, grid_for(n), dim3(kThreads), 0, stream, la);
        else if (source == FROM_ROWS) hipLaunchKernelGGL(link_kernel<SRC_ROWS>, grid_for(n), dim3(kThreads), 0, stream, la);
        else hipLaunchKernelGGL(link_kernel<SRC_NONE>, grid_for(n), dim3(kThreads), 0, stream, la);
        CFGZIP_TRY(check_launch());
        if (source == FROM_REWALK)  // the chain links: head_pos[i] == i - 1 for every unsettled i
            return launch_rewalk(verify_chain_rewalk_kernel<false>, verify_chain_rewalk_kernel<true>, ra,
                                 (int)ceil_div(n, kBatchTokens - 1), stream);
        return CFGZIP_OK;
    };
    // compares every unsettled position i with position head_pos[i] (collision rounds)
    auto verify_pairs = [&]() -> int {
        if (source == FROM_STORE) {
            StoreVerifyArgs sva{};
            sva.src = store_src;
            sva.n = n;
            sva.vals = vals;
            sva.head_pos = w.head_pos;
            sva.resolved = w.resolved;
            sva.mismatch = w.mismatch;
            sva.ctr = w.ctr;
            hipLaunchKernelGGL(verify_store_kernel, grid_for(n), dim3(kThreads), 0, stream, sva);
            return check_launch();
        }
        if (source == FROM_ROWS) {
            int n_cu = 256;
            int dev = 0;
            CFGZIP_TRY(check_hip(hipGetDevice(&dev)));
            CFGZIP_TRY(check_hip(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev)));
            if (n_cu <= 0) n_cu = 256;
            const int64_t wave_grid = ceil_div(std::min<int64_t>(n, (int64_t)n_cu * 32), kThreads / 64);
            hipLaunchKernelGGL(verify_stored_kernel, dim3((unsigned)wave_grid), dim3(kThreads), 0,
                               stream, sig, S, vals, w.head_pos, w.resolved, n, w.mismatch, w.ctr);
            return check_launch();
        }
        return launch_rewalk(verify_pairs_rewalk_kernel<false>, verify_pairs_rewalk_kernel<true>, ra,
                             (int)ceil_div(n, kBatchTokens / 2), stream);
    };
    // 5./6. class ids by ascending smallest member id, representatives
    // `settle_listed`: right after the link kernel, the same launch also compares the links it listed
    auto number_classes = [&](const int32_t *anchor, bool settle_listed) -> int {
        MarkArgs ma{};
        ma.n = n;
        ma.mark_blocks = (int)ceil_div(n, kThreads);
        ma.anchor = anchor;
        ma.min_id = w.min_id;
        ma.head_bits = w.head_bits;
        int verify_blocks = 0;
        if (settle_listed && source == FROM_STORE) {
            ma.other_list = w.other_list;
            ma.store = store_src;
            ma.resolved = w.resolved;
            ma.mismatch = w.mismatch;
            ma.ctr = w.ctr;
            verify_blocks = (int)std::min<int64_t>(ceil_div(n, kThreads / 64), 2048);
        }
        hipLaunchKernelGGL(mark_heads_kernel, dim3((unsigned)(ma.mark_blocks + verify_blocks)),
                           dim3(kThreads), 0, stream, ma);
        CFGZIP_TRY(check_launch());
        AssignArgs aa{};
        aa.n = n;
        aa.n_words = n_words;
        aa.anchor = anchor;
        aa.vals = vals;
        aa.min_id = w.min_id;
        aa.head_bits = w.head_bits;
        aa.word_prefix = w.word_prefix;
        aa.rep_key = w.rep_key;
        aa.ctr = w.ctr;
        aa.host_ctr = pinned;
        aa.class_of_token = class_of_token;
        aa.rep_of_class = rep_of_class;
        aa.num_classes_dev = num_classes_dev;
        const unsigned grid = (unsigned)ceil_div(n, kAssignTile);
        if (n_words <= kRankLdsWords) {
            const size_t dyn = (size_t)n_words * 8;
            auto kern = assign_classes_kernel<true>;
            if (dyn > 48 * 1024)
                CFGZIP_TRY(check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                                         (int)dyn)));
            hipLaunchKernelGGL(kern, dim3(grid), dim3(kAssignThreads), dyn, stream, aa);
        } else {
            // large vocabularies: the word prefix sums by a scan of their own (w.cand is free here)
            hipLaunchKernelGGL(popcount_words_kernel, grid_for(n_words), dim3(kThreads), 0, stream,
                               w.head_bits, n_words, w.cand);
            CFGZIP_TRY(check_launch());
            CFGZIP_TRY((device_scan<false, false>(w.cand, w.word_prefix, n_words, w.tile_tmp,
                                                  &w.ctr->num_classes, stream)));
            hipLaunchKernelGGL(assign_classes_kernel<false>, dim3(grid), dim3(kAssignThreads), 0, stream, aa);
        }
        return check_launch();
    };
    Counters host_ctr{};
    // after a numbering: its last kernel has left the counters in pinned memory
    auto read_counters = [&]() -> int {
        CFGZIP_TRY(check_hip(hipStreamSynchronize(stream)));
        host_ctr = *pinned;
        return CFGZIP_OK;
    };
    // in the collision rounds, between numberings: a copy
    auto copy_counters = [&]() -> int {
        CFGZIP_TRY(check_hip(hipMemcpyAsync(&host_ctr, w.ctr, sizeof(Counters),
                                            hipMemcpyDeviceToHost, stream)));
        return check_hip(hipStreamSynchronize(stream));
    };

    // 4. the numbering is enqueued right behind the links on the assumption that none differs
    //    (then the segments are the classes), and redone in the rare other case
    CFGZIP_TRY(link());
    CFGZIP_TRY(number_classes(w.seg_head, true));
    CFGZIP_TRY(read_counters());
    if (source == FROM_STORE && host_ctr.store_state) {
        // the workspace did not hold this call's walk vectors (or they had overflowed): take the
        // links again from the next source; an overflowed store still has this call's tables
        const bool tables_ok = host_ctr.store_state == kStoreOverflowed;
        source = sig ? FROM_ROWS : FROM_REWALK;
        if (source == FROM_REWALK) CFGZIP_TRY(prepare_rewalk(tables_ok));
        hipLaunchKernelGGL(reset_numbering_kernel, grid_for(std::max(n, n_words)), dim3(kThreads), 0, stream,
                           n, w.min_id, w.rep_key, w.head_bits, n_words, w.ctr);
        CFGZIP_TRY(check_launch());
        CFGZIP_TRY(link());
        CFGZIP_TRY(number_classes(w.seg_head, true));
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
        CFGZIP_TRY(copy_counters());
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
            CFGZIP_TRY(copy_counters());
        }
        hipLaunchKernelGGL(anchors_kernel, grid_for(std::max(n, n_words)), dim3(kThreads), 0, stream, n,
                           w.chain_start, w.head_pos, w.anchor, w.min_id, w.rep_key, w.head_bits, n_words);
        CFGZIP_TRY(check_launch());
        hipLaunchKernelGGL(class_minima_kernel, grid_for(n), dim3(kThreads), 0, stream, n, w.anchor, vals,
                           tok_off, w.min_id, w.rep_key);
        CFGZIP_TRY(check_launch());
        CFGZIP_TRY(number_classes(w.anchor, false));
        CFGZIP_TRY(read_counters());
    }
    if (num_classes_host) *num_classes_host = host_ctr.num_classes;
    if (collisions_host) *collisions_host = collisions;
    return CFGZIP_OK;
}
