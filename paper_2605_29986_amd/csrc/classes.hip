// cfgzip_build_classes: group tokens with equal signature, number the classes
// and pick representatives (paper Section 3.1 "Pre-Computation").
//
// Pipeline (all on the device):
//   1. stable LSD radix sort of (hash, token id), 8 bits per pass;
//   2. equal-hash segments; every member's signature is compared with its
//      segment head's (read from sig, or re-walked when sig is not stored);
//   3. members that differ from their head (hash collisions) are split off in
//      rounds: the first unresolved member of a segment becomes a new head and
//      the rest are compared with it, until nothing is unresolved - exact for
//      any hash that is a function of the signature;
//   4. class id = rank of the class head's token id among all heads (heads are
//      the smallest ids of their classes because the sort is stable), by a
//      prefix sum over token ids;
//   5. representative = min over members of (byte length, token id).

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

// ---------------------------------------------------------------- radix sort

__global__ __launch_bounds__(kThreads) void radix_hist_kernel(const uint64_t *__restrict__ keys,
                                                              int n, int shift, uint32_t *hist,
                                                              int nb) {
    __shared__ uint32_t bins[kBins];
    bins[threadIdx.x] = 0;
    __syncthreads();
    const int base = blockIdx.x * kTile;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int idx = base + j * kThreads + threadIdx.x;
        if (idx < n) atomicAdd(&bins[(uint32_t)(keys[idx] >> shift) & (kBins - 1)], 1u);
    }
    __syncthreads();
    hist[(size_t)threadIdx.x * nb + blockIdx.x] = bins[threadIdx.x];
}

// In-place exclusive sum scan of `n` uint32 by one workgroup of 1024 threads.
__global__ __launch_bounds__(1024) void scan_u32_single_block_kernel(uint32_t *data, int n) {
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t carry_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int base = 0; base < n; base += 1024) {
        const int idx = base + threadIdx.x;
        const uint32_t v = idx < n ? data[idx] : 0u;
        uint32_t inc = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            uint32_t o = __shfl_up(inc, off, 64);
            if (lane >= off) inc += o;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        uint32_t wave_prefix = 0;
        for (int w = 0; w < wave; ++w) wave_prefix += wave_tot[w];
        const uint32_t carry = carry_s;
        if (idx < n) data[idx] = carry + wave_prefix + inc - v;
        __syncthreads();
        if (threadIdx.x == 1023) carry_s = carry + wave_prefix + inc;
        __syncthreads();
    }
}

// Stable scatter of one pass.  A wave owns a contiguous chunk of the tile and
// visits it 64 keys at a time, so (wave, visit, lane) order is index order.
__global__ __launch_bounds__(kThreads) void radix_scatter_kernel(
    const uint64_t *__restrict__ keys_in, const int32_t *__restrict__ vals_in,
    uint64_t *__restrict__ keys_out, int32_t *__restrict__ vals_out, int n, int shift,
    const uint32_t *__restrict__ hist_scanned, int nb) {
    __shared__ uint32_t wave_count[kThreads / 64][kBins];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < (kThreads / 64) * kBins; i += kThreads)
        (&wave_count[0][0])[i] = 0;
    __syncthreads();

    volatile uint32_t *my_count = wave_count[wave];
    const int chunk = blockIdx.x * kTile + wave * (64 * kItems);
    uint64_t key[kItems];
    uint32_t rank[kItems];
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int idx = chunk + j * 64 + lane;
        const bool valid = idx < n;
        key[j] = valid ? keys_in[idx] : 0ull;
        const uint32_t d = (uint32_t)(key[j] >> shift) & (kBins - 1);
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
        const int d = threadIdx.x;  // kThreads == kBins
        uint32_t run = hist_scanned[(size_t)d * nb + blockIdx.x];
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
        if (idx < n) {
            const uint32_t d = (uint32_t)(key[j] >> shift) & (kBins - 1);
            const uint32_t pos = wave_count[wave][d] + rank[j];
            keys_out[pos] = key[j];
            vals_out[pos] = vals_in ? vals_in[idx] : idx;
        }
    }
}
static_assert(kThreads == kBins, "one thread per bin in the scatter kernel");

// ---------------------------------------------------------------- generic scans over int32

template <bool MAX>
__device__ __forceinline__ int32_t scan_op(int32_t a, int32_t b) {
    return MAX ? max(a, b) : a + b;
}

// Phase 1: per-tile totals.
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

// Phase 2: exclusive scan of the tile totals by one workgroup (values >= 0, identity 0).
template <bool MAX>
__global__ __launch_bounds__(1024) void scan_tiles_kernel(int32_t *tile_tot, int nt,
                                                          int32_t *grand_total) {
    __shared__ int32_t wave_tot[16];
    __shared__ int32_t carry_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int base = 0; base < nt; base += 1024) {
        const int idx = base + threadIdx.x;
        const int32_t v = idx < nt ? tile_tot[idx] : 0;
        int32_t inc = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            int32_t o = __shfl_up(inc, off, 64);
            if (lane >= off) inc = scan_op<MAX>(inc, o);
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        int32_t prefix = carry_s;
        for (int w = 0; w < wave; ++w) prefix = scan_op<MAX>(prefix, wave_tot[w]);
        // exclusive value: everything before this element
        int32_t before = __shfl_up(inc, 1, 64);
        if (lane == 0) before = 0;
        if (idx < nt) tile_tot[idx] = scan_op<MAX>(prefix, before);
        __syncthreads();
        if (threadIdx.x == 1023) carry_s = scan_op<MAX>(prefix, inc);
        __syncthreads();
    }
    if (threadIdx.x == 0 && grand_total) *grand_total = carry_s;
}

// Phase 3: scan inside each tile, seeded with the tile's exclusive prefix.
template <bool MAX, bool INCLUSIVE>
__global__ __launch_bounds__(kThreads) void scan_final_kernel(const int32_t *__restrict__ in, int n,
                                                              const int32_t *__restrict__ tile_prefix,
                                                              int32_t *__restrict__ out) {
    __shared__ int32_t wave_tot[kThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
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
    int32_t prefix = tile_prefix[blockIdx.x];
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
}

template <bool MAX, bool INCLUSIVE>
int device_scan(const int32_t *in, int32_t *out, int n, int32_t *tile_tmp, int32_t *grand_total,
                hipStream_t stream) {
    const int nt = (int)ceil_div(n, kTile);
    hipLaunchKernelGGL(scan_reduce_kernel<MAX>, dim3(nt), dim3(kThreads), 0, stream, in, n, tile_tmp);
    CFGZIP_TRY(check_launch());
    hipLaunchKernelGGL(scan_tiles_kernel<MAX>, dim3(1), dim3(1024), 0, stream, tile_tmp, nt,
                       grand_total);
    CFGZIP_TRY(check_launch());
    hipLaunchKernelGGL((scan_final_kernel<MAX, INCLUSIVE>), dim3(nt), dim3(kThreads), 0, stream, in,
                       n, tile_tmp, out);
    return check_launch();
}

// ---------------------------------------------------------------- segments, verification, rounds

struct Counters {
    int32_t unresolved;
    int32_t num_classes;
    int32_t pad[6];
};

// cand[i] = i if sorted position i starts an equal-hash segment, else 0 (max-scan input);
// also clears the per-token arrays used later.
__global__ void segment_start_kernel(const uint64_t *__restrict__ keys, int n, int32_t *cand,
                                     int32_t *is_head_token, uint64_t *rep_key, int32_t *mismatch) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    cand[i] = (i == 0 || keys[i] != keys[i - 1]) ? i : 0;
    is_head_token[i] = 0;
    rep_key[i] = ~0ull;
    mismatch[i] = 0;
}

// resolved[i] = 1 for segment heads; head_pos starts as the segment head.
__global__ void init_round0_kernel(const int32_t *__restrict__ seg_head, int n, int32_t *head_pos,
                                   int32_t *resolved, Counters *ctr) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) ctr->unresolved = 0;
    if (i >= n) return;
    head_pos[i] = seg_head[i];
    resolved[i] = seg_head[i] == i ? 1 : 0;
}

// One wave per sorted position: compares the stored signature rows of the
// member and of its candidate head.
__global__ __launch_bounds__(kThreads) void verify_stored_kernel(
    const uint16_t *__restrict__ sig, int S, const int32_t *__restrict__ vals,
    const int32_t *__restrict__ head_pos, const int32_t *__restrict__ resolved, int n,
    int32_t *mismatch) {
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
        if (__ballot(diff) != 0ull && lane == 0) mismatch[i] = 1;
    }
}

// A workgroup takes 32 consecutive sorted positions at a time.  Every unresolved member and
// its candidate head are walked with the image walk (walk_device.hpp); the pair is then
// compared without materialising either signature: directly on w when both byte strings
// start with the same byte (idx[row] is onto, so sig equal <=> w equal), else through
// sig[q] = w[idx[row][q]] for every q.
constexpr int kMaxLdsWalkEntries = 72 * 1024;  // 144 KB of uint16; beyond that w lives in global memory
constexpr int kGlobalWalkGrid = 256;

template <bool W_GLOBAL>
__global__ __launch_bounds__(kThreads) void verify_rewalk_kernel(
    Tables T, int S, int wcap, uint16_t *w_global, const uint8_t *__restrict__ tok_bytes,
    const int64_t *__restrict__ tok_off, const int32_t *__restrict__ vals,
    const int32_t *__restrict__ head_pos, const int32_t *__restrict__ resolved, int n,
    int32_t *mismatch) {
    extern __shared__ __align__(16) uint16_t dyn_lds[];
    __shared__ Batch B;
    __shared__ uint8_t ldsb[kByteCap];
    uint16_t *w = W_GLOBAL ? w_global + (size_t)blockIdx.x * wcap : dyn_lds;
    constexpr int kPairs = kBatchTokens / 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool vec = (S % 8) == 0;
    const int n_chunks = (n + kPairs - 1) / kPairs;
    for (int chunk = blockIdx.x; chunk < n_chunks; chunk += gridDim.x) {
        const int i_end = min(n, (chunk + 1) * kPairs);
        int icur = chunk * kPairs;
        while (icur < i_end) {  // workgroup-uniform
            __syncthreads();
            if (threadIdx.x < 64) {
                // lanes 2p, 2p+1: member and head of sorted position icur + p
                const int i = icur + (lane >> 1);
                int64_t beg = 0, len = -1;
                if (i < i_end && !resolved[i]) {
                    const int32_t tok = (lane & 1) ? vals[head_pos[i]] : vals[i];
                    beg = tok_off[tok];
                    len = tok_off[tok + 1] - beg;
                    if (len < 0) len = 0;
                }
                const int k = batch_fill(B, T, tok_bytes, beg, len, wcap, 2, 2);
                if (lane < k) B.aux[lane] = len >= 0 ? 1 : 0;
            }
            __syncthreads();
            const int pairs = min(B.k / 2, i_end - icur);
            batch_stage_bytes(B, tok_bytes, ldsb);
            __syncthreads();
            batch_walk<4, false>(T, T.Tt, S, tok_bytes, B, ldsb, w);
            __syncthreads();
            for (int p = wave; p < pairs; p += kThreads / 64) {
                if (!B.aux[2 * p]) continue;  // wave-uniform
                const int rm = B.row[2 * p], rh = B.row[2 * p + 1];
                const uint16_t *wm = w + B.wstart[2 * p], *wh = w + B.wstart[2 * p + 1];
                bool diff = false;
                if (rm == rh) {
                    const int cnt = B.wstart[2 * p + 1] - B.wstart[2 * p];
                    for (int j = lane; j < cnt; j += 64) diff |= wm[j] != wh[j];
                } else if (vec) {
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
                if (__ballot(diff) != 0ull && lane == 0) mismatch[icur + p] = 1;
            }
            icur += pairs;
        }
    }
}

// Unresolved members whose comparison found no difference join their head's class.
__global__ void settle_kernel(int n, int32_t *resolved, int32_t *mismatch, Counters *ctr) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n || resolved[i]) return;
    if (mismatch[i]) {
        mismatch[i] = 0;
        atomicAdd(&ctr->unresolved, 1);
    } else {
        resolved[i] = 1;
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
    if (h == i) resolved[i] = 1;  // first unresolved member of its segment: a new class head
}

// ---------------------------------------------------------------- numbering and representatives

__global__ void mark_heads_kernel(int n, const int32_t *__restrict__ head_pos,
                                  const int32_t *__restrict__ vals, int32_t *is_head_token) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && head_pos[i] == i) is_head_token[vals[i]] = 1;
}

// Sorted neighbours mostly share a class, so a wave first reduces (length, id) over its lanes
// of equal class and issues one atomic per distinct class instead of one per token.
__global__ __launch_bounds__(kThreads) void assign_classes_kernel(
    int n, const int32_t *__restrict__ head_pos, const int32_t *__restrict__ vals,
    const int32_t *__restrict__ id_of_head_token, const int64_t *__restrict__ tok_off,
    int32_t *class_of_token, uint64_t *rep_key) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool valid = i < n;
    int32_t k = -1;
    uint64_t packed = ~0ull;
    if (valid) {
        const int32_t tok = vals[i];
        k = id_of_head_token[vals[head_pos[i]]];
        class_of_token[tok] = k;
        int64_t len = tok_off[tok + 1] - tok_off[tok];
        if (len > 0x7FFFFFFF) len = 0x7FFFFFFF;
        packed = ((uint64_t)len << 32) | (uint32_t)tok;
    }
    uint64_t todo = __ballot(valid);
    const int lane = threadIdx.x & 63;
    while (todo) {
        const int leader = __ffsll((unsigned long long)todo) - 1;
        const int32_t k0 = __shfl(k, leader, 64);
        const bool mine = valid && k == k0;
        uint64_t m = mine ? packed : ~0ull;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint64_t o = __shfl_xor(m, off, 64);
            m = o < m ? o : m;
        }
        if (lane == leader)
            atomicMin(reinterpret_cast<unsigned long long *>(rep_key + k0), (unsigned long long)m);
        todo &= ~__ballot(mine);
    }
}

__global__ void write_reps_kernel(int n, const uint64_t *__restrict__ rep_key, const Counters *ctr,
                                  int32_t *rep_of_class, int32_t *num_classes_dev) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    const int C = ctr->num_classes;
    if (k == 0 && num_classes_dev) *num_classes_dev = C;
    if (k < n && k < C) rep_of_class[k] = (int32_t)(rep_key[k] & 0xFFFFFFFFull);
}

struct BuildWorkspace {
    void *sig_ws;
    uint64_t *keys[2];
    int32_t *vals[2];
    uint32_t *hist;
    int32_t *seg_head, *head_pos, *resolved, *mismatch, *next_head, *cand;
    int32_t *is_head_token, *id_of_head_token, *tile_tmp;
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
    w.sig_ws = c.take<char>(sig_workspace_bytes(S));
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

}  // namespace
}  // namespace cfgzip

using namespace cfgzip;

extern "C" size_t cfgzip_build_classes_workspace_bytes(int32_t V, int32_t S) {
    if (V <= 0 || S <= 0 || S > 65536) return 0;
    return carve_build_ws(nullptr, V, S).bytes;
}

extern "C" int cfgzip_build_classes(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                                    const uint16_t *table, int32_t S, const uint16_t *sig,
                                    const uint64_t *hash, int32_t *class_of_token,
                                    int32_t *rep_of_class, int32_t *num_classes_dev,
                                    int32_t *num_classes_host, int32_t *collisions_host, void *ws,
                                    size_t ws_bytes, void *stream_) {
    if (!tok_off || !table || !hash || !class_of_token || !rep_of_class) return CFGZIP_E_INVALID;
    if (V <= 0 || S <= 0 || S > 65536) return CFGZIP_E_INVALID;
    if (!aligned_to(tok_off, 8) || !aligned_to(hash, 8) || !aligned_to(sig, 2) ||
        !aligned_to(table, 2) || !aligned_to(class_of_token, 4) || !aligned_to(rep_of_class, 4))
        return CFGZIP_E_INVALID;
    if (!ws || !aligned_to(ws, 256)) return CFGZIP_E_WORKSPACE;
    BuildWorkspace w = carve_build_ws(ws, V, S);
    if (ws_bytes < w.bytes) return CFGZIP_E_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int n = V;
    const int nb = (int)ceil_div(n, kTile);

    // 1. sort (hash, token id)
    const uint64_t *kin = hash;
    const int32_t *vin = nullptr;
    int cur = 0;
    for (int shift = 0; shift < 64; shift += kRadixBits) {
        hipLaunchKernelGGL(radix_hist_kernel, dim3(nb), dim3(kThreads), 0, stream, kin, n, shift,
                           w.hist, nb);
        CFGZIP_TRY(check_launch());
        hipLaunchKernelGGL(scan_u32_single_block_kernel, dim3(1), dim3(1024), 0, stream, w.hist,
                           nb * kBins);
        CFGZIP_TRY(check_launch());
        hipLaunchKernelGGL(radix_scatter_kernel, dim3(nb), dim3(kThreads), 0, stream, kin, vin,
                           w.keys[cur], w.vals[cur], n, shift, w.hist, nb);
        CFGZIP_TRY(check_launch());
        kin = w.keys[cur];
        vin = w.vals[cur];
        cur ^= 1;
    }
    const uint64_t *keys = kin;
    const int32_t *vals = vin;

    // 2. equal-hash segments
    hipLaunchKernelGGL(segment_start_kernel, grid_for(n), dim3(kThreads), 0, stream, keys, n, w.cand,
                       w.is_head_token, w.rep_key, w.mismatch);
    CFGZIP_TRY(check_launch());
    CFGZIP_TRY((device_scan<true, true>(w.cand, w.seg_head, n, w.tile_tmp, nullptr, stream)));
    hipLaunchKernelGGL(init_round0_kernel, grid_for(n), dim3(kThreads), 0, stream, w.seg_head, n,
                       w.head_pos, w.resolved, w.ctr);
    CFGZIP_TRY(check_launch());

    Tables T{};
    if (!sig) CFGZIP_TRY(prepare_tables(table, S, 0, false, w.sig_ws, &T, stream));
    int n_cu = 256;
    {
        int dev = 0;
        CFGZIP_TRY(check_hip(hipGetDevice(&dev)));
        CFGZIP_TRY(check_hip(
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev)));
        if (n_cu <= 0) n_cu = 256;
    }
    auto verify = [&]() -> int {
        if (sig) {
            const int64_t waves = std::min<int64_t>(n, (int64_t)n_cu * 32);
            hipLaunchKernelGGL(verify_stored_kernel, dim3((unsigned)ceil_div(waves, kThreads / 64)),
                               dim3(kThreads), 0, stream, sig, S, vals, w.head_pos, w.resolved, n,
                               w.mismatch);
        } else {
            const int wcap = walk_cap_for(S);
            const int n_chunks = (int)ceil_div(n, kBatchTokens / 2);
            if (wcap > kMaxLdsWalkEntries) {
                hipLaunchKernelGGL(verify_rewalk_kernel<true>,
                                   dim3((unsigned)std::min(n_chunks, kGlobalWalkGrid)),
                                   dim3(kThreads), 0, stream, T, S, wcap, w.verify_w, tok_bytes,
                                   tok_off, vals, w.head_pos, w.resolved, n, w.mismatch);
            } else {
                const size_t dyn = (size_t)wcap * 2;
                auto kern = verify_rewalk_kernel<false>;
                if (dyn > 48 * 1024)
                    CFGZIP_TRY(check_hip(hipFuncSetAttribute(
                        reinterpret_cast<const void *>(kern),
                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn)));
                hipLaunchKernelGGL(kern, dim3((unsigned)std::min(n_chunks, n_cu * 8)),
                                   dim3(kThreads), dyn, stream, T, S, wcap, nullptr, tok_bytes,
                                   tok_off, vals, w.head_pos, w.resolved, n, w.mismatch);
            }
        }
        CFGZIP_TRY(check_launch());
        hipLaunchKernelGGL(settle_kernel, grid_for(n), dim3(kThreads), 0, stream, n, w.resolved,
                           w.mismatch, w.ctr);
        return check_launch();
    };
    auto read_unresolved = [&](int32_t *out) -> int {
        CFGZIP_TRY(check_hip(hipMemcpyAsync(out, &w.ctr->unresolved, sizeof(int32_t),
                                            hipMemcpyDeviceToHost, stream)));
        return check_hip(hipStreamSynchronize(stream));
    };

    // 3. compare with segment heads; split off colliding members in rounds
    CFGZIP_TRY(verify());
    int32_t unresolved = 0;
    CFGZIP_TRY(read_unresolved(&unresolved));
    const int32_t collisions = unresolved;
    int64_t rounds = 0;
    while (unresolved > 0) {
        if (++rounds > (int64_t)V) return CFGZIP_E_COLLISION;  // cannot happen: a round settles >= 1
        hipLaunchKernelGGL(round_reset_kernel, grid_for(n), dim3(kThreads), 0, stream, n, w.next_head,
                           w.ctr);
        CFGZIP_TRY(check_launch());
        hipLaunchKernelGGL(round_propose_kernel, grid_for(n), dim3(kThreads), 0, stream, n,
                           w.resolved, w.seg_head, w.next_head);
        CFGZIP_TRY(check_launch());
        hipLaunchKernelGGL(round_assign_kernel, grid_for(n), dim3(kThreads), 0, stream, n, w.resolved,
                           w.seg_head, w.next_head, w.head_pos);
        CFGZIP_TRY(check_launch());
        CFGZIP_TRY(verify());
        CFGZIP_TRY(read_unresolved(&unresolved));
    }

    // 4. class ids by ascending head token id; 5. representatives
    hipLaunchKernelGGL(mark_heads_kernel, grid_for(n), dim3(kThreads), 0, stream, n, w.head_pos, vals,
                       w.is_head_token);
    CFGZIP_TRY(check_launch());
    CFGZIP_TRY((device_scan<false, false>(w.is_head_token, w.id_of_head_token, n, w.tile_tmp,
                                          &w.ctr->num_classes, stream)));
    hipLaunchKernelGGL(assign_classes_kernel, grid_for(n), dim3(kThreads), 0, stream, n, w.head_pos,
                       vals, w.id_of_head_token, tok_off, class_of_token, w.rep_key);
    CFGZIP_TRY(check_launch());
    hipLaunchKernelGGL(write_reps_kernel, grid_for(n), dim3(kThreads), 0, stream, n, w.rep_key, w.ctr,
                       rep_of_class, num_classes_dev);
    CFGZIP_TRY(check_launch());
    int32_t C = 0;
    CFGZIP_TRY(check_hip(hipMemcpyAsync(&C, &w.ctr->num_classes, sizeof(int32_t),
                                        hipMemcpyDeviceToHost, stream)));
    CFGZIP_TRY(check_hip(hipStreamSynchronize(stream)));
    if (num_classes_host) *num_classes_host = C;
    if (collisions_host) *collisions_host = collisions;
    return CFGZIP_OK;
}
