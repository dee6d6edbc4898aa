// cfgzip_signatures: byte-walk signatures of all tokens and their hash
// (paper Section 3.2.1 / Algorithm 1, regular case; see walk_device.hpp for the
// image walk that keeps the work per token proportional to the number of
// distinct states its first byte leaves, not to S).
//
// Per call:  one kernel transposes the table and builds the per-first-byte image
// tables (a workgroup per image row), then
// one kernel in which a workgroup takes 64 consecutive tokens at a time, stages
// their bytes in LDS, walks all (token, image state) pairs as one flat list of
// independent lanes, reduces the hash in LDS and expands w through idx into the
// stored signature rows with 16-byte stores.  Automata whose transposed table
// fits next to that in LDS are walked from LDS, larger ones from the
// L2-resident copy in the workspace.  Two variants of the call share these kernels:
// cfgzip_signatures_composed (longer tokens continue the walk of a short token that is a
// prefix of theirs; paper Appendix A, Lemma 1) and cfgzip_signatures_static (tables in
// memory that belongs to the library, for callers that cannot allocate).

#include <algorithm>
#include <mutex>

#include "common.hpp"
#include "walk_device.hpp"

namespace cfgzip {
namespace {

// native 16-byte vector (the nontemporal builtins do not take HIP's uint4 struct)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// table read from L2 (S > 256): threads per workgroup and tokens per chunk
constexpr int kWalkThreads = 256;
constexpr int kWalkChunkTokens = 32;  // (measured 16, 24, 32, 40, 48, 64: 32 is best when rows are stored, flat otherwise)

struct WalkArgs {
    const uint8_t *tok_bytes;
    const int64_t *tok_off;
    int32_t V;
    int32_t S;
    int32_t wcap;  // entries of w in LDS
    int32_t chunk_tokens;  // consecutive tokens a workgroup takes at a time, <= kBatchTokens
    Tables T;
    WalkStoreView store;
    uint16_t *sig_out;   // [V][S] or null
    uint64_t *hash_out;  // [V] or null
    // composition over token prefixes (null / 0: plain walks of all tokens)
    const int32_t *parent;      // [V] id of a token of at most kComposePrefix bytes that is a proper prefix, or -1
    const uint8_t *parent_len;  // [V] its length
    int32_t phase;              // 1: only tokens of at most kComposePrefix bytes; 2: only the longer ones
};

// Composition (paper Appendix A, Lemma 1: the relation is a monoid homomorphism, so
// sig(tu) = sig(u) o sig(t)): a token may continue the walk of a shorter token that is a prefix of
// it.  Prefixes of up to this many bytes are used; the short tokens are walked in a first launch,
// the others, starting from their prefix's kept vector, in a second.
constexpr int kComposePrefix = 3;

constexpr int kStateWords = 65536 / 32;  // presence bitmap over every uint16 value
constexpr int kAccCap = 4096;            // ranks whose multiplier sums are reduced in LDS

// All tables of a call in one launch, one workgroup per image row b.  Rows 0..255: column b of
// the caller's table becomes row b of Tt (each thread keeps to its own states q = tid, tid + 1024,
// .., so what it reads back later is what it wrote), then the distinct states of the column, their
// ranks, and the multiplier sum of every rank.  Row 256 (the identity map of the empty token)
// also clears the padding behind Tt and writes the walk store's header.
__global__ __launch_bounds__(1024) void tables_kernel(const uint16_t *__restrict__ table,
                                                      uint16_t *Tt, int S, uint64_t seed,
                                                      int32_t *nimg, uint16_t *img, uint16_t *idx,
                                                      uint64_t *wsum, WalkStore *store, int V) {
    __shared__ uint32_t present[kStateWords];
    __shared__ uint32_t wprefix[kStateWords];
    __shared__ uint32_t wave_tot[16];
    __shared__ unsigned long long acc[kAccCap];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    uint16_t *col = Tt + (size_t)b * S;  // rows 0..255 only

    for (int i = tid; i < kStateWords; i += 1024) present[i] = 0;  // a table entry may be any uint16
    if (wsum)
        for (int i = tid; i < kAccCap && i < S; i += 1024) acc[i] = 0ull;
    __syncthreads();
    if (b < 256) {
        for (int q = tid; q < S; q += 1024) {
            const uint32_t s = table[(size_t)q * 256 + b];
            col[q] = (uint16_t)s;
            // most states of a lexer's column are the same few: look before the atomic
            if (!((present[s >> 5] >> (s & 31)) & 1u)) atomicOr(&present[s >> 5], 1u << (s & 31));
        }
    } else {
        for (int w = tid; w < kStateWords; w += 1024) {
            const int lo = w * 32;
            present[w] = lo + 32 <= S ? 0xFFFFFFFFu : (lo < S ? (1u << (S - lo)) - 1u : 0u);
        }
        uint16_t *pad = Tt + (size_t)256 * S;
        for (int i = tid; i < kTablePad; i += 1024) pad[i] = 0;
        if (store && tid == 0) {
            store->magic = kWalkStoreMagic;
            store->V = V;
            store->S = S;
            store->stride = walk_store_stride(S);
            store->overflow = 0;
        }
    }
    __syncthreads();
    auto state_of = [&](int q) -> uint32_t { return b < 256 ? (uint32_t)col[q] : (uint32_t)q; };
    // exclusive prefix of the per-word population counts; thread i owns words 2i, 2i+1
    const uint32_t c0 = __popc(present[2 * tid]), c1 = __popc(present[2 * tid + 1]);
    int incl = wave_inclusive_sum((int)(c0 + c1));
    if (lane == 63) wave_tot[wave] = (uint32_t)incl;
    __syncthreads();
    uint32_t before = 0;
    for (int wv = 0; wv < wave; ++wv) before += wave_tot[wv];
    const uint32_t excl = before + (uint32_t)incl - (c0 + c1);
    wprefix[2 * tid] = excl;
    wprefix[2 * tid + 1] = excl + c0;
    uint32_t n = 0;
    for (int wv = 0; wv < 16; ++wv) n += wave_tot[wv];  // distinct states, <= S
    if (tid == 0) nimg[b] = (int32_t)n;
    // img: the set bits in ascending order
    {
        uint32_t r = excl;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t bits = present[2 * tid + h];
            while (bits) {
                const int bit = __ffs(bits) - 1;
                bits &= bits - 1;
                img[(size_t)b * S + r++] = (uint16_t)((2 * tid + h) * 32 + bit);
            }
        }
    }
    if (wsum)
        for (uint32_t r = kAccCap + tid; r < n; r += 1024) wsum[(size_t)b * S + r] = 0ull;
    __syncthreads();
    for (int q0 = 0; q0 < S; q0 += 1024) {  // whole waves go round together: they vote below
        const int q = q0 + tid;
        const bool in = q < S;
        const uint32_t s = in ? state_of(q) : 0u;
        const uint32_t r = wprefix[s >> 5] + __popc(present[s >> 5] & ((1u << (s & 31)) - 1u));
        if (in) idx[(size_t)b * S + q] = (uint16_t)r;
        if (wsum) {
            const unsigned long long a = in ? (splitmix64_at(seed, (uint32_t)q) | 1ull) : 0ull;
            // A lexer's column sends most states to one or two ranks; thousands of atomics on one
            // LDS address are served one after the other.  The lanes that share the rank of the
            // wave's first active lane add up in registers first, twice over.
            bool pending = in;
#pragma unroll 1
            for (int round = 0; round < 2; ++round) {
                const uint64_t todo = __ballot(pending);
                if (!todo) break;
                const int leader = __ffsll((unsigned long long)todo) - 1;
                const uint32_t r0 = __shfl(r, leader, 64);
                const bool mine = pending && r == r0;
                if (__popcll(__ballot(mine)) < 4) break;  // not worth the reduction
                unsigned long long sum = mine ? a : 0ull;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) sum += __shfl_xor(sum, off, 64);
                if (mine) pending = false;
                if (lane == leader) {
                    if (r0 < kAccCap) atomicAdd(&acc[r0], sum);
                    else atomicAdd(reinterpret_cast<unsigned long long *>(wsum + (size_t)b * S + r0), sum);
                }
            }
            if (pending) {
                if (r < kAccCap) atomicAdd(&acc[r], a);
                else atomicAdd(reinterpret_cast<unsigned long long *>(wsum + (size_t)b * S + r), a);
            }
        }
    }
    __syncthreads();
    if (wsum)
        for (uint32_t r = tid; r < n && r < kAccCap; r += 1024) wsum[(size_t)b * S + r] = acc[r];
}

template <bool LDS_TABLE>
__global__ __launch_bounds__(LDS_TABLE ? 1024 : kWalkThreads) void signatures_kernel(WalkArgs a) {
    extern __shared__ __align__(16) uint16_t dyn_lds[];  // [table S*256 if LDS_TABLE][w wcap]
    __shared__ Batch B;
    __shared__ uint8_t ldsb[kByteCap];
    const int S = a.S;
    if (LDS_TABLE) {
        const int n16 = S * 32;  // S*512 bytes / 16
        const uint4 *src = reinterpret_cast<const uint4 *>(a.T.Tt);
        uint4 *dst = reinterpret_cast<uint4 *>(dyn_lds);
        for (int i = threadIdx.x; i < n16; i += blockDim.x) dst[i] = src[i];
    }
    const uint16_t *tab = LDS_TABLE ? dyn_lds : a.T.Tt;
    // the walk vectors go through LDS only when rows are expanded from them
    uint16_t *w = (LDS_TABLE || a.sig_out) ? dyn_lds + (LDS_TABLE ? (size_t)S * 256 : 0) : nullptr;
    const int lane = threadIdx.x & 63;
    const bool first_wave = threadIdx.x < 64;
    const bool vec = (S % 8) == 0 && (reinterpret_cast<uintptr_t>(a.sig_out) % 16) == 0;

    const int64_t n_chunks = ((int64_t)a.V + a.chunk_tokens - 1) / a.chunk_tokens;
    for (int64_t chunk = blockIdx.x; chunk < n_chunks; chunk += gridDim.x) {
        const int64_t t_end = min((int64_t)a.V, (chunk + 1) * a.chunk_tokens);
        int64_t tcur = chunk * a.chunk_tokens;
        while (tcur < t_end) {  // workgroup-uniform
            __syncthreads();    // previous batch fully consumed (and the table loaded)
            if (first_wave) {
                const int64_t t = tcur + lane;
                int64_t beg = 0, len = -1;
                int32_t parent = -1, parent_len = 0;
                if (t < t_end) {
                    beg = a.tok_off[t];
                    len = a.tok_off[t + 1] - beg;
                    if (len < 0) len = 0;  // offsets must not decrease; stay in bounds if they do
                    if (a.phase == 2 && a.parent) {
                        parent = a.parent[t];
                        parent_len = a.parent_len[t];
                    }
                }
                // a token that belongs to the other launch keeps its slot, with no walks: its
                // outputs are not touched
                const bool other_launch = (a.phase == 1 && len > kComposePrefix) ||
                                          (a.phase == 2 && len <= kComposePrefix);
                const int kk = batch_fill(B, a.T, a.tok_bytes, beg, other_launch ? -1 : len, a.wcap, 1, 1,
                                          parent, parent_len);
                if (lane < kk) B.aux[lane] = (len >= 0 && !other_launch) ? 1 : 0;
            }
            __syncthreads();
            const int k = (int)min((int64_t)B.k, t_end - tcur);
            batch_stage_bytes(B, a.tok_bytes, ldsb);
            __syncthreads();
            // the walk vectors are also kept for the class builder: token t at t * stride
            const uint32_t stride = walk_store_stride(S);
            uint16_t *keep = a.store.header ? a.store.wvec + (size_t)tcur * stride : nullptr;
            // launch 2 of a composed call: slots with a parent start from its kept vector
            const uint16_t *kept = (a.phase == 2 && a.parent && a.store.header) ? a.store.wvec : nullptr;
            if (a.hash_out) batch_walk<true>(a.T, tab, S, a.tok_bytes, B, ldsb, w, keep, stride, kept);
            else batch_walk<false>(a.T, tab, S, a.tok_bytes, B, ldsb, w, keep, stride, kept);
            __syncthreads();
            if (a.hash_out && (int)threadIdx.x < k && B.aux[threadIdx.x])
                a.hash_out[tcur + threadIdx.x] = B.hash[threadIdx.x];
            if (a.store.header && (int)threadIdx.x < k && B.aux[threadIdx.x]) {
                // image row of the kept vector (the walk wrote the vector and its zero padding)
                const uint32_t m = threadIdx.x;
                a.store.wrow[tcur + m] = pack_walk_row((uint32_t)B.row[m], (uint32_t)B.cnt[m], stride);
                // (the empty token's identity vector is never looked at: its row says it all)
                if ((uint32_t)B.cnt[m] > stride && B.row[m] != 256) a.store.header->overflow = 1;
            }
            if (a.sig_out) {
                // sig[t][q] = w[idx[row][q]]
                if (vec) {
                    // four 16-byte pieces per thread at a time: their index reads are in flight together
                    const uint32_t s8 = (uint32_t)S / 8;
                    const uint32_t items = (uint32_t)k * s8;
                    constexpr int kAhead = 4;
                    for (uint32_t x0 = threadIdx.x; x0 < items; x0 += kAhead * blockDim.x) {
                        uint4 id[kAhead];
#pragma unroll
                        for (int u = 0; u < kAhead; ++u) {
                            const uint32_t x = min(x0 + u * blockDim.x, items - 1);  // repeats the last past the end
                            const uint32_t m = x / s8, q0 = (x - m * s8) * 8;
                            id[u] = *reinterpret_cast<const uint4 *>(a.T.idx + (size_t)B.row[m] * S + q0);
                        }
#pragma unroll
                        for (int u = 0; u < kAhead; ++u) {
                            const uint32_t x = x0 + u * blockDim.x;
                            if (x < items && B.aux[x / s8]) {
                                const uint32_t m = x / s8, q0 = (x - m * s8) * 8;
                                const uint16_t *wm = w + B.wstart[m];
                                uint4 o;
                                o.x = (uint32_t)wm[id[u].x & 0xFFFFu] | ((uint32_t)wm[id[u].x >> 16] << 16);
                                o.y = (uint32_t)wm[id[u].y & 0xFFFFu] | ((uint32_t)wm[id[u].y >> 16] << 16);
                                o.z = (uint32_t)wm[id[u].z & 0xFFFFu] | ((uint32_t)wm[id[u].z >> 16] << 16);
                                o.w = (uint32_t)wm[id[u].w & 0xFFFFu] | ((uint32_t)wm[id[u].w >> 16] << 16);
                                // written once, not read again by this call: keep it out of the
                                // caches that hold the table
                                const u32x4 ov = {o.x, o.y, o.z, o.w};
                                __builtin_nontemporal_store(
                                    ov, reinterpret_cast<u32x4 *>(a.sig_out + (size_t)(tcur + m) * S + q0));
                            }
                        }
                    }
                } else {
                    const uint32_t items = (uint32_t)k * (uint32_t)S;
                    for (uint32_t x = threadIdx.x; x < items; x += blockDim.x) {
                        const uint32_t m = x / (uint32_t)S, q = x - m * (uint32_t)S;
                        if (!B.aux[m]) continue;
                        a.sig_out[(size_t)(tcur + m) * S + q] =
                            w[B.wstart[m] + a.T.idx[(size_t)B.row[m] * S + q]];
                    }
                }
            }
            tcur += k;
        }
    }
}

// ---- composition over token prefixes: which short token is a prefix of which long one ----------
// Tokens of 2 .. kComposePrefix bytes go into an open-addressing table keyed by their bytes
// (length and bytes fit a 32-bit key, so a key match is a byte-string match); every longer token
// then looks its own prefixes up, longest first.
constexpr unsigned long long kPrefixEmpty = ~0ull;

struct ComposeArgs {
    const uint8_t *tok_bytes;
    const int64_t *tok_off;
    int32_t V;
    unsigned long long *slots;  // [capacity]: (key << 32) | token id, or kPrefixEmpty
    uint32_t capacity_mask;     // capacity - 1, capacity a power of two
    int32_t *parent;            // [V]
    uint8_t *parent_len;        // [V]
};

__device__ __forceinline__ uint32_t prefix_key(const uint8_t *p, int len) {
    uint32_t key = (uint32_t)len << 24;
    for (int k = 0; k < len; ++k) key |= (uint32_t)p[k] << (8 * (2 - k));
    return key;
}
__device__ __forceinline__ uint32_t prefix_slot(uint32_t key, uint32_t mask) {
    return (key * 2654435761u >> 7) & mask;
}

__global__ void prefix_clear_kernel(unsigned long long *slots, uint32_t capacity) {
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < capacity; i += gridDim.x * blockDim.x)
        slots[i] = kPrefixEmpty;
}

// a thread per token; the short ones claim a slot (the first of several equal byte strings wins)
__global__ void prefix_insert_kernel(ComposeArgs a) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= a.V) return;
    const int64_t beg = a.tok_off[t], len = a.tok_off[t + 1] - beg;
    a.parent[t] = -1;
    a.parent_len[t] = 0;
    if (len < 2 || len > kComposePrefix) return;
    const uint32_t key = prefix_key(a.tok_bytes + beg, (int)len);
    const unsigned long long mine = ((unsigned long long)key << 32) | (uint32_t)t;
    uint32_t s = prefix_slot(key, a.capacity_mask);
    for (uint32_t probes = 0; probes <= a.capacity_mask; ++probes, s = (s + 1) & a.capacity_mask) {
        const unsigned long long old = atomicCAS(&a.slots[s], kPrefixEmpty, mine);
        if (old == kPrefixEmpty || (uint32_t)(old >> 32) == key) return;  // claimed, or already there
    }
}

// a thread per token; the long ones look their prefixes up
__global__ void prefix_find_kernel(ComposeArgs a) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= a.V) return;
    const int64_t beg = a.tok_off[t], len = a.tok_off[t + 1] - beg;
    if (len <= kComposePrefix) return;
    for (int k = kComposePrefix; k >= 2; --k) {
        const uint32_t key = prefix_key(a.tok_bytes + beg, k);
        uint32_t s = prefix_slot(key, a.capacity_mask);
        for (uint32_t probes = 0; probes <= a.capacity_mask; ++probes, s = (s + 1) & a.capacity_mask) {
            const unsigned long long e = a.slots[s];
            if (e == kPrefixEmpty) break;
            if ((uint32_t)(e >> 32) == key) {
                a.parent[t] = (int32_t)(uint32_t)e;
                a.parent_len[t] = (uint8_t)k;
                return;
            }
        }
    }
}

// the composition's own part of the workspace, behind the signature workspace
struct ComposeWorkspace {
    unsigned long long *slots;
    uint32_t capacity;
    int32_t *parent;
    uint8_t *parent_len;
    size_t bytes;
};

ComposeWorkspace carve_compose_ws(void *ws, int32_t V) {
    Carver c(ws);
    ComposeWorkspace w;
    uint32_t cap = 1024;
    while (cap < (1u << 31) && cap < 2u * (uint32_t)V) cap <<= 1;  // (V < 2^31: the product cannot wrap)
    w.capacity = cap;
    w.slots = c.take<unsigned long long>(cap);
    w.parent = c.take<int32_t>((size_t)V);
    w.parent_len = c.take<uint8_t>((size_t)V);
    w.bytes = c.used;
    return w;
}

constexpr size_t kLdsTableLimit = 128 * 1024;  // S <= 256

int device_cu_count(int *out) {
    int dev = 0;
    CFGZIP_TRY(check_hip(hipGetDevice(&dev)));
    int n = 0;
    CFGZIP_TRY(check_hip(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev)));
    *out = n > 0 ? n : 256;
    return CFGZIP_OK;
}

// Layout of the signature workspace.
struct SigWorkspace {
    uint16_t *Tt;
    int32_t *nimg;
    uint16_t *img, *idx;
    uint64_t *wsum;
    WalkStoreView store;  // V > 0 only
    size_t bytes;
};

// The header comes first, so that a reader that only knows "this is some signature workspace"
// can look at it before trusting any size-dependent offset.
SigWorkspace carve_sig_ws(void *ws, int32_t V, int32_t S) {
    Carver c(ws);
    SigWorkspace w;
    WalkStore *header = c.take<WalkStore>(1);
    w.Tt = c.take<uint16_t>((size_t)256 * S + kTablePad);
    w.nimg = c.take<int32_t>(kImageRows);
    w.img = c.take<uint16_t>((size_t)kImageRows * S);
    w.idx = c.take<uint16_t>((size_t)kImageRows * S);
    w.wsum = c.take<uint64_t>((size_t)kImageRows * S);
    w.store = WalkStoreView{nullptr, nullptr, nullptr};
    if (V > 0) {
        w.store.header = header;
        w.store.wrow = c.take<uint16_t>((size_t)V);
        w.store.wvec = c.take<uint16_t>((size_t)V * walk_store_stride(S));
    }
    w.bytes = c.used;
    return w;
}

}  // namespace

int prepare_tables(const uint16_t *table, int32_t S, uint64_t hash_seed, bool want_wsum, int32_t V,
                   void *ws, Tables *out, WalkStoreView *store, hipStream_t stream) {
    SigWorkspace w = carve_sig_ws(ws, V, S);
    hipLaunchKernelGGL(tables_kernel, dim3(kImageRows), dim3(1024), 0, stream, table, w.Tt, S, hash_seed,
                       w.nimg, w.img, w.idx, want_wsum ? w.wsum : nullptr, w.store.header, V);
    CFGZIP_TRY(check_launch());
    out->Tt = w.Tt;
    out->nimg = w.nimg;
    out->img = w.img;
    out->idx = w.idx;
    out->wsum = want_wsum ? w.wsum : nullptr;
    if (store) *store = w.store;
    return CFGZIP_OK;
}

size_t sig_workspace_bytes(int32_t V, int32_t S) { return carve_sig_ws(nullptr, V, S).bytes; }

void view_signature_workspace(void *ws, int32_t V, int32_t S, Tables *tables, WalkStoreView *store) {
    SigWorkspace w = carve_sig_ws(ws, V, S);
    tables->Tt = w.Tt;
    tables->nimg = w.nimg;
    tables->img = w.img;
    tables->idx = w.idx;
    tables->wsum = w.wsum;
    *store = w.store;
}

}  // namespace cfgzip

using namespace cfgzip;

extern "C" size_t cfgzip_signatures_workspace_bytes(int32_t V, int32_t S) {
    if (V <= 0 || S <= 0 || S > 65536) return 0;
    return sig_workspace_bytes(V, S);
}

namespace {

// Shared by both entry points: `ws` holds at least sig_workspace_bytes(store_V, S) bytes;
// store_V = V keeps the walk vectors for the class builder, store_V = 0 keeps nothing.
// `compose_ws` (or null): the composition's part of the workspace; the tokens are then walked
// in two launches, the longer ones starting from the kept vector of a short token that is a
// prefix of theirs (needs store_V = V).
int run_signatures(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V, const uint16_t *table,
                   int32_t S, uint16_t *sig_out, uint64_t *hash_out, uint64_t hash_seed, void *ws,
                   int32_t store_V, hipStream_t stream, void *compose_ws = nullptr) {
    WalkArgs a{};
    if (compose_ws) {
        const ComposeWorkspace cw = carve_compose_ws(compose_ws, V);
        ComposeArgs ca{tok_bytes, tok_off, V, cw.slots, cw.capacity - 1, cw.parent, cw.parent_len};
        hipLaunchKernelGGL(prefix_clear_kernel, dim3((unsigned)std::min<int64_t>(1024, ceil_div(cw.capacity, 256))),
                           dim3(256), 0, stream, cw.slots, cw.capacity);
        CFGZIP_TRY(check_launch());
        hipLaunchKernelGGL(prefix_insert_kernel, dim3((unsigned)ceil_div(V, 256)), dim3(256), 0, stream, ca);
        CFGZIP_TRY(check_launch());
        hipLaunchKernelGGL(prefix_find_kernel, dim3((unsigned)ceil_div(V, 256)), dim3(256), 0, stream, ca);
        CFGZIP_TRY(check_launch());
        a.parent = cw.parent;
        a.parent_len = cw.parent_len;
    }
    a.tok_bytes = tok_bytes;
    a.tok_off = tok_off;
    a.V = V;
    a.S = S;
    a.sig_out = sig_out;
    a.hash_out = hash_out;
    CFGZIP_TRY(prepare_tables(table, S, hash_seed, hash_out != nullptr, store_V, ws, &a.T, &a.store, stream));

    int n_cu = 256;
    CFGZIP_TRY(device_cu_count(&n_cu));
    const bool lds_table = (size_t)S * 512 <= kLdsTableLimit;
    a.chunk_tokens = lds_table ? kBatchTokens : kWalkChunkTokens;
    const int64_t n_chunks = ceil_div(V, a.chunk_tokens);
    // the signatures kernel walks one token at a time in the worst case: S entries suffice
    a.wcap = std::max(kMinWalkCap, (S + kWalkGroup - 1) / kWalkGroup * kWalkGroup);
    if (lds_table) {
        const size_t dyn = (size_t)S * 512 + (size_t)a.wcap * 2;
        auto kern = signatures_kernel<true>;
        if (dyn > 48 * 1024)
            CFGZIP_TRY(check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     (int)dyn)));
        // loading the table costs a workgroup about as much as walking a few batches
        const int per_cu = (int)std::max<size_t>(1, std::min<size_t>(2, (150 * 1024) / (dyn + 8192)));
        const int64_t grid = std::min<int64_t>(ceil_div(n_chunks, 2), (int64_t)n_cu * per_cu);
        for (int phase = compose_ws ? 1 : 0; phase <= (compose_ws ? 2 : 0); ++phase) {
            a.phase = phase;
            hipLaunchKernelGGL(kern, dim3((unsigned)std::max<int64_t>(1, grid)), dim3(1024), dyn, stream, a);
            CFGZIP_TRY(check_launch());
        }
    } else {
        const size_t dyn = sig_out ? (size_t)a.wcap * 2 : 0;
        if (!sig_out) a.wcap = 0x3FFFFFFF;  // no LDS buffer bounds a batch's walks
        auto kern = signatures_kernel<false>;
        if (dyn > 48 * 1024)
            CFGZIP_TRY(check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     (int)dyn)));
        // one workgroup per chunk: the hardware hands out chunks as workgroups retire, which
        // balances chunks of very different cost
        const int64_t grid = std::min<int64_t>(n_chunks, 0x7FFFFFFF);
        for (int phase = compose_ws ? 1 : 0; phase <= (compose_ws ? 2 : 0); ++phase) {
            a.phase = phase;
            hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kWalkThreads), dyn, stream, a);
            CFGZIP_TRY(check_launch());
        }
    }
    return CFGZIP_OK;
}

int check_signature_args(const int64_t *tok_off, int32_t V, const uint16_t *table, int32_t S,
                         const uint16_t *sig_out, const uint64_t *hash_out) {
    if (!tok_off || !table || V <= 0 || S <= 0 || S > 65536) return CFGZIP_E_INVALID;
    if (!sig_out && !hash_out) return CFGZIP_E_INVALID;
    if (!aligned_to(tok_off, 8) || !aligned_to(table, 2) || !aligned_to(sig_out, 2) ||
        !aligned_to(hash_out, 8))
        return CFGZIP_E_INVALID;
    return CFGZIP_OK;
}

// ---- the entry point that allocates nothing ------------------------------------------------
// Its tables live in device memory that belongs to the loaded library itself.  Each GPU has its
// own copy of the array at its own address; host code never uses the array's name as an
// address, only the pointer hipGetSymbolAddress returns for the current device.
constexpr int32_t kStaticMaxStates = CFGZIP_STATIC_MAX_STATES;
constexpr size_t static_scratch_bytes(size_t S) {
    // mirrors carve_sig_ws(ws, 0, S): header, Tt, nimg, img, idx, wsum, each rounded up to 256 bytes
    return 256 + ((256 * S + kTablePad) * 2 + 255) / 256 * 256 + (kImageRows * 4 + 255) / 256 * 256 +
           2 * ((kImageRows * S * 2 + 255) / 256 * 256) + (kImageRows * S * 8 + 255) / 256 * 256;
}
constexpr size_t kStaticScratchBytes = static_scratch_bytes(kStaticMaxStates);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // per device, filled at the first call on that device

int static_scratch_for_current_device(void **out) {
    int dev = 0;
    CFGZIP_TRY(check_hip(hipGetDevice(&dev)));
    if (dev < 0 || dev >= kMaxDevices) return CFGZIP_E_INVALID;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        CFGZIP_TRY(check_hip(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))));
        if (!ptr) return CFGZIP_E_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CFGZIP_OK;
}

}  // namespace

extern "C" int cfgzip_signatures(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                                 const uint16_t *table, int32_t S, uint16_t *sig_out,
                                 uint64_t *hash_out, uint64_t hash_seed, void *ws, size_t ws_bytes,
                                 void *stream_) {
    CFGZIP_TRY(check_signature_args(tok_off, V, table, S, sig_out, hash_out));
    if (!ws || ws_bytes < sig_workspace_bytes(V, S) || !aligned_to(ws, 256)) return CFGZIP_E_WORKSPACE;
    // tok_bytes may be null only if every token is empty; the kernels never read it then.
    return run_signatures(tok_bytes, tok_off, V, table, S, sig_out, hash_out, hash_seed, ws, V,
                          static_cast<hipStream_t>(stream_));
}

extern "C" size_t cfgzip_signatures_composed_workspace_bytes(int32_t V, int32_t S) {
    if (V <= 0 || S <= 0 || S > 65536) return 0;
    return sig_workspace_bytes(V, S) + carve_compose_ws(nullptr, V).bytes;
}

extern "C" int cfgzip_signatures_composed(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                                          const uint16_t *table, int32_t S, uint16_t *sig_out,
                                          uint64_t *hash_out, uint64_t hash_seed, void *ws,
                                          size_t ws_bytes, void *stream_) {
    CFGZIP_TRY(check_signature_args(tok_off, V, table, S, sig_out, hash_out));
    const size_t sig_bytes = sig_workspace_bytes(V, S);
    if (!ws || !aligned_to(ws, 256) || ws_bytes < sig_bytes + carve_compose_ws(nullptr, V).bytes)
        return CFGZIP_E_WORKSPACE;
    return run_signatures(tok_bytes, tok_off, V, table, S, sig_out, hash_out, hash_seed, ws, V,
                          static_cast<hipStream_t>(stream_), static_cast<char *>(ws) + sig_bytes);
}

extern "C" int cfgzip_signatures_static(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                                        const uint16_t *table, int32_t S, uint16_t *sig_out,
                                        uint64_t *hash_out, uint64_t hash_seed, void *stream_) {
    CFGZIP_TRY(check_signature_args(tok_off, V, table, S, sig_out, hash_out));
    if (S > kStaticMaxStates || sig_workspace_bytes(0, S) > kStaticScratchBytes) return CFGZIP_E_TOO_LARGE;
    void *ws = nullptr;
    CFGZIP_TRY(static_scratch_for_current_device(&ws));
    // every table entry the kernels read is written by this call's own table kernels first, so
    // what the previous call left in the array does not matter
    return run_signatures(tok_bytes, tok_off, V, table, S, sig_out, hash_out, hash_seed, ws, 0,
                          static_cast<hipStream_t>(stream_));
}
