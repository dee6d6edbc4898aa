// Signatures over a non-deterministic byte automaton (paper Section 3.2.1 for a right-linear
// grammar with several productions q -> a q' per state and byte).  The displacement of token t
// is then the relation R_t = {(q, q') : q' reachable from q on bytes(t)}, the boolean product of
// the per-byte transition relations; it is kept as one bit row per start state.
//
// A thread owns one (token, start state) pair and carries the set of current states as W words
// in registers.  Per byte it ORs together the successor rows of the set's members, visiting set
// bits only, so the cost follows the number of live states (one or a few for a lexer), not S;
// a set that has become empty stops early.  Automata of more than 256 states (up to 1,024) keep
// the sets in LDS instead.  The 64-bit hash is the same multilinear form as for
// the byte walk, over the relation read as 16-bit entries, so any split over threads gives the
// same bits.

#include <algorithm>

#include "common.hpp"
#include "walk_device.hpp"  // splitmix64_at: the multipliers of the signature hash

namespace cfgzip {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxRegisterStates = 256;  // up to here a thread keeps its set in registers
constexpr int kMaxNfaStates = 1024;
constexpr int kStagedBytes = 64;  // token bytes read once into LDS; longer tokens go on from global

struct NfaArgs {
    const uint8_t *tok_bytes;
    const int64_t *tok_off;
    const uint32_t *nfa;  // [256][S][W]
    uint32_t *rel;        // [V][S][W]
    uint64_t *hash;       // [V] or null
    uint64_t seed;
    int V, S;
    int threads_per_token;  // 64, 128 or 256: S rounded up
    uint32_t last_word_mask;  // the bits of a row's last word that are states
};

// A thread owns one (token, start state) pair.  (Two or four start states per thread, for more
// row reads in flight, made the kernel slower - 209 and 277 us against 164 us on 32,000 tokens x
// 256 states: it is bound by instruction issue, not by the latency of its reads.)
template <int W>
__global__ __launch_bounds__(kThreads) void nfa_walk_kernel(NfaArgs a) {
    __shared__ unsigned long long hash_sum[kThreads / 64];
    __shared__ uint8_t head_bytes[kThreads / 64][kStagedBytes];  // each token's first bytes
    const int slot = threadIdx.x / a.threads_per_token;
    const int q = threadIdx.x % a.threads_per_token;
    const int t = blockIdx.x * (kThreads / a.threads_per_token) + slot;
    if (threadIdx.x < kThreads / 64) hash_sum[threadIdx.x] = 0;
    int64_t b0 = 0, b1 = 0;
    if (t < a.V) {
        b0 = a.tok_off[t];
        b1 = a.tok_off[t + 1];
        if (q < kStagedBytes && b0 + q < b1) head_bytes[slot][q] = a.tok_bytes[b0 + q];
    }
    __syncthreads();
    uint64_t h = 0;
    if (t < a.V && q < a.S) {
        uint32_t cur[W];
#pragma unroll
        for (int w = 0; w < W; ++w) cur[w] = (q >> 5) == w ? 1u << (q & 31) : 0u;
        const size_t matrix = (size_t)a.S * W;
        for (int64_t p = b0; p < b1; ++p) {
            const int ch = p - b0 < kStagedBytes ? head_bytes[slot][p - b0] : a.tok_bytes[p];
            const uint32_t *step = a.nfa + ch * matrix;
            uint32_t nxt[W];
#pragma unroll
            for (int w = 0; w < W; ++w) nxt[w] = 0;
#pragma unroll
            for (int w = 0; w < W; ++w) {
                uint32_t bits = cur[w];
                while (bits) {
                    const int x = w * 32 + __ffs(bits) - 1;
                    bits &= bits - 1;
                    const uint32_t *row = step + (size_t)x * W;
                    if (W % 4 == 0) {  // rows are whole 16-byte units (the base is 16-byte aligned)
#pragma unroll
                        for (int k = 0; k < W / 4; ++k) {
                            const uint4 v = reinterpret_cast<const uint4 *>(row)[k];
                            nxt[4 * k] |= v.x;
                            nxt[4 * k + 1] |= v.y;
                            nxt[4 * k + 2] |= v.z;
                            nxt[4 * k + 3] |= v.w;
                        }
                    } else {
#pragma unroll
                        for (int k = 0; k < W; ++k) nxt[k] |= row[k];
                    }
                }
            }
            nxt[W - 1] &= a.last_word_mask;  // a stray pad bit must not become a state number
            uint32_t any = 0;
#pragma unroll
            for (int w = 0; w < W; ++w) {
                cur[w] = nxt[w];
                any |= nxt[w];
            }
            if (!any) break;  // no state left: the row stays empty
        }
        uint32_t *out = a.rel + ((size_t)t * a.S + q) * W;
        if (W % 4 == 0) {
#pragma unroll
            for (int k = 0; k < W / 4; ++k)
                reinterpret_cast<uint4 *>(out)[k] =
                    make_uint4(cur[4 * k], cur[4 * k + 1], cur[4 * k + 2], cur[4 * k + 3]);
        } else {
#pragma unroll
            for (int w = 0; w < W; ++w) out[w] = cur[w];
        }
#pragma unroll
        for (int w = 0; w < W; ++w) {
            if (a.hash && cur[w]) {  // most words of a relation are empty: their terms are zero
                const uint32_t e = 2u * (uint32_t)(q * W + w);  // 16-bit entries 2(qW+w), 2(qW+w)+1
                if (cur[w] & 0xFFFFu)
                    h += (splitmix64_at(a.seed, e) | 1ull) * (uint64_t)(cur[w] & 0xFFFFu);
                if (cur[w] >> 16)
                    h += (splitmix64_at(a.seed, e + 1u) | 1ull) * (uint64_t)(cur[w] >> 16);
            }
        }
    }
    if (a.hash) {
        if (h) atomicAdd(&hash_sum[slot], (unsigned long long)h);
        __syncthreads();
        if (q == 0 && t < a.V) a.hash[t] = hash_sum[slot];
    }
}

// More than 256 states: the sets no longer fit in registers.  A workgroup takes 256 start states
// of one token; a thread keeps its current and next set in LDS, word w of thread t at [w][t] (so
// the threads of a wave hit different banks), and per byte ORs the successor rows of the set's
// members into the next set.  The hash is accumulated per token with one atomic per workgroup
// (hash_out is cleared by a launch before).
__global__ __launch_bounds__(kThreads) void nfa_walk_lds_kernel(NfaArgs a, int W, int q_blocks) {
    extern __shared__ uint32_t sets[];  // [2][W][kThreads]
    __shared__ unsigned long long hash_sum;
    const int t = blockIdx.x / q_blocks;
    const int q = (blockIdx.x % q_blocks) * kThreads + threadIdx.x;
    uint32_t *cur = sets + threadIdx.x, *nxt = sets + (size_t)W * kThreads + threadIdx.x;
    if (threadIdx.x == 0) hash_sum = 0;
    __syncthreads();
    uint64_t h = 0;
    if (q < a.S) {
        for (int w = 0; w < W; ++w) cur[(size_t)w * kThreads] = (q >> 5) == w ? 1u << (q & 31) : 0u;
        const int64_t b0 = a.tok_off[t], b1 = a.tok_off[t + 1];
        const size_t matrix = (size_t)a.S * W;
        for (int64_t p = b0; p < b1; ++p) {
            const uint32_t *step = a.nfa + (size_t)a.tok_bytes[p] * matrix;
            for (int w = 0; w < W; ++w) nxt[(size_t)w * kThreads] = 0;
            for (int w = 0; w < W; ++w) {
                uint32_t bits = cur[(size_t)w * kThreads];
                while (bits) {
                    const int x = w * 32 + __ffs(bits) - 1;
                    bits &= bits - 1;
                    const uint32_t *row = step + (size_t)x * W;
                    for (int k = 0; k < W; ++k) nxt[(size_t)k * kThreads] |= row[k];
                }
            }
            nxt[(size_t)(W - 1) * kThreads] &= a.last_word_mask;  // a stray pad bit must not become a state number
            uint32_t any = 0;
            for (int w = 0; w < W; ++w) any |= nxt[(size_t)w * kThreads];
            uint32_t *tmp = cur;
            cur = nxt;
            nxt = tmp;
            if (!any) break;  // no state left: the row stays empty
        }
        uint32_t *out = a.rel + ((size_t)t * a.S + q) * W;
        for (int w = 0; w < W; ++w) {
            const uint32_t v = cur[(size_t)w * kThreads];
            out[w] = v;
            if (a.hash && v) {
                const uint32_t e = 2u * (uint32_t)(q * W + w);
                if (v & 0xFFFFu) h += (splitmix64_at(a.seed, e) | 1ull) * (uint64_t)(v & 0xFFFFu);
                if (v >> 16) h += (splitmix64_at(a.seed, e + 1u) | 1ull) * (uint64_t)(v >> 16);
            }
        }
    }
    if (a.hash) {
        if (h) atomicAdd(&hash_sum, (unsigned long long)h);
        __syncthreads();
        if (threadIdx.x == 0 && hash_sum)
            atomicAdd(reinterpret_cast<unsigned long long *>(a.hash + t), hash_sum);
    }
}

__global__ void clear_u64_kernel(uint64_t *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

template <int W>
int launch_nfa(const NfaArgs &a, hipStream_t stream) {
    const int per_block = kThreads / a.threads_per_token;
    hipLaunchKernelGGL(nfa_walk_kernel<W>, dim3((unsigned)ceil_div(a.V, per_block)), dim3(kThreads), 0,
                       stream, a);
    return check_launch();
}

}  // namespace
}  // namespace cfgzip

using namespace cfgzip;

extern "C" int cfgzip_nfa_signatures(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                                     const int32_t *nfa, int32_t S, int32_t *rel_out,
                                     uint64_t *hash_out, uint64_t hash_seed, void *stream_) {
    if (!tok_off || !nfa || !rel_out) return CFGZIP_E_INVALID;
    if (V <= 0 || S <= 0 || S > kMaxNfaStates) return CFGZIP_E_INVALID;
    if (!aligned_to(tok_off, 8) || !aligned_to(nfa, 16) || !aligned_to(rel_out, 16) ||
        !aligned_to(hash_out, 8))
        return CFGZIP_E_INVALID;
    NfaArgs a{};
    a.tok_bytes = tok_bytes;
    a.tok_off = tok_off;
    a.nfa = reinterpret_cast<const uint32_t *>(nfa);
    a.rel = reinterpret_cast<uint32_t *>(rel_out);
    a.hash = hash_out;
    a.seed = hash_seed;
    a.V = V;
    a.S = S;
    a.threads_per_token = 64;  // whole waves, a power of two so that a block holds whole tokens
    while (a.threads_per_token < S) a.threads_per_token *= 2;
    a.last_word_mask = (S & 31) ? (1u << (S & 31)) - 1u : 0xFFFFFFFFu;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (S > kMaxRegisterStates) {
        const int W = (S + 31) / 32, q_blocks = (S + kThreads - 1) / kThreads;
        if ((int64_t)V * q_blocks > 0x7FFFFFFF) return CFGZIP_E_INVALID;
        if (hash_out) {
            hipLaunchKernelGGL(clear_u64_kernel, dim3((unsigned)ceil_div(V, kThreads)), dim3(kThreads), 0,
                               stream, hash_out, V);
            CFGZIP_TRY(check_launch());
        }
        const size_t dyn = (size_t)2 * W * kThreads * sizeof(uint32_t);
        if (dyn > 48 * 1024)
            CFGZIP_TRY(check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(nfa_walk_lds_kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn)));
        hipLaunchKernelGGL(nfa_walk_lds_kernel, dim3((unsigned)(V * q_blocks)), dim3(kThreads), dyn, stream,
                           a, W, q_blocks);
        return check_launch();
    }
    switch ((S + 31) / 32) {
        case 1: return launch_nfa<1>(a, stream);
        case 2: return launch_nfa<2>(a, stream);
        case 3: return launch_nfa<3>(a, stream);
        case 4: return launch_nfa<4>(a, stream);
        case 5: return launch_nfa<5>(a, stream);
        case 6: return launch_nfa<6>(a, stream);
        case 7: return launch_nfa<7>(a, stream);
        default: return launch_nfa<8>(a, stream);
    }
}
