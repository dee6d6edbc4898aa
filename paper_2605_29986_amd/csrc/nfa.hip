// Signatures over a non-deterministic byte automaton (paper Section 3.2.1 for a right-linear
// grammar with several productions q -> a q' per state and byte).  The displacement of token t
// is then the relation R_t = {(q, q') : q' reachable from q on bytes(t)}, the boolean product of
// the per-byte transition relations; it is kept as one bit row per start state.
//
// A thread owns one (token, start state) pair and carries the set of current states as W words
// in registers.  Per byte it ORs together the successor rows of the set's members, visiting set
// bits only, so the cost follows the number of live states (one or a few for a lexer), not S;
// a set that has become empty stops early.  The 64-bit hash is the same multilinear form as for
// the byte walk, over the relation read as 16-bit entries, so any split over threads gives the
// same bits.

#include <algorithm>

#include "common.hpp"
#include "walk_device.hpp"  // splitmix64_at: the multipliers of the signature hash

namespace cfgzip {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxNfaStates = 256;
constexpr int kStagedBytes = 64;  // token bytes read once into LDS; longer tokens go on from global

struct NfaArgs {
    const uint8_t *tok_bytes;
    const int64_t *tok_off;
    const uint32_t *nfa;  // [256][S][W]
    uint32_t *rel;        // [V][S][W]
    uint64_t *hash;       // [V] or null
    uint64_t seed;
    int V, S;
    int threads_per_token;  // 64, 128 or 256: covers S with the rows each thread owns
    uint32_t last_word_mask;  // the bits of a row's last word that are states
};

// A thread owns R start states of one token, q, q + threads_per_token, ..  R = 1 is what is
// launched: with 2 or 4 chains per thread the kernel got slower (209 and 277 us against 164 us
// on 32,000 tokens x 256 states), so it is not waiting on the latency of its row reads.
template <int W, int R>
__global__ __launch_bounds__(kThreads) void nfa_walk_kernel(NfaArgs a) {
    __shared__ unsigned long long hash_sum[kThreads / 64];
    __shared__ uint8_t head_bytes[kThreads / 64][kStagedBytes];  // each token's first bytes
    const int slot = threadIdx.x / a.threads_per_token;
    const int q0 = threadIdx.x % a.threads_per_token;
    const int t = blockIdx.x * (kThreads / a.threads_per_token) + slot;
    if (threadIdx.x < kThreads / 64) hash_sum[threadIdx.x] = 0;
    int64_t b0 = 0, b1 = 0;
    if (t < a.V) {
        b0 = a.tok_off[t];
        b1 = a.tok_off[t + 1];
        if (q0 < kStagedBytes && b0 + q0 < b1) head_bytes[slot][q0] = a.tok_bytes[b0 + q0];
    }
    __syncthreads();
    uint64_t h = 0;
    if (t < a.V) {
        uint32_t cur[R][W];
        bool live[R];  // start state exists and its set is not empty yet
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int q = q0 + r * a.threads_per_token;
            live[r] = q < a.S;
#pragma unroll
            for (int w = 0; w < W; ++w) cur[r][w] = (live[r] && (q >> 5) == w) ? 1u << (q & 31) : 0u;
        }
        for (int64_t p = b0; p < b1; ++p) {
            bool any_live = false;
#pragma unroll
            for (int r = 0; r < R; ++r) any_live |= live[r];
            if (!any_live) break;
            const int ch = p - b0 < kStagedBytes ? head_bytes[slot][p - b0] : a.tok_bytes[p];
            const uint32_t *step = a.nfa + (size_t)ch * a.S * W;
            uint32_t nxt[R][W];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int w = 0; w < W; ++w) nxt[r][w] = 0;
#pragma unroll
            for (int w = 0; w < W; ++w) {
                uint32_t bits[R];
                uint32_t left = 0;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    bits[r] = cur[r][w];
                    left |= bits[r];
                }
                while (left) {
                    // one member of each chain's set: the reads of all chains are issued together
                    const uint32_t *row[R];
                    uint32_t take[R];
                    left = 0;
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        take[r] = bits[r] ? 0xFFFFFFFFu : 0u;
                        const int x = bits[r] ? w * 32 + __ffs(bits[r]) - 1 : 0;  // row 0: read, not used
                        bits[r] &= bits[r] - 1;  // 0 stays 0
                        left |= bits[r];
                        row[r] = step + (size_t)x * W;
                    }
                    if (W % 4 == 0) {  // rows are whole 16-byte units (the base is 16-byte aligned)
                        uint4 v[R][W / 4 > 0 ? W / 4 : 1];
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int k = 0; k < W / 4; ++k) v[r][k] = reinterpret_cast<const uint4 *>(row[r])[k];
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int k = 0; k < W / 4; ++k) {
                                nxt[r][4 * k] |= v[r][k].x & take[r];
                                nxt[r][4 * k + 1] |= v[r][k].y & take[r];
                                nxt[r][4 * k + 2] |= v[r][k].z & take[r];
                                nxt[r][4 * k + 3] |= v[r][k].w & take[r];
                            }
                    } else {
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int k = 0; k < W; ++k) nxt[r][k] |= row[r][k] & take[r];
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                nxt[r][W - 1] &= a.last_word_mask;  // a stray pad bit must not become a state number
                uint32_t any = 0;
#pragma unroll
                for (int w = 0; w < W; ++w) {
                    cur[r][w] = nxt[r][w];
                    any |= nxt[r][w];
                }
                live[r] = any != 0;  // an empty set stays empty
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int q = q0 + r * a.threads_per_token;
            if (q >= a.S) continue;
            uint32_t *out = a.rel + ((size_t)t * a.S + q) * W;
            if (W % 4 == 0) {
#pragma unroll
                for (int k = 0; k < W / 4; ++k)
                    reinterpret_cast<uint4 *>(out)[k] = make_uint4(cur[r][4 * k], cur[r][4 * k + 1],
                                                                   cur[r][4 * k + 2], cur[r][4 * k + 3]);
            } else {
#pragma unroll
                for (int w = 0; w < W; ++w) out[w] = cur[r][w];
            }
#pragma unroll
            for (int w = 0; w < W; ++w) {
                if (a.hash && cur[r][w]) {  // most words of a relation are empty: their terms are zero
                    const uint32_t e = 2u * (uint32_t)(q * W + w);  // 16-bit entries 2(qW+w), 2(qW+w)+1
                    if (cur[r][w] & 0xFFFFu)
                        h += (splitmix64_at(a.seed, e) | 1ull) * (uint64_t)(cur[r][w] & 0xFFFFu);
                    if (cur[r][w] >> 16)
                        h += (splitmix64_at(a.seed, e + 1u) | 1ull) * (uint64_t)(cur[r][w] >> 16);
                }
            }
        }
    }
    if (a.hash) {
        if (h) atomicAdd(&hash_sum[slot], (unsigned long long)h);
        __syncthreads();
        if (q0 == 0 && t < a.V) a.hash[t] = hash_sum[slot];
    }
}

constexpr int kRowsPerThread = 1;

template <int W>
int launch_nfa(const NfaArgs &a, hipStream_t stream) {
    const int per_block = kThreads / a.threads_per_token;
    hipLaunchKernelGGL((nfa_walk_kernel<W, kRowsPerThread>), dim3((unsigned)ceil_div(a.V, per_block)),
                       dim3(kThreads), 0, stream, a);
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
    while (a.threads_per_token * kRowsPerThread < S) a.threads_per_token *= 2;
    a.last_word_mask = (S & 31) ? (1u << (S & 31)) - 1u : 0xFFFFFFFFu;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
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
