// Engine side for grammars given as a deterministic byte automaton (paper Section 2.2: a token
// is allowed iff the extended sequence is still a prefix of the language; Section 3.1
// "Inference": the engine runs on the vocabulary E of class representatives and is advanced
// with r[c[t]] in place of the sampled token t).
//
// With sig_rep[k][q] = state reached from q on the bytes of class k's representative (the
// signatures of the representatives) and live[q] = "an accepting state is reachable from q":
//   state_mask[q] bit k = live[sig_rep[k][q]]      class-level mask of every automaton state,
//                                                  computed once per grammar
//   cls_bits[b]         = state_mask[state[b]]     the engine's mask m over E for sequence b
//   state[b]           <- sig_rep[c[tok[b]]][state[b]]

#include <algorithm>

#include "common.hpp"

namespace cfgzip {
namespace {

constexpr int kThreads = 256;
constexpr int kStateWords = 65536 / 32;  // one bit per uint16 value

// Lanes are 64 consecutive states; a wave builds one 32-class word per state at a time from
// 32 coalesced reads of signature rows, looking `live` up in an LDS bitmap.
__global__ __launch_bounds__(kThreads) void state_masks_kernel(const uint16_t *__restrict__ sig_rep,
                                                               int C, int S,
                                                               const uint8_t *__restrict__ live,
                                                               int32_t *__restrict__ state_mask,
                                                               int Wc) {
    __shared__ uint32_t live_bits[kStateWords];
    for (int w = threadIdx.x; w < kStateWords; w += kThreads) {
        uint32_t bits = 0;
        for (int j = 0; j < 32; ++j) {
            const int q = w * 32 + j;
            if (q < S && live[q]) bits |= 1u << j;
        }
        live_bits[w] = bits;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = blockIdx.x * 64 + lane;
    if (q >= S) return;
    const int waves = kThreads / 64;
    for (int wi = blockIdx.y * waves + wave; wi < Wc; wi += gridDim.y * waves) {
        uint32_t word = 0;
#pragma unroll 8
        for (int j = 0; j < 32; ++j) {
            const int k = wi * 32 + j;
            if (k < C) {
                const uint32_t s = sig_rep[(size_t)k * S + q];
                word |= ((live_bits[s >> 5] >> (s & 31)) & 1u) << j;
            }
        }
        state_mask[(size_t)q * Wc + wi] = (int32_t)word;
    }
}

__global__ __launch_bounds__(kThreads) void class_masks_kernel(const int32_t *__restrict__ state_mask,
                                                               int S, int Wc,
                                                               const int32_t *__restrict__ states,
                                                               int32_t *__restrict__ cls_bits) {
    const int b = blockIdx.x;
    const int32_t q = states[b];
    const bool ok = q >= 0 && q < S;
    for (int w = threadIdx.x; w < Wc; w += kThreads)
        cls_bits[(size_t)b * Wc + w] = ok ? state_mask[(size_t)q * Wc + w] : 0;
}

__global__ void advance_states_kernel(const uint16_t *__restrict__ sig_rep, int C, int S,
                                      const int32_t *__restrict__ class_of_token, int V,
                                      const int32_t *__restrict__ tok, int B, int32_t *states) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int32_t t = tok[b], q = states[b];
    int32_t next = -1;
    if (t >= 0 && t < V && q >= 0 && q < S) {
        const int32_t k = class_of_token[t];
        if (k >= 0 && k < C) next = (int32_t)sig_rep[(size_t)k * S + q];
    }
    states[b] = next;
}

// Offsets of the representatives' byte strings: one workgroup; thread i sums the lengths of a
// contiguous run of classes, the runs' totals are scanned in LDS, and the thread writes its run's
// offsets.  An id outside [0, V) counts as an empty string.
constexpr int kScanThreads = 1024;
__global__ __launch_bounds__(kScanThreads) void rep_offsets_kernel(const int64_t *__restrict__ tok_off,
                                                                   int V,
                                                                   const int32_t *__restrict__ rep,
                                                                   int C, int64_t *__restrict__ rep_off) {
    __shared__ int64_t partial[kScanThreads];
    const int i = threadIdx.x;
    const int per = (C + kScanThreads - 1) / kScanThreads;
    const int k0 = min(C, i * per), k1 = min(C, k0 + per);
    auto length = [&](int k) -> int64_t {
        const int32_t t = rep[k];
        return (t >= 0 && t < V) ? tok_off[t + 1] - tok_off[t] : 0;
    };
    int64_t sum = 0;
    for (int k = k0; k < k1; ++k) sum += length(k);
    partial[i] = sum;
    __syncthreads();
    for (int off = 1; off < kScanThreads; off <<= 1) {  // inclusive scan of the run totals
        const int64_t add = i >= off ? partial[i - off] : 0;
        __syncthreads();
        partial[i] += add;
        __syncthreads();
    }
    int64_t at = partial[i] - sum;
    for (int k = k0; k < k1; ++k) {
        rep_off[k] = at;
        at += length(k);
    }
    if (i == kScanThreads - 1) rep_off[C] = partial[i];
}

// A thread per class copies its representative's bytes; bytes beyond the capacity are dropped.
__global__ void rep_bytes_kernel(const uint8_t *__restrict__ tok_bytes,
                                 const int64_t *__restrict__ tok_off, int V,
                                 const int32_t *__restrict__ rep, int C,
                                 const int64_t *__restrict__ rep_off, uint8_t *__restrict__ rep_bytes,
                                 int64_t capacity) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= C) return;
    const int32_t t = rep[k];
    if (t < 0 || t >= V) return;
    const int64_t src = tok_off[t], n = tok_off[t + 1] - src, dst = rep_off[k];
    for (int64_t j = 0; j < n && dst + j < capacity; ++j) rep_bytes[dst + j] = tok_bytes[src + j];
}

// ---- the same engine over a non-deterministic byte automaton: the state is a set of states ----
//   state_mask[q] bit k = some state that the representative of class k reaches from q is live
//   cls_bits[b]         = union of state_mask[q] over the states q of sets[b]
//   sets[b]            <- union over q in sets[b] of rel_rep[c[tok[b]]][q]

// A thread per (state q, word of 32 classes): 32 relation rows tested against the live bitmap.
__global__ __launch_bounds__(kThreads) void nfa_state_masks_kernel(const uint32_t *__restrict__ rel_rep,
                                                                   int C, int S, int W,
                                                                   const uint8_t *__restrict__ live,
                                                                   int32_t *__restrict__ state_mask,
                                                                   int Wc) {
    __shared__ uint32_t live_bits[kStateWords];
    for (int w = threadIdx.x; w < kStateWords; w += kThreads) {
        uint32_t bits = 0;
        for (int j = 0; j < 32; ++j) {
            const int q = w * 32 + j;
            if (q < S && live[q]) bits |= 1u << j;
        }
        live_bits[w] = bits;
    }
    __syncthreads();
    const int64_t item = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (item >= (int64_t)S * Wc) return;
    const int q = (int)(item / Wc), wi = (int)(item % Wc);
    uint32_t word = 0;
    for (int j = 0; j < 32; ++j) {
        const int k = wi * 32 + j;
        if (k >= C) break;
        const uint32_t *row = rel_rep + ((size_t)k * S + q) * W;
        uint32_t hit = 0;
        for (int w = 0; w < W; ++w) hit |= row[w] & live_bits[w];
        if (hit) word |= 1u << j;
    }
    state_mask[(size_t)q * Wc + wi] = (int32_t)word;
}

// A workgroup per sequence; a thread per word of the class mask goes through the set's members.
__global__ __launch_bounds__(kThreads) void nfa_class_masks_kernel(const int32_t *__restrict__ state_mask,
                                                                   int S, int W, int Wc,
                                                                   const uint32_t *__restrict__ sets,
                                                                   int32_t *__restrict__ cls_bits) {
    const int b = blockIdx.x;
    const uint32_t *set = sets + (size_t)b * W;
    for (int wc = threadIdx.x; wc < Wc; wc += kThreads) {
        uint32_t acc = 0;
        for (int w = 0; w < W; ++w) {
            uint32_t bits = set[w];  // the same for every thread
            while (bits) {
                const int q = w * 32 + __ffs(bits) - 1;
                bits &= bits - 1;
                if (q < S) acc |= (uint32_t)state_mask[(size_t)q * Wc + wc];
            }
        }
        cls_bits[(size_t)b * Wc + wc] = (int32_t)acc;
    }
}

// A workgroup per sequence; the old set is read whole before any word of the new one is written.
__global__ __launch_bounds__(kThreads) void nfa_advance_kernel(const uint32_t *__restrict__ rel_rep, int C,
                                                               int S, int W,
                                                               const int32_t *__restrict__ class_of_token,
                                                               int V, const int32_t *__restrict__ tok,
                                                               uint32_t *sets) {
    __shared__ uint32_t old_set[kStateWords];
    const int b = blockIdx.x;
    uint32_t *set = sets + (size_t)b * W;
    for (int w = threadIdx.x; w < W; w += kThreads) old_set[w] = set[w];
    __syncthreads();
    const int32_t t = tok[b];
    const int32_t k = (t < 0 || t >= V) ? -1 : class_of_token[t];
    for (int wo = threadIdx.x; wo < W; wo += kThreads) {
        uint32_t acc = 0;
        if (k >= 0 && k < C) {
            for (int w = 0; w < W; ++w) {
                uint32_t bits = old_set[w];
                while (bits) {
                    const int q = w * 32 + __ffs(bits) - 1;
                    bits &= bits - 1;
                    if (q < S) acc |= rel_rep[((size_t)k * S + q) * W + wo];
                }
            }
        }
        set[wo] = acc;
    }
}

}  // namespace
}  // namespace cfgzip

using namespace cfgzip;

extern "C" int cfgzip_nfa_state_masks(const int32_t *rel_rep, int32_t C, int32_t S, const uint8_t *live,
                                      int32_t *state_mask, void *stream) {
    if (!rel_rep || !live || !state_mask || C <= 0 || S <= 0 || S > 65536) return CFGZIP_E_INVALID;
    if (!aligned_to(rel_rep, 4) || !aligned_to(state_mask, 4)) return CFGZIP_E_INVALID;
    const int Wc = (int)words_for(C), W = (int)words_for(S);
    const int64_t items = (int64_t)S * Wc;
    hipLaunchKernelGGL(nfa_state_masks_kernel, dim3((unsigned)ceil_div(items, kThreads)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<const uint32_t *>(rel_rep), C, S, W,
                       live, state_mask, Wc);
    return check_launch();
}

extern "C" int cfgzip_nfa_class_masks(const int32_t *state_mask, int32_t S, int32_t C,
                                      const int32_t *state_sets, int32_t B, int32_t *cls_bits,
                                      void *stream) {
    if (!state_mask || !state_sets || !cls_bits || S <= 0 || S > 65536 || C <= 0 || B <= 0)
        return CFGZIP_E_INVALID;
    if (!aligned_to(state_mask, 4) || !aligned_to(state_sets, 4) || !aligned_to(cls_bits, 4))
        return CFGZIP_E_INVALID;
    hipLaunchKernelGGL(nfa_class_masks_kernel, dim3(B), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       state_mask, S, (int)words_for(S), (int)words_for(C),
                       reinterpret_cast<const uint32_t *>(state_sets), cls_bits);
    return check_launch();
}

extern "C" int cfgzip_nfa_advance_states(const int32_t *rel_rep, int32_t C, int32_t S,
                                         const int32_t *class_of_token, int32_t V, const int32_t *tok,
                                         int32_t B, int32_t *state_sets, void *stream) {
    if (!rel_rep || !class_of_token || !tok || !state_sets) return CFGZIP_E_INVALID;
    if (C <= 0 || S <= 0 || S > 65536 || V <= 0 || B <= 0) return CFGZIP_E_INVALID;
    hipLaunchKernelGGL(nfa_advance_kernel, dim3(B), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const uint32_t *>(rel_rep), C, S, (int)words_for(S), class_of_token, V,
                       tok, reinterpret_cast<uint32_t *>(state_sets));
    return check_launch();
}

extern "C" int cfgzip_representative_vocabulary(const uint8_t *tok_bytes, const int64_t *tok_off,
                                                int32_t V, const int32_t *rep_of_class, int32_t C,
                                                int64_t *rep_off, uint8_t *rep_bytes,
                                                int64_t capacity, void *stream) {
    if (!tok_off || !rep_of_class || !rep_off || V <= 0 || C <= 0 || capacity < 0) return CFGZIP_E_INVALID;
    if (capacity > 0 && (!rep_bytes || !tok_bytes)) return CFGZIP_E_INVALID;
    if (!aligned_to(tok_off, 8) || !aligned_to(rep_off, 8) || !aligned_to(rep_of_class, 4))
        return CFGZIP_E_INVALID;
    hipLaunchKernelGGL(rep_offsets_kernel, dim3(1), dim3(kScanThreads), 0,
                       static_cast<hipStream_t>(stream), tok_off, V, rep_of_class, C, rep_off);
    CFGZIP_TRY(check_launch());
    if (capacity == 0) return CFGZIP_OK;
    hipLaunchKernelGGL(rep_bytes_kernel, dim3((C + kThreads - 1) / kThreads), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), tok_bytes, tok_off, V, rep_of_class, C,
                       rep_off, rep_bytes, capacity);
    return check_launch();
}

extern "C" int cfgzip_state_masks(const uint16_t *sig_rep, int32_t C, int32_t S, const uint8_t *live,
                                  int32_t *state_mask, void *stream) {
    if (!sig_rep || !live || !state_mask || C <= 0 || S <= 0 || S > 65536) return CFGZIP_E_INVALID;
    if (!aligned_to(sig_rep, 2) || !aligned_to(state_mask, 4)) return CFGZIP_E_INVALID;
    const int Wc = (int)words_for(C);
    const int tiles = (int)ceil_div(S, 64);
    // enough workgroups to fill the chip even for small automata
    int rows = (int)std::min<int64_t>(ceil_div(Wc, kThreads / 64), std::max<int64_t>(1, 2048 / tiles));
    hipLaunchKernelGGL(state_masks_kernel, dim3(tiles, rows), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), sig_rep, C, S, live, state_mask, Wc);
    return check_launch();
}

extern "C" int cfgzip_class_masks(const int32_t *state_mask, int32_t S, int32_t C,
                                  const int32_t *states, int32_t B, int32_t *cls_bits, void *stream) {
    if (!state_mask || !states || !cls_bits || S <= 0 || C <= 0 || B <= 0) return CFGZIP_E_INVALID;
    if (!aligned_to(state_mask, 4) || !aligned_to(states, 4) || !aligned_to(cls_bits, 4))
        return CFGZIP_E_INVALID;
    hipLaunchKernelGGL(class_masks_kernel, dim3(B), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), state_mask, S, (int)words_for(C), states,
                       cls_bits);
    return check_launch();
}

extern "C" int cfgzip_advance_states(const uint16_t *sig_rep, int32_t C, int32_t S,
                                     const int32_t *class_of_token, int32_t V, const int32_t *tok,
                                     int32_t B, int32_t *states, void *stream) {
    if (!sig_rep || !class_of_token || !tok || !states || C <= 0 || S <= 0 || V <= 0 || B <= 0)
        return CFGZIP_E_INVALID;
    hipLaunchKernelGGL(advance_states_kernel, dim3((B + kThreads - 1) / kThreads), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), sig_rep, C, S, class_of_token, V, tok, B,
                       states);
    return check_launch();
}
