// Device-side byte walk shared by the signature kernels and by the class
// builder's re-walk verification (paper Section 3.2.1 / Algorithm 1 restricted to
// a deterministic byte automaton:  sig[t][q] = delta*(q, bytes(t))).
//
// Table layout used on the device: the caller's table[q][b] is transposed once
// into Tt[b][q] so that one token byte selects one contiguous column of S
// uint16 entries; a wavefront's lanes are start states, the byte is uniform.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cfgzip {

// Tt is over-allocated by this many entries so that a table entry >= S (a
// caller error) still indexes inside the workspace.
constexpr int kTablePad = 65536;

__device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint32_t index) {
    // index-th output (0-based) of the SplitMix64 generator seeded with `seed`
    uint64_t z = seed + (uint64_t)(index + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v, int width = 64) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        if (off < width) v += __shfl_xor(v, off, 64);
    }
    return v;
}

// Walks M tokens at once from K start states per lane.  `tab` points at Tt
// (global or LDS).  beg/len are wave-uniform.  cur[m][k] must hold the start
// states on entry and holds the end states on return.
template <int K, int M>
__device__ __forceinline__ void walk_uniform(const uint16_t *tab, int S,
                                             const uint8_t *__restrict__ tok_bytes,
                                             const int64_t (&beg)[M], const int (&len)[M],
                                             uint32_t (&cur)[M][K]) {
    const int lane = threadIdx.x & 63;
    int maxlen = 0;
#pragma unroll
    for (int m = 0; m < M; ++m) maxlen = max(maxlen, len[m]);
    for (int base = 0; base < maxlen; base += 64) {
        uint32_t mybyte[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int idx = base + lane;
            mybyte[m] = idx < len[m] ? (uint32_t)tok_bytes[beg[m] + idx] : 0u;
        }
        const int steps = min(64, maxlen - base);
        for (int p = 0; p < steps; ++p) {
#pragma unroll
            for (int m = 0; m < M; ++m) {
                if (base + p < len[m]) {  // wave-uniform
                    const uint32_t b = __builtin_amdgcn_readlane(mybyte[m], p);
                    const uint16_t *col = tab + (size_t)b * S;
#pragma unroll
                    for (int k = 0; k < K; ++k) cur[m][k] = col[cur[m][k]];
                }
            }
        }
    }
}

}  // namespace cfgzip
