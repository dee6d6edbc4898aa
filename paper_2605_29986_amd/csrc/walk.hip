// cfgzip_signatures: byte-walk signatures of all tokens and their hash
// (paper Section 3.2.1 / Algorithm 1, regular case; see walk_device.hpp).
//
// Work item = (group of M tokens, block of 64*K start states), one wavefront
// each; lanes are start states, so every table read of a step goes to one
// column Tt[byte][*].  Automata whose whole transposed table fits in LDS are
// walked from LDS; larger ones are walked from the L2-resident copy in the
// workspace.  Automata with fewer than 64 states pack several tokens per wave.

#include <algorithm>

#include "common.hpp"
#include "walk_device.hpp"

namespace cfgzip {
namespace {

struct WalkArgs {
    const uint8_t *tok_bytes;
    const int64_t *tok_off;
    int32_t V;
    int32_t S;
    const uint16_t *Tt;   // [256][S] (+ pad), workspace
    const uint64_t *mult; // [S] hash multipliers a_q, workspace
    uint16_t *sig_out;    // [V][S] or null
    uint64_t *hash_out;   // [V] or null
};

// Tt[b][q] = table[q][b]
__global__ __launch_bounds__(256) void transpose_table_kernel(const uint16_t *__restrict__ table,
                                                              uint16_t *__restrict__ Tt, int S) {
    __shared__ uint16_t tile[64][65];
    const int q0 = blockIdx.x * 64, b0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;  // 64 x 4
    for (int r = ty; r < 64; r += 4) {
        const int q = q0 + r;
        tile[r][tx] = q < S ? table[(size_t)q * 256 + b0 + tx] : (uint16_t)0;
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        const int q = q0 + tx;
        if (q < S) Tt[(size_t)(b0 + r) * S + q] = tile[tx][r];
    }
}

__global__ void fill_pad_and_multipliers_kernel(uint16_t *Tt_pad, int n_pad, uint64_t *mult, int S,
                                                uint64_t seed) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_pad) Tt_pad[i] = 0;
    if (i < S) mult[i] = splitmix64_at(seed, (uint32_t)i) | 1ull;
}

__global__ void zero_u64_kernel(uint64_t *p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// S >= 64 (or any S when no narrow variant applies): lanes = start states.
template <int K, int M, bool LDS_TABLE>
__global__ __launch_bounds__(LDS_TABLE ? 1024 : 256) void walk_wide_kernel(WalkArgs a) {
    extern __shared__ uint16_t t_lds[];
    if (LDS_TABLE) {
        const int n16 = a.S * 32;  // S*512 bytes / 16
        const uint4 *src = reinterpret_cast<const uint4 *>(a.Tt);
        uint4 *dst = reinterpret_cast<uint4 *>(t_lds);
        for (int i = threadIdx.x; i < n16; i += blockDim.x) dst[i] = src[i];
        __syncthreads();
    }
    const uint16_t *tab = LDS_TABLE ? t_lds : a.Tt;

    const int lane = threadIdx.x & 63;
    const int waves_per_block = blockDim.x >> 6;
    const int64_t gw = (int64_t)blockIdx.x * waves_per_block + (threadIdx.x >> 6);
    const int64_t total_waves = (int64_t)gridDim.x * waves_per_block;
    constexpr int SB = 64 * K;
    const int S = a.S;
    const int nsb = (S + SB - 1) / SB;
    const int64_t n_items = ((int64_t)a.V + M - 1) / M * nsb;

    for (int64_t i = gw; i < n_items; i += total_waves) {
        const int sb = (int)(i % nsb);
        const int64_t t0 = (i / nsb) * M;
        int64_t beg[M];
        int len[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const bool tv = t0 + m < a.V;
            const int64_t o0 = tv ? a.tok_off[t0 + m] : 0;
            const int64_t o1 = tv ? a.tok_off[t0 + m + 1] : 0;
            beg[m] = o0;
            len[m] = __builtin_amdgcn_readfirstlane((int)(o1 - o0));
        }
        int q[K];
        uint32_t cur[M][K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            q[k] = sb * SB + k * 64 + lane;
#pragma unroll
            for (int m = 0; m < M; ++m) cur[m][k] = q[k] < S ? (uint32_t)q[k] : 0u;
        }
        walk_uniform<K, M>(tab, S, a.tok_bytes, beg, len, cur);

#pragma unroll
        for (int m = 0; m < M; ++m) {
            if (t0 + m >= a.V) continue;
            if (a.sig_out) {
#pragma unroll
                for (int k = 0; k < K; ++k)
                    if (q[k] < S) a.sig_out[(size_t)(t0 + m) * S + q[k]] = (uint16_t)cur[m][k];
            }
            if (a.hash_out) {
                uint64_t h = 0;
#pragma unroll
                for (int k = 0; k < K; ++k)
                    if (q[k] < S) h += a.mult[q[k]] * (uint64_t)cur[m][k];
                h = wave_sum_u64(h);
                if (lane == 0) {
                    if (nsb == 1) a.hash_out[t0 + m] = h;
                    else atomicAdd(reinterpret_cast<unsigned long long *>(a.hash_out + t0 + m),
                                   (unsigned long long)h);
                }
            }
        }
    }
}

// S < 64: a wave holds 64 / SP tokens, SP = smallest power of two >= S; table in LDS.
__global__ __launch_bounds__(256) void walk_narrow_kernel(WalkArgs a, int SP) {
    extern __shared__ uint16_t t_lds[];
    {
        const int n16 = a.S * 32;
        const uint4 *src = reinterpret_cast<const uint4 *>(a.Tt);
        uint4 *dst = reinterpret_cast<uint4 *>(t_lds);
        for (int i = threadIdx.x; i < n16; i += blockDim.x) dst[i] = src[i];
        __syncthreads();
    }
    const int S = a.S;
    const int per_thread_block = blockDim.x / SP;  // tokens per workgroup pass
    const int slot = threadIdx.x / SP;
    const int q = threadIdx.x % SP;
    for (int64_t t = (int64_t)blockIdx.x * per_thread_block + slot; t < a.V;
         t += (int64_t)gridDim.x * per_thread_block) {
        // lanes of one token slot that lie beyond S idle through the walk
        const int64_t beg = a.tok_off[t];
        const int len = (int)(a.tok_off[t + 1] - beg);
        uint32_t cur = q < S ? (uint32_t)q : 0u;
        for (int p = 0; p < len; ++p) {
            const uint32_t b = a.tok_bytes[beg + p];
            cur = t_lds[b * S + cur];
        }
        if (q < S && a.sig_out) a.sig_out[(size_t)t * S + q] = (uint16_t)cur;
        if (a.hash_out) {
            uint64_t h = q < S ? a.mult[q] * (uint64_t)cur : 0ull;
            h = wave_sum_u64(h, SP);
            if (q == 0) a.hash_out[t] = h;
        }
    }
}

constexpr size_t kLdsTableLimit = 144 * 1024;

template <int K, int M>
int launch_wide(const WalkArgs &a, bool lds, int n_cu, hipStream_t stream) {
    if (lds) {
        auto kern = walk_wide_kernel<K, M, true>;
        const size_t bytes = (size_t)a.S * 512;
        if (bytes > 64 * 1024)
            CFGZIP_TRY(check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     (int)bytes)));
        const int per_cu = (int)std::max<size_t>(1, std::min<size_t>(2, (160 * 1024) / bytes));
        hipLaunchKernelGGL(kern, dim3(n_cu * per_cu), dim3(1024), bytes, stream, a);
    } else {
        auto kern = walk_wide_kernel<K, M, false>;
        hipLaunchKernelGGL(kern, dim3(n_cu * 8), dim3(256), 0, stream, a);
    }
    return check_launch();
}

int device_cu_count(int *out) {
    int dev = 0;
    CFGZIP_TRY(check_hip(hipGetDevice(&dev)));
    int n = 0;
    CFGZIP_TRY(check_hip(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev)));
    *out = n > 0 ? n : 256;
    return CFGZIP_OK;
}

}  // namespace

// Layout of the signature workspace: Tt (+pad), then the hash multipliers.
struct SigWorkspace {
    uint16_t *Tt;
    uint64_t *mult;
    size_t bytes;
};

static SigWorkspace carve_sig_ws(void *ws, int32_t S) {
    Carver c(ws);
    SigWorkspace w;
    w.Tt = c.take<uint16_t>((size_t)256 * S + kTablePad);
    w.mult = c.take<uint64_t>((size_t)S);
    w.bytes = c.used;
    return w;
}

// Builds Tt and the multipliers in the workspace.  Shared with the class builder.
int prepare_tables(const uint16_t *table, int32_t S, uint64_t hash_seed, void *ws,
                   const uint16_t **Tt_out, const uint64_t **mult_out, hipStream_t stream) {
    SigWorkspace w = carve_sig_ws(ws, S);
    hipLaunchKernelGGL(transpose_table_kernel, dim3((S + 63) / 64, 4), dim3(256), 0, stream, table,
                       w.Tt, S);
    CFGZIP_TRY(check_launch());
    const int n = std::max(kTablePad, S);
    hipLaunchKernelGGL(fill_pad_and_multipliers_kernel, dim3((n + 255) / 256), dim3(256), 0, stream,
                       w.Tt + (size_t)256 * S, kTablePad, w.mult, S, hash_seed);
    CFGZIP_TRY(check_launch());
    *Tt_out = w.Tt;
    *mult_out = w.mult;
    return CFGZIP_OK;
}

size_t sig_workspace_bytes(int32_t S) { return carve_sig_ws(nullptr, S).bytes; }

}  // namespace cfgzip

using namespace cfgzip;

extern "C" size_t cfgzip_signatures_workspace_bytes(int32_t V, int32_t S) {
    if (V <= 0 || S <= 0 || S > 65536) return 0;
    return sig_workspace_bytes(S);
}

extern "C" int cfgzip_signatures(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                                 const uint16_t *table, int32_t S, uint16_t *sig_out,
                                 uint64_t *hash_out, uint64_t hash_seed, void *ws, size_t ws_bytes,
                                 void *stream_) {
    if (!tok_off || !table || V <= 0 || S <= 0 || S > 65536) return CFGZIP_E_INVALID;
    if (!sig_out && !hash_out) return CFGZIP_E_INVALID;
    if (!aligned_to(tok_off, 8) || !aligned_to(table, 2) || !aligned_to(sig_out, 2) ||
        !aligned_to(hash_out, 8))
        return CFGZIP_E_INVALID;
    if (!ws || ws_bytes < sig_workspace_bytes(S) || !aligned_to(ws, 256)) return CFGZIP_E_WORKSPACE;
    // tok_bytes may be null only if every token is empty; the kernels never read it then.
    hipStream_t stream = static_cast<hipStream_t>(stream_);

    WalkArgs a{};
    a.tok_bytes = tok_bytes;
    a.tok_off = tok_off;
    a.V = V;
    a.S = S;
    a.sig_out = sig_out;
    a.hash_out = hash_out;
    CFGZIP_TRY(prepare_tables(table, S, hash_seed, ws, &a.Tt, &a.mult, stream));

    int n_cu = 256;
    CFGZIP_TRY(device_cu_count(&n_cu));
    const bool lds = (size_t)S * 512 <= kLdsTableLimit;

    if (S < 64) {
        int SP = 1;
        while (SP < S) SP <<= 1;
        const int tokens_per_block = 256 / SP;
        int64_t blocks = ceil_div(V, tokens_per_block);
        blocks = std::min<int64_t>(blocks, (int64_t)n_cu * 8);
        hipLaunchKernelGGL(walk_narrow_kernel, dim3((int)blocks), dim3(256), (size_t)S * 512, stream,
                           a, SP);
        return check_launch();
    }
    const int nsb4 = (S + 255) / 256;
    if (hash_out && S > 256) {
        hipLaunchKernelGGL(zero_u64_kernel, dim3((V + 255) / 256), dim3(256), 0, stream, hash_out,
                           (int64_t)V);
        CFGZIP_TRY(check_launch());
    }
    (void)nsb4;
    if (S <= 64) return launch_wide<1, 4>(a, lds, n_cu, stream);
    if (S <= 128) return launch_wide<2, 4>(a, lds, n_cu, stream);
    return launch_wide<4, 2>(a, lds, n_cu, stream);
}
