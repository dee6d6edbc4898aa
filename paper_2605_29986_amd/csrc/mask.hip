// Per-decode-step kernels: class mask -> token mask, -inf masking of logits,
// sampled token -> representative (paper Section 3.1 "Inference", Figure 1;
// Section 2.2 for the meaning of a mask).
//
// One kernel template covers expand, apply and the fused expand+apply.  The
// path is HBM-bound: every logit is read once and written once with 16-byte
// accesses, the class-level mask rows of a row chunk live in LDS, and the class
// ids of a thread's eight columns stay in registers across the rows.

#include <type_traits>

#include "common.hpp"

namespace cfgzip {

static thread_local hipError_t g_last_hip_error = hipSuccess;
void set_last_hip_error(hipError_t e) { g_last_hip_error = e; }

namespace {

constexpr int kThreads = 256;
constexpr int kCols = 8;                       // columns (tokens) per thread
constexpr int kTileCols = kThreads * kCols;    // 2048 columns per workgroup
constexpr int kUnroll = 2;                     // rows in flight per thread
constexpr int kRowsStream = 4;                 // rows per workgroup when logits are streamed
constexpr int kRowsStreamFusedBf16 = 2;        // the same for bf16 logits masked from class bits (measured best of 1, 2, 3, 4, 8)
constexpr int kRowsExpand = 16;                // rows per workgroup for mask expansion alone
constexpr int kMaxRowsPerBlock = 16;           // the larger of the two

enum : int { LOGITS_NONE = 0, LOGITS_BF16 = 1, LOGITS_F32 = 2 };

// native 16-byte vector (the nontemporal builtins do not take HIP's uint4 struct)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// streaming 16-byte accesses: every logit is touched exactly once per call
__device__ __forceinline__ u32x4 load16(const void *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}
__device__ __forceinline__ void store16(void *p, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
}

struct MaskArgs {
    void *logits;
    int64_t row_stride;  // elements
    int32_t B, V;
    const int32_t *bits_in;  // class bits [B][Wc] or token bits [B][Wv]
    int32_t Wc, Wv;
    const int32_t *class_of_token;
    int32_t *tok_bits_out;
    int32_t rows_per_block;
    int32_t col_tiles;
    // engine step (all null otherwise): the class-mask row of sequence b is row q[b] of
    // state_mask, q[b] the sequence's automaton state after the token sampled last
    const int32_t *state_mask;  // [S][Wc]
    const uint16_t *sig_rep;    // [C][S]
    const int32_t *tok_prev;    // [B] or null: no advance
    const int32_t *states_in;   // [B]
    int32_t *states_out;        // [B]
    int32_t S, C;
    // decode step (null otherwise): the first workgroup also maps the sampled tokens to their
    // representatives once its own rows are streamed
    const int32_t *map_tok;       // [B]
    const int32_t *rep_of_class;  // [map_C]
    int32_t *map_out;             // [B]
    int32_t map_C;
};

__device__ __forceinline__ uint32_t select_bf16_pair(uint32_t x, uint32_t two_bits) {
    // two_bits: bit 0 -> low half allowed, bit 1 -> high half allowed
    uint32_t keep = ((0u - (two_bits & 1u)) & 0x0000FFFFu) | ((0u - (two_bits >> 1)) & 0xFFFF0000u);
    return (x & keep) | (0xFF80FF80u & ~keep);
}

// LOGITS: which logits to mask (none = mask expansion only).
// FROM_CLASS: bits_in is a class-level mask gathered through class_of_token.
// WRITE_BITS: also store the token-level mask.
// VEC: logits rows and class_of_token allow 16-byte accesses at column multiples of 8.
template <int LOGITS, bool FROM_CLASS, bool WRITE_BITS, bool VEC>
__device__ __forceinline__ void mask_tile(const MaskArgs &a, uint32_t *cls_lds) {

    const int ct = blockIdx.x % a.col_tiles;
    const int rc = blockIdx.x / a.col_tiles;
    const int r0 = rc * a.rows_per_block;
    const int nrows = min(a.rows_per_block, a.B - r0);
    const int col0 = (ct * kThreads + (int)threadIdx.x) * kCols;

    if (FROM_CLASS) {
        const int n = nrows * a.Wc;
        if (a.state_mask) {
            // engine step: advance the rows' automaton states on the representative of the token
            // sampled last, then take each row's class mask from the table of per-state masks
            __shared__ int32_t q_s[kMaxRowsPerBlock];
            if ((int)threadIdx.x < nrows) {
                const int b = r0 + threadIdx.x;
                int32_t q = a.states_in[b];
                if (a.tok_prev) {
                    const int32_t t = a.tok_prev[b];
                    int32_t next = -1;
                    if (t >= 0 && t < a.V && q >= 0 && q < a.S) {
                        const int32_t k = a.class_of_token[t];
                        if (k >= 0 && k < a.C) next = (int32_t)a.sig_rep[(size_t)k * a.S + q];
                    }
                    q = next;
                }
                q_s[threadIdx.x] = (q >= 0 && q < a.S) ? q : -1;
                if (ct == 0) a.states_out[b] = q;  // one column tile writes the new states
            }
            __syncthreads();
            for (int i = threadIdx.x; i < n; i += kThreads) {
                const int r = i / a.Wc, w = i - r * a.Wc;
                const int32_t q = q_s[r];
                cls_lds[i] = q >= 0 ? (uint32_t)a.state_mask[(size_t)q * a.Wc + w] : 0u;
            }
        } else {
            const uint32_t *src = reinterpret_cast<const uint32_t *>(a.bits_in) + (int64_t)r0 * a.Wc;
            for (int i = threadIdx.x; i < n; i += kThreads) cls_lds[i] = src[i];
        }
        __syncthreads();
    }
    if (col0 >= a.Wv * 32) return;  // past the padded end of a mask row: nothing to do

    const int nvalid = min(kCols, max(0, a.V - col0));
    const uint32_t valid_mask = (1u << nvalid) - 1u;
    const bool full = nvalid == kCols;

    uint32_t woff[kCols], shift[kCols];
    if (FROM_CLASS) {
        int32_t k[kCols];
        if (VEC && full) {
            const int4 *p = reinterpret_cast<const int4 *>(a.class_of_token + col0);
            int4 lo = p[0], hi = p[1];
            k[0] = lo.x; k[1] = lo.y; k[2] = lo.z; k[3] = lo.w;
            k[4] = hi.x; k[5] = hi.y; k[6] = hi.z; k[7] = hi.w;
        } else {
#pragma unroll
            for (int j = 0; j < kCols; ++j) k[j] = j < nvalid ? a.class_of_token[col0 + j] : 0;
        }
#pragma unroll
        for (int j = 0; j < kCols; ++j) {
            woff[j] = (uint32_t)k[j] >> 5;
            shift[j] = (uint32_t)k[j] & 31u;
        }
    }

    auto row_mask = [&](int r) -> uint32_t {  // r relative to r0
        uint32_t m = 0;
        if (FROM_CLASS) {
            const uint32_t *row = cls_lds + r * a.Wc;
#pragma unroll
            for (int j = 0; j < kCols; ++j) m |= ((row[woff[j]] >> shift[j]) & 1u) << j;
        } else {
            const uint8_t *row = reinterpret_cast<const uint8_t *>(a.bits_in) +
                                 (int64_t)(r0 + r) * a.Wv * 4;
            m = row[col0 >> 3];
        }
        return m & valid_mask;
    };
    auto store_bits = [&](int r, uint32_t m) {
        if (WRITE_BITS) {
            uint8_t *row = reinterpret_cast<uint8_t *>(a.tok_bits_out) + (int64_t)(r0 + r) * a.Wv * 4;
            row[col0 >> 3] = (uint8_t)m;
        }
    };

    if (LOGITS == LOGITS_NONE) {
        for (int r = 0; r < nrows; ++r) store_bits(r, row_mask(r));
        return;
    }

    if (VEC && full) {
        if (LOGITS == LOGITS_BF16) {
            uint16_t *base = reinterpret_cast<uint16_t *>(a.logits) + (int64_t)r0 * a.row_stride + col0;
            auto masked = [](u32x4 x, uint32_t m) -> u32x4 {
                u32x4 y;
                y.x = select_bf16_pair(x.x, m & 3u);
                y.y = select_bf16_pair(x.y, (m >> 2) & 3u);
                y.z = select_bf16_pair(x.z, (m >> 4) & 3u);
                y.w = select_bf16_pair(x.w, (m >> 6) & 3u);
                return y;
            };
            int r = 0;
            for (; r + kUnroll <= nrows; r += kUnroll) {
                u32x4 x[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) x[u] = load16(base + (int64_t)(r + u) * a.row_stride);
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const uint32_t m = row_mask(r + u);
                    store16(base + (int64_t)(r + u) * a.row_stride, masked(x[u], m));
                    store_bits(r + u, m);
                }
            }
            for (; r < nrows; ++r) {
                const uint32_t m = row_mask(r);
                store16(base + (int64_t)r * a.row_stride, masked(load16(base + (int64_t)r * a.row_stride), m));
                store_bits(r, m);
            }
        } else {  // fp32: two 16-byte accesses per thread and row
            uint32_t *base = reinterpret_cast<uint32_t *>(a.logits) + (int64_t)r0 * a.row_stride + col0;
            constexpr uint32_t NINF = 0xFF800000u;
            constexpr int U = 4;  // rows in flight (eight 16-byte loads): measured best of 1, 2, 4
            auto do_rows = [&](int r, auto count) {
                constexpr int N = decltype(count)::value;
                u32x4 x[N][2];
#pragma unroll
                for (int u = 0; u < N; ++u) {
                    x[u][0] = load16(base + (int64_t)(r + u) * a.row_stride);
                    x[u][1] = load16(base + (int64_t)(r + u) * a.row_stride + 4);
                }
#pragma unroll
                for (int u = 0; u < N; ++u) {
                    const uint32_t m = row_mask(r + u);
                    u32x4 lo = x[u][0], hi = x[u][1];
                    lo.x = (m & 1u) ? lo.x : NINF;
                    lo.y = (m & 2u) ? lo.y : NINF;
                    lo.z = (m & 4u) ? lo.z : NINF;
                    lo.w = (m & 8u) ? lo.w : NINF;
                    hi.x = (m & 16u) ? hi.x : NINF;
                    hi.y = (m & 32u) ? hi.y : NINF;
                    hi.z = (m & 64u) ? hi.z : NINF;
                    hi.w = (m & 128u) ? hi.w : NINF;
                    store16(base + (int64_t)(r + u) * a.row_stride, lo);
                    store16(base + (int64_t)(r + u) * a.row_stride + 4, hi);
                    store_bits(r + u, m);
                }
            };
            int r = 0;
            for (; r + U <= nrows; r += U) do_rows(r, std::integral_constant<int, U>{});
            for (; r < nrows; ++r) do_rows(r, std::integral_constant<int, 1>{});
        }
        return;
    }

    // element-wise path: ragged last columns of a row, or rows that are not 16-byte aligned
    for (int r = 0; r < nrows; ++r) {
        uint32_t m = row_mask(r);
        if (LOGITS == LOGITS_BF16) {
            uint16_t *p = reinterpret_cast<uint16_t *>(a.logits) + (int64_t)(r0 + r) * a.row_stride + col0;
            for (int j = 0; j < nvalid; ++j)
                if (!((m >> j) & 1u)) p[j] = 0xFF80u;
        } else {
            uint32_t *p = reinterpret_cast<uint32_t *>(a.logits) + (int64_t)(r0 + r) * a.row_stride + col0;
            for (int j = 0; j < nvalid; ++j)
                if (!((m >> j) & 1u)) p[j] = 0xFF800000u;
        }
        store_bits(r, m);
    }
}

// out = rep_of_class[class_of_token[t]], or -1 when the token id or its class id is out of range
__device__ __forceinline__ int32_t representative_of(int32_t t, const int32_t *class_of_token,
                                                     int32_t V, const int32_t *rep_of_class,
                                                     int32_t C) {
    if (t < 0 || t >= V) return -1;
    const int32_t k = class_of_token[t];
    return (k >= 0 && k < C) ? rep_of_class[k] : -1;
}

template <int LOGITS, bool FROM_CLASS, bool WRITE_BITS, bool VEC>
__global__ __launch_bounds__(kThreads) void mask_kernel(MaskArgs a) {
    extern __shared__ uint32_t cls_lds[];  // [rows_per_block][Wc] when FROM_CLASS
    mask_tile<LOGITS, FROM_CLASS, WRITE_BITS, VEC>(a, cls_lds);
    // The first workgroup is the first to be scheduled and to finish its rows; the B dependent
    // look-ups then overlap with the streaming of all the others.
    if (a.map_tok && blockIdx.x == 0)
        for (int b = threadIdx.x; b < a.B; b += kThreads)
            a.map_out[b] = representative_of(a.map_tok[b], a.class_of_token, a.V, a.rep_of_class, a.map_C);
}

__global__ void map_to_rep_kernel(const int32_t *tok, int32_t B, const int32_t *class_of_token,
                                  int32_t V, const int32_t *rep_of_class, int32_t C, int32_t *out) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    out[b] = representative_of(tok[b], class_of_token, V, rep_of_class, C);
}

constexpr size_t kMaxLds = 160 * 1024;

template <int LOGITS, bool FROM_CLASS, bool WRITE_BITS, bool VEC>
int launch_mask(const MaskArgs &args, int grid, size_t lds_bytes, hipStream_t stream) {
    auto kern = mask_kernel<LOGITS, FROM_CLASS, WRITE_BITS, VEC>;
    if (lds_bytes > 64 * 1024) {
        CFGZIP_TRY(check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 (int)lds_bytes)));
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds_bytes, stream, args);
    return check_launch();
}

template <int LOGITS, bool FROM_CLASS>
int dispatch_mask(const MaskArgs &args, bool write_bits, bool vec, int grid, size_t lds,
                  hipStream_t stream) {
    if (write_bits) {
        return vec ? launch_mask<LOGITS, FROM_CLASS, true, true>(args, grid, lds, stream)
                   : launch_mask<LOGITS, FROM_CLASS, true, false>(args, grid, lds, stream);
    }
    if (LOGITS == LOGITS_NONE) return CFGZIP_E_INVALID;  // nothing to do
    return vec ? launch_mask<LOGITS, FROM_CLASS, false, true>(args, grid, lds, stream)
               : launch_mask<LOGITS, FROM_CLASS, false, false>(args, grid, lds, stream);
}

// Shared host path of cfgzip_expand_mask and cfgzip_apply_mask.
struct EngineStep {
    const int32_t *state_mask;
    const uint16_t *sig_rep;
    const int32_t *tok_prev;
    const int32_t *states_in;
    int32_t *states_out;
    int32_t S;
};
struct MapStep {
    const int32_t *tok;
    const int32_t *rep_of_class;
    int32_t *out;
};

int run_mask(void *logits, int logits_kind, int32_t B, int32_t V, int64_t row_stride,
             const int32_t *bits, bool from_class, const int32_t *class_of_token, int32_t C,
             int32_t *tok_bits_out, hipStream_t stream, const EngineStep *engine = nullptr,
             const MapStep *map = nullptr) {
    MaskArgs a{};
    if (map) {
        a.map_tok = map->tok;
        a.rep_of_class = map->rep_of_class;
        a.map_out = map->out;
        a.map_C = C;
    }
    if (engine) {
        a.state_mask = engine->state_mask;
        a.sig_rep = engine->sig_rep;
        a.tok_prev = engine->tok_prev;
        a.states_in = engine->states_in;
        a.states_out = engine->states_out;
        a.S = engine->S;
        a.C = C;
    }
    a.logits = logits;
    a.row_stride = row_stride;
    a.B = B;
    a.V = V;
    a.bits_in = bits;
    a.Wc = from_class ? (int32_t)words_for(C) : 0;
    a.Wv = (int32_t)words_for(V);
    a.class_of_token = class_of_token;
    a.tok_bits_out = tok_bits_out;

    size_t row_bytes = (size_t)a.Wc * 4;
    // Measured on MI355X at batch 256 x 128,256 bf16: small row chunks (many workgroups, two
    // rows in flight per thread) stream fastest; the class ids of a tile are re-read from L2.
    int rows = logits_kind == LOGITS_NONE ? kRowsExpand : kRowsStream;
    // (the engine step's staging phase wants the larger chunk: it is paid per workgroup)
    if (logits_kind == LOGITS_BF16 && from_class && !engine) rows = kRowsStreamFusedBf16;
    if (from_class) {
        if (row_bytes > kMaxLds) return CFGZIP_E_INVALID;  // one class-mask row must fit in LDS
        while (rows > 1 && rows * row_bytes > 64 * 1024) rows /= 2;
    }
    if (rows > B) rows = B;
    a.rows_per_block = rows;
    a.col_tiles = (int32_t)ceil_div((int64_t)a.Wv * 32, kTileCols);
    int64_t grid = (int64_t)a.col_tiles * ceil_div(B, rows);
    if (grid > 0x7FFFFFFF) return CFGZIP_E_INVALID;
    size_t lds = from_class ? (size_t)rows * row_bytes : 0;

    size_t esz = logits_kind == LOGITS_BF16 ? 2 : 4;
    bool vec = true;
    if (logits_kind != LOGITS_NONE)
        vec = aligned_to(logits, 16) && (row_stride * (int64_t)esz) % 16 == 0;
    if (from_class) vec = vec && aligned_to(class_of_token, 16);

    const bool wb = tok_bits_out != nullptr;
    switch (logits_kind) {
        case LOGITS_NONE:
            return dispatch_mask<LOGITS_NONE, true>(a, wb, vec, (int)grid, lds, stream);
        case LOGITS_BF16:
            return from_class ? dispatch_mask<LOGITS_BF16, true>(a, wb, vec, (int)grid, lds, stream)
                              : dispatch_mask<LOGITS_BF16, false>(a, wb, vec, (int)grid, lds, stream);
        default:
            return from_class ? dispatch_mask<LOGITS_F32, true>(a, wb, vec, (int)grid, lds, stream)
                              : dispatch_mask<LOGITS_F32, false>(a, wb, vec, (int)grid, lds, stream);
    }
}

}  // namespace
}  // namespace cfgzip

using namespace cfgzip;

extern "C" int cfgzip_last_hip_error(void) { return (int)g_last_hip_error; }

extern "C" int cfgzip_version(void) { return 100; }

extern "C" int cfgzip_expand_mask(const int32_t *cls_bits, int32_t B, int32_t C,
                                  const int32_t *class_of_token, int32_t V, int32_t *tok_bits,
                                  void *stream) {
    if (!cls_bits || !class_of_token || !tok_bits || B <= 0 || C <= 0 || V <= 0)
        return CFGZIP_E_INVALID;
    if (!aligned_to(cls_bits, 4) || !aligned_to(class_of_token, 4) || !aligned_to(tok_bits, 4))
        return CFGZIP_E_INVALID;
    return run_mask(nullptr, LOGITS_NONE, B, V, 0, cls_bits, true, class_of_token, C, tok_bits,
                    static_cast<hipStream_t>(stream));
}

extern "C" int cfgzip_apply_mask(void *logits, int32_t dtype, int32_t B, int32_t V,
                                 int64_t row_stride, const int32_t *bits, int32_t bits_kind,
                                 const int32_t *class_of_token, int32_t C, int32_t *tok_bits_out,
                                 void *stream) {
    if (!logits || !bits || B <= 0 || V <= 0 || row_stride < V) return CFGZIP_E_INVALID;
    if (dtype != CFGZIP_DTYPE_F32 && dtype != CFGZIP_DTYPE_BF16) return CFGZIP_E_INVALID;
    if (bits_kind != CFGZIP_BITS_TOKEN && bits_kind != CFGZIP_BITS_CLASS) return CFGZIP_E_INVALID;
    const size_t esz = dtype == CFGZIP_DTYPE_BF16 ? 2 : 4;
    if (!aligned_to(logits, esz) || !aligned_to(bits, 4)) return CFGZIP_E_INVALID;
    const bool from_class = bits_kind == CFGZIP_BITS_CLASS;
    if (from_class) {
        if (!class_of_token || C <= 0 || !aligned_to(class_of_token, 4)) return CFGZIP_E_INVALID;
        if (tok_bits_out && !aligned_to(tok_bits_out, 4)) return CFGZIP_E_INVALID;
    } else {
        if (tok_bits_out) return CFGZIP_E_INVALID;  // token bits are the input already
    }
    return run_mask(logits, dtype == CFGZIP_DTYPE_BF16 ? LOGITS_BF16 : LOGITS_F32, B, V, row_stride,
                    bits, from_class, class_of_token, C, tok_bits_out,
                    static_cast<hipStream_t>(stream));
}

extern "C" int cfgzip_engine_step(void *logits, int32_t dtype, int32_t B, int32_t V,
                                  int64_t row_stride, const int32_t *state_mask, int32_t S, int32_t C,
                                  const int32_t *class_of_token, const uint16_t *sig_rep,
                                  const int32_t *tok_prev, const int32_t *states_in,
                                  int32_t *states_out, int32_t *tok_bits_out, void *stream) {
    if (!logits || !state_mask || !class_of_token || !states_in || !states_out) return CFGZIP_E_INVALID;
    if (B <= 0 || V <= 0 || S <= 0 || S > 65536 || C <= 0 || row_stride < V) return CFGZIP_E_INVALID;
    if (tok_prev && !sig_rep) return CFGZIP_E_INVALID;
    if (states_in == states_out) return CFGZIP_E_INVALID;  // every column tile reads the old states
    if (dtype != CFGZIP_DTYPE_F32 && dtype != CFGZIP_DTYPE_BF16) return CFGZIP_E_INVALID;
    const size_t esz = dtype == CFGZIP_DTYPE_BF16 ? 2 : 4;
    if (!aligned_to(logits, esz) || !aligned_to(state_mask, 4) || !aligned_to(class_of_token, 4) ||
        !aligned_to(sig_rep, 2) || !aligned_to(tok_prev, 4) || !aligned_to(states_in, 4) ||
        !aligned_to(states_out, 4) || !aligned_to(tok_bits_out, 4))
        return CFGZIP_E_INVALID;
    EngineStep e{state_mask, sig_rep, tok_prev, states_in, states_out, S};
    return run_mask(logits, dtype == CFGZIP_DTYPE_BF16 ? LOGITS_BF16 : LOGITS_F32, B, V, row_stride,
                    state_mask, true, class_of_token, C, tok_bits_out,
                    static_cast<hipStream_t>(stream), &e);
}

extern "C" int cfgzip_decode_step(void *logits, int32_t dtype, int32_t B, int32_t V,
                                  int64_t row_stride, const int32_t *cls_bits,
                                  const int32_t *class_of_token, int32_t C, int32_t *tok_bits_out,
                                  const int32_t *tok, const int32_t *rep_of_class, int32_t *rep_out,
                                  void *stream) {
    if (!logits || !cls_bits || !class_of_token || !tok || !rep_of_class || !rep_out)
        return CFGZIP_E_INVALID;
    if (B <= 0 || V <= 0 || C <= 0 || row_stride < V) return CFGZIP_E_INVALID;
    if (dtype != CFGZIP_DTYPE_F32 && dtype != CFGZIP_DTYPE_BF16) return CFGZIP_E_INVALID;
    const size_t esz = dtype == CFGZIP_DTYPE_BF16 ? 2 : 4;
    if (!aligned_to(logits, esz) || !aligned_to(cls_bits, 4) || !aligned_to(class_of_token, 4) ||
        !aligned_to(tok_bits_out, 4) || !aligned_to(tok, 4) || !aligned_to(rep_of_class, 4) ||
        !aligned_to(rep_out, 4))
        return CFGZIP_E_INVALID;
    MapStep m{tok, rep_of_class, rep_out};
    return run_mask(logits, dtype == CFGZIP_DTYPE_BF16 ? LOGITS_BF16 : LOGITS_F32, B, V, row_stride,
                    cls_bits, true, class_of_token, C, tok_bits_out, static_cast<hipStream_t>(stream),
                    nullptr, &m);
}

extern "C" int cfgzip_map_to_rep(const int32_t *tok, int32_t B, const int32_t *class_of_token,
                                 int32_t V, const int32_t *rep_of_class, int32_t C, int32_t *out,
                                 void *stream) {
    if (!tok || !class_of_token || !rep_of_class || !out || B <= 0 || V <= 0 || C <= 0)
        return CFGZIP_E_INVALID;
    const int threads = 256;
    hipLaunchKernelGGL(map_to_rep_kernel, dim3((B + threads - 1) / threads), dim3(threads), 0,
                       static_cast<hipStream_t>(stream), tok, B, class_of_token, V, rep_of_class, C,
                       out);
    return check_launch();
}
