// Displacement sets of tokens over a context-free grammar in Greibach normal form (paper
// Section 3.2.1, Algorithm 1) and the stack-adjacency relation that prunes the stack
// backtrack (Section 3.2.2, Appendix C).
//
// A configuration of Algorithm 1 is (input queue, output stack, symbol consumed last).  A
// workgroup of one wave owns one token and advances the SET of its live configurations one
// byte at a time:
//   - a configuration with a non-empty output stack pops the top symbol A and pushes the body
//     of every production A -> a beta whose terminal is the byte read;
//   - one with an empty output stack backtracks: every production A -> a beta with that
//     terminal, whose head A is stack-adjacent to the symbol consumed last (any head at the
//     very first byte), appends A to the input queue and starts the output stack with beta.
// Successors are appended to a second LDS buffer through one LDS counter, duplicates are
// dropped, and the buffers swap.  What is left after the last byte, without the third
// component, is the displacement; it is written as a fixed-length row in a canonical order
// together with an order-free 64-bit hash, so that equal sets give equal rows and the class
// builder can group tokens by comparing rows.
//
// Everything is bounded: queue, stack, number of successors per byte and row length each have
// a cap; a token that crosses one gets a row and hash of its own (its class is a singleton,
// which costs compression and never correctness).

#include <algorithm>

#include "common.hpp"

namespace cfgzip {
namespace {

constexpr int kMaxBody = 4;
constexpr int kMaxIn = 8;
constexpr int kMaxOut = 12;
constexpr int kMaxFrontier = 128;
constexpr int kRowLen = 256;
constexpr int kRecLen = 2 + kMaxIn + kMaxOut;  // ni, no, queue, stack
constexpr int kPrevAt = kRecLen;               // symbol consumed last, "none" before any
constexpr int kMaxSymbols = 4096;
constexpr int kMaxByteSymbols = 255;           // up to here a symbol (and "none") fits a byte

// A record in LDS: kRecLen entries, the symbol consumed last, zero padding up to an odd number
// of 32-bit words (lanes that read one record each then hit different banks).  Grammars with
// at most kMaxByteSymbols symbols use byte entries: half the LDS per token, twice the waves
// per compute unit.
template <typename Sym>
struct Rec {
    static constexpr int kStride = sizeof(Sym) == 1 ? 28 : 26;  // entries: 7 or 13 words
    static constexpr int kWords = kStride * (int)sizeof(Sym) / 4;
    static constexpr int kOrderWords = (kRecLen * (int)sizeof(Sym) + 3) / 4;
    static constexpr int kBits = 8 * (int)sizeof(Sym);
    static constexpr int kNone = (1 << kBits) - 1;
};

constexpr int kStatusOk = 0;
constexpr int kStatusOverflow = 1;
constexpr int kStatusBadGrammar = 2;

struct GrammarHeader {
    int32_t invalid;  // set by the index kernel when the productions break a stated rule
    int32_t pad[63];
};

struct Grammar {
    const uint16_t *head;
    const uint8_t *byte;
    const uint8_t *len;
    const uint16_t *body;  // [P][kMaxBody]
    int P, N, W;           // W = words per bit row over the symbols
};

struct GrammarWorkspace {
    GrammarHeader *hdr;
    int32_t *byte_off;  // [257]: productions with terminal b are byte_off[b] .. byte_off[b+1]-1
    uint32_t *unary;    // [W]: symbols with a production without body
    uint32_t *reach[2]; // [N][W]: reachability over "right-most body symbol" edges
    uint32_t *adj;      // [N][W]: bit Y of row Z <=> (Y, Z) stack-adjacent
    int32_t *pair_first;  // [256][N]: 1 + index of the first production with (terminal, head), 0 = none
    size_t clear_words; // words from hdr to the end that start at zero
    size_t bytes;
};

GrammarWorkspace carve_grammar_ws(void *ws, int N) {
    GrammarWorkspace g{};
    const size_t W = (size_t)ceil_div(N, 32);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = static_cast<char *>(ws) + off;
        off += (bytes + 255) / 256 * 256;
        return p;
    };
    g.hdr = reinterpret_cast<GrammarHeader *>(take(sizeof(GrammarHeader)));
    g.byte_off = reinterpret_cast<int32_t *>(take(257 * sizeof(int32_t)));
    g.unary = reinterpret_cast<uint32_t *>(take(W * 4));
    g.reach[0] = reinterpret_cast<uint32_t *>(take((size_t)N * W * 4));
    g.adj = reinterpret_cast<uint32_t *>(take((size_t)N * W * 4));
    g.pair_first = reinterpret_cast<int32_t *>(take((size_t)256 * N * 4));
    g.clear_words = off / 4;
    g.reach[1] = reinterpret_cast<uint32_t *>(take((size_t)N * W * 4));  // fully written
    g.bytes = off;
    return g;
}

__global__ void clear_words_kernel(uint32_t *p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

// (byte, head, body) of production i strictly below that of production j, bodies compared
// symbol by symbol, a proper prefix first
__device__ bool production_less(const Grammar &g, int i, int j) {
    if (g.byte[i] != g.byte[j]) return g.byte[i] < g.byte[j];
    if (g.head[i] != g.head[j]) return g.head[i] < g.head[j];
    const int li = min((int)g.len[i], kMaxBody), lj = min((int)g.len[j], kMaxBody);
    for (int k = 0; k < min(li, lj); ++k) {
        const uint16_t x = g.body[i * kMaxBody + k], y = g.body[j * kMaxBody + k];
        if (x != y) return x < y;
    }
    return li < lj;
}

// One thread per production and per symbol: checks the rules the other kernels rely on
// (symbols < N, body length <= kMaxBody, strictly ascending order), finds where each
// terminal's productions start, marks unary symbols and seeds the reachability matrix with
// the identity and the edges head -> right-most body symbol (Appendix C's graph).
__global__ void grammar_index_kernel(Grammar g, GrammarWorkspace w) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < g.N) atomicOr(&w.reach[0][(size_t)i * g.W + (i >> 5)], 1u << (i & 31));
    if (i >= g.P) return;
    const int len = g.len[i];
    bool ok = g.head[i] < g.N && len <= kMaxBody;
    if (ok)
        for (int k = 0; k < len; ++k) ok = ok && g.body[i * kMaxBody + k] < g.N;
    if (ok && i > 0) ok = production_less(g, i - 1, i);
    if (!ok) {
        w.hdr->invalid = 1;
        return;
    }
    const int b = g.byte[i];
    const int first = i == 0 ? 0 : g.byte[i - 1] + 1;
    for (int x = first; x <= b; ++x) w.byte_off[x] = i;  // empty when the bytes are equal
    if (i == g.P - 1)
        for (int x = b + 1; x <= 256; ++x) w.byte_off[x] = g.P;
    const int A = g.head[i];
    if (i == 0 || g.byte[i - 1] != b || g.head[i - 1] != A) w.pair_first[(size_t)b * g.N + A] = i + 1;
    if (len == 0) {
        atomicOr(&w.unary[A >> 5], 1u << (A & 31));
    } else {
        const int last = g.body[i * kMaxBody + len - 1];
        atomicOr(&w.reach[0][(size_t)A * g.W + (last >> 5)], 1u << (last & 31));
    }
}

// One doubling step of the transitive closure: out[X] = union of in[Y] over Y in in[X].  Every
// row holds its own symbol, so rows only grow; ceil(log2 N) steps reach every path.
__global__ __launch_bounds__(64) void closure_round_kernel(const uint32_t *__restrict__ in,
                                                           uint32_t *__restrict__ out, int N,
                                                           int W) {
    const int X = blockIdx.x, lane = threadIdx.x;
    uint32_t acc0 = 0, acc1 = 0;
    for (int w = 0; w < W; ++w) {
        uint32_t bits = in[(size_t)X * W + w];
        while (bits) {
            const int Y = w * 32 + __ffs(bits) - 1;
            bits &= bits - 1;
            if (Y < N) {
                if (lane < W) acc0 |= in[(size_t)Y * W + lane];
                if (lane + 64 < W) acc1 |= in[(size_t)Y * W + lane + 64];
            }
        }
    }
    if (lane < W) out[(size_t)X * W + lane] = acc0;
    if (lane + 64 < W) out[(size_t)X * W + lane + 64] = acc1;
}

// Appendix C: for a production A -> a B_1 .. B_n Z beta (n >= 1), every unary symbol reachable
// from B_n is consumed right before Z.  One thread per (production, n, word).
__global__ void adjacency_kernel(Grammar g, GrammarWorkspace w, const uint32_t *__restrict__ reach) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int word = (int)(idx % g.W);
    const int64_t pair = idx / g.W;
    const int n = (int)(pair % (kMaxBody - 1)) + 1;
    const int64_t i = pair / (kMaxBody - 1);
    if (i >= g.P || w.hdr->invalid) return;
    if (n >= (int)g.len[i]) return;
    const int Bn = g.body[i * kMaxBody + n - 1], Z = g.body[i * kMaxBody + n];
    if (Bn >= g.N || Z >= g.N) return;
    const uint32_t bits = reach[(size_t)Bn * g.W + word] & w.unary[word];
    if (bits) atomicOr(&w.adj[(size_t)Z * g.W + word], bits);
}

__global__ void copy_words_kernel(const uint32_t *__restrict__ src, int32_t *__restrict__ dst,
                                  size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        dst[i] = (int32_t)src[i];
}

int enqueue_grammar_tables(const Grammar &g, const GrammarWorkspace &w, hipStream_t stream) {
    hipLaunchKernelGGL(clear_words_kernel, dim3((unsigned)std::min<int64_t>(1024, ceil_div((int64_t)w.clear_words, 256))),
                       dim3(256), 0, stream, reinterpret_cast<uint32_t *>(w.hdr), w.clear_words);
    CFGZIP_TRY(check_launch());
    hipLaunchKernelGGL(grammar_index_kernel, dim3((unsigned)ceil_div(std::max(g.P, g.N), 256)),
                       dim3(256), 0, stream, g, w);
    CFGZIP_TRY(check_launch());
    int rounds = 0;
    while ((1 << rounds) < g.N) ++rounds;
    int cur = 0;
    for (int r = 0; r < rounds; ++r, cur ^= 1) {
        hipLaunchKernelGGL(closure_round_kernel, dim3(g.N), dim3(64), 0, stream, w.reach[cur],
                           w.reach[cur ^ 1], g.N, g.W);
        CFGZIP_TRY(check_launch());
    }
    const int64_t items = (int64_t)g.P * (kMaxBody - 1) * g.W;
    hipLaunchKernelGGL(adjacency_kernel, dim3((unsigned)ceil_div(items, 256)), dim3(256), 0, stream,
                       g, w, w.reach[cur]);
    return check_launch();
}

// ---- per-token displacement --------------------------------------------------------------

struct DisplacementArgs {
    Grammar g;
    const GrammarHeader *hdr;
    const int32_t *byte_off;
    const int32_t *pair_first;
    const uint32_t *adj;
    const uint8_t *tok_bytes;
    const int64_t *tok_off;
    uint16_t *rows;
    uint64_t *hash;
    int32_t *status;
    uint64_t seed;
};

template <typename Sym>
__device__ inline uint64_t mix_record(const Sym *rec, uint64_t seed) {
    uint64_t h = seed ^ 0x9E3779B97F4A7C15ull;
    for (int k = 0; k < kRecLen; ++k) h = (h ^ rec[k]) * 0x100000001B3ull;
    h ^= h >> 30;
    h *= 0xBF58476D1CE4E5B9ull;
    h ^= h >> 27;
    h *= 0x94D049BB133111EBull;
    h ^= h >> 31;
    return h;
}

template <typename Sym>
__device__ inline bool records_equal(const uint32_t *a, const uint32_t *b) {
    for (int k = 0; k < Rec<Sym>::kWords; ++k)
        if (a[k] != b[k]) return false;
    return true;
}

// ascending order of the entries: in the first word that differs, the lowest entry that
// differs decides (entry e of a word sits at bits e * kBits and up).  Called once the symbol
// consumed last has been cleared, so the words beyond entry kRecLen - 1 are equal.
template <typename Sym>
__device__ inline bool record_less(const uint32_t *a, const uint32_t *b) {
    for (int k = 0; k < Rec<Sym>::kOrderWords; ++k) {
        const uint32_t x = a[k], y = b[k];
        if (x != y) {
            const int shift = (__ffs(x ^ y) - 1) & ~(Rec<Sym>::kBits - 1);
            const uint32_t mask = (uint32_t)Rec<Sym>::kNone;
            return ((x >> shift) & mask) < ((y >> shift) & mask);
        }
    }
    return false;
}

// Drops every record of src[0..m) that equals an earlier one and packs the rest into dst;
// returns how many are left.  Called by the whole wave; m <= kMaxFrontier.
template <typename Sym>
__device__ int drop_duplicates(const Sym (*src)[Rec<Sym>::kStride], Sym (*dst)[Rec<Sym>::kStride],
                               int m, int lane) {
    int kept = 0;
    for (int base = 0; base < kMaxFrontier; base += 64) {
        const int i = base + lane;
        bool keep = i < m;
        if (keep) {
            const uint32_t *mine = reinterpret_cast<const uint32_t *>(src[i]);
            for (int j = 0; j < i; ++j)
                if (records_equal<Sym>(mine, reinterpret_cast<const uint32_t *>(src[j]))) {
                    keep = false;
                    break;
                }
        }
        const uint64_t mask = __ballot(keep);
        if (keep) {
            const int pos = kept + __popcll(mask & ((1ull << lane) - 1ull));
            const uint32_t *s = reinterpret_cast<const uint32_t *>(src[i]);
            uint32_t *d = reinterpret_cast<uint32_t *>(dst[pos]);
            for (int k = 0; k < Rec<Sym>::kWords; ++k) d[k] = s[k];
        }
        kept += __popcll(mask);
    }
    return kept;
}

template <typename Sym>
__global__ __launch_bounds__(64) void displacement_kernel(DisplacementArgs a) {
    constexpr int kRecStride = Rec<Sym>::kStride;
    constexpr int kNone = Rec<Sym>::kNone;
    __shared__ __align__(8) Sym buf[2][kMaxFrontier][kRecStride];
    __shared__ __align__(8) uint16_t row[kRowLen];
    __shared__ int n_emit, crossed, total_len;
    __shared__ unsigned long long hash_sum;

    const int t = blockIdx.x, lane = threadIdx.x;
    const Grammar &g = a.g;
    uint16_t *out_row = a.rows + (size_t)t * kRowLen;
    if (a.hdr->invalid) {  // the same value for every lane
        reinterpret_cast<uint2 *>(out_row)[lane] = make_uint2(0, 0);
        if (lane == 0) {
            a.hash[t] = 0;
            if (a.status) a.status[t] = kStatusBadGrammar;
        }
        return;
    }
    const int64_t b0 = a.tok_off[t], b1 = a.tok_off[t + 1];

    // the start configuration: nothing consumed, nothing pushed
    if (lane < kRecStride) buf[0][0][lane] = (Sym)(lane == kPrevAt ? kNone : 0);
    if (lane == 0) crossed = 0;
    int n = 1, cur = 0;
    bool overflow = false;
    __syncthreads();

    for (int64_t p = b0; p < b1 && n > 0; ++p) {
        const int ch = a.tok_bytes[p];
        const int lo = a.byte_off[ch], hi = a.byte_off[ch + 1];
        if (lane == 0) n_emit = 0;
        __syncthreads();
        Sym(*src)[kRecStride] = buf[cur];
        Sym(*dst)[kRecStride] = buf[cur ^ 1];

        // pops: a lane per configuration (few productions per (terminal, head))
        for (int c = lane; c < n; c += 64) {
            const Sym *rec = src[c];
            const int no = rec[1];
            if (no == 0) continue;
            const int top = rec[2 + kMaxIn];
            const int first = a.pair_first[(size_t)ch * g.N + top] - 1;
            if (first < 0) continue;
            for (int i = first; i < hi && g.head[i] == top; ++i) {
                const int len = g.len[i];
                const uint2 body2 = reinterpret_cast<const uint2 *>(g.body)[i];
                const uint16_t body[kMaxBody] = {(uint16_t)(body2.x & 0xFFFF), (uint16_t)(body2.x >> 16),
                                                 (uint16_t)(body2.y & 0xFFFF), (uint16_t)(body2.y >> 16)};
                const int slot = atomicAdd(&n_emit, 1);
                if (no - 1 + len > kMaxOut) {
                    crossed = 1;
                } else if (slot < kMaxFrontier) {
                    Sym *o = dst[slot];
                    o[0] = rec[0];
                    o[1] = (Sym)(no - 1 + len);
                    for (int k = 0; k < kMaxIn; ++k) o[2 + k] = rec[2 + k];
                    for (int k = 0; k < kMaxOut; ++k) {
                        Sym v = 0;
                        if (k < len) v = (Sym)body[k];
                        else if (k - len + 1 < no) v = rec[2 + kMaxIn + k - len + 1];
                        o[2 + kMaxIn + k] = v;
                    }
                    o[kPrevAt] = (Sym)top;
                    for (int k = kPrevAt + 1; k < kRecStride; ++k) o[k] = 0;
                }
            }
        }
        // stack backtracks: the wave per configuration (every production of the terminal)
        for (int c = 0; c < n; ++c) {
            const Sym *rec = src[c];
            if (rec[1] != 0) continue;  // the same for every lane
            const int ni = rec[0];
            const int prev = rec[kPrevAt];
            for (int i = lo + lane; i < hi; i += 64) {
                const int A = g.head[i];
                if (prev != kNone &&
                    !((a.adj[(size_t)A * g.W + (prev >> 5)] >> (prev & 31)) & 1u))
                    continue;
                const int len = g.len[i];
                const uint2 body2 = reinterpret_cast<const uint2 *>(g.body)[i];
                const uint16_t body[kMaxBody] = {(uint16_t)(body2.x & 0xFFFF), (uint16_t)(body2.x >> 16),
                                                 (uint16_t)(body2.y & 0xFFFF), (uint16_t)(body2.y >> 16)};
                const int slot = atomicAdd(&n_emit, 1);
                if (ni + 1 > kMaxIn) {
                    crossed = 1;
                } else if (slot < kMaxFrontier) {
                    Sym *o = dst[slot];
                    o[0] = (Sym)(ni + 1);
                    o[1] = (Sym)len;
                    for (int k = 0; k < kMaxIn; ++k)
                        o[2 + k] = k < ni ? rec[2 + k] : (k == ni ? (Sym)A : (Sym)0);
                    for (int k = 0; k < kMaxOut; ++k)
                        o[2 + kMaxIn + k] = k < len ? (Sym)body[k] : (Sym)0;
                    o[kPrevAt] = (Sym)A;
                    for (int k = kPrevAt + 1; k < kRecStride; ++k) o[k] = 0;
                }
            }
        }
        __syncthreads();
        const int m = n_emit;
        if (m > kMaxFrontier || crossed) {
            overflow = true;
            break;
        }
        n = drop_duplicates<Sym>(dst, src, m, lane);  // back into the buffer just read
        __syncthreads();
    }

    Sym(*front)[kRecStride] = buf[cur];
    Sym(*other)[kRecStride] = buf[cur ^ 1];
    int start0 = 0, start1 = 0;  // where this lane's records begin in the row
    if (!overflow) {
        // the displacement forgets the symbol consumed last
        for (int c = lane; c < n; c += 64) front[c][kPrevAt] = 0;
        if (lane == 0) {
            total_len = 1;
            hash_sum = 0;
        }
        __syncthreads();
        n = drop_duplicates<Sym>(front, other, n, lane);
        __syncthreads();
        // canonical order by counting: a record starts behind all smaller ones
        for (int c = lane, u = 0; c < n; c += 64, ++u) {
            const uint32_t *mine = reinterpret_cast<const uint32_t *>(other[c]);
            int start = 1;
            for (int j = 0; j < n; ++j) {
                const Sym *r = other[j];
                if (j != c && record_less<Sym>(reinterpret_cast<const uint32_t *>(r), mine))
                    start += 2 + r[0] + r[1];
            }
            if (u == 0) start0 = start; else start1 = start;
            atomicAdd(&total_len, 2 + other[c][0] + other[c][1]);
        }
        __syncthreads();
        if (total_len > kRowLen) overflow = true;
    }
    reinterpret_cast<uint2 *>(row)[lane] = make_uint2(0, 0);
    __syncthreads();
    if (overflow) {
        if (lane == 0) {
            row[0] = 0xFFFF;
            row[1] = (uint16_t)(t & 0xFFFF);
            row[2] = (uint16_t)((uint32_t)t >> 16);
        }
        __syncthreads();
        if (lane == 0) {
            a.hash[t] = mix_record(row, a.seed);
            if (a.status) a.status[t] = kStatusOverflow;
        }
    } else {
        if (lane == 0) row[0] = (uint16_t)n;
        for (int c = lane, u = 0; c < n; c += 64, ++u) {
            const Sym *r = other[c];
            int pos = u == 0 ? start0 : start1;
            const int ni = r[0], no = r[1];
            row[pos++] = (uint16_t)ni;
            row[pos++] = (uint16_t)no;
            for (int k = 0; k < ni; ++k) row[pos++] = r[2 + k];
            for (int k = 0; k < no; ++k) row[pos++] = r[2 + kMaxIn + k];
            atomicAdd(&hash_sum, (unsigned long long)mix_record(r, a.seed));
        }
        __syncthreads();
        if (lane == 0) {
            a.hash[t] = hash_sum;
            if (a.status) a.status[t] = kStatusOk;
        }
    }
    reinterpret_cast<uint2 *>(out_row)[lane] = reinterpret_cast<const uint2 *>(row)[lane];
}

int check_grammar_args(const uint16_t *prod_head, const uint8_t *prod_byte, const uint8_t *prod_len,
                       const uint16_t *prod_body, int32_t P, int32_t N) {
    if (!prod_head || !prod_byte || !prod_len || !prod_body) return CFGZIP_E_INVALID;
    if (P <= 0 || N <= 0 || N > kMaxSymbols) return CFGZIP_E_INVALID;
    if (!aligned_to(prod_head, 2) || !aligned_to(prod_body, 8)) return CFGZIP_E_INVALID;
    return CFGZIP_OK;
}

}  // namespace
}  // namespace cfgzip

using namespace cfgzip;

extern "C" size_t cfgzip_displacements_workspace_bytes(int32_t N) {
    if (N <= 0 || N > kMaxSymbols) return 0;
    return carve_grammar_ws(nullptr, N).bytes;
}

extern "C" int cfgzip_stack_adjacency(const uint16_t *prod_head, const uint8_t *prod_byte,
                                      const uint8_t *prod_len, const uint16_t *prod_body, int32_t P,
                                      int32_t N, int32_t *adj_out, int32_t *invalid_out, void *ws,
                                      size_t ws_bytes, void *stream_) {
    CFGZIP_TRY(check_grammar_args(prod_head, prod_byte, prod_len, prod_body, P, N));
    if (!adj_out || !aligned_to(adj_out, 4) || !aligned_to(invalid_out, 4)) return CFGZIP_E_INVALID;
    if (!ws || !aligned_to(ws, 256)) return CFGZIP_E_WORKSPACE;
    GrammarWorkspace w = carve_grammar_ws(ws, N);
    if (ws_bytes < w.bytes) return CFGZIP_E_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    Grammar g{prod_head, prod_byte, prod_len, prod_body, P, N, (int)ceil_div(N, 32)};
    CFGZIP_TRY(enqueue_grammar_tables(g, w, stream));
    const size_t words = (size_t)N * g.W;
    hipLaunchKernelGGL(copy_words_kernel, dim3((unsigned)std::min<int64_t>(1024, ceil_div((int64_t)words, 256))),
                       dim3(256), 0, stream, w.adj, adj_out, words);
    CFGZIP_TRY(check_launch());
    if (invalid_out) {
        hipLaunchKernelGGL(copy_words_kernel, dim3(1), dim3(64), 0, stream,
                           reinterpret_cast<const uint32_t *>(&w.hdr->invalid), invalid_out,
                           (size_t)1);
        CFGZIP_TRY(check_launch());
    }
    return CFGZIP_OK;
}

extern "C" int cfgzip_displacements(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                                    const uint16_t *prod_head, const uint8_t *prod_byte,
                                    const uint8_t *prod_len, const uint16_t *prod_body, int32_t P,
                                    int32_t N, uint16_t *rows_out, uint64_t *hash_out,
                                    int32_t *status_out, uint64_t hash_seed, void *ws,
                                    size_t ws_bytes, void *stream_) {
    CFGZIP_TRY(check_grammar_args(prod_head, prod_byte, prod_len, prod_body, P, N));
    if (!tok_off || !rows_out || !hash_out || V <= 0) return CFGZIP_E_INVALID;
    if (!aligned_to(tok_off, 8) || !aligned_to(rows_out, 8) || !aligned_to(hash_out, 8) ||
        !aligned_to(status_out, 4))
        return CFGZIP_E_INVALID;
    if (!ws || !aligned_to(ws, 256)) return CFGZIP_E_WORKSPACE;
    GrammarWorkspace w = carve_grammar_ws(ws, N);
    if (ws_bytes < w.bytes) return CFGZIP_E_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    Grammar g{prod_head, prod_byte, prod_len, prod_body, P, N, (int)ceil_div(N, 32)};
    CFGZIP_TRY(enqueue_grammar_tables(g, w, stream));
    DisplacementArgs a{};
    a.g = g;
    a.hdr = w.hdr;
    a.byte_off = w.byte_off;
    a.pair_first = w.pair_first;
    a.adj = w.adj;
    a.tok_bytes = tok_bytes;
    a.tok_off = tok_off;
    a.rows = rows_out;
    a.hash = hash_out;
    a.status = status_out;
    a.seed = hash_seed;
    if (N <= kMaxByteSymbols)
        hipLaunchKernelGGL(displacement_kernel<uint8_t>, dim3((unsigned)V), dim3(64), 0, stream, a);
    else
        hipLaunchKernelGGL(displacement_kernel<uint16_t>, dim3((unsigned)V), dim3(64), 0, stream, a);
    return check_launch();
}
