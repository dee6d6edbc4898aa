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
// Successors are appended to a second LDS buffer through one LDS counter; duplicates are
// dropped while the survivors are packed back into the first.  What is left after the last byte, without the third
// component, is the displacement; it is written as a fixed-length row in a canonical order
// together with an order-free 64-bit hash, so that equal sets give equal rows and the class
// builder can group tokens by comparing rows.
//
// Everything is bounded: queue, stack, number of successors per byte and row length each have
// a cap.  All tokens are first taken under small caps (little LDS per token, many waves per
// compute unit); the few that cross them are queued and taken again under larger ones by a
// second, persistent kernel.  A token that crosses those too, or whose set does not fit the row,
// gets a row and hash of its own (its class is a singleton, which costs compression and never
// correctness).

#include <algorithm>

#include "common.hpp"

namespace cfgzip {
namespace {

constexpr int kRowChunk = 256;                 // row entries staged in LDS at a time
constexpr int kMaxRowLen = 4096;
constexpr int kMaxSymbols = 4096;
constexpr int kMaxByteSymbols = 255;           // up to here a symbol (and "none") fits a byte

// caps of the first pass over all tokens and of the second pass over those it could not finish.
// The second pass runs in two steps: with the first pass's frontier capacity (half the LDS, twice
// the waves per compute unit; enough for most of what the first pass hands on), then with the full
// one for what is still left.  A token that gets through the narrower step would have got through
// the wider one with the same result, so the two steps together are one pass under kFrontier2.
constexpr int kIn1 = 12, kOut1 = 12, kFrontier1 = 128;
constexpr int kIn2 = 32, kOut2 = 32, kFrontier2 = 256;
constexpr int kFrontier2Narrow = 128;
// the second pass keeps the current byte's productions and the relation in LDS when they fit
constexpr int kStageCap = 128;      // productions of one terminal
constexpr int kStageBodyCap = 512;  // body symbols of those productions together
constexpr int kAdjLdsWords = 512;   // N * W(N) words: N <= 128

// A record in LDS: ni, no, MAX_IN queue entries, MAX_OUT stack entries (top first), the symbol
// consumed last, zero padding up to an odd number of 32-bit words (lanes that read one record
// each then hit different banks).  Grammars with at most kMaxByteSymbols symbols use byte
// entries: half the LDS per token, twice the waves per compute unit.
template <typename Sym, int MAX_IN, int MAX_OUT>
struct Rec {
    static constexpr int kLen = 2 + MAX_IN + MAX_OUT;
    static constexpr int kStackAt = 2 + MAX_IN;
    static constexpr int kPrevAt = kLen;  // "none" before anything was consumed
    static constexpr int kWords = (((kLen + 1) * (int)sizeof(Sym) + 3) / 4) | 1;
    static constexpr int kStride = kWords * 4 / (int)sizeof(Sym);
    static constexpr int kOrderWords = (kLen * (int)sizeof(Sym) + 3) / 4;
    static constexpr int kBits = 8 * (int)sizeof(Sym);
    static constexpr int kNone = (1 << kBits) - 1;
};

constexpr int kStatusOk = 0;
constexpr int kStatusOverflow = 1;
constexpr int kStatusBadGrammar = 2;

struct GrammarHeader {
    int32_t invalid;      // set by the index kernel when the productions break a stated rule
    // two lists of tokens handed on: by the first pass, and by the pass after it
    int32_t retry_count[2];
    int32_t retry_next[2];  // next entry of each list to be taken
    int32_t pad[59];
};

struct Grammar {
    const uint16_t *head;
    const uint8_t *byte;
    const int32_t *body_off;  // [P + 1]: the body of production i is body[body_off[i] .. body_off[i+1])
    const uint16_t *body;
    int P, N, W;              // W = words per bit row over the symbols
    int body_total;           // body symbols the caller says there are (the offsets are checked against it)
};

__device__ __forceinline__ int body_len(const Grammar &g, int i) { return g.body_off[i + 1] - g.body_off[i]; }

struct GrammarWorkspace {
    GrammarHeader *hdr;
    int32_t *byte_off;  // [257]: productions with terminal b are byte_off[b] .. byte_off[b+1]-1
    uint32_t *unary;    // [W]: symbols with a production without body
    uint32_t *reach[2]; // [N][W]: reachability over "right-most body symbol" edges
    uint32_t *adj;      // [N][W]: bit Y of row Z <=> (Y, Z) stack-adjacent
    int32_t *pair_first;  // [256][N]: 1 + index of the first production with (terminal, head), 0 = none
    uint4 *prod_short;    // [P]: first four body symbols (16 bits each), body length, body offset: one load per production
    int32_t *retry_list[2];  // [V] each: ids of the tokens handed on
    size_t clear_words; // words from hdr to the end that start at zero
    size_t bytes;
};

GrammarWorkspace carve_grammar_ws(void *ws, int N, int V, int P) {
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
    g.prod_short = reinterpret_cast<uint4 *>(take((size_t)P * sizeof(uint4)));  // fully written for a valid grammar
    g.retry_list[0] = reinterpret_cast<int32_t *>(take((size_t)V * 4));
    g.retry_list[1] = reinterpret_cast<int32_t *>(take((size_t)V * 4));
    g.bytes = off;
    return g;
}

__global__ void clear_words_kernel(uint32_t *p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

// (byte, head, body) of production i strictly below that of production j, bodies compared
// symbol by symbol, a proper prefix first.  Both bodies lie inside the body array.
__device__ bool production_less(const Grammar &g, int i, int j) {
    if (g.byte[i] != g.byte[j]) return g.byte[i] < g.byte[j];
    if (g.head[i] != g.head[j]) return g.head[i] < g.head[j];
    const int li = body_len(g, i), lj = body_len(g, j);
    const uint16_t *bi = g.body + g.body_off[i], *bj = g.body + g.body_off[j];
    for (int k = 0; k < min(li, lj); ++k)
        if (bi[k] != bj[k]) return bi[k] < bj[k];
    return li < lj;
}

// One thread per production and per symbol: checks the rules the other kernels rely on
// (body offsets ascending from 0 to the stated total, symbols < N, strictly ascending order of
// the productions), finds where each terminal's productions start, marks unary symbols and
// seeds the reachability matrix with the identity and the edges head -> right-most body symbol
// (Appendix C's graph).
__global__ void grammar_index_kernel(Grammar g, GrammarWorkspace w) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < g.N) atomicOr(&w.reach[0][(size_t)i * g.W + (i >> 5)], 1u << (i & 31));
    if (i >= g.P) return;
    const int off = g.body_off[i], end = g.body_off[i + 1];
    bool ok = g.head[i] < g.N && off >= 0 && end >= off && end <= g.body_total;
    if (ok && i == 0) ok = off == 0;
    if (ok && i == g.P - 1) ok = end == g.body_total;
    if (ok && i > 0) {  // the body before this one must be in bounds before it is compared
        const int poff = g.body_off[i - 1];
        ok = poff >= 0 && poff <= off;
    }
    const int len = end - off;
    if (ok)
        for (int k = 0; k < len; ++k) ok = ok && g.body[off + k] < g.N;
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
    {
        uint32_t sym[4] = {0, 0, 0, 0};
        for (int k = 0; k < min(len, 4); ++k) sym[k] = g.body[off + k];
        w.prod_short[i] = make_uint4(sym[0] | (sym[1] << 16), sym[2] | (sym[3] << 16), (uint32_t)len, (uint32_t)off);
    }
    if (len == 0) {
        atomicOr(&w.unary[A >> 5], 1u << (A & 31));
    } else {
        const int last = g.body[end - 1];
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
// from B_n is consumed right before Z.  One thread per (production, word); it goes through the
// neighbouring pairs of the body.
__global__ void adjacency_kernel(Grammar g, GrammarWorkspace w, const uint32_t *__restrict__ reach) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int word = (int)(idx % g.W);
    const int64_t i = idx / g.W;
    if (i >= g.P || w.hdr->invalid) return;
    const int off = g.body_off[i], end = g.body_off[i + 1];
    for (int p = off; p + 1 < end; ++p) {
        const int Bn = g.body[p], Z = g.body[p + 1];
        const uint32_t bits = reach[(size_t)Bn * g.W + word] & w.unary[word];
        if (bits) atomicOr(&w.adj[(size_t)Z * g.W + word], bits);
    }
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
    const int64_t items = (int64_t)g.P * g.W;
    hipLaunchKernelGGL(adjacency_kernel, dim3((unsigned)ceil_div(items, 256)), dim3(256), 0, stream,
                       g, w, w.reach[cur]);
    return check_launch();
}

// ---- per-token displacement --------------------------------------------------------------

struct DisplacementArgs {
    Grammar g;
    GrammarHeader *hdr;
    const int32_t *byte_off;
    const int32_t *pair_first;
    const uint4 *prod_short;
    const uint32_t *adj;
    const uint8_t *tok_bytes;
    const int64_t *tok_off;
    uint16_t *rows;
    uint64_t *hash;
    int32_t *status;
    int32_t *retry_list[2];
    uint64_t seed;
    int V, row_len;
};

// 64-bit mix of a record's entries ni, no, queue, stack (FNV-1a style pass, SplitMix64 finaliser)
struct RecordMix {
    uint64_t h;
    __device__ explicit RecordMix(uint64_t seed) : h(seed ^ 0x9E3779B97F4A7C15ull) {}
    __device__ void add(uint32_t x) { h = (h ^ x) * 0x100000001B3ull; }
    __device__ uint64_t done() const {
        uint64_t z = h;
        z ^= z >> 30;
        z *= 0xBF58476D1CE4E5B9ull;
        z ^= z >> 27;
        z *= 0x94D049BB133111EBull;
        z ^= z >> 31;
        return z;
    }
};

template <typename R>
__device__ inline bool records_equal(const uint32_t *a, const uint32_t *b) {
    for (int k = 0; k < R::kWords; ++k)
        if (a[k] != b[k]) return false;
    return true;
}

// Canonical order: by (ni, no), then the queue, then the stack.  With equal ni and no the
// padding of two records sits at the same entries, so this is the ascending order of the padded
// entries: in the first word that differs, the lowest entry that differs decides (entry e of a
// word sits at bits e * kBits and up).  Called once the symbol consumed last has been cleared,
// so the words beyond the last entry are equal.
template <typename R>
__device__ inline bool record_less(const uint32_t *a, const uint32_t *b) {
    for (int k = 0; k < R::kOrderWords; ++k) {
        const uint32_t x = a[k], y = b[k];
        if (x != y) {
            const int shift = (__ffs(x ^ y) - 1) & ~(R::kBits - 1);
            const uint32_t mask = (uint32_t)R::kNone;
            return ((x >> shift) & mask) < ((y >> shift) & mask);
        }
    }
    return false;
}

// Drops every record of src[0..m) that equals an earlier one and packs the rest into dst;
// returns how many are left.  Called by the whole wave; m <= FRONTIER.  A 16-bit fingerprint of
// every record goes to `fp` first: a lane then scans the fingerprints before its own without
// branching (independent LDS reads) and compares whole records only where one matches.
// `empty_list` receives the positions (in dst) of the records whose stack is empty, `n_empty`
// how many there are: the next byte's backtrack visits only those.
template <typename Sym, typename R, int FRONTIER>
__device__ int drop_duplicates(const Sym (*src)[R::kStride], Sym (*dst)[R::kStride], int m, int lane,
                               uint16_t *fp, uint8_t *empty_list, int &n_empty) {
    for (int i = lane; i < m; i += 64) {
        const uint32_t *w = reinterpret_cast<const uint32_t *>(src[i]);
        uint32_t h = 0;
#pragma unroll
        for (int k = 0; k < R::kWords; ++k) h = h * 0x9E3779B1u + w[k];
        fp[i] = (uint16_t)((h >> 16) ^ h);
    }
    __syncthreads();
    int kept = 0;
    n_empty = 0;
    for (int base = 0; base < FRONTIER; base += 64) {
        if (base >= m) break;  // the same for every lane
        const int i = base + lane;
        bool keep = i < m;
        if (keep) {
            const uint32_t mine_fp = fp[i];
            bool candidate = false;
            const int last = min(m, base + 64) - 1;  // the same bound for every lane: no divergence
#pragma unroll 4
            for (int j = 0; j < last; ++j) candidate |= (j < i) & (fp[j] == mine_fp);
            if (candidate) {
                const uint32_t *mine = reinterpret_cast<const uint32_t *>(src[i]);
                for (int j = 0; j < i; ++j)
                    if (fp[j] == mine_fp &&
                        records_equal<R>(mine, reinterpret_cast<const uint32_t *>(src[j]))) {
                        keep = false;
                        break;
                    }
            }
        }
        const uint64_t mask = __ballot(keep);
        const bool empty = keep && src[i][1] == 0;
        const uint64_t empty_mask = __ballot(empty);
        const uint64_t below = (1ull << lane) - 1ull;
        if (keep) {
            const int pos = kept + __popcll(mask & below);
            const uint32_t *s = reinterpret_cast<const uint32_t *>(src[i]);
            uint32_t *d = reinterpret_cast<uint32_t *>(dst[pos]);
            for (int k = 0; k < R::kWords; ++k) d[k] = s[k];
            if (empty) empty_list[n_empty + __popcll(empty_mask & below)] = (uint8_t)pos;
        }
        kept += __popcll(mask);
        n_empty += __popcll(empty_mask);
    }
    return kept;
}

// LDS of one workgroup (one wave)
template <typename Sym, typename R, int FRONTIER, bool STAGE>
struct TokenLds {
    __align__(8) Sym buf[2][FRONTIER][R::kStride];
    __align__(8) uint16_t row[kRowChunk];
    int n_emit, crossed, total_len, next_item;
    unsigned long long hash_sum;
    uint16_t fingerprint[FRONTIER];
    uint8_t empty_list[FRONTIER];  // positions of the live configurations with an empty stack
    // STAGE only: the productions lo .. hi-1 of the byte being read (heads, body offsets
    // relative to the first, body symbols), and the relation
    uint16_t sp_body[STAGE ? kStageBodyCap : 1];
    uint16_t sp_off[STAGE ? kStageCap + 1 : 1];
    uint16_t sp_head[STAGE ? kStageCap : 1];
    uint32_t adj[STAGE ? kAdjLdsWords : 1];
};

// The displacement of token t under the caps MAX_IN, MAX_OUT, FRONTIER, by the whole wave.
// HAND_ON >= 0: a token that crosses a cap is appended to that retry list (and still gets the
// overflow row, which a later pass overwrites if it gets through).
template <typename Sym, int MAX_IN, int MAX_OUT, int FRONTIER, int HAND_ON, bool STAGE>
__device__ void token_displacement(const DisplacementArgs &a, int t,
                                   TokenLds<Sym, Rec<Sym, MAX_IN, MAX_OUT>, FRONTIER, STAGE> &L,
                                   bool adj_in_lds) {
    using R = Rec<Sym, MAX_IN, MAX_OUT>;
    constexpr int kStride = R::kStride;
    constexpr int kNone = R::kNone;
    static_assert(FRONTIER % 64 == 0 && FRONTIER <= 256, "whole waves of records; positions fit a byte");
    constexpr int kPerLane = FRONTIER / 64;
    const int lane = threadIdx.x;
    const Grammar &g = a.g;
    const int64_t b0 = a.tok_off[t], b1 = a.tok_off[t + 1];

    // the start configuration: nothing consumed, nothing pushed
    for (int k = lane; k < kStride; k += 64) L.buf[0][0][k] = (Sym)(k == R::kPrevAt ? kNone : 0);
    if (lane == 0) {
        L.crossed = 0;
        L.empty_list[0] = 0;
    }
    int n = 1, n_empty = 1;
    bool caps_crossed = false;
    __syncthreads();

    Sym(*src)[kStride] = L.buf[0];  // the live set is always handed back to buf[0]
    Sym(*dst)[kStride] = L.buf[1];
    for (int64_t p = b0; p < b1 && n > 0; ++p) {
        const int ch = a.tok_bytes[p];
        const int lo = a.byte_off[ch], hi = a.byte_off[ch + 1];
        if (lane == 0) L.n_emit = 0;
        const int body_lo = hi > lo ? g.body_off[lo] : 0;
        const bool staged = STAGE && hi - lo <= kStageCap &&
                            (hi > lo ? g.body_off[hi] - body_lo : 0) <= kStageBodyCap;  // the same for every lane
        if (staged) {
            for (int i = lo + lane; i < hi; i += 64) L.sp_head[i - lo] = g.head[i];
            for (int i = lo + lane; i <= hi; i += 64) L.sp_off[i - lo] = (uint16_t)(g.body_off[i] - body_lo);
            const int symbols = hi > lo ? g.body_off[hi] - body_lo : 0;
            for (int x = lane; x < symbols; x += 64) L.sp_body[x] = g.body[body_lo + x];
        }
        __syncthreads();
        auto head_of = [&](int i) -> int { return staged ? L.sp_head[i - lo] : g.head[i]; };
        // a production's body: staged symbols in LDS, or the packed record (its first four symbols,
        // length and offset in one 16-byte load) with the symbol array behind it for longer bodies
        auto body_of = [&](int i) -> uint4 {
            if (staged) return make_uint4(0, 0, (uint32_t)(L.sp_off[i - lo + 1] - L.sp_off[i - lo]), L.sp_off[i - lo]);
            return a.prod_short[i];
        };
        auto body_sym = [&](const uint4 &b, int k) -> int {
            if (staged) return L.sp_body[b.w + k];
            if (k < 4) return (int)(((k < 2 ? b.x : b.y) >> (16 * (k & 1))) & 0xFFFFu);
            return g.body[b.w + k];
        };

        // pops: a lane per configuration (few productions per (terminal, head))
        for (int c = lane; c < n; c += 64) {
            const Sym *rec = src[c];
            const int no = rec[1];
            if (no == 0) continue;
            const int top = rec[R::kStackAt];
            const int first = a.pair_first[(size_t)ch * g.N + top] - 1;
            if (first < 0) continue;
            for (int i = first; i < hi && head_of(i) == top; ++i) {
                const uint4 body = body_of(i);
                const int len = (int)body.z;
                const int slot = atomicAdd(&L.n_emit, 1);
                if (no - 1 + len > MAX_OUT) {
                    L.crossed = 1;
                } else if (slot < FRONTIER) {
                    // the old record, then the stack rewritten: the body on top of what was below
                    Sym *o = dst[slot];
                    const uint32_t *rw = reinterpret_cast<const uint32_t *>(rec);
                    uint32_t *ow = reinterpret_cast<uint32_t *>(o);
                    for (int k = 0; k < R::kWords; ++k) ow[k] = rw[k];
                    const int new_no = no - 1 + len;
                    for (int k = 0; k < new_no; ++k)
                        o[R::kStackAt + k] = k < len ? (Sym)body_sym(body, k) : rec[R::kStackAt + k - len + 1];
                    if (len == 0) o[R::kStackAt + new_no] = 0;  // the stack got shorter by one
                    o[1] = (Sym)new_no;
                    o[R::kPrevAt] = (Sym)top;
                }
            }
        }
        // stack backtracks: the wave per configuration with an empty stack (every production of
        // the terminal)
        for (int e = 0; e < n_empty; ++e) {
            const Sym *rec = src[L.empty_list[e]];
            const int ni = rec[0];
            const int prev = rec[R::kPrevAt];
            for (int i = lo + lane; i < hi; i += 64) {
                const int A = head_of(i);
                if (prev != kNone) {
                    const size_t w = (size_t)A * g.W + (prev >> 5);
                    const uint32_t bits = (STAGE && adj_in_lds) ? L.adj[w] : a.adj[w];
                    if (!((bits >> (prev & 31)) & 1u)) continue;
                }
                const uint4 body = body_of(i);
                const int len = (int)body.z;
                const int slot = atomicAdd(&L.n_emit, 1);
                if (ni + 1 > MAX_IN || len > MAX_OUT) {
                    L.crossed = 1;
                } else if (slot < FRONTIER) {
                    // the old record (its stack is empty) with A appended to the queue, the body
                    // as the new stack
                    Sym *o = dst[slot];
                    const uint32_t *rw = reinterpret_cast<const uint32_t *>(rec);
                    uint32_t *ow = reinterpret_cast<uint32_t *>(o);
                    for (int k = 0; k < R::kWords; ++k) ow[k] = rw[k];
                    o[0] = (Sym)(ni + 1);
                    o[1] = (Sym)len;
                    o[2 + ni] = (Sym)A;
                    for (int k = 0; k < len; ++k) o[R::kStackAt + k] = (Sym)body_sym(body, k);
                    o[R::kPrevAt] = (Sym)A;
                }
            }
        }
        __syncthreads();
        const int m = L.n_emit;
        if (m > FRONTIER || L.crossed) {
            caps_crossed = true;
            break;
        }
        // back into the buffer just read
        n = drop_duplicates<Sym, R, FRONTIER>(dst, src, m, lane, L.fingerprint, L.empty_list, n_empty);
        __syncthreads();
    }

    int start[kPerLane];  // where this lane's records begin in the row
    bool overflow = caps_crossed;
    int total = 1;
    if (!caps_crossed) {
        // the displacement forgets the symbol consumed last
        for (int c = lane; c < n; c += 64) src[c][R::kPrevAt] = 0;
        if (lane == 0) {
            L.total_len = 1;
            L.hash_sum = 0;
        }
        __syncthreads();
        n = drop_duplicates<Sym, R, FRONTIER>(src, dst, n, lane, L.fingerprint, L.empty_list, n_empty);
        __syncthreads();
        // canonical order by counting: a record starts behind all smaller ones
#pragma unroll
        for (int u = 0; u < kPerLane; ++u) {
            const int c = lane + 64 * u;
            start[u] = 1;
            if (c < n) {
                const uint32_t *mine = reinterpret_cast<const uint32_t *>(dst[c]);
                for (int j = 0; j < n; ++j) {
                    const Sym *r = dst[j];
                    if (j != c && record_less<R>(reinterpret_cast<const uint32_t *>(r), mine))
                        start[u] += 2 + r[0] + r[1];
                }
                atomicAdd(&L.total_len, 2 + dst[c][0] + dst[c][1]);
            }
        }
        __syncthreads();
        total = L.total_len;
        if (total > a.row_len) overflow = true;
    }

    if (overflow) {
        if (lane == 0) {
            RecordMix mix(a.seed);
            mix.add(0xFFFFu);
            mix.add((uint32_t)t & 0xFFFFu);
            mix.add((uint32_t)t >> 16);
            a.hash[t] = mix.done();
            if (a.status) a.status[t] = kStatusOverflow;
            if (HAND_ON >= 0 && caps_crossed)
                a.retry_list[HAND_ON < 0 ? 0 : HAND_ON][atomicAdd(&a.hdr->retry_count[HAND_ON < 0 ? 0 : HAND_ON], 1)] = t;
        }
    } else {
        uint64_t h = 0;
#pragma unroll
        for (int u = 0; u < kPerLane; ++u) {
            const int c = lane + 64 * u;
            if (c < n) {
                const Sym *r = dst[c];
                RecordMix mix(a.seed);
                mix.add(r[0]);
                mix.add(r[1]);
                for (int k = 0; k < r[0]; ++k) mix.add(r[2 + k]);
                for (int k = 0; k < r[1]; ++k) mix.add(r[R::kStackAt + k]);
                h += mix.done();
            }
        }
        if (h) atomicAdd(&L.hash_sum, (unsigned long long)h);
    }

    // the row, kRowChunk entries at a time through LDS; chunks behind the data are plain zeros
    uint16_t *out_row = a.rows + (size_t)t * a.row_len;
    const int used = overflow ? 3 : total;
    for (int base = 0; base < a.row_len; base += kRowChunk) {
        uint2 *out = reinterpret_cast<uint2 *>(out_row + base);
        if (base >= used) {  // the same for every lane
            out[lane] = make_uint2(0, 0);
            continue;
        }
        reinterpret_cast<uint2 *>(L.row)[lane] = make_uint2(0, 0);
        __syncthreads();
        if (overflow) {
            if (lane == 0) {
                L.row[0] = 0xFFFF;
                L.row[1] = (uint16_t)(t & 0xFFFF);
                L.row[2] = (uint16_t)((uint32_t)t >> 16);
            }
        } else {
            if (lane == 0 && base == 0) L.row[0] = (uint16_t)n;
#pragma unroll
            for (int u = 0; u < kPerLane; ++u) {
                const int c = lane + 64 * u;
                if (c >= n) continue;
                const Sym *r = dst[c];
                const int ni = r[0], no = r[1];
                const int first = start[u] - base;  // position of the record's first entry in this chunk
                if (first >= kRowChunk || first + 2 + ni + no <= 0) continue;
                for (int e = max(0, -first); e < 2 + ni + no && first + e < kRowChunk; ++e) {
                    const int v = e < 2 ? r[e] : (e < 2 + ni ? r[e] : r[R::kStackAt + e - 2 - ni]);
                    L.row[first + e] = (uint16_t)v;
                }
            }
        }
        __syncthreads();
        out[lane] = reinterpret_cast<const uint2 *>(L.row)[lane];
    }
    __syncthreads();
    if (!overflow && lane == 0) {
        a.hash[t] = L.hash_sum;
        if (a.status) a.status[t] = kStatusOk;
    }
    __syncthreads();  // the next token of a persistent workgroup starts from settled LDS
}

// first pass: a workgroup of one wave per token
template <typename Sym>
__global__ __launch_bounds__(64) void displacement_kernel(DisplacementArgs a) {
    __shared__ TokenLds<Sym, Rec<Sym, kIn1, kOut1>, kFrontier1, false> lds;
    const int t = blockIdx.x;
    if (a.hdr->invalid) {  // the same value for every lane
        for (int base = 0; base < a.row_len; base += kRowChunk)
            reinterpret_cast<uint2 *>(a.rows + (size_t)t * a.row_len + base)[threadIdx.x] = make_uint2(0, 0);
        if (threadIdx.x == 0) {
            a.hash[t] = 0;
            if (a.status) a.status[t] = kStatusBadGrammar;
        }
        return;
    }
    token_displacement<Sym, kIn1, kOut1, kFrontier1, 0, false>(a, t, lds, false);
}

// second pass: persistent workgroups of one wave take retry list LIST entry by entry; what they
// cannot finish goes to list HAND_ON (none if negative)
template <typename Sym, int FRONTIER, int LIST, int HAND_ON>
__global__ __launch_bounds__(64) void displacement_retry_kernel(DisplacementArgs a) {
    __shared__ TokenLds<Sym, Rec<Sym, kIn2, kOut2>, FRONTIER, true> lds;
    const int count = min(a.hdr->retry_count[LIST], a.V);
    if (count == 0) return;
    const bool adj_in_lds = a.g.N * a.g.W <= kAdjLdsWords;
    if (adj_in_lds)
        for (int i = threadIdx.x; i < a.g.N * a.g.W; i += 64) lds.adj[i] = a.adj[i];
    for (;;) {
        if (threadIdx.x == 0) lds.next_item = atomicAdd(&a.hdr->retry_next[LIST], 1);
        __syncthreads();
        const int i = lds.next_item;
        __syncthreads();
        if (i >= count) break;  // the same for every lane
        token_displacement<Sym, kIn2, kOut2, FRONTIER, HAND_ON, true>(a, a.retry_list[LIST][i], lds, adj_in_lds);
    }
}

template <typename Sym>
int launch_displacements(const DisplacementArgs &a, int n_cu, hipStream_t stream) {
    hipLaunchKernelGGL(displacement_kernel<Sym>, dim3((unsigned)a.V), dim3(64), 0, stream, a);
    CFGZIP_TRY(check_launch());
    // as many one-wave workgroups as the LDS of all compute units holds at once
    auto grid_for_lds = [&](size_t lds) {
        return (unsigned)std::min<int64_t>(a.V, (int64_t)n_cu * std::max<size_t>(1, (160 * 1024) / lds));
    };
    hipLaunchKernelGGL((displacement_retry_kernel<Sym, kFrontier2Narrow, 0, 1>),
                       dim3(grid_for_lds(sizeof(TokenLds<Sym, Rec<Sym, kIn2, kOut2>, kFrontier2Narrow, true>))),
                       dim3(64), 0, stream, a);
    CFGZIP_TRY(check_launch());
    hipLaunchKernelGGL((displacement_retry_kernel<Sym, kFrontier2, 1, -1>),
                       dim3(grid_for_lds(sizeof(TokenLds<Sym, Rec<Sym, kIn2, kOut2>, kFrontier2, true>))),
                       dim3(64), 0, stream, a);
    return check_launch();
}

int check_grammar_args(const uint16_t *prod_head, const uint8_t *prod_byte, const int32_t *prod_body_off,
                       const uint16_t *prod_body, int32_t body_total, int32_t P, int32_t N) {
    if (!prod_head || !prod_byte || !prod_body_off) return CFGZIP_E_INVALID;
    if (P <= 0 || N <= 0 || N > kMaxSymbols || body_total < 0) return CFGZIP_E_INVALID;
    if (body_total > 0 && !prod_body) return CFGZIP_E_INVALID;
    if (!aligned_to(prod_head, 2) || !aligned_to(prod_body_off, 4) || !aligned_to(prod_body, 2))
        return CFGZIP_E_INVALID;
    return CFGZIP_OK;
}

}  // namespace
}  // namespace cfgzip

using namespace cfgzip;

extern "C" size_t cfgzip_displacements_workspace_bytes(int32_t V, int32_t N, int32_t P) {
    if (V < 0 || N <= 0 || N > kMaxSymbols || P <= 0) return 0;
    return carve_grammar_ws(nullptr, N, V, P).bytes;
}

extern "C" int cfgzip_stack_adjacency(const uint16_t *prod_head, const uint8_t *prod_byte,
                                      const int32_t *prod_body_off, const uint16_t *prod_body,
                                      int32_t body_total, int32_t P, int32_t N, int32_t *adj_out,
                                      int32_t *invalid_out, void *ws, size_t ws_bytes, void *stream_) {
    CFGZIP_TRY(check_grammar_args(prod_head, prod_byte, prod_body_off, prod_body, body_total, P, N));
    if (!adj_out || !aligned_to(adj_out, 4) || !aligned_to(invalid_out, 4)) return CFGZIP_E_INVALID;
    if (!ws || !aligned_to(ws, 256)) return CFGZIP_E_WORKSPACE;
    GrammarWorkspace w = carve_grammar_ws(ws, N, 0, P);
    if (ws_bytes < w.bytes) return CFGZIP_E_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    Grammar g{prod_head, prod_byte, prod_body_off, prod_body, P, N, (int)ceil_div(N, 32), body_total};
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
                                    const int32_t *prod_body_off, const uint16_t *prod_body,
                                    int32_t body_total, int32_t P, int32_t N, uint16_t *rows_out,
                                    int32_t row_len, uint64_t *hash_out, int32_t *status_out,
                                    uint64_t hash_seed, void *ws, size_t ws_bytes, void *stream_) {
    CFGZIP_TRY(check_grammar_args(prod_head, prod_byte, prod_body_off, prod_body, body_total, P, N));
    if (!tok_off || !rows_out || !hash_out || V <= 0) return CFGZIP_E_INVALID;
    if (row_len < kRowChunk || row_len > kMaxRowLen || row_len % kRowChunk) return CFGZIP_E_INVALID;
    if (!aligned_to(tok_off, 8) || !aligned_to(rows_out, 8) || !aligned_to(hash_out, 8) ||
        !aligned_to(status_out, 4))
        return CFGZIP_E_INVALID;
    if (!ws || !aligned_to(ws, 256)) return CFGZIP_E_WORKSPACE;
    GrammarWorkspace w = carve_grammar_ws(ws, N, V, P);
    if (ws_bytes < w.bytes) return CFGZIP_E_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    Grammar g{prod_head, prod_byte, prod_body_off, prod_body, P, N, (int)ceil_div(N, 32), body_total};
    CFGZIP_TRY(enqueue_grammar_tables(g, w, stream));
    DisplacementArgs a{};
    a.g = g;
    a.hdr = w.hdr;
    a.byte_off = w.byte_off;
    a.pair_first = w.pair_first;
    a.prod_short = w.prod_short;
    a.adj = w.adj;
    a.tok_bytes = tok_bytes;
    a.tok_off = tok_off;
    a.rows = rows_out;
    a.hash = hash_out;
    a.status = status_out;
    a.retry_list[0] = w.retry_list[0];
    a.retry_list[1] = w.retry_list[1];
    a.seed = hash_seed;
    a.V = V;
    a.row_len = row_len;
    int n_cu = 256;
    {
        int dev = 0;
        CFGZIP_TRY(check_hip(hipGetDevice(&dev)));
        CFGZIP_TRY(check_hip(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev)));
        if (n_cu <= 0) n_cu = 256;
    }
    return N <= kMaxByteSymbols ? launch_displacements<uint8_t>(a, n_cu, stream)
                                : launch_displacements<uint16_t>(a, n_cu, stream);
}
