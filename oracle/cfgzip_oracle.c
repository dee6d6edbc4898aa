/*
 * CPU oracle for the CFGzip hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct C.  It shares no code with the HIP library and
 * must never be called from the product path; only the tests, the smoke check
 * and the benchmark's CPU-baseline leg use it.
 *
 * What each function follows in the paper ("Accelerating Constrained Decoding
 * with Token Space Compression"):
 *
 *   oracle_signatures     Displacement of a token (Section 3.2.1, Algorithm 1)
 *                         restricted to right-linear grammars, i.e. to a
 *                         deterministic byte automaton: the PDA stack holds one
 *                         symbol, the stack-adjacency relation (Appendix C) is
 *                         empty, and the displacement of token t collapses to
 *                         the map  q -> delta*(q, bytes(t)).  Written out as
 *                         that walk, from every state.
 *   oracle_build_classes  Section 3.1 "Pre-Computation": group tokens with equal
 *                         signature; representative = byte-wise shortest member
 *                         (tie: smallest token id); vectors c (token -> class)
 *                         and r (class -> representative).  Class ids are issued
 *                         in order of first appearance when scanning token ids
 *                         upwards.  No hashing: full signatures are compared.
 *   oracle_expand_mask    Section 3.1 "Inference" / Figure 1(b): token-level mask
 *                         bit i = class-level mask bit c[i].
 *   oracle_apply_mask_*   Section 2.2 logit masking: a disallowed token's logit
 *                         becomes -infinity, an allowed one is left untouched
 *                         (bit-for-bit).
 *   oracle_map_to_rep     Section 3.1 "Inference" / Figure 1(a): sampled token
 *                         t(i) -> r[c[i]].
 *   oracle_live_states    Section 2.2: a generated prefix is valid iff it is in Pr(L(G)), i.e.
 *                         can be extended to a word of the language.  For a
 *                         deterministic byte automaton with accepting states F:
 *                         state q is live iff some byte string leads from q into F.
 *   oracle_state_masks    Section 2.2 + Section 3.1 "Inference": the engine runs on the
 *                         vocabulary E of representatives; its mask over E in automaton
 *                         state q allows class k iff the state reached from q on the
 *                         representative's bytes is live.
 *   oracle_class_masks    the engine's mask m over E for each sequence of a batch (the row
 *                         of its current state).
 *   oracle_advance_states Section 3.1 "Inference": the engine's state is updated with the
 *                         representative r[c[t]] of the sampled token t.
 *   oracle_representative_vocabulary  Section 3.1 "Inference": the engine is initialised with
 *                         the vocabulary E of the representatives' byte strings.
 *   oracle_nfa_signatures Section 3.2.1 for a right-linear grammar that is NOT deterministic
 *                         (several productions q -> a q' per state and byte): the
 *                         displacement of t is the relation {(q, q') : q' reachable from q
 *                         on bytes(t)}, kept as one bit row per start state.
 *   oracle_nfa_live_states, oracle_nfa_state_masks, oracle_nfa_class_masks,
 *   oracle_nfa_advance_states
 *                         The engine side (Section 2.2, Section 3.1 "Inference") when the
 *                         automaton is not deterministic: the engine's state is a SET of
 *                         automaton states; a class is allowed iff its representative leads
 *                         from some state of the set to a live state; the set advances to
 *                         everything the representative reaches from it.
 *   oracle_hash           The library's signature hash (not in the paper; a
 *                         device of this implementation) written from its
 *                         formula:  H(t) = sum_q a_q * sig[t][q]  mod 2^64 with
 *                         a_q = (q-th output of the SplitMix64 generator seeded
 *                         with `seed`) | 1.
 *
 * Bit masks: int32 words, bit (i & 31) of word (i >> 5); 1 = allowed; rows are
 * padded to whole words; pad bits are written as 0 and ignored on input.
 */

#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* sig[t][q] = state reached from q after reading every byte of token t. */
void oracle_signatures(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                       const uint16_t *table /* [S][256] */, int32_t S,
                       uint16_t *sig /* [V][S] */) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int32_t t = 0; t < V; ++t) {
        for (int32_t q = 0; q < S; ++q) {
            uint16_t s = (uint16_t)q;
            for (int64_t p = tok_off[t]; p < tok_off[t + 1]; ++p)
                s = table[(size_t)s * 256 + tok_bytes[p]];
            sig[(size_t)t * S + q] = s;
        }
    }
}

/* ---- grouping -------------------------------------------------------- */

static const uint16_t *g_sig;
static int32_t g_S;

static int cmp_by_signature_then_id(const void *pa, const void *pb) {
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    const uint16_t *ra = g_sig + (size_t)a * g_S, *rb = g_sig + (size_t)b * g_S;
    for (int32_t q = 0; q < g_S; ++q) {
        if (ra[q] != rb[q]) return ra[q] < rb[q] ? -1 : 1;
    }
    return (a > b) - (a < b);
}

static int cmp_int32(const void *pa, const void *pb) {
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/*
 * Groups tokens by equal signature.  Returns the number of classes C, fills
 * class_of_token[V] and the first C entries of rep_of_class.
 * Not re-entrant (the comparator reads file-scope pointers).
 */
int32_t oracle_build_classes(const uint16_t *sig /* [V][S] */, const int64_t *tok_off,
                             int32_t V, int32_t S,
                             int32_t *class_of_token /* [V] */,
                             int32_t *rep_of_class /* [V] capacity */) {
    if (V <= 0) return 0;
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)V);
    int32_t *first = (int32_t *)malloc(sizeof(int32_t) * (size_t)V); /* smallest member of each group */
    int32_t *group_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)V);
    for (int32_t t = 0; t < V; ++t) order[t] = t;
    g_sig = sig;
    g_S = S;
    qsort(order, (size_t)V, sizeof(int32_t), cmp_by_signature_then_id);

    /* equal signatures are now adjacent, members of a group in ascending id */
    int32_t G = 0;
    for (int32_t i = 0; i < V; ++i) {
        int same = i > 0 && memcmp(sig + (size_t)order[i] * S, sig + (size_t)order[i - 1] * S,
                                   sizeof(uint16_t) * (size_t)S) == 0;
        if (!same) first[G++] = order[i];
        group_of[order[i]] = G - 1;
    }
    /* class id = rank of the group's smallest member among all groups' smallest members */
    int32_t *sorted_first = (int32_t *)malloc(sizeof(int32_t) * (size_t)G);
    memcpy(sorted_first, first, sizeof(int32_t) * (size_t)G);
    qsort(sorted_first, (size_t)G, sizeof(int32_t), cmp_int32);
    int32_t *id_of_group = (int32_t *)malloc(sizeof(int32_t) * (size_t)G);
    for (int32_t k = 0; k < G; ++k) class_of_token[sorted_first[k]] = k; /* temp: on the first members */
    for (int32_t g = 0; g < G; ++g) id_of_group[g] = class_of_token[first[g]];
    for (int32_t t = 0; t < V; ++t) class_of_token[t] = id_of_group[group_of[t]];

    /* representative: shortest member, ties to the smallest token id */
    for (int32_t k = 0; k < G; ++k) rep_of_class[k] = -1;
    for (int32_t t = 0; t < V; ++t) {
        int32_t k = class_of_token[t];
        int32_t r = rep_of_class[k];
        if (r < 0) {
            rep_of_class[k] = t;
        } else {
            int64_t lt = tok_off[t + 1] - tok_off[t], lr = tok_off[r + 1] - tok_off[r];
            if (lt < lr) rep_of_class[k] = t; /* t > r always, so ties keep r */
        }
    }
    free(order);
    free(first);
    free(group_of);
    free(sorted_first);
    free(id_of_group);
    return G;
}

/* ---- decode-step path ------------------------------------------------ */

static int get_bit(const int32_t *row, int64_t i) {
    return (int)(((uint32_t)row[i >> 5] >> (i & 31)) & 1u);
}

void oracle_expand_mask(const int32_t *cls_bits /* [B][W(C)] */, int32_t B, int32_t C,
                        const int32_t *class_of_token /* [V] */, int32_t V,
                        int32_t *tok_bits /* [B][W(V)] */) {
    int64_t Wc = ((int64_t)C + 31) / 32, Wv = ((int64_t)V + 31) / 32;
#pragma omp parallel for schedule(static)
    for (int32_t b = 0; b < B; ++b) {
        const int32_t *in = cls_bits + b * Wc;
        int32_t *out = tok_bits + b * Wv;
        for (int64_t w = 0; w < Wv; ++w) out[w] = 0;
        for (int32_t i = 0; i < V; ++i) {
            if (get_bit(in, class_of_token[i]))
                out[i >> 5] = (int32_t)((uint32_t)out[i >> 5] | (1u << (i & 31)));
        }
    }
}

/* logits as raw 32-bit patterns (fp32); -inf = 0xFF800000 */
void oracle_apply_mask_f32(uint32_t *logits /* [B][row_stride] */, int32_t B, int32_t V,
                           int64_t row_stride, const int32_t *tok_bits /* [B][W(V)] */) {
    int64_t Wv = ((int64_t)V + 31) / 32;
#pragma omp parallel for schedule(static)
    for (int32_t b = 0; b < B; ++b)
        for (int32_t i = 0; i < V; ++i)
            if (!get_bit(tok_bits + b * Wv, i)) logits[b * row_stride + i] = 0xFF800000u;
}

/* logits as raw 16-bit patterns (bf16); -inf = 0xFF80 */
void oracle_apply_mask_bf16(uint16_t *logits, int32_t B, int32_t V, int64_t row_stride,
                            const int32_t *tok_bits) {
    int64_t Wv = ((int64_t)V + 31) / 32;
#pragma omp parallel for schedule(static)
    for (int32_t b = 0; b < B; ++b)
        for (int32_t i = 0; i < V; ++i)
            if (!get_bit(tok_bits + b * Wv, i)) logits[b * row_stride + i] = 0xFF80u;
}

/* out[b] = r[c[tok[b]]]; a token id outside [0, V) maps to -1 */
void oracle_map_to_rep(const int32_t *tok, int32_t B, const int32_t *class_of_token, int32_t V,
                       const int32_t *rep_of_class, int32_t C, int32_t *out) {
    (void)C;
    for (int32_t b = 0; b < B; ++b) {
        int32_t t = tok[b];
        out[b] = (t < 0 || t >= V) ? -1 : rep_of_class[class_of_token[t]];
    }
}

/* ---- the engine side for a deterministic byte automaton --------------- */

/* live[q] = 1 iff an accepting state can be reached from q (with zero or more bytes). */
void oracle_live_states(const uint16_t *table /* [S][256] */, int32_t S,
                        const uint8_t *accept /* [S] */, uint8_t *live /* [S] */) {
    for (int32_t q = 0; q < S; ++q) live[q] = accept[q] ? 1 : 0;
    int changed = 1;
    while (changed) {
        changed = 0;
        for (int32_t q = 0; q < S; ++q) {
            if (live[q]) continue;
            for (int b = 0; b < 256; ++b) {
                if (live[table[(size_t)q * 256 + b]]) {
                    live[q] = 1;
                    changed = 1;
                    break;
                }
            }
        }
    }
}

/* state_mask[q] bit k = live[ sig_rep[k][q] ]: class k is allowed in automaton state q. */
void oracle_state_masks(const uint16_t *sig_rep /* [C][S] */, int32_t C, int32_t S,
                        const uint8_t *live /* [S] */, int32_t *state_mask /* [S][W(C)] */) {
    int64_t Wc = ((int64_t)C + 31) / 32;
    for (int32_t q = 0; q < S; ++q) {
        int32_t *row = state_mask + q * Wc;
        for (int64_t w = 0; w < Wc; ++w) row[w] = 0;
        for (int32_t k = 0; k < C; ++k) {
            if (live[sig_rep[(size_t)k * S + q]])
                row[k >> 5] = (int32_t)((uint32_t)row[k >> 5] | (1u << (k & 31)));
        }
    }
}

/* cls_bits[b] = state_mask[states[b]]; a state outside [0, S) allows nothing. */
void oracle_class_masks(const int32_t *state_mask /* [S][W(C)] */, int32_t S, int32_t C,
                        const int32_t *states /* [B] */, int32_t B,
                        int32_t *cls_bits /* [B][W(C)] */) {
    int64_t Wc = ((int64_t)C + 31) / 32;
    for (int32_t b = 0; b < B; ++b) {
        int32_t q = states[b];
        for (int64_t w = 0; w < Wc; ++w)
            cls_bits[b * Wc + w] = (q < 0 || q >= S) ? 0 : state_mask[q * Wc + w];
    }
}

/* states[b] <- state reached from states[b] on the representative of tok[b]'s class;
 * an id or state out of range gives -1. */
void oracle_advance_states(const uint16_t *sig_rep /* [C][S] */, int32_t C, int32_t S,
                           const int32_t *class_of_token /* [V] */, int32_t V,
                           const int32_t *tok /* [B] */, int32_t B, int32_t *states /* [B] */) {
    for (int32_t b = 0; b < B; ++b) {
        int32_t t = tok[b], q = states[b];
        if (t < 0 || t >= V || q < 0 || q >= S) {
            states[b] = -1;
            continue;
        }
        int32_t k = class_of_token[t];
        states[b] = (k < 0 || k >= C) ? -1 : (int32_t)sig_rep[(size_t)k * S + q];
    }
}

/* ---- the library's signature hash, from its formula ------------------- */

/* SplitMix64 (Steele, Lea, Flood 2014; Vigna's public-domain formulation):
 * state += 0x9E3779B97F4A7C15; z = state; z = (z ^ z>>30) * 0xBF58476D1CE4E5B9;
 * z = (z ^ z>>27) * 0x94D049BB133111EB; output z ^ z>>31. */
uint64_t oracle_splitmix64_next(uint64_t *state) {
    uint64_t z = (*state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

void oracle_hash(const uint16_t *sig /* [V][S] */, int32_t V, int32_t S, uint64_t seed,
                 uint64_t *hash_out /* [V] */) {
    uint64_t *a = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)S);
    uint64_t state = seed;
    for (int32_t q = 0; q < S; ++q) a[q] = oracle_splitmix64_next(&state) | 1ull;
    for (int32_t t = 0; t < V; ++t) {
        uint64_t h = 0;
        for (int32_t q = 0; q < S; ++q) h += a[q] * (uint64_t)sig[(size_t)t * S + q];
        hash_out[t] = h;
    }
    free(a);
}

/* Non-deterministic byte automaton: nfa[b][q] is the bit row (W = ceil(S/32) words, bit q' & 31
 * of word q' >> 5) of the states that may follow q on byte b.  out[t][q] = bit row of the states
 * reachable from q on the bytes of token t (the identity for an empty token).  Pad bits 0. */
void oracle_nfa_signatures(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                           const uint32_t *nfa /* [256][S][W] */, int32_t S,
                           uint32_t *out /* [V][S][W] */) {
    const int32_t W = (S + 31) / 32;
#pragma omp parallel for schedule(dynamic, 64)
    for (int32_t t = 0; t < V; ++t) {
        uint32_t *cur = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)W);
        uint32_t *nxt = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)W);
        for (int32_t q = 0; q < S; ++q) {
            for (int32_t w = 0; w < W; ++w) cur[w] = 0;
            cur[q >> 5] = 1u << (q & 31);
            for (int64_t p = tok_off[t]; p < tok_off[t + 1]; ++p) {
                const uint32_t *step = nfa + (size_t)tok_bytes[p] * S * W;
                for (int32_t w = 0; w < W; ++w) nxt[w] = 0;
                for (int32_t x = 0; x < S; ++x)
                    if ((cur[x >> 5] >> (x & 31)) & 1u)
                        for (int32_t w = 0; w < W; ++w) nxt[w] |= step[(size_t)x * W + w];
                uint32_t *tmp = cur; cur = nxt; nxt = tmp;
            }
            for (int32_t w = 0; w < W; ++w) out[((size_t)t * S + q) * W + w] = cur[w];
        }
        free(cur);
        free(nxt);
    }
}

/* ---- engine side for a non-deterministic byte automaton ------------------------------- */

static int bit_of(const uint32_t *row, int32_t i) { return (row[i >> 5] >> (i & 31)) & 1u; }

/* live[q] = 1 iff an accepting state can be reached from q (q itself counts). */
void oracle_nfa_live_states(const uint32_t *nfa /* [256][S][W] */, int32_t S,
                            const uint8_t *accept /* [S] */, uint8_t *live /* [S] */) {
    const int32_t W = (S + 31) / 32;
    for (int32_t q = 0; q < S; ++q) live[q] = accept[q] ? 1 : 0;
    int changed = 1;
    while (changed) {
        changed = 0;
        for (int32_t q = 0; q < S; ++q) {
            if (live[q]) continue;
            for (int b = 0; b < 256 && !live[q]; ++b)
                for (int32_t x = 0; x < S; ++x)
                    if (live[x] && bit_of(nfa + ((size_t)b * S + q) * W, x)) {
                        live[q] = 1;
                        changed = 1;
                        break;
                    }
        }
    }
}

/* state_mask[q] bit k = 1 iff the representative of class k leads from q to some live state:
 * exists q' with (q, q') in rel_rep[k] and live[q']. */
void oracle_nfa_state_masks(const uint32_t *rel_rep /* [C][S][W] */, int32_t C, int32_t S,
                            const uint8_t *live /* [S] */, int32_t *state_mask /* [S][W(C)] */) {
    const int32_t W = (S + 31) / 32;
    const int64_t Wc = ((int64_t)C + 31) / 32;
    for (int32_t q = 0; q < S; ++q) {
        int32_t *row = state_mask + q * Wc;
        for (int64_t w = 0; w < Wc; ++w) row[w] = 0;
        for (int32_t k = 0; k < C; ++k) {
            const uint32_t *reach = rel_rep + ((size_t)k * S + q) * W;
            int ok = 0;
            for (int32_t x = 0; x < S && !ok; ++x) ok = bit_of(reach, x) && live[x];
            if (ok) row[k >> 5] = (int32_t)((uint32_t)row[k >> 5] | (1u << (k & 31)));
        }
    }
}

/* cls_bits[b] = union of state_mask[q] over the states q of sets[b]. */
void oracle_nfa_class_masks(const int32_t *state_mask /* [S][W(C)] */, int32_t S, int32_t C,
                            const uint32_t *sets /* [B][W(S)] */, int32_t B,
                            int32_t *cls_bits /* [B][W(C)] */) {
    const int32_t W = (S + 31) / 32;
    const int64_t Wc = ((int64_t)C + 31) / 32;
    for (int32_t b = 0; b < B; ++b) {
        for (int64_t w = 0; w < Wc; ++w) cls_bits[b * Wc + w] = 0;
        for (int32_t q = 0; q < S; ++q)
            if (bit_of(sets + (size_t)b * W, q))
                for (int64_t w = 0; w < Wc; ++w)
                    cls_bits[b * Wc + w] = (int32_t)((uint32_t)cls_bits[b * Wc + w] | (uint32_t)state_mask[q * Wc + w]);
    }
}

/* sets[b] <- everything the representative of tok[b]'s class reaches from a state of sets[b];
 * a token id or class id out of range leaves the empty set. */
void oracle_nfa_advance_states(const uint32_t *rel_rep /* [C][S][W] */, int32_t C, int32_t S,
                               const int32_t *class_of_token /* [V] */, int32_t V,
                               const int32_t *tok /* [B] */, int32_t B, uint32_t *sets /* [B][W] */) {
    const int32_t W = (S + 31) / 32;
    uint32_t *next = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)W);
    for (int32_t b = 0; b < B; ++b) {
        uint32_t *set = sets + (size_t)b * W;
        for (int32_t w = 0; w < W; ++w) next[w] = 0;
        const int32_t t = tok[b];
        const int32_t k = (t < 0 || t >= V) ? -1 : class_of_token[t];
        if (k >= 0 && k < C)
            for (int32_t q = 0; q < S; ++q)
                if (bit_of(set, q))
                    for (int32_t w = 0; w < W; ++w) next[w] |= rel_rep[((size_t)k * S + q) * W + w];
        for (int32_t w = 0; w < W; ++w) set[w] = next[w];
    }
    free(next);
}

/* Byte strings of the representatives, class after class: rep_off[k] .. rep_off[k+1] delimit
 * bytes(r[k]) in rep_bytes; an id outside [0, V) stands for the empty string.  Returns the total
 * number of bytes; with rep_bytes == NULL only the offsets are written. */
int64_t oracle_representative_vocabulary(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                                         const int32_t *rep, int32_t C, int64_t *rep_off,
                                         uint8_t *rep_bytes) {
    int64_t at = 0;
    for (int32_t k = 0; k < C; ++k) {
        rep_off[k] = at;
        int32_t t = rep[k];
        if (t < 0 || t >= V) continue;
        for (int64_t p = tok_off[t]; p < tok_off[t + 1]; ++p) {
            if (rep_bytes) rep_bytes[at] = tok_bytes[p];
            ++at;
        }
    }
    rep_off[C] = at;
    return at;
}
