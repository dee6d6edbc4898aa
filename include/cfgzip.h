/*
 * cfgzip.h - C ABI of the MI355X (gfx950) CFGzip hot-path library.
 *
 * CFGzip ("Accelerating Constrained Decoding with Token Space Compression")
 * collapses a tokenizer vocabulary T into equivalence classes E of tokens that a
 * grammar engine cannot tell apart, so that the engine works on |E| << |T|
 * representatives.  This library holds the data-parallel part:
 *
 *   offline   per-token signatures, grouping into classes, representatives
 *             (paper Section 3.1 "Pre-Computation", Section 3.2 for what a
 *             signature is);
 *   per step  class-level mask -> token-level mask, -inf masking of logits,
 *             sampled token -> class representative
 *             (paper Section 3.1 "Inference", Figure 1; Section 2.2 for what a
 *             mask means).
 *
 * Signature.  The paper's relation is equality of displacement sets over the
 * one-state pushdown automaton of a grammar in Greibach normal form (Section
 * 3.2.1, Algorithm 1).  Three forms of it are covered:
 *   - a deterministic byte automaton (a right-linear grammar): the stack holds one
 *     symbol, no stack backtrack can follow the first one, and the displacement of
 *     token t is the map  q -> delta*(q, bytes(t))  over all automaton states q;
 *     that vector is the signature sig[t][q], S entries of uint16
 *     (cfgzip_signatures);
 *   - a non-deterministic byte automaton: the relation R_t of the state pairs that
 *     bytes(t) connects, S bit rows (cfgzip_nfa_signatures);
 *   - a grammar in Greibach normal form: the displacement set itself, written as a
 *     fixed-length row (cfgzip_stack_adjacency, cfgzip_displacements).
 * cfgzip_build_classes groups tokens by any of the three.
 *
 * Conventions for every call
 *   - Every pointer is a DEVICE pointer owned by the caller unless the comment
 *     says "host".  The library allocates no device memory, frees nothing and keeps no
 *     pointer after a call returns.  Scratch memory comes in as `ws`, sized by
 *     the matching *_workspace_bytes query (a host-only computation).  (cfgzip_build_classes
 *     keeps 32 bytes of pinned host memory per calling thread, through which its counts reach
 *     the host.)
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Work
 *     is enqueued on it; calls do not synchronise, except cfgzip_build_classes
 *     (it must hand the class count back to the host).
 *   - Return value: CFGZIP_OK, or a negative CFGZIP_E* code.  On
 *     CFGZIP_E_INVALID nothing was enqueued.  On CFGZIP_E_HIP the failing HIP
 *     status is kept per host thread and read with cfgzip_last_hip_error().
 *   - Ids (token ids, class ids) are int32.  Bit masks are int32 words: bit
 *     (i & 31) of word (i >> 5) belongs to item i; 1 = allowed.  A mask row over
 *     n items has W(n) = ceil(n / 32) words; pad bits are written as 0 and
 *     ignored when read.
 *   - Values the host cannot check without reading device memory (table entries
 *     < S, class ids < C, sampled ids < V) are the caller's responsibility where
 *     a comment says so; cfgzip_map_to_rep range-checks on the device.
 */
#ifndef CFGZIP_H
#define CFGZIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CFGZIP_OK 0
#define CFGZIP_E_INVALID (-1)   /* null pointer, non-positive size, S > 65536, bad enum, misaligned pointer */
#define CFGZIP_E_WORKSPACE (-2) /* ws == NULL or ws_bytes smaller than the query says */
#define CFGZIP_E_HIP (-3)       /* a HIP call failed; see cfgzip_last_hip_error() */
#define CFGZIP_E_COLLISION (-4) /* hash collisions could not be resolved within the round limit */
#define CFGZIP_E_TOO_LARGE (-5) /* a size beyond what an entry point with built-in scratch memory takes */

#define CFGZIP_DTYPE_F32 0
#define CFGZIP_DTYPE_BF16 1

#define CFGZIP_BITS_TOKEN 0 /* `bits` is a token-level mask  [B][W(V)] */
#define CFGZIP_BITS_CLASS 1 /* `bits` is a class-level mask  [B][W(C)], gathered through class_of_token */

/* hipError_t (as int) of the last failing HIP call made by this host thread; 0 if none. */
int cfgzip_last_hip_error(void);

/* Library version: major * 100 + minor. */
int cfgzip_version(void);

/*
 * Signatures of all tokens (paper Section 3.2.1 / Algorithm 1, regular case):
 *     sig[t][q] = state reached from q after reading bytes(t),  0 <= t < V, 0 <= q < S,
 * and/or their 64-bit hash
 *     hash[t] = sum_{q<S} a_q * sig[t][q]  (mod 2^64),
 *     a_q = (q-th output of SplitMix64 seeded with hash_seed) | 1.
 * The sum is order-free, so the hash does not depend on how states are split
 * over lanes, waves or kernels.  The hash is a device of this library (the
 * paper never hashes); class ids never depend on it.
 *
 *   tok_bytes  uint8 [tok_off[V]]   concatenated token bytes
 *   tok_off    int64 [V + 1]        CSR offsets, tok_off[0] = 0, non-decreasing; an empty
 *                                   token (equal offsets) has the identity signature
 *   table      uint16 [S][256]      table[q][b] = next state; every entry must be < S
 *                                   (caller's responsibility)
 *   S          1 .. 65536
 *   sig_out    uint16 [V][S] or NULL (NULL: signatures are hashed on the fly, never stored)
 *   hash_out   uint64 [V]   or NULL (at least one of sig_out / hash_out must be given)
 *   ws         cfgzip_signatures_workspace_bytes(V, S) bytes, 256-byte aligned.  After the call
 *              it holds, besides tables, the compressed form in which the signatures were
 *              computed (per token the states reached from the distinct states its first
 *              byte leaves; up to 512 bytes per token).  Handing the untouched workspace
 *              to cfgzip_build_classes lets it compare those instead of walking again.
 */
size_t cfgzip_signatures_workspace_bytes(int32_t V, int32_t S);
int cfgzip_signatures(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                      const uint16_t *table, int32_t S,
                      uint16_t *sig_out, uint64_t *hash_out, uint64_t hash_seed,
                      void *ws, size_t ws_bytes, void *stream);

/*
 * cfgzip_signatures by composition (paper Appendix A, Lemma 1: the relation is compatible with
 * concatenation, so the signature of a concatenation is the composition of the signatures,
 *     sig(tu)[q] = sig(u)[sig(t)[q]] ).
 * A token whose byte string starts with the byte string of a shorter token need not be walked
 * from its first byte: its walk continues from that token's end states.  Tokens of up to three
 * bytes are walked first; every longer token then starts from the longest of them that is a
 * prefix of it (if any) and reads only its remaining bytes.  Arguments and results are those of
 * cfgzip_signatures, bit for bit; only the work differs (fewer table reads, four more launches).
 *   ws   cfgzip_signatures_composed_workspace_bytes(V, S) bytes, 256-byte aligned; it begins with
 *        a signature workspace as cfgzip_signatures leaves it (usable as signatures_ws of
 *        cfgzip_build_classes)
 */
size_t cfgzip_signatures_composed_workspace_bytes(int32_t V, int32_t S);
int cfgzip_signatures_composed(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                               const uint16_t *table, int32_t S,
                               uint16_t *sig_out, uint64_t *hash_out, uint64_t hash_seed,
                               void *ws, size_t ws_bytes, void *stream);

/*
 * cfgzip_signatures for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments and results as cfgzip_signatures without `ws`; the tables the
 * kernels need live in a device array that is part of the loaded library
 * (about 14.2 MiB per GPU, held until the process ends), so the call allocates nothing.
 *   S   1 .. CFGZIP_STATIC_MAX_STATES; a larger automaton is refused with CFGZIP_E_TOO_LARGE
 *       (nothing enqueued)
 * The compressed signatures are not kept: cfgzip_build_classes after this call is given
 * signatures_ws = NULL.  All calls on one GPU share that GPU's array: two calls that overlap
 * in time on the same GPU (different streams or host threads) race; calls on one stream, or
 * ordered by events, are fine.  Nothing in the array needs clearing between calls.
 */
#define CFGZIP_STATIC_MAX_STATES 4096
int cfgzip_signatures_static(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                             const uint16_t *table, int32_t S,
                             uint16_t *sig_out, uint64_t *hash_out, uint64_t hash_seed,
                             void *stream);

/*
 * Equivalence classes, class ids and representatives (paper Section 3.1
 * "Pre-Computation"): tokens with equal signature form a class; the vector c
 * maps token id -> class id, the vector r maps class id -> representative, the
 * byte-wise shortest member (ties: smallest token id).  Class ids are issued in
 * order of each class's smallest token id, so c[0] = 0.
 *
 * Method: radix sort by (hash, first byte) with the token id as value, equal-hash
 * segments, then every member's full signature is compared with its left
 * neighbour's in the segment (equality is transitive); members that differ (a
 * hash collision) start a chain of their own and the chains of a segment are
 * matched against each other in further rounds, so the result is exact for any
 * `hash` that is a function of the signature (equal signatures must carry equal
 * hashes).  The comparison reads, in order of preference: the compressed
 * signatures in `signatures_ws`; the rows of `sig`; or, with neither, signatures
 * recomputed from the automaton.
 *
 *   tok_bytes, tok_off, V, table, S   as for cfgzip_signatures.  `table` may be NULL when `sig`
 *              is given and `signatures_ws` is NULL: the rows of `sig` are then the only source
 *              and may be any fixed-length encoding in which equal rows mean equivalent tokens
 *              (S = row length), e.g. the rows of cfgzip_displacements
 *   sig        uint16 [V][S] from cfgzip_signatures, or NULL
 *   hash       uint64 [V]    from cfgzip_signatures (or any function of the signature)
 *   signatures_ws  the workspace of a finished cfgzip_signatures call with the same
 *              vocabulary, table, V and S, not written to since, or NULL.  It is only read.
 *              If it turns out not to hold that call's data (other V or S, or its
 *              compressed signatures did not fit) the next source is used.
 *   class_of_token   out, int32 [V]
 *   rep_of_class     out, int32 [V] capacity; the first C entries are written
 *   num_classes_dev  out, int32 [1] device, or NULL
 *   num_classes_host out, int32 [1] HOST, or NULL
 *   collisions_host  out, int32 [1] HOST, or NULL: number of tokens whose signature
 *                    differed from that of their left neighbour in an equal-hash
 *                    segment (0 unless hashes collide)
 *   ws         cfgzip_build_classes_workspace_bytes(V, S) bytes, 256-byte aligned
 * Synchronises `stream` before returning.
 */
size_t cfgzip_build_classes_workspace_bytes(int32_t V, int32_t S);
int cfgzip_build_classes(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                         const uint16_t *table, int32_t S,
                         const uint16_t *sig, const uint64_t *hash, void *signatures_ws,
                         int32_t *class_of_token, int32_t *rep_of_class,
                         int32_t *num_classes_dev, int32_t *num_classes_host,
                         int32_t *collisions_host,
                         void *ws, size_t ws_bytes, void *stream);

/*
 * Class-level mask -> token-level mask (paper Section 3.1 "Inference",
 * Figure 1(b)):  tok_bits[b] bit i = cls_bits[b] bit class_of_token[i].
 *
 *   cls_bits        int32 [B][W(C)]
 *   class_of_token  int32 [V], every entry in [0, C) (caller's responsibility)
 *   tok_bits        out, int32 [B][W(V)], pad bits 0
 */
int cfgzip_expand_mask(const int32_t *cls_bits, int32_t B, int32_t C,
                       const int32_t *class_of_token, int32_t V,
                       int32_t *tok_bits, void *stream);

/*
 * Logit masking in place (paper Section 2.2: a disallowed token's logit is set
 * to -infinity; Section 3.1 "Inference": z_i <- z_i * m_{c_i} read as a select,
 * since a product with -inf would give +inf or NaN on log-probabilities):
 *     logits[b][i] unchanged, bit for bit, if token i is allowed in row b,
 *     else the dtype's -inf pattern (fp32 0xFF800000, bf16 0xFF80).
 *
 *   logits      [B] rows of V elements, consecutive rows row_stride ELEMENTS apart
 *               (row_stride >= V); element size 4 (F32) or 2 (BF16) bytes; the base
 *               pointer must be aligned to the element size
 *   bits_kind   CFGZIP_BITS_TOKEN: bits = int32 [B][W(V)] token-level mask;
 *               CFGZIP_BITS_CLASS: bits = int32 [B][W(C)] class-level mask, gathered through
 *               class_of_token (expand and apply fused; no token mask round trip)
 *   class_of_token, C   used for CFGZIP_BITS_CLASS only (else NULL / 0)
 *   tok_bits_out        CFGZIP_BITS_CLASS only: NULL, or int32 [B][W(V)] that also receives
 *                       the token-level mask
 */
int cfgzip_apply_mask(void *logits, int32_t dtype, int32_t B, int32_t V, int64_t row_stride,
                      const int32_t *bits, int32_t bits_kind,
                      const int32_t *class_of_token, int32_t C,
                      int32_t *tok_bits_out, void *stream);

/*
 * Sampled token -> class representative (paper Section 3.1 "Inference",
 * Figure 1(a)):  out[b] = rep_of_class[class_of_token[tok[b]]].
 * A token id outside [0, V), or a class id outside [0, C), yields -1.
 *
 *   tok  int32 [B];  out  int32 [B]
 */
int cfgzip_map_to_rep(const int32_t *tok, int32_t B,
                      const int32_t *class_of_token, int32_t V,
                      const int32_t *rep_of_class, int32_t C,
                      int32_t *out, void *stream);

/*
 * One decode step of the per-step path in a single launch (paper Section 3.1 "Inference",
 * Figure 1, both halves): cfgzip_apply_mask with CFGZIP_BITS_CLASS on `logits`, and
 * cfgzip_map_to_rep on the tokens sampled in the step before,
 *     rep_out[b] = rep_of_class[class_of_token[tok[b]]]   (-1 when out of range).
 * The two are independent (the mask does not depend on `tok`); one workgroup of the masking
 * kernel does the B look-ups once its own rows are done.  Arguments as for the two calls;
 * tok_bits_out may be NULL.
 */
int cfgzip_decode_step(void *logits, int32_t dtype, int32_t B, int32_t V, int64_t row_stride,
                       const int32_t *cls_bits, const int32_t *class_of_token, int32_t C,
                       int32_t *tok_bits_out,
                       const int32_t *tok, const int32_t *rep_of_class, int32_t *rep_out,
                       void *stream);

/*
 * Engine side for grammars given as a deterministic byte automaton.  The paper's engine works
 * on the vocabulary E of class representatives (Section 3.1 "Inference"); for a byte
 * automaton with accepting states that engine is a table look-up, and these three calls are
 * it.  A token may follow a prefix iff the extended sequence is still a prefix of the
 * language (Section 2.2), i.e. iff the state it leads to is live: an accepting state can be
 * reached from it.
 *
 *   sig_rep   uint16 [C][S]  signatures of the C representatives (cfgzip_signatures on the
 *                            representatives' byte strings): sig_rep[k][q] = state reached
 *                            from q on the bytes of r[k]
 *   live      uint8 [S]      1 iff an accepting state is reachable from the state
 *
 * cfgzip_state_masks (once per grammar):
 *     state_mask[q] bit k = live[sig_rep[k][q]]        int32 [S][W(C)], pad bits 0
 * cfgzip_class_masks (per decode step): the engine's mask over E for each sequence,
 *     cls_bits[b] = state_mask[states[b]]              int32 [B][W(C)]; a state outside
 *     [0, S) gives an all-zero row
 * cfgzip_advance_states (per decode step): the engine consumes the representative of the
 *     sampled token's class instead of the token,
 *     states[b] <- sig_rep[class_of_token[tok[b]]][states[b]]     int32 [B], in place;
 *     a token id, class id or state out of range gives -1
 */
/*
 * The vocabulary E the engine is initialised with (paper Section 3.1 "Inference"): the byte
 * strings of the representatives, in class order, in the same CSR form as the token vocabulary:
 *     rep_off[k] .. rep_off[k+1]  =  position of bytes(r[k]) in rep_bytes,  rep_off[0] = 0.
 *   rep_of_class  int32 [C]; an id outside [0, V) gives an empty string
 *   rep_off       out, int64 [C + 1]
 *   rep_bytes     out, uint8 [capacity]; bytes that would fall beyond `capacity` are not written
 *                 (rep_off[C] still tells how many there are).  tok_off[V] bytes always suffice,
 *                 since representatives are distinct tokens.  capacity = 0: offsets only.
 */
int cfgzip_representative_vocabulary(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                                     const int32_t *rep_of_class, int32_t C,
                                     int64_t *rep_off, uint8_t *rep_bytes, int64_t capacity,
                                     void *stream);

int cfgzip_state_masks(const uint16_t *sig_rep, int32_t C, int32_t S, const uint8_t *live,
                       int32_t *state_mask, void *stream);
/*
 * cfgzip_engine_step: one decode step of that engine in a single launch (the three calls below
 * followed by cfgzip_apply_mask, without the class masks going through memory):
 *     q[b] = tok_prev ? sig_rep[class_of_token[tok_prev[b]]][states_in[b]] : states_in[b]
 *            (-1 if the token id, its class id or the state is out of range)
 *     states_out[b] = q[b]
 *     logits row b masked with the class mask state_mask[q[b]] gathered through class_of_token
 *     (all of row b becomes -inf if q[b] is not a state); tok_bits_out as for cfgzip_apply_mask.
 *   tok_prev    int32 [B] tokens sampled in the previous step, or NULL (first step: no advance)
 *   states_in   int32 [B];  states_out  int32 [B], a different array (callers alternate two)
 *   logits, dtype, row_stride, tok_bits_out   as for cfgzip_apply_mask
 */
int cfgzip_engine_step(void *logits, int32_t dtype, int32_t B, int32_t V, int64_t row_stride,
                       const int32_t *state_mask, int32_t S, int32_t C,
                       const int32_t *class_of_token, const uint16_t *sig_rep,
                       const int32_t *tok_prev, const int32_t *states_in, int32_t *states_out,
                       int32_t *tok_bits_out, void *stream);
int cfgzip_class_masks(const int32_t *state_mask, int32_t S, int32_t C, const int32_t *states,
                       int32_t B, int32_t *cls_bits, void *stream);
int cfgzip_advance_states(const uint16_t *sig_rep, int32_t C, int32_t S,
                          const int32_t *class_of_token, int32_t V, const int32_t *tok, int32_t B,
                          int32_t *states, void *stream);

/*
 * General case: grammars in Greibach normal form (paper Section 2.1), every production
 *     A -> a B_1 .. B_n,   one terminal byte a, n >= 0 non-terminals (any number),
 * non-terminals numbered 0 .. N-1, N <= 4096, given as flat arrays
 *     prod_head uint16 [P], prod_byte uint8 [P],
 *     prod_body_off int32 [P + 1], prod_body uint16 [body_total]
 *     (the body of production i is prod_body[prod_body_off[i] .. prod_body_off[i+1]);
 *      prod_body_off[0] = 0, prod_body_off[P] = body_total; prod_body may be NULL if body_total = 0)
 * in strictly ascending order of (byte, head, body), bodies compared symbol by symbol with a
 * proper prefix first (so no production occurs twice).  The order, the offsets and the value
 * ranges are checked on the device; a grammar that breaks them is reported, not computed (below).
 *
 * cfgzip_stack_adjacency (paper Section 3.2.2, Appendix C): the relation "Y can be consumed
 * right before Z":  for every production A -> a B_1 .. B_n Z beta with n >= 1, every Y that is
 * reachable from B_n along right-most body symbols (B_n itself included) and has a production
 * without body.
 *     adj_out      int32 [N][W(N)]   bit Y of row Z <=> (Y, Z) stack-adjacent
 *     invalid_out  int32 [1] or NULL 1 if the grammar broke a rule above (adj_out then
 *                                    holds no result), else 0
 *
 * cfgzip_displacements (paper Section 3.2.1, Algorithm 1, with the backtrack restricted to
 * stack-adjacent symbols): the displacement set of every token, i.e. the pairs (input queue,
 * output stack) with which the token can be read by the one-state pushdown automaton of the
 * grammar; the first backtrack may take any production of the first byte.  Each set is
 * written as a row of row_len 16-bit values so that equal sets give equal rows:
 *     row[0] = number of pairs; then one record per pair,
 *     ni, no, the ni queue symbols, the no stack symbols (top first),
 *     in ascending order of (ni, no), then of the queue, then of the stack; the rest is 0.
 * hash_out[t] is the sum over the pairs of a 64-bit mix of the record and hash_seed (a
 * function of the set, for cfgzip_build_classes; never part of a result).
 * Bounds.  With C_p the set of configurations (queue, stack, symbol consumed last) that
 * Algorithm 1 reaches after p bytes of the token: no successor of a configuration of C_p may
 * hold more than 32 queue symbols or more than 32 stack symbols, and the successors of C_p, one
 * per configuration and applicable production (counted before equal ones fall together), may
 * number at most 256.  (Tokens are first tried in smaller buffers and taken again when those do
 * not suffice; which attempt finishes a token shows in no output.)  A token that breaks one of
 * the bounds, or whose set needs more than row_len entries, gets status
 * CFGZIP_DISP_OVERFLOW and a row no other token has (0xFFFF, id & 0xFFFF, id >> 16, 0 ..):
 * it forms a class of its own.  With status CFGZIP_DISP_OK the row holds exactly the set
 * Algorithm 1 returns.
 *     rows_out    uint16 [V][row_len], 8-byte aligned
 *     row_len     a multiple of 256, 256 .. 4096 (CFGZIP_DISP_ROW is the usual choice)
 *     hash_out    uint64 [V]
 *     status_out  int32 [V] or NULL: CFGZIP_DISP_OK, CFGZIP_DISP_OVERFLOW, or
 *                 CFGZIP_DISP_BAD_GRAMMAR for every token (rows and hashes then 0)
 *     ws          cfgzip_displacements_workspace_bytes(V, N, P) bytes, 256-byte aligned
 *                 (cfgzip_stack_adjacency alone: V = 0)
 * Grouping: cfgzip_build_classes(tok_bytes, tok_off, V, NULL, row_len, rows, hash, NULL, ..).
 */
#define CFGZIP_DISP_ROW 256
#define CFGZIP_DISP_OK 0
#define CFGZIP_DISP_OVERFLOW 1
#define CFGZIP_DISP_BAD_GRAMMAR 2
size_t cfgzip_displacements_workspace_bytes(int32_t V, int32_t N, int32_t P);
int cfgzip_stack_adjacency(const uint16_t *prod_head, const uint8_t *prod_byte,
                           const int32_t *prod_body_off, const uint16_t *prod_body,
                           int32_t body_total, int32_t P, int32_t N,
                           int32_t *adj_out, int32_t *invalid_out,
                           void *ws, size_t ws_bytes, void *stream);
int cfgzip_displacements(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                         const uint16_t *prod_head, const uint8_t *prod_byte,
                         const int32_t *prod_body_off, const uint16_t *prod_body,
                         int32_t body_total, int32_t P, int32_t N,
                         uint16_t *rows_out, int32_t row_len, uint64_t *hash_out,
                         int32_t *status_out, uint64_t hash_seed,
                         void *ws, size_t ws_bytes, void *stream);

/*
 * Non-deterministic byte automata (paper Section 3.2.1 for a right-linear grammar with several
 * productions q -> a q' per state and byte): the displacement of token t is the relation
 *     R_t = {(q, q') : q' can be reached from q on bytes(t)},
 * the boolean product of the per-byte relations; R of the empty token is the identity.
 *
 *   nfa       int32 [256][S][W(S)]  bit q' of row nfa[b][q] <=> q' may follow q on byte b
 *                                   (pad bits must be 0); 16-byte aligned, as is rel_out
 *   S         1 .. 1024 (up to 256 states a thread keeps its state set in registers, beyond
 *             that in LDS)
 *   rel_out   int32 [V][S][W(S)]    bit q' of row rel_out[t][q] <=> (q, q') in R_t; pad bits 0
 *   hash_out  uint64 [V] or NULL    the hash of cfgzip_signatures taken over the relation read
 *                                   as 2 * S * W(S) 16-bit entries (low half of a word first)
 * Grouping: cfgzip_build_classes(tok_bytes, tok_off, V, NULL, 2 * S * W(S), (uint16*)rel_out,
 * hash_out, NULL, ..).  A deterministic automaton gives one-bit rows and the classes of the
 * byte walk.
 */
int cfgzip_nfa_signatures(const uint8_t *tok_bytes, const int64_t *tok_off, int32_t V,
                          const int32_t *nfa, int32_t S, int32_t *rel_out, uint64_t *hash_out,
                          uint64_t hash_seed, void *stream);

/*
 * Engine side for a non-deterministic byte automaton (paper Section 2.2 and Section 3.1
 * "Inference", as cfgzip_state_masks / cfgzip_class_masks / cfgzip_advance_states above): the
 * engine's state per sequence is a SET of automaton states, a bit row int32 [W(S)].
 *   rel_rep   int32 [C][S][W(S)]  relations of the C representatives (cfgzip_nfa_signatures on the
 *                                 representatives' byte strings, or rows of its output)
 *   live      uint8 [S]           1 iff an accepting state can be reached from the state
 * cfgzip_nfa_state_masks (once per grammar):
 *     state_mask[q] bit k = some state that r[k] reaches from q is live      int32 [S][W(C)]
 * cfgzip_nfa_class_masks (per step):
 *     cls_bits[b] = union of state_mask[q] over the states q of state_sets[b]  int32 [B][W(C)]
 * cfgzip_nfa_advance_states (per step), in place:
 *     state_sets[b] <- union over q in state_sets[b] of rel_rep[class_of_token[tok[b]]][q];
 *     a token id or class id out of range leaves the empty set (which allows nothing)
 */
int cfgzip_nfa_state_masks(const int32_t *rel_rep, int32_t C, int32_t S, const uint8_t *live,
                           int32_t *state_mask, void *stream);
int cfgzip_nfa_class_masks(const int32_t *state_mask, int32_t S, int32_t C,
                           const int32_t *state_sets, int32_t B, int32_t *cls_bits, void *stream);
int cfgzip_nfa_advance_states(const int32_t *rel_rep, int32_t C, int32_t S,
                              const int32_t *class_of_token, int32_t V, const int32_t *tok, int32_t B,
                              int32_t *state_sets, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CFGZIP_H */
