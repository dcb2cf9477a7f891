/*
 * aasd.h - C ABI of the MI355X (gfx950) hot path of Alignment-Augmented
 * Speculative Decoding: alignment sampling over prefill logits, n-gram draft
 * retrieval over the token buffer (stateless, or through a persistent draft
 * pool), conditional verification of draft candidates against the target
 * model's logits, and the draft-tree form of the same path (tree build with
 * its attention mask, verification over the tree's nodes).
 *
 * Conventions shared by every entry point
 *   - Pointers named in "DEVICE" lists are device (HBM) pointers owned by the
 *     caller; the library never allocates, frees or retains them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; outputs are valid once the caller has
 *     synchronised the stream.  There is no host synchronisation inside.
 *   - Return value: AASD_OK (0) or a negative aasd_status.  Every argument is
 *     checked before the first launch: with AASD_ERR_INVALID_ARG,
 *     AASD_ERR_UNSUPPORTED or AASD_ERR_WORKSPACE nothing has been enqueued.
 *     AASD_ERR_LAUNCH means that the HIP runtime refused a launch; kernels that
 *     the same call launched before it may already be enqueued, and the outputs
 *     are then undefined.  aasd_last_error() returns a thread-local message for
 *     the last failing call on the calling thread.  No exception crosses the ABI.
 *   - A call with zero rows / zero sequences succeeds and enqueues nothing.
 *   - Logits must be finite or -inf, with at least one finite value per row;
 *     NaN or +inf logits give unspecified numbers (never a fault).
 *   - All reductions have a fixed order and no floating-point atomics are
 *     used: the same inputs give byte-identical outputs on every run.
 *   - The library reads no environment variable and keeps no state between
 *     calls besides the last error message and, once aasd_verify_static has
 *     been called on a GPU, the address and the state of that GPU's scratch
 *     array.  (Measurement and test hooks, off by default, are declared apart
 *     in aasd_hooks.h.)
 */
#ifndef AASD_H
#define AASD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    AASD_OK = 0,
    AASD_ERR_INVALID_ARG = -1, /* null required pointer, size or parameter out of range */
    AASD_ERR_UNSUPPORTED = -2, /* valid request this build cannot serve (e.g. misaligned base pointer) */
    AASD_ERR_WORKSPACE = -3,   /* workspace missing or too small */
    AASD_ERR_LAUNCH = -4       /* the HIP runtime refused a launch */
} aasd_status;

typedef enum { AASD_F32 = 0, AASD_BF16 = 1 } aasd_dtype;

/* how the extra draft tokens of a misaligned position are chosen */
typedef enum {
    AASD_EXTRAS_TOP = 0,   /* best-ranked first (Fig. 2: the rank-1 and rank-2 tokens) */
    AASD_EXTRAS_SAMPLE = 1, /* seeded draws without replacement, proportional to probability, among them */
    AASD_EXTRAS_GUMBEL = 2  /* seeded draws without replacement from the whole row (Sec. 3.2 read literally) */
} aasd_extras_mode;

/* aasd_verify flags */
#define AASD_VERIFY_NO_CLAMP 1u /* threshold alpha*H+beta without the min with Delta (Eq. 3 when alpha = 0) */
#define AASD_VERIFY_ZEROED_WORKSPACE 2u /* the caller vouches for the workspace's counters: one launch instead of two (see aasd_verify) */

/* limits */
#define AASD_MAX_EXTRAS 4      /* m */
#define AASD_MAX_CANDSET 8     /* c */
#define AASD_MAX_KEY 8         /* n_max */
#define AASD_MAX_DRAFT 16      /* k */
#define AASD_MAX_CANDIDATES 32 /* C */
#define AASD_MAX_TREE_NODES 512 /* nodes of a draft tree, root included (16 candidates x 8 tokens x (1 + 2 extras) + 1 = 385) */

const char *aasd_version(void);
const char *aasd_last_error(void);

/*
 * Alignment sampling over the prefill logits (Sec. 2.3 for aligned/misaligned
 * positions; Sec. 3.2 and the caption of Fig. 2 for the extra tokens; Sec. 4.1
 * for the cap of two extras per position).
 *
 * For every row r of logits[rows, V] (row-major, consecutive rows `row_stride`
 * elements apart, temperature-1 softmax):
 *   argmax[r]     smallest token id that attains the row maximum (the greedy pick)
 *   entropy[r]    H = -sum_v p_v ln p_v in nats
 *   p_max[r]      max_v p_v
 *   and, when next_tok[r] is a token id (the prompt token that follows row r):
 *   rank[r]       number of tokens with a strictly larger logit than next_tok[r]
 *   misaligned[r] 1 iff rank[r] > 0, i.e. the prompt's next token is not a greedy pick
 *   p_next[r]     probability of next_tok[r]
 *   extras[r,:]   for misaligned rows, up to m of the tokens that are strictly more likely
 *                 than next_tok[r], taken from the c best tokens of the row (logit descending,
 *                 id ascending): in TOP mode the best min(m, .) of them in rank order; in
 *                 SAMPLE mode, if more than m qualify, m draws without replacement with
 *                 probability proportional to p.  Draw j of row r uses the first word of
 *                 Philox4x32-10(counter = (lo32(id), hi32(id), j, 0x41415344),
 *                 key = (lo32(seed), hi32(seed))), id = row_id_base + r, as u = (word >> 8) / 2^24
 *                 and picks the first remaining candidate whose running weight sum exceeds
 *                 u * (total remaining weight).  Unused slots hold -1.
 *                 In GUMBEL mode the extras of a misaligned row are min(m, V-1) draws without
 *                 replacement, with probability proportional to p, from ALL tokens of the row but
 *                 next_tok[r] (c is not used): the tokens with the largest keys z_v + G_v, key
 *                 descending, id ascending, where G_v = -ln(-ln(1 - x_v)) is a standard Gumbel
 *                 variate, x_v = ((word >> 9) + 1/2) / 2^23 and word is word (v mod 4) of
 *                 Philox4x32-10(counter = (lo32(id), hi32(id), v div 4, 0x47554D42), key as above).
 *                 Keys are formed in fp32 (error below 1e-5).
 *   n_extras[r]   number of valid entries in extras[r,:]
 *   Rows with next_tok[r] < 0 (or >= V) get misaligned = 0, p_next = 0, rank = -1, no extras.
 *
 * DEVICE in : logits (dtype dt; base pointer aligned to the element size), next_tok[rows]
 *             (NULL = no row has a next token)
 * DEVICE out: argmax[rows] i32, misaligned[rows] u8, entropy[rows] f32, p_next[rows] f32,
 *             p_max[rows] f32 (all required); rank[rows] i32 (NULL = not wanted);
 *             extras[rows, m] i32 and n_extras[rows] u8 (required when m > 0; with m = 0 an n_extras
 *             array, if given, is set to 0);
 *             near_count: one u32 that is INCREMENTED by the number of SAMPLE draws that fell
 *             within 1e-6 (relative to the total weight) of a boundary between two picks, in
 *             GUMBEL mode by the number of rows in which a pick's key is within 5e-5 of the next
 *             smaller key (NULL = not wanted; the caller zeroes it).
 * workspace : DEVICE scratch of at least aasd_align_sample_workspace_bytes(rows, V, dt) bytes,
 *             16-byte aligned; it needs no initialisation and holds nothing of value afterwards.
 * Parameters: 0 <= m <= 4, max(m,1) <= c <= 8, rows >= 0, V >= 1, row_stride >= V.
 */
size_t aasd_align_sample_workspace_bytes(int64_t rows, int32_t V, int32_t dt);
int aasd_align_sample(const void *logits, int32_t dt, int64_t rows, int32_t V, int64_t row_stride,
                      const int32_t *next_tok, int32_t m, int32_t c, int32_t mode, uint64_t seed,
                      uint64_t row_id_base, int32_t *argmax, uint8_t *misaligned, float *entropy,
                      float *p_next, float *p_max, int32_t *rank, int32_t *extras,
                      uint8_t *n_extras, uint32_t *near_count, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * n-gram draft retrieval (Sec. 3.1; Algorithm 1: draft-pool initialisation and the
 * longest-key-first lookup).  Stateless: instead of keeping the dictionary, each call
 * scans the token buffer and returns the positions the dictionary would hold.
 *
 * For every sequence b with context tokens[b, 0 .. len[b]):
 *   for n = n_max down to n_min, the hits of key length n are the positions p in
 *   [n, len-1] whose n preceding tokens equal the last n tokens of the context; the
 *   first n with at least one hit wins (key_len[b] = n, 0 if none).  The candidates are
 *   the hits in descending p (latest occurrence first), at most C of them (n_cand[b]).
 *   Candidate c copies draft_len[b,c] = min(k, len - p) tokens tokens[p ..] into
 *   drafts[b,c,:] (-1 padded), records p in src_pos[b,c] (-1 if absent), and marks
 *   strict[b,c,j] = 1 iff the j-th token was copied from generated context
 *   (p + j >= prompt_len[b]); such tokens are to be verified strictly (Sec. 3.3).
 *   With an alignment table (extras/n_extras from aasd_align_sample, row
 *   b*extras_stride + i = prefill row i of sequence b), draft_extras[b,c,j,:] holds
 *   the extra tokens of the prefill row that predicted position p + j (row p+j-1,
 *   only when p + j <= prompt_len - 1), else -1.
 *
 * DEVICE in : tokens[B, tok_stride] i32, len[B] i32 (0 <= len <= tok_stride; other
 *             values are treated as an empty context), prompt_len[B] i32,
 *             extras / n_extras (both NULL, or both given with 1 <= m <= 4)
 * DEVICE out: drafts[B,C,k] i32, draft_len[B,C] i32, src_pos[B,C] i32, n_cand[B] i32,
 *             key_len[B] i32, strict[B,C,k] u8 (all required);
 *             draft_extras[B,C,k,m] i32 (NULL = not wanted; needs the table)
 * Parameters: 1 <= n_min <= n_max <= 8, 1 <= k <= 16, 1 <= C <= 32, B >= 0, tok_stride >= 1.
 */
int aasd_retrieve_drafts(const int32_t *tokens, int64_t tok_stride, const int32_t *len,
                         const int32_t *prompt_len, int32_t B, int32_t n_min, int32_t n_max,
                         int32_t k, int32_t C, const int32_t *extras, const uint8_t *n_extras,
                         int32_t m, int64_t extras_stride, int32_t *drafts, int32_t *draft_len,
                         int32_t *src_pos, int32_t *n_cand, int32_t *key_len,
                         int32_t *draft_extras, uint8_t *strict, void *stream);

/* Bytes of device workspace aasd_verify needs for B sequences of C candidates of k tokens over
 * a vocabulary of V logits of type dt (0 on invalid arguments). */
size_t aasd_verify_workspace_bytes(int32_t B, int32_t C, int32_t k, int32_t V, int32_t dt);

/*
 * Conditional verification (Sec. 3.3, Eq. 4-6; the cascade rule of Sec. 2.1; "the longest
 * draft candidate that passes" of Sec. 3.3).
 *
 * logits[B, R, V] with R = 1 + C*k rows per sequence: row 0 is the distribution after the
 * last committed token, row 1 + c*k + (j-1) the distribution after the j-th (1-based)
 * draft token of candidate c.  Element (b, r, v) is at b*seq_stride + r*row_stride + v.
 * The j-th token t of candidate c is verified by row rho = 0 (j = 1) or 1 + c*k + (j-2):
 *   p     = softmax(row rho)[t]
 *   Delta = max_v softmax(row rho)[v]                                  (Eq. 6)
 *   delta = min(alpha * H(row rho) + beta, Delta), H in nats           (Eq. 5)
 *           (strict token: delta = Delta; AASD_VERIFY_NO_CLAMP: delta = alpha*H + beta)
 *   pass  = p >= delta, and a token whose logit equals the row maximum always
 *           passes (not under AASD_VERIFY_NO_CLAMP)                    (Eq. 4)
 * A token id outside [0, V) fails.  accept_len[b] is the largest number of leading passes
 * over the candidates (at most draft_len), best_cand[b] the lowest candidate index that
 * reaches it, next_token[b] the greedy pick of the row after the last accepted token
 * (row 0 if nothing was accepted).
 *
 * DEVICE in : logits, drafts[B,C,k] i32, draft_len[B,C] i32 (clamped to [0,k]),
 *             strict[B,C,k] u8 (NULL = no token is strict)
 * DEVICE out: accept_len[B], best_cand[B], next_token[B] i32 (required);
 *             row_entropy[B,R] f32, row_pmax[B,R] f32, row_argmax[B,R] i32 (each NULL = not wanted);
 *             tok_p[B,C,k], tok_delta[B,C,k] f32 (0 beyond draft_len; NULL = not wanted);
 *             near_count[B] u32 = number of evaluated tokens (up to and including each
 *             candidate's first failure) with |p - delta| < 1e-6 (NULL = not wanted)
 * workspace : DEVICE scratch of at least aasd_verify_workspace_bytes(B, C, k, V, dt) bytes, 128-byte
 *             aligned; it needs no initialisation and holds nothing of value afterwards.
 *             The call enqueues two kernels (row sweep, then decisions).  With
 *             AASD_VERIFY_ZEROED_WORKSPACE it may enqueue ONE instead (it does for a small call, up
 *             to 32 MiB of logits, the case of a decode step of a few sequences, where the launches
 *             are what the call costs the host; replayed from a graph the two kernels are as fast),
 *             in which the last workgroup to finish a
 *             sequence's rows also takes that sequence's decisions; this form counts finished
 *             workgroups in counters at the start of the workspace, which must be zero when the
 *             kernel starts and are zero again when it ends.  By setting the flag the caller vouches
 *             for that: the workspace was zero-filled once, and has since been used only by calls of
 *             aasd_verify with this flag and the same B, C, k, V, dt that ran to completion (calls
 *             that share a workspace must not overlap in either form).  The two forms add the same
 *             terms in a different order: their decisions agree (except within rounding of a
 *             threshold), row_argmax exactly, probabilities and entropies to fp32 rounding.
 * Parameters: 1 <= k <= 16, 1 <= C <= 32, V >= 1, row_stride >= V, seq_stride >= R*row_stride.
 */
int aasd_verify(const void *logits, int32_t dt, int32_t B, int32_t C, int32_t k, int32_t V,
                int64_t row_stride, int64_t seq_stride, const int32_t *drafts,
                const int32_t *draft_len, const uint8_t *strict, float alpha, float beta,
                uint32_t flags, int32_t *accept_len, int32_t *best_cand, int32_t *next_token,
                float *row_entropy, float *row_pmax, int32_t *row_argmax, float *tok_p,
                float *tok_delta, uint32_t *near_count, void *workspace, size_t workspace_bytes,
                void *stream);

/*
 * aasd_verify for callers that cannot allocate device memory or pass a workspace along: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It is aasd_verify
 * (same arguments, same kernels, same outputs) with the workspace replaced by scratch memory that is
 * built into the library: 4.25 MiB per GPU, held from the first call on a GPU until the process ends.
 * The call itself allocates nothing and frees nothing.
 *   - Limit: the partial results of the call must fit aasd_verify_static_max_bytes() = 4 MiB, i.e.
 *     aasd_verify_workspace_bytes(B, C, k, V, dt) minus its counters; this covers every decode step up to
 *     32768 rows (B * (1 + C*k)).  Larger calls return AASD_ERR_UNSUPPORTED and enqueue nothing: use
 *     aasd_verify with a workspace for them.
 *   - Small calls run as one launch (the form AASD_VERIFY_ZEROED_WORKSPACE selects in aasd_verify;
 *     the flag itself is not accepted here): the library keeps its own counters at zero.
 *   - Every call on one GPU uses that GPU's one scratch array: calls that overlap in time on the same GPU
 *     (two streams, two threads) race and give undefined outputs; calls ordered on one stream are safe.
 *   - The device must be the calling thread's current device when the call is made.
 */
size_t aasd_verify_static_max_bytes(void);
int aasd_verify_static(const void *logits, int32_t dt, int32_t B, int32_t C, int32_t k, int32_t V,
                       int64_t row_stride, int64_t seq_stride, const int32_t *drafts,
                       const int32_t *draft_len, const uint8_t *strict, float alpha, float beta,
                       uint32_t flags, int32_t *accept_len, int32_t *best_cand, int32_t *next_token,
                       float *row_entropy, float *row_pmax, int32_t *row_argmax, float *tok_p,
                       float *tok_delta, uint32_t *near_count, void *stream);

/*
 * Persistent draft pool (Sec. 3.1; Algorithm 1: the dictionary from n-grams to the positions after their
 * occurrences, initialised over the prompt and then extended by the windows that end in the new tokens).
 * aasd_pool_retrieve returns exactly what aasd_retrieve_drafts returns for the same arguments, but
 * follows hash chains kept in `pool` instead of scanning the context.
 *
 * `pool` is DEVICE memory owned by the caller, at least aasd_pool_bytes(B, capacity, n_min, n_max) bytes,
 * 16-byte aligned; the same B, capacity, n_min, n_max must be passed to every call on one pool.  It needs
 * no initialisation before the first aasd_pool_update with reset != 0.
 *
 * aasd_pool_update: with reset != 0, forget everything and index tokens[b, 0 .. len[b]) for every key length
 * in [n_min, n_max]; with reset == 0, index the positions added since the previous call (len[b] may only
 * grow between calls, and tokens that were indexed must not change).  len[b] beyond capacity is cut there.
 * aasd_pool_retrieve: the context tokens[b, 0 .. len[b]) must have been indexed at least up to len[b]; it may
 * be called with a smaller len[b] than was indexed (later positions are ignored).  All other arguments,
 * outputs and limits are those of aasd_retrieve_drafts.
 * aasd_pool_step: one decode step in one launch, aasd_pool_update(reset = 0) followed by aasd_pool_retrieve.
 * Calls on one pool must be ordered (same stream, or synchronised by the caller).
 * Parameters: 1 <= capacity <= 2^24 tokens per sequence, 1 <= n_min <= n_max <= 8, B >= 0.
 */
size_t aasd_pool_bytes(int32_t B, int32_t capacity, int32_t n_min, int32_t n_max);
int aasd_pool_update(void *pool, size_t pool_bytes, int32_t B, int32_t capacity, int32_t n_min,
                     int32_t n_max, const int32_t *tokens, int64_t tok_stride, const int32_t *len,
                     int32_t reset, void *stream);
int aasd_pool_retrieve(const void *pool, size_t pool_bytes, int32_t B, int32_t capacity, int32_t n_min,
                       int32_t n_max, const int32_t *tokens, int64_t tok_stride, const int32_t *len,
                       const int32_t *prompt_len, int32_t k, int32_t C, const int32_t *extras,
                       const uint8_t *n_extras, int32_t m, int64_t extras_stride, int32_t *drafts,
                       int32_t *draft_len, int32_t *src_pos, int32_t *n_cand, int32_t *key_len,
                       int32_t *draft_extras, uint8_t *strict, void *stream);
int aasd_pool_step(void *pool, size_t pool_bytes, int32_t B, int32_t capacity, int32_t n_min,
                   int32_t n_max, const int32_t *tokens, int64_t tok_stride, const int32_t *len,
                   const int32_t *prompt_len, int32_t k, int32_t C, const int32_t *extras,
                   const uint8_t *n_extras, int32_t m, int64_t extras_stride, int32_t *drafts,
                   int32_t *draft_len, int32_t *src_pos, int32_t *n_cand, int32_t *key_len,
                   int32_t *draft_extras, uint8_t *strict, void *stream);

/*
 * Top-k verification, the ablation of Sec. 4.4 (topk = 5 there): same rows, cascade, longest candidate
 * and next token as aasd_verify, but a draft token is accepted iff fewer than `topk` tokens of the row
 * that verifies it have a strictly larger logit (ties with the topk-th largest logit pass).  No
 * probabilities are formed: comparisons of logits only, so every output is exact.
 *
 * DEVICE in : logits[B, 1 + C*k, V] (layout as aasd_verify), drafts[B,C,k], draft_len[B,C]
 * DEVICE out: accept_len[B], best_cand[B], next_token[B] i32 (required); row_argmax[B, 1 + C*k] i32 and
 *             tok_pass[B,C,k] u8 (1 = within the top `topk`; 0 otherwise and beyond draft_len) (NULL = not wanted)
 * workspace : DEVICE scratch of at least aasd_verify_topk_workspace_bytes(B, C, k, V, dt) bytes, 16-byte
 *             aligned; needs no initialisation.
 * Parameters: 1 <= topk <= 8; the others as for aasd_verify.
 */
size_t aasd_verify_topk_workspace_bytes(int32_t B, int32_t C, int32_t k, int32_t V, int32_t dt);
int aasd_verify_topk(const void *logits, int32_t dt, int32_t B, int32_t C, int32_t k, int32_t V,
                     int64_t row_stride, int64_t seq_stride, const int32_t *drafts,
                     const int32_t *draft_len, int32_t topk, int32_t *accept_len, int32_t *best_cand,
                     int32_t *next_token, int32_t *row_argmax, uint8_t *tok_pass, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * Draft tree and tree attention mask (Sec. 3.2, Eq. 2): the retrieved candidates and the
 * alignment extras of their positions are merged into one tree under the last committed token,
 * so that one forward pass of the target model can verify all of them.
 *
 * For every sequence: node 0 is the root (the last committed token, root_tok[b]).  Layer j of the
 * tree is built from the j-th tokens of the candidates, in the order (candidate, slot) with slot 0
 * the retrieved token and slots 1..m its extras from draft_extras: a (parent, token) pair that
 * already exists is reused, otherwise it becomes the next node, so candidates that share a prefix
 * share nodes.  Extras are siblings of the retrieved token and have no continuation of their own.
 * Nodes are numbered in creation order (parents before children); nodes beyond max_nodes are dropped
 * together with what would hang below them.  A token id < 0 inside draft_len ends its candidate.
 * A node is strict iff every occurrence that maps to it is a retrieved token flagged strict.
 *
 * DEVICE in : drafts[B,C,k] i32, draft_len[B,C] i32, strict[B,C,k] u8 (NULL = none strict),
 *             draft_extras[B,C,k,m] i32 (NULL = no extras), root_tok[B] i32 (NULL = -1)
 * DEVICE out: node_token, node_parent, node_depth [B,max_nodes] i32 (unused slots -1, -1, 0; the
 *             root has parent -1), node_strict[B,max_nodes] u8, n_nodes[B] i32 (all required);
 *             mask[B, max_nodes, W] u32 with W = (max_nodes+31)/32: bit a of row i is set iff node a
 *             is node i or an ancestor of it (NULL = not wanted);
 *             cand_node[B,C,k] i32: the node of every candidate token, -1 if none (NULL = not wanted)
 * Parameters: 1 <= k <= 16, 1 <= C <= 32, 0 <= m <= 4, 1 <= max_nodes <= 512, B >= 0.
 */
int aasd_build_tree(const int32_t *drafts, const int32_t *draft_len, const uint8_t *strict,
                    const int32_t *draft_extras, int32_t m, const int32_t *root_tok, int32_t B,
                    int32_t C, int32_t k, int32_t max_nodes, int32_t *node_token,
                    int32_t *node_parent, int32_t *node_depth, uint8_t *node_strict,
                    int32_t *n_nodes, uint32_t *mask, int32_t *cand_node, void *stream);

/*
 * Conditional verification over a draft tree (Sec. 3.3, Eq. 4-6, applied to the nodes of Eq. 2).
 * logits[B, N, V]: row i is the distribution after node i (element (b, i, v) at
 * b*seq_stride + i*row_stride + v); rows at or beyond n_nodes[b] are not read.  Node i >= 1 with
 * token t is verified by the row of its parent exactly as in aasd_verify (p, Delta, delta, pass,
 * strict nodes, AASD_VERIFY_NO_CLAMP).  A node is accepted iff it and all its ancestors pass.
 * The deepest accepted node wins (lowest node index on ties): accept_len[b] is its depth,
 * best_node[b] its index, accept_path[b, 0..15] the nodes from depth 1 down to it (-1 padded),
 * next_token[b] the greedy pick of its row (of the root's row if nothing was accepted).
 * Parents must precede their children (node_parent[i] < i); a node that breaks this is rejected.
 *
 * DEVICE in : logits, node_token[B,N], node_parent[B,N] i32, node_strict[B,N] u8 (NULL = none),
 *             n_nodes[B] i32 (clamped to [1, N])
 * DEVICE out: accept_len[B], best_node[B], next_token[B] i32 (required); accept_path[B,16] i32;
 *             row_entropy, row_pmax [B,N] f32 and row_argmax[B,N] i32 (0, 0, -1 for unused rows);
 *             node_p, node_delta [B,N] f32; near_count[B] u32 = evaluated nodes (all ancestors
 *             accepted) with |p - delta| < 1e-6 (each NULL = not wanted)
 * workspace : DEVICE scratch of at least aasd_verify_tree_workspace_bytes(B, N, V, dt) bytes, 16-byte
 *             aligned; needs no initialisation.
 * Parameters: 1 <= N <= 512, V >= 1, row_stride >= V, seq_stride >= N*row_stride, B >= 0.
 */
size_t aasd_verify_tree_workspace_bytes(int32_t B, int32_t N, int32_t V, int32_t dt);
int aasd_verify_tree(const void *logits, int32_t dt, int32_t B, int32_t N, int32_t V,
                     int64_t row_stride, int64_t seq_stride, const int32_t *node_token,
                     const int32_t *node_parent, const uint8_t *node_strict,
                     const int32_t *n_nodes, float alpha, float beta, uint32_t flags,
                     int32_t *accept_len, int32_t *best_node, int32_t *accept_path,
                     int32_t *next_token, float *row_entropy, float *row_pmax,
                     int32_t *row_argmax, float *node_p, float *node_delta,
                     uint32_t *near_count, void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* AASD_H */
