/*
 * CPU oracle for the data-parallel hot path of Alignment-Augmented Speculative
 * Decoding (AASD).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * single-threaded transcription of the paper's definitions in fp64, written so
 * that it can be checked against the paper by eye.  It shares no code, header,
 * table or constant generator with the HIP library; only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.
 *
 * All pointers are HOST pointers owned by the caller.  Every function returns 0
 * on success and a negative value on an invalid argument.
 *
 * Paper passages followed (section / equation / algorithm):
 *   - aligned / misaligned tokens: Sec. 2.3 (the "A,B,C,D -> B,C,F,E" example)
 *   - alignment sampling:          Sec. 3.2, Fig. 2 caption, Sec. 4.1 (at most two extras)
 *   - draft pool and lookup:       Sec. 3.1, Algorithm 1 (pool init, longest key first)
 *   - conditional verification:    Sec. 3.3, Eq. 3-6; cascade rule Sec. 2.1;
 *                                  "longest candidate that passes" Sec. 3.3
 */
#ifndef AASD_ORACLE_H
#define AASD_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* logits element types (bit patterns are widened exactly to double) */
#define ORC_F32 0
#define ORC_BF16 1

/* extra-token selection modes for alignment sampling */
#define ORC_EXTRAS_TOP 0
#define ORC_EXTRAS_SAMPLE 1
#define ORC_EXTRAS_GUMBEL 2 /* m_x seeded draws without replacement from the WHOLE row (Gumbel-top-k) */

/* verification flags */
#define ORC_VERIFY_NO_CLAMP 1u /* Eq. 3 style: threshold alpha*H+beta, no min with Delta */

/* Philox4x32 with 10 rounds (Salmon et al., SC'11).  Integer only. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* Widen one row to double.  z must hold V doubles. */
int orc_widen_row(const void *row, int dtype, int32_t V, double *z);

/* Softmax of one row (temperature 1, Eq. 1's p_M).  p must hold V doubles. */
int orc_row_softmax(const void *row, int dtype, int32_t V, double *p);

/* Row statistics used by both alignment sampling and verification:
 *   m      = max_v z_v
 *   S      = sum_v exp(z_v - m)            (so max_v p_v = 1/S, Eq. 6's Delta)
 *   H      = -sum_{p_v>0} p_v ln p_v       (Eq. 5's entropy term, nats)
 *   argmax = smallest v with z_v == m      (greedy pick, Sec. 2.3)            */
int orc_row_stats(const void *row, int dtype, int32_t V, double *m, double *S, double *H,
                  int32_t *argmax);

/* Alignment sampling over prefill logits [rows, V] (Sec. 2.3, Sec. 3.2, Fig. 2).
 *   next_tok[r]  prompt token that follows row r, or -1 (NULL pointer = all -1)
 *   m_x          max extra tokens per position (Sec. 4.1 uses 2), 0..4
 *   c            candidate-set size (top-c by logit), m_x..8
 *   mode         ORC_EXTRAS_TOP | ORC_EXTRAS_SAMPLE | ORC_EXTRAS_GUMBEL
 * Outputs (any may be NULL):
 *   argmax[rows], misaligned[rows], entropy[rows], p_next[rows], p_max[rows],
 *   rank[rows]   (#tokens with a strictly larger logit than next_tok; -1 if none)
 *   extras[rows,m_x] (-1 padded), n_extras[rows]
 *   draw_margin[rows,m_x]  SAMPLE mode: for each seeded draw the distance
 *                min_i |u*W - cum_i| / W to the nearest CDF edge; -1 where no
 *                random number was consumed.  GUMBEL mode: the gap between the
 *                key z_v + G_v of the j-th pick and the next smaller key
 *                (+inf if there is none).                                    */
int orc_align_sample(const void *logits, int dtype, int64_t rows, int32_t V, int64_t row_stride,
                     const int32_t *next_tok, int32_t m_x, int32_t c, int mode, uint64_t seed,
                     uint64_t row_id_base, int32_t *argmax, uint8_t *misaligned, double *entropy,
                     double *p_next, double *p_max, int32_t *rank, int32_t *extras,
                     uint8_t *n_extras, double *draw_margin);

/* n-gram draft retrieval over the token buffer (Sec. 3.1, Algorithm 1).
 * Stateless brute force over the context instead of a dictionary: it returns the
 * positions the dictionary would hold for the longest key that occurs. */
int orc_retrieve_drafts(const int32_t *tokens, int64_t tok_stride, const int32_t *len,
                        const int32_t *prompt_len, int32_t B, int32_t n_min, int32_t n_max,
                        int32_t k, int32_t C, const int32_t *extras, const uint8_t *n_extras,
                        int32_t m_x, int64_t extras_stride, int32_t *drafts, int32_t *draft_len,
                        int32_t *src_pos, int32_t *n_cand, int32_t *key_len,
                        int32_t *draft_extras, uint8_t *strict);

/* Conditional verification (Sec. 3.3, Eq. 4-6) of C candidate drafts of up to k
 * tokens per sequence against logits[B, R, V], R = 1 + C*k.
 * Row 0 follows the last committed token; row 1 + c*k + (j-1) follows the j-th
 * (1-based) draft token of candidate c.
 * Outputs (any may be NULL): accept_len[B], best_cand[B], next_token[B],
 *   row_entropy/row_pmax/row_argmax [B,R], tok_p/tok_delta [B,C,k] (0 beyond
 *   draft_len), tok_margin[B,C,k] = |p - delta| for tokens that were evaluated
 *   (up to and including the first failure of each candidate) else -1,
 *   near_count[B] = number of evaluated tokens with margin < 1e-6.            */
int orc_verify(const void *logits, int dtype, int32_t B, int32_t C, int32_t k, int32_t V,
               int64_t row_stride, int64_t seq_stride, const int32_t *drafts,
               const int32_t *draft_len, const uint8_t *strict, double alpha, double beta,
               uint32_t flags, int32_t *accept_len, int32_t *best_cand, int32_t *next_token,
               double *row_entropy, double *row_pmax, int32_t *row_argmax, double *tok_p,
               double *tok_delta, double *tok_margin, uint32_t *near_count);

/* Top-k verification, the ablation of Sec. 4.4 (k = 5 there): a draft token is accepted iff fewer than
 * `topk` tokens of the row that verifies it have a strictly larger logit; rows, cascade, longest
 * candidate and next token as in orc_verify.  Outputs (any may be NULL): accept_len[B], best_cand[B],
 * next_token[B], row_argmax[B,R], tok_rank[B,C,k] (number of strictly larger logits; -1 beyond
 * draft_len or for a token id outside the vocabulary).                                          */
int orc_verify_topk(const void *logits, int dtype, int32_t B, int32_t C, int32_t k, int32_t V,
                    int64_t row_stride, int64_t seq_stride, const int32_t *drafts,
                    const int32_t *draft_len, int32_t topk, int32_t *accept_len,
                    int32_t *best_cand, int32_t *next_token, int32_t *row_argmax,
                    int32_t *tok_rank);

/* Draft tree (Sec. 3.2, Eq. 2): the candidate n-grams and the alignment extras of their positions
 * merged into one tree under the last committed token, plus the tree attention mask.
 *   Node 0 is the root.  Layer j (depth j) is built from the j-th tokens of the candidates in the
 *   order (candidate, slot), slot 0 = the retrieved token, slots 1..m_x = its extras; a (parent,
 *   token) pair that already exists is reused, otherwise it becomes the next node.  Extras are
 *   siblings of the retrieved token and have no continuation of their own.  Nodes beyond
 *   max_nodes (at most 512) are dropped (and with them whatever would hang below).  A node is strict iff every
 *   occurrence that maps to it is a strict retrieved token.
 * Outputs (any may be NULL): node_token/node_parent/node_depth [B,max_nodes] (-1 / -1 / 0 for
 *   unused slots; root: token root_tok[b] or -1, parent -1), node_strict [B,max_nodes],
 *   n_nodes[B], mask[B,max_nodes,W] with W = (max_nodes+31)/32: bit a of row i is set iff node a
 *   is node i or one of its ancestors; cand_node[B,C,k] = node of each candidate token (-1 if
 *   it has none).                                                                              */
int orc_build_tree(const int32_t *drafts, const int32_t *draft_len, const uint8_t *strict,
                   const int32_t *draft_extras, int32_t m_x, const int32_t *root_tok, int32_t B,
                   int32_t C, int32_t k, int32_t max_nodes, int32_t *node_token,
                   int32_t *node_parent, int32_t *node_depth, uint8_t *node_strict,
                   int32_t *n_nodes, uint32_t *mask, int32_t *cand_node);

/* Conditional verification over a draft tree: logits[B, N, V], row i = distribution after node i.
 * Node i >= 1 is verified by the row of its parent exactly as in orc_verify; a node is accepted iff
 * it and all its ancestors pass.  The deepest accepted node wins (lowest index on ties).
 * Outputs (any may be NULL): accept_len[B] (its depth), best_node[B], accept_path[B,16] (nodes from
 * depth 1 to the best node, -1 padded), next_token[B] (greedy pick of the best node's row),
 * row_entropy/row_pmax/row_argmax [B,N] (rows >= n_nodes: 0/0/-1), node_p/node_delta [B,N],
 * node_margin[B,N] = |p - delta| for evaluated nodes (parent accepted) else -1, near_count[B]. */
int orc_verify_tree(const void *logits, int dtype, int32_t B, int32_t N, int32_t V,
                    int64_t row_stride, int64_t seq_stride, const int32_t *node_token,
                    const int32_t *node_parent, const uint8_t *node_strict,
                    const int32_t *n_nodes, double alpha, double beta, uint32_t flags,
                    int32_t *accept_len, int32_t *best_node, int32_t *accept_path,
                    int32_t *next_token, double *row_entropy, double *row_pmax,
                    int32_t *row_argmax, double *node_p, double *node_delta, double *node_margin,
                    uint32_t *near_count);

#ifdef __cplusplus
}
#endif
#endif /* AASD_ORACLE_H */
