/*
 * CPU ORACLE for fused uniform neighbor sampling + GraphSAGE-mean aggregation.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, single-threaded
 * C++17 program written from the paper's definitions; it shares no code, header, table or
 * helper with the HIP path and must never be called from it.  Only the test-suite, the
 * smoke check and the benchmark's "cpu_baseline" leg may load it.
 *
 * What it follows (paper = arXiv 2511.13645, "FuseSampleAgg"):
 *   - Sec. 3.2, sampled-neighborhood mean  h_nei(v) = (1/t) sum_{u in U(v)} X[u],
 *     t = min(k, |N(v)|), U(v) a uniform sample without replacement from N(v);
 *   - Sec. 3.2, 2-hop nested mean  X^_r = mean over u in U1(r) of ( mean over w in W(u) of X[w] ),
 *     with empty neighborhoods skipped;
 *   - Sec. 3.3, Prop. 1 (for fixed sampled IDs the result is the plain mean over those rows),
 *     Lemma 1 (every neighbor is included with probability k/|N(v)|), and the paragraph on
 *     seed-controlled sampling and saved-index replay in backward.
 * The paper names neither a sampling algorithm nor a random-number generator.  This build
 * fixes them: Floyd's k-of-n selection driven by Philox4x32-10 (Salmon et al., SC'11), one
 * generator call per Floyd step, key = the 64-bit user seed, counter = (node, hop, step, 0),
 * output word 0 mapped to [0, n) by multiply-high.
 *
 * Parity pins (tests/, run without a GPU): Philox known-answer vectors; exhaustive
 * enumeration of Floyd's draws (every k-subset reached exactly k! times); chi-square and
 * inclusion-probability tests over many seeds; invariants on random graphs; closed forms
 * (k >= max degree reduces to a row-normalised sparse product computed by scipy);
 * finite differences and the adjoint identity for the backward pass.
 *
 * All pointers are HOST pointers.  Means and gradients are computed and returned in
 * double precision (fp64); the caller rounds if it wants another type.
 */
#ifndef FSA_ORACLE_H
#define FSA_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types, the oracle's own numbering */
enum { ORC_X_F32 = 0, ORC_X_BF16 = 1, ORC_X_F64 = 2 }; /* storage type of the feature table  */
enum { ORC_I32 = 0, ORC_I64 = 1 };                     /* storage type of indptr             */

/* Philox4x32 with 10 rounds (Salmon et al., SC'11, Sec. 3.3 / Table 2 constants). */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* One bounded draw for Floyd step `step` of row `node` at hop `hop`:
 * r = Philox(ctr=(node, hop, step, 0), key=(seed lo, seed hi))[0];  returns (r * n) >> 32,
 * a value in [0, n).  n must be >= 1. */
uint32_t orc_draw(uint64_t seed, uint32_t node, uint32_t hop, uint32_t step, uint32_t n);

/* Floyd's selection of k distinct positions out of deg, given the k draws t[i] in
 * [0, deg-k+i].  deg <= k: positions 0..deg-1 (t unused).  Writes pos[0..ret-1] in step
 * order and returns how many were written, min(k, deg). */
int32_t orc_floyd_select(int64_t deg, int32_t k, const uint32_t* t, int64_t* pos);

/* Sample row `node` of a CSR graph: positions (relative to the row start) and neighbor IDs
 * in slot order; slots >= ret get pos = -1, ids = -1.  Either output may be NULL. */
int32_t orc_sample_row(const void* indptr, int indptr_type, const int32_t* indices,
                       int64_t node, uint32_t hop, int32_t k, uint64_t seed,
                       int64_t* pos, int32_t* ids);

/* Sec. 3.2: fused sample + mean.  num_hops in {1,2}; fanouts[0]=k1, fanouts[1]=k2.
 * out     [B,D]      fp64  1-hop: h_nei(seed); 2-hop: the nested mean (zero row if empty)
 * out_h1  [B,k1,D]   fp64  2-hop only, nullable: inner mean of every hop-1 slot (zero if empty)
 * ids1    [B,k1]     nullable; ids2 [B,k1,k2] 2-hop only, nullable; -1 padded.
 * Returns 0, or a negative value on a bad argument. */
int orc_sample_mean_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                        int64_t num_nodes, const void* x, int x_dtype, int64_t D,
                        const int32_t* seeds, int64_t B, const int32_t* fanouts, int num_hops,
                        uint64_t seed, double* out, double* out_h1,
                        int32_t* ids1, int32_t* ids2);

/* Prop. 1: the same means from given IDs.  ids2 == NULL means 1-hop.  A negative entry is
 * an empty slot; in 2-hop, slot j takes part only if ids1[b,j] >= 0 and it has at least one
 * non-negative ids2[b,j,:]. */
int orc_mean_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                        const int32_t* ids1, const int32_t* ids2,
                        int64_t B, int32_t k1, int32_t k2,
                        double* out, double* out_h1);

/* Adjoint of the replay forward with respect to X, accumulated into grad_x [N,D] fp64.
 * grad_out [B,D] fp64; grad_h1 [B,k1,D] fp64, nullable, 2-hop only. */
int orc_mean_bwd(const double* grad_out, const double* grad_h1,
                 const int32_t* ids1, const int32_t* ids2,
                 int64_t B, int32_t k1, int32_t k2, int64_t D,
                 double* grad_x, int64_t num_nodes);

/* ---- weighted mean (Sec. 3.2, "Extension Feasibility": the same fusion with weighted
 * numerators and denominators streamed per sampled neighborhood) -------------------------
 * edge_weight [E] fp32, aligned with `indices`, non-negative and finite.  Sampling is
 * unchanged (uniform over edge slots); only the average is weighted:
 *   1-hop  out[b] = sum_i w1[b,i] X[ids1[b,i]] / W,  W = sum_i w1[b,i];  W == 0 -> zero row
 *   2-hop  inner_j = sum_i w2[b,j,i] X[ids2[b,j,i]] / W2_j;  slot j takes part iff
 *          ids1[b,j] >= 0 and W2_j > 0;  out[b] = sum_j w1[b,j] inner_j / sum_j w1[b,j]
 *          over the slots that take part (zero row if that divisor is 0).
 * The forward emits the weight of every sampled edge (w1 [B,k1], w2 [B,k1,k2], 0 in unused
 * slots); replay and backward take them back together with the IDs.  Parity pins: unit
 * weights reproduce the unweighted functions bit for bit; a fanout >= every degree reduces
 * to weighted-adjacency products computed by scipy; finite differences for the backward. */
int orc_sample_wmean_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                         const float* edge_weight, int64_t num_nodes,
                         const void* x, int x_dtype, int64_t D,
                         const int32_t* seeds, int64_t B, const int32_t* fanouts, int num_hops,
                         uint64_t seed, double* out, double* out_h1,
                         int32_t* ids1, int32_t* ids2, float* w1, float* w2);
int orc_wmean_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                         const int32_t* ids1, const int32_t* ids2, const float* w1, const float* w2,
                         int64_t B, int32_t k1, int32_t k2, double* out, double* out_h1);
int orc_wmean_bwd(const double* grad_out, const double* grad_h1,
                  const int32_t* ids1, const int32_t* ids2, const float* w1, const float* w2,
                  int64_t B, int32_t k1, int32_t k2, int64_t D, double* grad_x, int64_t num_nodes);

/* ---- three hops: the nested mean of Sec. 3.2 taken one level deeper (the paper discusses
 * deeper hops under "Extension Feasibility" and "Limitations" without a formula; this is the
 * same construction applied once more) ------------------------------------------------------
 *   U = sample(seed, hop 0, k1);  V_j = sample(U[j], hop 1, k2);  W_ji = sample(V_j[i], hop 2, k3)
 *   out_h2[b,j,i] = mean of X over W_ji                                  (zero row if empty)
 *   out_h1[b,j]   = mean over the i with a non-empty W_ji of out_h2[b,j,i];  cnt2[b,j] = their number
 *   out[b]        = mean over the j with cnt2[b,j] > 0 of out_h1[b,j]
 *   out_m1[b]     = mean of X over U                    (the plain hop-1 mean, layer-wise SAGE)
 * ids1 [B,k1], ids2 [B,k1,k2], ids3 [B,k1,k2,k3] are required (-1 padded, all -1 under an
 * unused slot); out_h1, out_h2, out_m1, cnt2 may be NULL.  Parity pins: a fanout >= every
 * degree reduces to products with the adjacency matrix computed by scipy (empty rows skipped
 * level by level); every ids3 row equals orc_sample_row at hop 2; the adjoint identity and
 * finite differences for the backward. */
int orc_sample_mean3_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                         int64_t num_nodes, const void* x, int x_dtype, int64_t D,
                         const int32_t* seeds, int64_t B, const int32_t* fanouts, uint64_t seed,
                         double* out, double* out_h1, double* out_h2, double* out_m1,
                         int32_t* ids1, int32_t* ids2, int32_t* ids3, int32_t* cnt2);
int orc_mean3_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                         const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                         int64_t B, int32_t k1, int32_t k2, int32_t k3,
                         double* out, double* out_h1, double* out_h2, double* out_m1,
                         int32_t* cnt2);
int orc_mean3_bwd(const double* grad_out, const double* grad_h1, const double* grad_h2,
                  const double* grad_m1,
                  const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                  int64_t B, int32_t k1, int32_t k2, int32_t k3, int64_t D,
                  double* grad_x, int64_t num_nodes);

/* Round fp64 values to bfloat16 bit patterns / fp32, round-to-nearest-even, directly from
 * the double (no intermediate float rounding). */
void orc_round_to_bf16(const double* src, int64_t n, uint16_t* dst);
void orc_round_to_f32(const double* src, int64_t n, float* dst);

#ifdef __cplusplus
}
#endif
#endif /* FSA_ORACLE_H */
