/*
 * fsa.h -- C ABI of the MI355X (gfx950) fused neighbor-sampling + mean-aggregation library.
 *
 * The operations are those of arXiv 2511.13645 ("FuseSampleAgg"):
 *   Sec. 3.2  for each seed v, draw up to k neighbors uniformly without replacement from its
 *             CSR row and emit  h_nei(v) = (1/t) sum_{u in U(v)} X[u],  t = min(k, |N(v)|),
 *             in one pass, with no sampled-subgraph ("block") tensor and no gathered-feature
 *             tensor; for fanouts (k1,k2) emit the nested mean
 *             X^_r = mean_{u in U1(r)} ( mean_{w in W(u)} X[w] ), skipping empty neighborhoods;
 *   Sec. 3.3  Prop. 1 (fixed IDs give the plain mean of the named rows), seed-controlled
 *             repeatable sampling, and saved-index replay so that backward reaches the same
 *             neighborhoods;
 *   Sec. 4    contiguous CSR (rowptr, col) and a contiguous row-major feature table.
 *
 * What the paper leaves open is fixed here, identically for every caller:
 *   - the sampler is Floyd's k-of-n selection driven by Philox4x32-10; Floyd step i of row
 *     `node` at hop h (0 = the seed's own row, 1 = a hop-1 node's row) uses word 0 of
 *     Philox(counter = (node, h, i, 0), key = (seed & 0xffffffff, seed >> 32)), mapped to
 *     [0, n) by (word * n) >> 32;  rows with deg <= k are taken whole in CSR order;
 *   - sampling is over edge slots, so a multigraph row may emit the same ID twice; each
 *     occurrence counts once in the sum and in the divisor;
 *   - emitted IDs are in Floyd step order, unused slots hold -1, and ids2[b,j,:] is all -1
 *     when ids1[b,j] is -1;
 *   - in the 2-hop mean a hop-1 node with an empty row leaves both the sum and the divisor;
 *     a seed with nothing to average gets a zero row (never NaN);
 *   - sums are accumulated in fp32 in a fixed order; outputs have the feature type (bf16 and
 *     fp16 outputs are rounded to nearest even from the fp32 result).
 * Because every draw is keyed by (seed, node, hop, step) the sampled IDs do not depend on
 * batch size, batch order, launch shape or how seeds are split over devices.
 *
 * Conventions for every entry point
 *   - All array arguments are DEVICE pointers on the current HIP device unless marked HOST.
 *     The caller owns every buffer; the library allocates nothing and keeps no state.
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*; NULL = default stream)
 *     and return without synchronising.  Outputs are valid once the stream has drained.
 *   - Return value: FSA_OK or a negative fsa_status.  Arguments are validated on the host
 *     before anything is launched: a validation error (every status but FSA_ERR_HIP) means
 *     nothing was launched and no output was written.  FSA_ERR_HIP means the HIP runtime
 *     refused a launch; an entry point that is a chain of launches (the layer-wise and
 *     three-hop calls) may then already have enqueued its earlier ones.  Every entry point
 *     discards an error that an earlier HIP call of the caller left pending before it
 *     launches, so FSA_ERR_HIP always refers to this call.  FSA_ERR_ARG is also returned when
 *     the fanouts need more LDS than the device offers.
 *     B == 0 returns FSA_OK without a launch (batch-sized arrays may then be NULL).
 *   - The library reads no environment variable and keeps no state between calls (one
 *     exception, stated there: fsa_mean3_bwd_noalloc remembers a device address).
 *   - grad_x (backward entry points) must be ordinary coarse-grained device memory
 *     (hipMalloc; not fine-grained, host-mapped or managed memory): the kernels add into it
 *     with hardware floating-point atomics resolved in the device's L2, which other kinds of
 *     memory do not honour.
 *   - Node IDs in `seeds`, `indices`, `ids1`, `ids2` must lie in [0, num_nodes) (or be
 *     negative padding in ids1/ids2); this is not checked on the device.  Rows must be
 *     shorter than 2^31 entries.
 */
#ifndef FSA_H
#define FSA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types: fp32, bfloat16, IEEE half.  The paper's kernels are FP32-only and name that
 * as a limitation (Sec. 5 "Limitations"); the 16-bit types are this library's extension. */
typedef enum { FSA_F32 = 0, FSA_BF16 = 1, FSA_F16 = 2 } fsa_dtype;
typedef enum { FSA_I32 = 0, FSA_I64 = 1 } fsa_itype;    /* indptr element type           */

typedef enum {
    FSA_OK = 0,
    FSA_ERR_NULL = -1,    /* a required pointer is NULL                                   */
    FSA_ERR_ARG = -2,     /* a size, fanout or hop count is out of range                  */
    FSA_ERR_DTYPE = -3,   /* unknown fsa_dtype / fsa_itype                                */
    FSA_ERR_ALIGN = -4,   /* a pointer is not aligned to its element size                 */
    FSA_ERR_HIP = -5,     /* the HIP runtime refused the launch                           */
    FSA_ERR_SCRATCH = -6  /* the call needs more scratch than the library's fixed array   */
} fsa_status;

enum { FSA_KMAX = 64 };   /* largest fanout per hop (one wavefront lane per Floyd step)   */

/*
 * Fused sample + mean, forward (Sec. 3.2; kernel mapping of Sec. 4 re-derived for 64-wide
 * wavefronts).
 *   indptr      [num_nodes+1]  int32 or int64 per indptr_type
 *   indices     [E]            int32 neighbor IDs
 *   x           [num_nodes,D]  row-major, contiguous, fsa_dtype x_dtype
 *   seeds       [B]            int32
 *   fanouts     HOST array of num_hops entries (k1[,k2]); num_hops in {1,2}; 1 <= k <= FSA_KMAX
 *   seed        sampler seed
 *   out         [B,D]      x_dtype   1-hop: h_nei(seed);  2-hop: nested mean         (required)
 *   out_h1      [B,k1,D]   x_dtype   2-hop: inner mean of every hop-1 slot, zero row for an
 *                                    empty slot; may be NULL; must be NULL for 1-hop
 *   out_ids1    [B,k1]     int32     sampled hop-1 IDs, -1 padded; may be NULL (no emit)
 *   out_ids2    [B,k1,k2]  int32     sampled hop-2 IDs, -1 padded; may be NULL; NULL for 1-hop
 * One kernel launch.  Deterministic and bit-reproducible for fixed arguments.
 */
int fsa_sample_mean_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                        int64_t num_nodes, const void* x, int x_dtype, int64_t D,
                        const int32_t* seeds, int64_t B, const int32_t* fanouts, int num_hops,
                        uint64_t seed, void* out, void* out_h1,
                        int32_t* out_ids1, int32_t* out_ids2, void* stream);

/*
 * Replay forward from saved IDs (Sec. 3.3, Prop. 1 and "Reproducibility").
 *   ids1 [B,k1], ids2 [B,k1,k2] int32; ids2 == NULL selects 1-hop (k2 ignored).
 * A negative entry is an empty slot and may appear anywhere.  In 2-hop, slot j takes part
 * only if ids1[b,j] >= 0 and ids2[b,j,:] holds at least one non-negative ID.
 * Given the arrays emitted by fsa_sample_mean_fwd and the same x, `out` and `out_h1` are
 * bitwise identical to that call's (same summation order).
 */
int fsa_mean_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                        const int32_t* ids1, const int32_t* ids2,
                        int64_t B, int32_t k1, int32_t k2,
                        void* out, void* out_h1, void* stream);

/*
 * Backward of the mean with respect to the feature table, replaying saved IDs (Sec. 3.3
 * "Reproducibility": gradients correspond to the same sampled neighborhoods).
 *   1-hop:  grad_x[ids1[b,i],:] += grad_out[b,:] / cnt_b
 *   2-hop:  grad_x[ids2[b,j,i],:] += (grad_out[b,:] / c1_b + grad_h1[b,j,:]) / c2_bj
 *           over slots j that take part (see replay), c1_b = number of such slots.
 *   grad_out [B,D] fp32;  grad_h1 [B,k1,D] fp32, may be NULL;  grad_x [num_nodes,D] fp32.
 * grad_x is ACCUMULATED INTO with fp32 atomics (the caller zeroes it or chains calls);
 * the order of additions, and therefore the last bits, vary from run to run.
 */
int fsa_mean_bwd(const float* grad_out, const float* grad_h1,
                 const int32_t* ids1, const int32_t* ids2,
                 int64_t B, int32_t k1, int32_t k2, int64_t D,
                 float* grad_x, int64_t num_nodes, void* stream);

/*
 * fsa_mean_bwd with a caller workspace (same arguments, same result within the same tolerance).
 * The atomic backward is bound by the L2 atomic unit (one 4-byte add per channel and clock), and
 * that cost grows with the row width.  Given a workspace, 2-hop calls with wide rows
 * (at least 1024 bytes, at most 8 x 64 chunks of 16 / 8 / 4 bytes -- the widest the row size and
 * the pointers' alignment allow -- and at least 32 MiB of row updates per call), and calls with
 * rows of 256 .. 1023 bytes and at least 393,216 leaf slots (B*k1*k2), take another route: the
 * leaf entries are binned by destination row, each bin is sorted in LDS, the gradients that reach
 * one row are summed in registers and the row is updated once with plain loads and stores by the
 * one workgroup that owns it (Sec. 3.3 only fixes WHICH rows receive gradient; how is ours).
 * Without overflow of a bin (rows sampled thousands of times in one batch) that route is
 * bit-reproducible.  Calls that are not eligible, a NULL workspace, one that is too small or not
 * 256-byte aligned: the call behaves exactly as fsa_mean_bwd.
 *   workspace        device memory, contents irrelevant on entry, overwritten
 *   workspace_bytes  its size; fsa_mean_bwd_workspace_bytes(B,k1,k2,D) returns what the call can
 *                    use (0: this shape always takes the atomic route)
 */
int64_t fsa_mean_bwd_workspace_bytes(int64_t B, int32_t k1, int32_t k2, int64_t D);
int fsa_mean_bwd_ws(const float* grad_out, const float* grad_h1,
                    const int32_t* ids1, const int32_t* ids2,
                    int64_t B, int32_t k1, int32_t k2, int64_t D,
                    float* grad_x, int64_t num_nodes,
                    void* workspace, int64_t workspace_bytes, void* stream);

/*
 * Reduced-precision backward (the paper lists FP32-only kernels as a limitation, Sec. 5
 * "Limitations"; this entry point lifts it).  Same operation as fsa_mean_bwd with
 *   grad_out / grad_h1 of type grad_dtype  (FSA_F32, FSA_BF16 or FSA_F16), and
 *   grad_x of type grad_x_dtype:
 *     FSA_F32             an fp32 master gradient: 16-bit upstream gradients are widened
 *                         exactly, all arithmetic and the atomics are fp32;
 *     FSA_BF16 / FSA_F16  grad_x in the 16-bit type; grad_dtype must be the same type or
 *                         FSA_F32.  Each contribution is formed in fp32, rounded once to the
 *                         16-bit type (nearest even) and added with packed two-element
 *                         hardware atomics, each of which rounds the running sum again: with
 *                         n additions into an element the error is bounded by about
 *                         (n + 1) * 2^-8 (bf16) or (n + 1) * 2^-10 (fp16) times the sum of
 *                         the absolute contributions, whatever way the atomic unit rounds
 *                         (plus (n + 1) subnormal spacings, 2^-24 for fp16, where values
 *                         fall below the smallest normal number).
 *                         fp16 sums can overflow to infinity.
 * With a 16-bit grad_x D must be even (FSA_ERR_ARG otherwise) and every array 4-byte aligned:
 * lanes read and add element pairs.  grad_dtype == grad_x_dtype == FSA_F32 is exactly
 * fsa_mean_bwd.  grad_x is accumulated into; the order of additions varies.
 */
int fsa_mean_bwd_lp(const void* grad_out, const void* grad_h1, int grad_dtype,
                    const int32_t* ids1, const int32_t* ids2,
                    int64_t B, int32_t k1, int32_t k2, int64_t D,
                    void* grad_x, int grad_x_dtype, int64_t num_nodes, void* stream);

/*
 * Layer-wise two-hop forward: fsa_sample_mean_fwd for fanouts (k1,k2) that ALSO emits the plain
 * hop-1 mean  out_m1[b] = mean of X over the sampled hop-1 nodes U1(seed)  -- what a layer-wise
 * GraphSAGE needs next to the nested mean, and the other way to read "the seed's mean" in a
 * two-hop call (Sec. 3.2 defines the nested mean only).  out_m1 [B,D] x_dtype, required; the
 * other arguments as in fsa_sample_mean_fwd with num_hops = 2.  Two launches on `stream`: the
 * fused two-hop kernel and the one-hop kernel, which draws the same U1 because hop-0 draws
 * depend only on (seed, node).  Replay: fsa_mean_replay_fwd(x, ids1) gives out_m1; backward:
 * fsa_mean_bwd with (grad_m1, ids1) next to the two-hop call.
 */
int fsa_sample_mean_layerwise_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                                  int64_t num_nodes, const void* x, int x_dtype, int64_t D,
                                  const int32_t* seeds, int64_t B, const int32_t* fanouts,
                                  uint64_t seed, void* out, void* out_h1, void* out_m1,
                                  int32_t* out_ids1, int32_t* out_ids2, void* stream);

/*
 * Three hops: the nested mean of Sec. 3.2 taken one level deeper (the paper names deeper hops
 * as an extension with more traffic and synchronisation, Sec. 3.2 "Extension Feasibility" and
 * Sec. 5; it gives no formula, so the same construction is applied once more):
 *   U = sample(seed, hop 0, k1);  V_j = sample(U[j], hop 1, k2);  W_ji = sample(V_j[i], hop 2, k3)
 *   out_h2[b,j,i] = mean of X over W_ji                                    (zero row if empty)
 *   out_h1[b,j]   = mean over the i with non-empty W_ji of out_h2[b,j,i];  out_cnt2[b,j] = their number
 *   out[b]        = mean over the j with out_cnt2[b,j] > 0 of out_h1[b,j]  (zero row if none)
 *   out_m1[b]     = mean of X over U
 * fanouts: HOST array of 3.  Required outputs: out [B,D], out_h1 [B,k1,D], out_m1 [B,D] (x_dtype),
 * out_ids1 [B,k1], out_cnt2 [B,k1] (int32).  Optional: out_h2 [B,k1,k2,D], out_ids2 [B,k1,k2],
 * out_ids3 [B,k1,k2,k3].  B*k1 must not exceed 2^31-1.
 * Built layer-wise from the kernels above, three launches on `stream`: the one-hop kernel on
 * the seeds; the fused two-hop kernel with the B*k1 hop-1 slots as roots and hop counters 1
 * and 2 (so no gathered leaf tensor exists: the only intermediate is out_h1 itself); a mean
 * over the slots of out_h1.  For 16-bit tables out is therefore formed from the ROUNDED out_h1
 * rows (two roundings instead of one).
 */
int fsa_sample_mean3_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                         int64_t num_nodes, const void* x, int x_dtype, int64_t D,
                         const int32_t* seeds, int64_t B, const int32_t* fanouts, uint64_t seed,
                         void* out, void* out_h1, void* out_h2, void* out_m1,
                         int32_t* out_ids1, int32_t* out_ids2, int32_t* out_ids3, int32_t* out_cnt2,
                         void* stream);

/*
 * Replay of the three-hop forward from saved IDs: the same three launches with the sampler
 * replaced by loads, bitwise equal to fsa_sample_mean3_fwd on the IDs it emitted.  Holes (-1)
 * may appear anywhere: (j,i) takes part iff ids1[b,j] >= 0, ids2[b,j,i] >= 0 and ids3[b,j,i,:]
 * has a non-negative entry.  out_m1 and out_h2 may be NULL.
 */
int fsa_mean3_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                         const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                         int64_t B, int32_t k1, int32_t k2, int32_t k3,
                         void* out, void* out_h1, void* out_h2, void* out_m1, int32_t* out_cnt2,
                         void* stream);

/*
 * Backward of the three-hop forward with respect to the feature table (fp32 throughout):
 *   grad_x[w,:] += ((grad_out[b,:]/c1_b + grad_h1[b,j,:]) / cnt2_bj + grad_h2[b,j,i,:]) / c3_bji
 *   for every valid leaf w of a (j,i) that took part, and
 *   grad_x[u,:] += grad_m1[b,:] / |U|  for every valid hop-1 node u.
 * grad_h1 [B,k1,D], grad_h2 [B,k1,k2,D], grad_m1 [B,D] may be NULL.  `work` is a caller-owned
 * scratch array of B*k1*D floats, overwritten (it carries the gradient of each hop-1 slot
 * between the two kernels).  grad_x is accumulated into with fp32 atomics.
 */
int fsa_mean3_bwd(const float* grad_out, const float* grad_h1, const float* grad_h2, const float* grad_m1,
                  const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                  int64_t B, int32_t k1, int32_t k2, int32_t k3, int64_t D,
                  float* grad_x, int64_t num_nodes, float* work, void* stream);

/*
 * fsa_mean3_bwd for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same
 * kernels and the same result as fsa_mean3_bwd; the scratch array (the gradient of each hop-1
 * slot, B*k1*D floats) lives in a fixed device array inside the library instead of `work`.
 *   - Limit: B*k1*D <= FSA_SCRATCH_FLOATS (32 MiB of floats), else FSA_ERR_SCRATCH and nothing
 *     is launched.  Every GPU the library runs on holds that array until the process ends.
 *   - The call allocates nothing and frees nothing.  Its first call on a device looks up the
 *     array's address on that device (with that device current) and keeps it for later calls.
 *   - All calls on one GPU share the array: calls that overlap on one GPU (different streams,
 *     or threads) race on it and must be serialised by the caller.  Every element a call reads
 *     is written by the same call first, so nothing needs clearing between calls.
 */
enum { FSA_SCRATCH_FLOATS = 8 * 1024 * 1024 };
int fsa_mean3_bwd_noalloc(const float* grad_out, const float* grad_h1, const float* grad_h2, const float* grad_m1,
                          const int32_t* ids1, const int32_t* ids2, const int32_t* ids3,
                          int64_t B, int32_t k1, int32_t k2, int32_t k3, int64_t D,
                          float* grad_x, int64_t num_nodes, void* stream);

/*
 * Weighted mean (Sec. 3.2, "Extension Feasibility": the same fusion with weighted numerators
 * and denominators streamed per sampled neighborhood).  edge_weight [E] fp32 is aligned with
 * `indices`; weights must be finite and non-negative.  Sampling is unchanged -- the same
 * draws and the same IDs as fsa_sample_mean_fwd for the same seed -- only the average is
 * weighted:
 *   1-hop  out[b] = sum_i w1[b,i] X[ids1[b,i]] / W_b,  W_b = sum_i w1[b,i];  W_b == 0 -> zero row
 *   2-hop  inner_j = sum_i w2[b,j,i] X[ids2[b,j,i]] / W2_bj;  slot j takes part iff
 *          ids1[b,j] >= 0 and W2_bj > 0;  out[b] = sum_j w1[b,j] inner_j / sum_j w1[b,j] over
 *          the slots that take part (zero row when that divisor is 0); out_h1[b,j,:] = inner_j
 *          (zero row for a slot that does not take part).
 * The sampling forward emits the weight of every sampled edge slot next to its ID
 * (out_w1 [B,k1], out_w2 [B,k1,k2], fp32, 0 in unused slots; each may be NULL); replay and
 * backward take the weights back together with the IDs.  Unit weights give the unweighted
 * means.  Everything else (layouts, stream, status codes, B == 0) is as for the unweighted
 * entry points; replay is bitwise equal to the sampling forward.
 *   backward 1-hop:  grad_x[ids1[b,i],:] += grad_out[b,:] * w1[b,i] / W_b
 *   backward 2-hop:  grad_x[ids2[b,j,i],:] += (grad_out[b,:] * w1[b,j] / A_b + grad_h1[b,j,:])
 *                                              * w2[b,j,i] / W2_bj,   A_b = sum of w1 over the
 *                    slots that take part (the first term is dropped when A_b == 0).
 */
int fsa_sample_wmean_fwd(const void* indptr, int indptr_type, const int32_t* indices,
                         const float* edge_weight, int64_t num_nodes,
                         const void* x, int x_dtype, int64_t D,
                         const int32_t* seeds, int64_t B, const int32_t* fanouts, int num_hops,
                         uint64_t seed, void* out, void* out_h1,
                         int32_t* out_ids1, int32_t* out_ids2, float* out_w1, float* out_w2,
                         void* stream);

int fsa_wmean_replay_fwd(const void* x, int x_dtype, int64_t D, int64_t num_nodes,
                         const int32_t* ids1, const int32_t* ids2,
                         const float* w1, const float* w2,
                         int64_t B, int32_t k1, int32_t k2,
                         void* out, void* out_h1, void* stream);

int fsa_wmean_bwd(const float* grad_out, const float* grad_h1,
                  const int32_t* ids1, const int32_t* ids2,
                  const float* w1, const float* w2,
                  int64_t B, int32_t k1, int32_t k2, int64_t D,
                  float* grad_x, int64_t num_nodes, void* stream);

/* Static, never-freed description of a status code. */
const char* fsa_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FSA_H */
