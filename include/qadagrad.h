/* qadagrad.h -- C ABI of libqadagrad: the data-parallel hot path of QCMD adagrad and QRDA
 * adagrad (arXiv 2208.05631, "Quantized Adaptive Subgradient Algorithms and Their
 * Applications") on one AMD MI355X (gfx950).
 *
 * One training step of Algorithm 1, with the M workers and the parameter server living as
 * slices of one GPU's memory:
 *
 *   worker m : g_m  = minibatch gradient of the logistic loss            qa_local_grad
 *              (codes_m, s_m) = threshold quantizer + 2-bit encoding      qa_quantize_pack
 *   server   : SynQ = (1/M) sum_m s_m * codes_m                           qa_aggregate_unpack
 *              q = SynQ, or q = Q(SynQ) (second quantization)             } fused into
 *   workers  : G += q^2, H = delta + sqrt(G), QCMD or QRDA update of x    } qa_step_qcmd / qa_step_qrda
 *
 * The same roles as separate calls, for a deployment in which server and workers are different
 * processes: qa_aggregate_quantize (server: messages in, q_t out as a message) and a step with
 * M = 1 on that message (worker).  With the indicator of Section 3.2 only the selected components
 * travel: qa_indicator, qa_quantize_pack_selected (worker), qa_indicator_or,
 * qa_aggregate_quantize_selected, qa_select_codes (server), qa_step_*_selected (worker).
 *
 * Conventions common to every call
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates, frees or keeps device memory, and keeps no state between calls
 *     (x, G, z and the step counter t live with the caller).
 *   - Calls are asynchronous: kernels are enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the call returns without synchronising.
 *   - The qa_layout struct and every scalar are HOST values.
 *   - Return value: QA_OK (0) or a negative QA_ERR_* code; nothing is launched when an
 *     argument check fails.  The library never aborts and never throws.
 *   - Buffers that are read or written with 128-bit accesses (g, x, G, z, gbar) must be
 *     16-byte aligned; codes, scales, thresholds 4-byte aligned; workspace 256-byte aligned.
 *
 * Arithmetic (identical to what the CPU checker under oracle/ states)
 *   - state, gradients, scales and thresholds are binary32; each element-wise formula is
 *     evaluated one correctly rounded binary32 operation at a time in the order given in
 *     the comments below, without fused multiply-add;
 *   - every sum over many terms (over a bucket, over the workers, over a row or a
 *     minibatch) is accumulated in binary64 and rounded once to binary32.
 */
#ifndef QADAGRAD_H
#define QADAGRAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QA_VERSION 100 /* 0.1.0 */

/* error codes */
#define QA_OK 0
#define QA_ERR_INVALID_ARG (-1) /* NULL required pointer, size/stride/scalar out of range   */
#define QA_ERR_ALIGNMENT (-2)   /* a buffer does not have the alignment stated above         */
#define QA_ERR_WORKSPACE (-3)   /* workspace NULL or smaller than qa_workspace_bytes says    */
#define QA_ERR_LAUNCH (-4)      /* the HIP runtime refused a launch (hipGetLastError != 0)   */
#define QA_ERR_UNSUPPORTED (-5) /* valid request this build does not implement               */
#define QA_ERR_TOO_LARGE (-6)   /* qa_quantize_pack_static: needs more than the static scratch */

/* second-quantization mode of the fused steps ("q_t = Q(SynQ_t)", Section 3.2, equation Qt;
 * the methods marked with a dagger in Section 5.1 skip it) */
#define QA_REQUANT_NONE 0   /* q = SynQ                                                      */
#define QA_REQUANT_BUCKET 1 /* q = Q(SynQ) with one threshold/scale per bucket of the layout */
#define QA_REQUANT_GLOBAL 2 /* q = Q(SynQ) with one threshold/scale for the whole vector     */

/* flags of qa_quantize_pack */
#define QA_THRESH_GIVEN 1u /* thresholds[] is an INPUT; only scales and codes are computed   */
#define QA_THRESH_EXACT 2u /* thresholds[] is an OUTPUT holding the exact least-squares optimum
                              found by ranking (Section 3.4) instead of the 0.75*mean|v| rule;
                              needs 64 <= bucket <= 4096 or (bucket == 0 and d <= 4096), and
                              a non-NULL thresholds array                                    */

/* operations for qa_workspace_bytes */
#define QA_OP_QUANTIZE 1
#define QA_OP_STEP 2
#define QA_OP_GRAD_CSR 3
#define QA_OP_GRAD_DENSE 4
#define QA_OP_SELECT 5        /* qa_quantize_pack_selected, qa_decode_selected, qa_select_codes   */
#define QA_OP_STEP_SELECTED 6 /* qa_step_*_selected, qa_aggregate_quantize_selected               */
#define QA_OP_QUANTIZE_EXACT 7 /* qa_quantize_pack with QA_THRESH_EXACT (any bucket size)          */

/* data formats of qa_local_grad */
#define QA_DENSE 0
#define QA_CSR 1

/* Shape of one step's messages (all HOST values).
 *
 * Encoding ("Encode" paragraph of Section 3.5: two bits per component plus one float):
 *   component i of worker m sits in bits [2*(i%16), 2*(i%16)+1] of the 32-bit word
 *   codes[m*code_stride + i/16];  00 = 0, 01 = +1, 11 = -1 (two's complement), 10 is never
 *   written and is read as 0; unused bits of the last word are 0.
 *   Its scale is scales[m*scale_stride + i/bucket] (bucket == 0: scales[m*scale_stride]).
 */
typedef struct {
  int64_t d;            /* number of coordinates, 1 <= d < 2^40                               */
  int32_t M;            /* number of workers, 1 <= M <= 4096                                  */
  int32_t bucket;       /* elements per threshold/scale: a power of two >= 64, or 0 = one per
                           vector (the paper's single float per message)                      */
  float thr_coef;       /* threshold = thr_coef * mean|v| ; 0.75 in Section 3.5               */
  int64_t code_stride;  /* 32-bit words between consecutive workers, >= ceil(d/16).  For large
                           d: a multiple of 256 (rows start on 1 KiB boundaries) such that
                           consecutive rows lie a few KiB apart modulo 16 KiB, e.g. 768 words
                           more than a multiple of 4096: with rows a power of two apart the M
                           code streams of a tile meet in the same memory channels (measured
                           at d = 2^30, M = 64: steps 0.5-3 %, aggregate-only calls 2-6 %
                           slower; 16 KiB modulo 32 KiB apart: 4 % slower still); rows off a
                           256-byte boundary cost about 4 %                                   */
  int64_t scale_stride; /* floats between consecutive workers in scales/thresholds, >= number
                           of buckets = ceil(d/bucket) (1 if bucket == 0)                     */
} qa_layout;

int qa_version(void);
const char* qa_strerror(int code);

/* Bytes of device workspace that `op` needs for this layout (0 if none).  For
 * QA_OP_GRAD_CSR / QA_OP_GRAD_DENSE only layout->d and layout->M are used (the size for
 * qa_local_grad_batched over M workers; qa_local_grad needs 1/M of it).  Returns 0 for a NULL or
 * invalid layout. */
size_t qa_workspace_bytes(const qa_layout* layout, int op);

/* Minibatch gradient of one worker for the logistic loss log(1 + exp(-y a.x)), y in {-1,+1}
 * (stochastic gradient of Section 3.1 for the L1-regularised logistic regression of
 * Section 5.1; the regulariser is handled by the update, not here):
 *     p_b    = a_{r_b} . x                        (sum in binary64, rounded to binary32)
 *     coef_b = -y_{r_b} / (1 + exp(y_{r_b} p_b)) / B     (binary64, rounded to binary32)
 *     g_j    = sum_b coef_b * a_{r_b, j}          (sum in binary64, rounded to binary32)
 *     loss   = (1/B) sum_b log(1 + exp(-y_{r_b} p_b))
 * format QA_DENSE: A_or_vals = A[n_rows][d] row-major, indptr = indices = NULL.
 * format QA_CSR  : A_or_vals = vals[nnz], indptr[n_rows+1] (int64), indices[nnz] (int32,
 *                  0 <= index < d; duplicate indices in a row add up).
 * batch_rows[B] holds row ids in [0, n_rows) and may repeat.  g_out[d] is fully overwritten
 * (zero where no batch row has an entry).  loss_out (one float, device) may be NULL.
 * ws: qa_workspace_bytes(layout with d, QA_OP_GRAD_CSR or QA_OP_GRAD_DENSE) bytes; its
 * contents on entry do not matter. */
int qa_local_grad(int format, const float* A_or_vals, const int64_t* indptr, const int32_t* indices,
                  int64_t n_rows, int64_t d, const float* y, const int32_t* batch_rows, int32_t B,
                  const float* x, float* g_out, float* loss_out, void* ws, size_t ws_bytes,
                  void* stream);

/* The same for M workers in one call ("for M worker ... do in parallel", Algorithm 1): worker m
 * uses batch_rows[m*B .. m*B+B), writes g_out[m*g_stride .. + d) and loss_out[m] (loss_out may
 * be NULL).  g_stride >= d and a multiple of 4.  All workers read the same x.
 * ws: qa_workspace_bytes(layout with d and M, QA_OP_GRAD_CSR or QA_OP_GRAD_DENSE). */
int qa_local_grad_batched(int format, const float* A_or_vals, const int64_t* indptr,
                          const int32_t* indices, int64_t n_rows, int64_t d, const float* y,
                          const int32_t* batch_rows, int32_t B, int32_t M, const float* x,
                          float* g_out, int64_t g_stride, float* loss_out, void* ws, size_t ws_bytes,
                          void* stream);

/* Threshold quantizer of Sections 3.4-3.5 and 2-bit encoding for M gradients
 * g[m*g_stride + i], m < M, i < d, bucket by bucket (bucket k = [k*b, min((k+1)*b, d)),
 * n = its true length):
 *     Delta = thr_coef * (sum |v_i|) / n                        (Section 3.5)
 *     code_i = +1 if v_i > Delta, -1 if v_i < -Delta, else 0     (definition of Q_Delta)
 *     s = (sum_{|v_i| > Delta} |v_i|) / #{|v_i| > Delta}, or 0 if that set is empty (s*_Delta)
 * Writes codes[m*code_stride + w] for every w < ceil(d/16), scales[m*scale_stride + k] and,
 * if thresholds != NULL and QA_THRESH_GIVEN is not set, thresholds[m*scale_stride + k].
 * With QA_THRESH_GIVEN thresholds must be non-NULL and is read instead of computed.
 * With QA_THRESH_EXACT each bucket's threshold is the largest magnitude NOT kept by the k that
 * maximises (sum of the k largest |v|)^2 / k (equal magnitudes are never split), so that the
 * strict comparisons keep exactly the optimal set; scale and codes follow as usual.  Buckets of
 * up to 4096 components are ranked inside one work-group; longer buckets, and one threshold for
 * a vector of more than 4096 components (Section 3.4's optimum over the whole gradient), are
 * ranked by a device-wide sort, worker after worker, in 17 bytes of workspace per component
 * (d < 2^32, else QA_ERR_TOO_LARGE); that form calls a library sort, which may enqueue memset
 * operations: do not record it into a HIP graph.  Candidates whose objectives agree to binary64 rounding
 * (likely only beyond some 1e7 components per bucket) may be resolved differently from a
 * strictly sequential summation.
 * g_stride >= d and a multiple of 4.  ws: qa_workspace_bytes(layout, QA_OP_QUANTIZE), or
 * qa_workspace_bytes(layout, QA_OP_QUANTIZE_EXACT) with QA_THRESH_EXACT (the two agree for
 * buckets of up to 4096 components). */
int qa_quantize_pack(const qa_layout* layout, const float* g, int64_t g_stride, uint32_t* codes,
                     float* scales, float* thresholds, uint32_t flags, void* ws, size_t ws_bytes,
                     void* stream);

/* qa_quantize_pack for callers that cannot allocate or pass device scratch: code recorded into a
 * HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and
 * results as qa_quantize_pack, bit for bit, without the workspace: the per-tile partial sums,
 * counts and thresholds that the multi-pass layouts need (one scale per vector, or buckets above
 * 4096) live in a 4 MiB array in the library's own device image instead.  The call allocates
 * nothing and frees nothing.
 *   - Limit: qa_workspace_bytes(layout, QA_OP_QUANTIZE) <= 4 MiB (QA_STATIC_SCRATCH_BYTES), about
 *     12 bytes per worker and 4096 coordinates: e.g. M * ceil(d/4096) <= 349 000.  Larger
 *     problems return QA_ERR_TOO_LARGE and launch nothing.  Layouts that need no workspace
 *     (bucket <= 4096, or a vector of at most 4096 coordinates) have no limit.  QA_THRESH_EXACT
 *     for buckets longer than 4096 components needs a sort's worth of scratch and is refused
 *     with QA_ERR_TOO_LARGE as well.
 *   - Each GPU holds one such array for the life of the process.  The first call on a device
 *     looks its address up (the device of the calling thread must be the one `stream` belongs
 *     to); make that first call outside stream capture.
 *   - All calls on one GPU share the array: two calls whose kernels may overlap (different
 *     streams, or several host threads) race on it.  Calls on one stream are ordered and safe.
 *     Nothing in the array needs clearing between calls. */
#define QA_STATIC_SCRATCH_BYTES (4u << 20)
int qa_quantize_pack_static(const qa_layout* layout, const float* g, int64_t g_stride,
                            uint32_t* codes, float* scales, float* thresholds, uint32_t flags,
                            void* stream);

/* Stochastic ternary quantizer, the "ternary" comparison of Section 5.1 (TernGrad, cited in
 * Section 2; the paper does not restate it): per bucket s = max|v_i|, component i is kept with
 * probability |v_i|/s and coded as its sign, so that E[s*code_i] = v_i.  Same outputs and
 * encoding as qa_quantize_pack (codes, scales; no thresholds).  The uniform numbers are
 * Philox4x32-10 (Salmon et al., SC'11) with key = seed, counter = (i/4 low, i/4 high, worker
 * m, step), component i taking output word i%4, u = (r >> 8) * 2^-24, kept iff u < |v_i|/s in
 * binary32: the result is a pure function of (g, seed, step).  Any bucket of the layout; no
 * workspace. */
int qa_quantize_pack_stochastic(const qa_layout* layout, const float* g, int64_t g_stride,
                                uint32_t* codes, float* scales, uint64_t seed, uint32_t step,
                                void* stream);

/* Server average (equation SynQ_t of Section 3.1; "Average the quantized gradients" in
 * Algorithm 1), materialised:  gbar_out[i] = (1/M) sum_m scales[m][i/bucket] * code[m][i],
 * sum and division in binary64, rounded once. */
int qa_aggregate_unpack(const qa_layout* layout, const uint32_t* codes, const float* scales,
                        float* gbar_out, void* stream);

/* One fused QCMD adagrad step (equations SynQ_t, Qt, Hq and QCMD; Algorithm 1 server and
 * final worker block).  Per coordinate, with q from the average as selected by `requant`:
 *     G = G + q*q ;  H = delta + sqrt(G)
 *     u = x - (eta*q)/H ;  tau = (lambda*eta)/H ;  r = |u| - tau
 *     x = r > 0 ? copysign(r, u) : +0
 *     if z_or_null: z = z + q            (keeps the running sum for a later QRDA step)
 * x, G (and z) are read and written in place.  eta > 0, lambda >= 0, delta > 0.
 * ws: qa_workspace_bytes(layout, QA_OP_STEP); only used when the second quantization cannot
 * be done in one pass (QA_REQUANT_GLOBAL, or QA_REQUANT_BUCKET with bucket > 4096); may be
 * NULL with ws_bytes 0 otherwise.  In that case the call enqueues several kernels (the two sums
 * behind the threshold and the scale of q, each followed by a small finalize kernel, then the
 * update); otherwise exactly one.  Nothing is copied or waited for: the call can be recorded
 * into a HIP graph. */
int qa_step_qcmd(const qa_layout* layout, const uint32_t* codes, const float* scales, float* x,
                 float* G, float* z_or_null, float eta, float lambda, float delta, int requant,
                 void* ws, size_t ws_bytes, void* stream);

/* The server's part of Algorithm 1 as one call: SynQ_t = (1/M) sum_m Q(g^(m)) followed by
 * q_t = Q(SynQ_t) (equations SynQ_t and Qt), returned as a one-worker message in the dense 2-bit
 * encoding: q_codes[w], w < ceil(d/16), and q_scales[k] (q_thresholds[k] if not NULL), with
 * k < ceil(d/bucket) buckets for QA_REQUANT_BUCKET and k = 0 for QA_REQUANT_GLOBAL (one threshold
 * and scale for the whole vector).  The result equals qa_aggregate_unpack followed by
 * qa_quantize_pack of that vector with M = 1 and the corresponding bucket; buckets of at most 4096
 * components (and vectors of at most 4096 with one scale) are done in a single pass that never
 * writes the average.  requant must be QA_REQUANT_BUCKET or QA_REQUANT_GLOBAL.
 * ws: qa_workspace_bytes(layout, QA_OP_STEP) (may be NULL when the single pass applies).
 * Stepping from the message (layout with M = 1, that bucket) gives the same state as the fused
 * step with the same requant. */
int qa_aggregate_quantize(const qa_layout* layout, const uint32_t* codes, const float* scales,
                          int requant, uint32_t* q_codes, float* q_scales, float* q_thresholds,
                          void* ws, size_t ws_bytes, void* stream);

/* One fused QRDA adagrad step (equations SynQ_t, Qt, Hq and QRDA).  Per coordinate:
 *     G = G + q*q ;  H = delta + sqrt(G) ;  z = z + q
 *     r = |z| - (float)t*lambda
 *     x = r > 0 ? -copysign((eta*r)/H, z) : +0
 * which is the printed sign(-z) (t eta / H) [ |z/t| - lambda ]_+ multiplied through by t.
 * t >= 1 is the 1-based index of this step (z holds t gradients after the call).
 * x is write-only; G and z are updated in place. */
int qa_step_qrda(const qa_layout* layout, const uint32_t* codes, const float* scales, float* x,
                 float* G, float* z, int64_t t, float eta, float lambda, float delta, int requant,
                 void* ws, size_t ws_bytes, void* stream);

/* ---- indicator, selection and sparse encoding (Section 3.2, equations "select" and "ind";
 * Algorithm 1: worker block and the server's decode; Encode paragraph: 32 + d + 2k bits) ----
 *
 * A worker sends only the components of its gradient whose parameter is, or would become,
 * non-zero, plus one bit per coordinate saying which ones.  The indicator of worker m is
 * ind[m*ind_stride + i/32], bit i%32; unused bits of the last word are 0.
 *
 * Sparse message of worker m, for every bucket size the layout allows: bucket k (coordinates
 * [k*b, min((k+1)*b, d)), b = bucket, or the whole vector for bucket == 0) owns the area of
 * ceil(b/16) words that starts at sel_codes[m*code_stride + k*ceil(b/16)]; the codes of its
 * marked components, in index order, are packed from bit 0 of that area; counts[m*scale_stride + k]
 * says how many there are, scales[m*scale_stride + k] is their scale.  Only the first
 * ceil(count/16) words of an area are meaningful (and written).  With bucket == 0 this is the
 * paper's message: one float, d indicator bits and 2k code bits in one stream.
 *
 * Buckets of 4096 (and a vector of at most 4096 coordinates with one scale) are served by
 * kernels that work tile by tile and need no workspace; the steps read such messages directly.
 * Buckets of 64 .. 2048 need none either.  Buckets above 4096 and one scale for a longer vector
 * span several tiles: every call first counts the marked components of each tile and scans the
 * counts (qa_workspace_bytes(layout, QA_OP_SELECT) bytes of workspace), and a bucket may hold
 * fewer than 2^32 coordinates (QA_ERR_UNSUPPORTED otherwise).  For all sizes other than 4096 the
 * steps on sparse messages decode into the workspace first and then take the dense path
 * (qa_workspace_bytes(layout, QA_OP_STEP_SELECTED) bytes).
 */
#define QA_METHOD_QCMD 0
#define QA_METHOD_QRDA 1

/* Indicators of all M workers.  Worker m forms, from its own full-precision gradient
 * g[m*g_stride + i], the parameter it would get:  H^ = delta + sqrt(G_i + g*g), then the QCMD
 * (method 0) or QRDA (method 1, with z_i + g and step index t) closed form with g in place of
 * q, evaluated exactly like qa_step_qcmd / qa_step_qrda; bit i = (x_i != 0 or x^_i != 0).
 * x, G, z are only read.  z may be NULL for QCMD.  ind_stride >= ceil(d/32). */
int qa_indicator(const qa_layout* layout, int method, const float* g, int64_t g_stride,
                 const float* x, const float* G, const float* z, int64_t t, float eta, float lambda,
                 float delta, uint32_t* ind_out, int64_t ind_stride, void* stream);

/* Synchronous indicator: ind_syn_out[w] = OR over the M workers of ind[m*ind_stride + w]. */
int qa_indicator_or(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                    uint32_t* ind_syn_out, void* stream);

/* Q(S(g, I)) for M workers: in every bucket k the marked components, in index order, form a
 * vector of length counts[m*scale_stride + k]; threshold (with that length as n), scale and
 * ternary codes as in qa_quantize_pack; its codes are packed from bit 0 of the bucket's area.
 * Only the first ceil(count/16) words of an area are written (unused bits of the last one
 * are 0), the rest is left untouched: the message
 * of a bucket is 32 + b + 2*count bits.  count == 0 gives scale 0, threshold 0, no codes.
 * thresholds may be NULL.  ws: qa_workspace_bytes(layout, QA_OP_SELECT) (0 bytes, ws may be NULL,
 * unless buckets span several tiles). */
int qa_quantize_pack_selected(const qa_layout* layout, const float* g, int64_t g_stride,
                              const uint32_t* ind, int64_t ind_stride, uint32_t* sel_codes,
                              uint32_t* counts, float* scales, float* thresholds, void* ws,
                              size_t ws_bytes, void* stream);

/* S^{-1} (Algorithm 1, server: "Decode ... to get Q(g^(m))"): writes the dense 2-bit codes of
 * qa_layout for all M workers, codes_out[m*code_stride + w], w < ceil(d/16): the j-th marked
 * component of a bucket gets the j-th code of its area, unmarked components get 0.  With the
 * scales from qa_quantize_pack_selected the result feeds qa_aggregate_unpack / qa_step_*.
 * ind_stride = 0 applies one indicator to all M messages.  ws as for qa_quantize_pack_selected. */
int qa_decode_selected(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                       const uint32_t* sel_codes, uint32_t* codes_out, void* ws, size_t ws_bytes,
                       void* stream);

/* S applied to coded messages (Algorithm 1, server: "Push S(q_t, I^Syn) and I^Syn to every
 * worker"): for each of the M messages codes[m*code_stride + w] (dense 2-bit layout, e.g. the
 * one-worker message that qa_aggregate_unpack followed by qa_quantize_pack produces for q_t), the
 * codes of the marked components, in index order, are packed per bucket exactly like the output of
 * qa_quantize_pack_selected: from bit 0 of the bucket's area, only the first ceil(count/16) words
 * of an area are written; counts[m*scale_stride + k] = marked components of bucket k.
 * ind_stride = 0 applies the same indicator (the synchronous one) to every message.
 * qa_decode_selected is the inverse on the marked components.  Not in place.  ws as for
 * qa_quantize_pack_selected. */
int qa_select_codes(const qa_layout* layout, const uint32_t* codes, const uint32_t* ind,
                    int64_t ind_stride, uint32_t* sel_codes, uint32_t* counts, void* ws,
                    size_t ws_bytes, void* stream);

/* The fused steps on sparse-encoded messages (Algorithm 1: the server's "Decode" followed by
 * SynQ_t and the update; on a worker, the update from the pushed S(q_t, I^Syn) with M = 1):
 * exactly qa_decode_selected into a dense code buffer followed by qa_step_qcmd / qa_step_qrda on
 * it, without that buffer.  ind / ind_stride / sel_codes as for qa_decode_selected, scales as
 * written by qa_quantize_pack_selected; ind_stride = 0 applies one indicator to all M messages.
 * Only the first ceil(count/16) words of a bucket's area are read, count = marked components of
 * the bucket.  Everything else (arguments, requant, errors) as for the dense steps.
 * ws: qa_workspace_bytes(layout, QA_OP_STEP_SELECTED); with buckets of 4096 that is the dense
 * steps' workspace (the kernel expands the messages itself), otherwise it also holds the decoded
 * code words of all M messages. */
int qa_step_qcmd_selected(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                          const uint32_t* sel_codes, const float* scales, float* x, float* G,
                          float* z_or_null, float eta, float lambda, float delta, int requant,
                          void* ws, size_t ws_bytes, void* stream);
int qa_step_qrda_selected(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                          const uint32_t* sel_codes, const float* scales, float* x, float* G,
                          float* z, int64_t t, float eta, float lambda, float delta, int requant,
                          void* ws, size_t ws_bytes, void* stream);

/* qa_aggregate_quantize on sparse-encoded messages (Algorithm 1, server: "Decode", "Compute the
 * synchronous indicator", "Average", "Quantize the aggregated gradient" in one call); ind /
 * ind_stride / sel_codes as for qa_decode_selected.  If ind_syn_out is not NULL it receives the
 * synchronous indicator, ceil(d/32) words, exactly as qa_indicator_or writes it.  qa_select_codes
 * with that indicator then turns q_codes into the message S(q_t, I^Syn) that is pushed to the
 * workers. */
int qa_aggregate_quantize_selected(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                                   const uint32_t* sel_codes, const float* scales, int requant,
                                   uint32_t* q_codes, float* q_scales, float* q_thresholds,
                                   uint32_t* ind_syn_out, void* ws, size_t ws_bytes, void* stream);

/* ---- a list of parameter tensors in one flat vector --------------------------------------------
 *
 * For models whose parameters are many tensors of very different sizes (the convolutional
 * networks of Section 5).  The paper does not say at which granularity their gradients are
 * quantized; this library's reading is: the quantizer of Sections 3.4-3.5 is applied to each
 * tensor's gradient on its own (own threshold, own scale), exactly as to a vector of that
 * length, and the update is the same per coordinate.  One launch covers the whole list.
 *
 * The tensors live in one flat vector of length d (x, G, z, the gradients and the 2-bit codes
 * all use the flat index): tensor s occupies [begin[s], begin[s] + length[s]); begin[s] is a
 * multiple of 16 (no code word is shared), the tensors are in ascending order and do not
 * overlap; length[s] may be 0.  Coordinates between tensors belong to no tensor: their gradient
 * is not read, their code fields inside a tensor's last word are written as 0, code words that
 * no tensor touches are neither written nor read, and the steps leave their x, G, z alone.
 * scales[m*scale_stride + s] / thresholds[...] belong to worker m's tensor s
 * (layout->bucket must be 0 and layout->scale_stride >= n_seg).
 *
 * A plan is the device-resident description of the list, built once and reused.  The caller owns
 * the table memory and keeps it unchanged while the plan is in use. */
typedef struct qa_segment_plan {
  int64_t d;         /* length of the flat vector                                            */
  int64_t n_seg;     /* number of tensors                                                    */
  int64_t n_pieces;  /* (4096-tile x tensor) intersections = work-groups per launch          */
  const void* table; /* device memory written by qa_segment_plan_init                        */
} qa_segment_plan;

/* Bytes of device memory a plan's table may need (an upper bound; 0 for invalid arguments). */
size_t qa_segment_plan_bytes(int64_t d, int64_t n_seg);

/* Validates begin/length (HOST arrays of n_seg entries) against the rules above, writes the
 * table (device, 8-byte aligned, at least qa_segment_plan_bytes) and fills *plan_out.  The copy
 * is enqueued on `stream` and waited for: this call synchronises that stream.  1 <= n_seg,
 * 1 <= d < 2^40. */
int qa_segment_plan_init(int64_t d, int64_t n_seg, const int64_t* begin, const int64_t* length,
                         void* table, size_t table_bytes, qa_segment_plan* plan_out, void* stream);

/* The same validation and table, on the HOST only (no device access): *n_pieces_out receives the
 * number of pieces; if table_host is non-NULL (at least qa_segment_plan_bytes) it receives the
 * table as int64 words: [0] tag, [1] d, [2] n_seg, [3] n_pieces, then begin[n_seg],
 * length[n_seg], first_piece[n_seg + 1], piece_tile[n_pieces], piece_tensor[n_pieces]
 * (piece p is the intersection of 4096-tile piece_tile[p] with tensor piece_tensor[p]; the pieces
 * of tensor s are first_piece[s] .. first_piece[s+1]-1).  For sizing and for inspection. */
int qa_segment_plan_host(int64_t d, int64_t n_seg, const int64_t* begin, const int64_t* length,
                         int64_t* table_host, size_t table_bytes, int64_t* n_pieces_out);

/* Workspace of the tensor-list calls below: op = QA_OP_QUANTIZE or QA_OP_STEP (the latter only
 * needed with requant != QA_REQUANT_NONE). */
size_t qa_segment_workspace_bytes(const qa_segment_plan* plan, int32_t M, int op);

/* qa_quantize_pack per tensor: thresholds (optional output) and scales per (worker, tensor),
 * codes at the flat index.  A tensor of length 0 gets threshold 0 and scale 0. */
int qa_quantize_pack_segments(const qa_layout* layout, const qa_segment_plan* plan, const float* g,
                              int64_t g_stride, uint32_t* codes, float* scales, float* thresholds,
                              void* ws, size_t ws_bytes, void* stream);

/* qa_step_qcmd / qa_step_qrda per tensor.  requant: QA_REQUANT_NONE, or QA_REQUANT_BUCKET = the
 * averaged gradient of each tensor is quantized again as a vector of that tensor's length
 * (QA_REQUANT_GLOBAL is refused: there is no whole-vector scale here). */
int qa_step_qcmd_segments(const qa_layout* layout, const qa_segment_plan* plan,
                          const uint32_t* codes, const float* scales, float* x, float* G,
                          float* z_or_null, float eta, float lambda, float delta, int requant,
                          void* ws, size_t ws_bytes, void* stream);
int qa_step_qrda_segments(const qa_layout* layout, const qa_segment_plan* plan,
                          const uint32_t* codes, const float* scales, float* x, float* G, float* z,
                          int64_t t, float eta, float lambda, float delta, int requant, void* ws,
                          size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QADAGRAD_H */
