/* C ABI of the MI355X (gfx950) ELMO classifier-head library.
 *
 * The library implements the hot path of ELMO (arxiv 2510.11168): the label-chunked training
 * step of a linear extreme-classification head whose weights live only in BF16 or FP8-E4M3,
 * with the weight gradient fused into the SGD update (Algorithm 1 "Float8 XMC classifier",
 * Sections 4.1-4.3), stochastic rounding (Section 3, Eq. 1), optional Kahan compensation in
 * BF16 (Section 3; Appendix "Precision Recovery"), and the top-k scoring needed by P@k
 * (Appendix, definition of P@k).
 *
 * General rules
 *  - Every pointer named W, comp, workspace, X, indptr, indices, dX_out, loss_out, idx_out,
 *    score_out, src, dst is a DEVICE pointer owned by the caller; the library never allocates or
 *    frees device memory and never synchronises the device (exception: ELMO_VALIDATE, below).
 *  - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the null stream);
 *    results are valid once the stream has reached that point.  Calls on one head must not
 *    overlap in time: they share its workspace.
 *  - Return value: 0 success; -1 invalid argument; -2 unsupported format/flag; -3 HIP runtime
 *    error; -4 invalid label data found by a previous validated step.  elmo_last_error() gives
 *    the text for the calling thread.
 *  - All matrices are row-major and densely packed.
 */
#ifndef ELMO_HEAD_H
#define ELMO_HEAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct elmo_head elmo_head_t; /* opaque, host-side */

/* Storage format of the classifier weights (Section 4.1 pure 16-bit; Section 4.3 8-bit).
 * ELMO_FP8_E4M3 is the OCP "FN" flavour: bias 7, largest finite value 448, no infinities. */
enum { ELMO_BF16 = 0, ELMO_FP8_E4M3 = 1, ELMO_FP32 = 2 /* optimiser moments of elmo_kahan_adamw only */ };

/* ELMO_SR: the update rounds with stochastic rounding (Eq. 1), otherwise to nearest even.
 * ELMO_KAHAN: a BF16 compensation buffer carries the rounding error of every update into the
 *             next one (the recurrence of Section 3 with s = w, v = -lr*grad), for all labels or,
 *             with elmo_head_opts.kahan_rows, for the head labels only.
 * ELMO_VALIDATE: each step checks the label data on the device (ids inside [0, L), ascending
 *             within a row) and the NEXT call on the head reads that flag back (one blocking
 *             4-byte copy) and fails with -4 if it was raised. */
enum { ELMO_SR = 1u, ELMO_KAHAN = 2u, ELMO_VALIDATE = 4u };

typedef struct {
  uint32_t flags;         /* ELMO_SR | ELMO_KAHAN | ELMO_VALIDATE */
  int32_t max_B;          /* largest batch any step / top-k call will use (>= 1) */
  int64_t max_nnz;        /* largest number of positives in one batch (>= 1) */
  void* W;                /* [L, d] weights in weight_dtype, updated in place by every step */
  size_t W_bytes;
  void* comp;             /* [kahan_rows, d] BF16 compensation, required iff ELMO_KAHAN, start at zero */
  size_t comp_bytes;
  int64_t kahan_rows;     /* with ELMO_KAHAN: only the labels [0, kahan_rows) carry compensation, the rest
                             are updated as without the flag ("Kahan summation for head labels", appendix
                             "Precision Recovery for Sensitive Applications": number the labels by falling
                             frequency and the top-p% head is this prefix; memory 2 bytes x kahan_rows x d).
                             0 = every label.  Otherwise L or a multiple of 128.  Must be 0 without the flag. */
  float weight_decay;     /* L2 weight decay of the classifier (the "WD ... XMC" column of the paper's
                             hyper-parameter table; Algorithm 1 itself has none): the update uses
                             g + weight_decay * w in place of the gradient g, two more FP32 operations, each
                             rounded.  0 = none (the two operations are skipped).  In [0, 1]. */
  float dropout_p;        /* dropout on the classifier weights inside the products (appendix "Low-Memory
                             Dropout for Classifier": the weights are masked after they are loaded, before
                             the matrix product, so no masked copy of W exists).  Per step every weight
                             element is dropped with probability T/256, T = round(256 * dropout_p), the
                             same mask for all samples of the batch; the logits and the input gradient use
                             the masked weights scaled by 256/(256-T), and the weight gradient is that of
                             the masked model (zero at dropped elements, scaled elsewhere).  The mask is
                             byte e % 16 >= T of Philox4x32-10 with key = seed of the step and counter =
                             (e / 16, step | 2^63), e = label * d + column; steps must stay below 2^63.
                             elmo_head_topk never drops.  0 = none.  In [0, 255/256]. */
  void* workspace;        /* scratch; contents need not survive between calls */
  size_t workspace_bytes;
} elmo_head_opts;

/* Bytes of the three buffers a head needs.  workspace = one chunk's logit-gradient buffer
 * (chunk x round_up(max_B, 64) BF16 values, the paper's per-chunk logits buffer of Section 4.4)
 * plus O(max_B * d) staging for the inputs and the input-gradient partial sums, plus the
 * per-batch label index.  Any of the three output pointers may be NULL. */
int elmo_head_sizes(int64_t L, int32_t d, int weight_dtype, int64_t chunk, int32_t max_B,
                    int64_t max_nnz, uint32_t flags, int64_t kahan_rows, size_t* W_bytes,
                    size_t* comp_bytes, size_t* workspace_bytes);

/* Bytes of the logit / logit-gradient buffer for `batch` samples and `labels` labels held in
 * 16 bits, batch * labels * 2 -- the quantity Section 4.4 divides by the number of chunks. */
size_t elmo_logit_buffer_bytes(int64_t batch, int64_t labels);

/* Create a head over caller-owned buffers.  Requirements: L >= 1; d a positive multiple of 128, at most 2^20;
 * chunk >= 1 (the labels processed per pass, Section 4.2 "chunking"; it need not divide L, the last
 * chunk is short.  The kernels work on whole 128-label tiles, so a pass takes round_up(chunk, 128)
 * labels; the updated weights do not depend on the chunk size at all and the input gradient only
 * through the order of its FP32 sums, so the rounding shows in the workspace size only); buffers at
 * least as large as elmo_head_sizes says and 256-byte aligned.  Launches nothing.  *out receives the
 * handle.  Heads may be created and stepped from several host threads (one head per thread at a
 * time); the library's one-time set-up is guarded. */
int elmo_head_create(int64_t L, int32_t d, int weight_dtype, int64_t chunk,
                     const elmo_head_opts* opts, elmo_head_t** out);

/* One training step of the head (Algorithm 1, XMC_update):
 *   for each chunk c of labels:  Z = Xq W_c^T ; G = sigmoid(Z) - Y_c ; dX += G W_c (old W_c);
 *                                W_c <- Q(W_c - lr * G^T X)   (fused, FP32 arithmetic)
 * X      [B, d] BF16 inputs (the encoder's output).  With FP8 weights the logits use X rounded
 *        to E4M3 (nearest even); the weight gradient always uses the BF16 X.
 * indptr [B+1], indices [nnz] int32: CSR of the positive label ids of each sample; within a row
 *        ids are distinct, ascending, in [0, L); nnz == indptr[B] <= max_nnz.
 * lr     learning rate; the gradient is summed over the batch (no 1/B).
 * seed, step: select the stochastic-rounding stream (Philox4x32-10, key = seed, counter =
 *        (flat element index / 8, step); element l*d+j uses 16-bit field (l*d+j) % 8).  The
 *        updated weights depend on (seed, step) only -- not on chunk or launch geometry.
 * dX_out [B, d] BF16 input gradient, or NULL.  loss_out: one float, the summed BCE loss
 *        sum(softplus(z) - y z) over the batch and all labels, or NULL.
 * The call only enqueues kernels on hip_stream (no allocation, no memset node, no host
 * synchronisation unless ELMO_VALIDATE is set), so after one ordinary call it can be captured
 * into a HIP graph; lr, seed and step are then part of the captured launches. */
int elmo_head_step(elmo_head_t* h, const void* X, int32_t B, const int32_t* indptr,
                   const int32_t* indices, int64_t nnz, float lr, uint64_t seed, uint64_t step,
                   void* dX_out, float* loss_out, void* hip_stream);

/* Top-k scoring (the top_k of the P@k definition): for each of the B rows of X the k labels with
 * the largest logit over all L labels, ordered by (logit descending, label id ascending).
 * idx_out [B, k] int32, score_out [B, k] float (either may be NULL).  1 <= k <= L.
 * Up to k = 128 the labels are swept once; larger k is produced in pages of 128 entries, one more
 * sweep per page (each page admits only what ranks strictly after the last entry of the page
 * before it), exact for any k. */
int elmo_head_topk(elmo_head_t* h, const void* X, int32_t B, int32_t k, int32_t* idx_out,
                   float* score_out, void* hip_stream);

/* Top-k scoring for callers that cannot allocate device memory or keep a head: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as
 * elmo_head_topk on a head over the same weights (same kernels), but the call takes the weights
 * directly and needs no workspace: its scratch (staged E4M3 copy of X, thresholds, candidate lists)
 * is a device array of 18 MiB inside the library, one copy per GPU the library runs on, held until
 * the process ends.  The call allocates and frees nothing and launches only kernels (no memset
 * node).  Limits, rejected with -1: B <= 128 queries, d a multiple of 128 up to 4096, 1 <= k <= L.
 * W [L, d] in weight_dtype (ELMO_BF16 or ELMO_FP8_E4M3), X [B, d] BF16, both device pointers,
 * 16-byte aligned; idx_out [B, k] int32, score_out [B, k] float (either may be NULL).
 * All calls on one GPU share that GPU's array and nothing of it survives a call: calls that overlap
 * in time on one GPU (two streams, two host threads) race.  The first call on a device looks the
 * array's address up (hipGetSymbolAddress); make that call outside any stream capture. */
int elmo_topk_static(const void* W, int64_t L, int32_t d, int weight_dtype, const void* X, int32_t B,
                     int32_t k, int32_t* idx_out, float* score_out, void* hip_stream);

/* Precision at k (evaluation section, P@k(y, y^) = (1/k) sum over l in top_k(y^) of y_l), as exact
 * integer numerators: hits_out[j-1] = number of (row, label) pairs with the label among the row's
 * first j entries of idx and among the row's positives, summed over the B rows, j = 1..k; then
 * P@j = hits_out[j-1] / (j * B).  idx [B, k] int32 as written by elmo_head_topk (best first);
 * indptr / indices: the CSR positives of the same B rows (ids ascending within a row); hits_out
 * [k] int64.  All device pointers; 1 <= k <= 2^20 and B * k < 2^31.  Needs no head. */
int elmo_precision_hits(const int32_t* idx, int32_t B, int32_t k, const int32_t* indptr,
                        const int32_t* indices, int64_t* hits_out, void* hip_stream);

int elmo_head_destroy(elmo_head_t* h);

/* Measurement hooks.  elmo_head_profile(h, 1) makes every later step / top-k call record a HIP
 * event on its stream at each boundary between kernel classes; elmo_head_profile(h, 0) stops.
 * elmo_head_profile_read waits for the last recorded event, then returns per class the summed
 * event-to-event time in milliseconds and the number of spans, and clears the record.  Classes:
 * 0 step set-up, 1 logits + epilogue, 2 input gradient, 3 fused update, 4 finalise, 5 top-k.
 * ms and launches are HOST arrays of 6 entries. */
int elmo_head_profile(elmo_head_t* h, int enable);
int elmo_head_profile_read(elmo_head_t* h, double ms[6], int64_t launches[6]);

/* Text of the last error on the calling thread; never NULL. */
const char* elmo_last_error(void);

/* Test hooks for the bit-exactness clause of the parity contract.
 * elmo_quantize: dst[i] = Q(src[i]) for i in [0, n): dtype ELMO_BF16 writes uint16, ELMO_FP8_E4M3
 * writes uint8; mode 0 = round to nearest even, mode 1 = stochastic rounding with the field of
 * flat element index first_elem + i (same stream as elmo_head_step).  src: device FP32. */
int elmo_quantize(const float* src, int64_t n, int dtype, int mode, uint64_t seed, uint64_t step,
                  uint64_t first_elem, void* dst, void* hip_stream);

/* Simulated low-precision formats (the bit-width study of Section 4.3, "simulating floating-point
 * numbers with a specific number of mantissa and exponent bits"): dst[i] = the FP32 value of src[i]
 * rounded to a format with exp_bits exponent and man_bits mantissa bits, mode and rounding fields as
 * in elmo_quantize.  The format follows the IEEE pattern (bias 2^(E-1)-1, top exponent code reserved,
 * gradual underflow): (8,7) is BF16, (5,10) FP16, (5,2) E5M2; finite overflow and infinities clip to
 * the largest finite value, NaN passes through.  2 <= exp_bits <= 8, 1 <= man_bits <= 22 (else -2).
 * src, dst: device FP32, n entries each (may be the same buffer). */
int elmo_quantize_em(const float* src, int64_t n, int exp_bits, int man_bits, int mode, uint64_t seed,
                     uint64_t step, uint64_t first_elem, float* dst, void* hip_stream);

/* AdamW with Kahan-compensated BF16 parameters, in place (Section 4.1: the encoder's parameters
 * are kept in BF16 and their optimiser step uses Kahan summation so that updates below half a
 * grid spacing are not cancelled).  Textbook AdamW (decoupled weight decay, bias-corrected
 * moments) in FP32 arithmetic, every operation rounded once:
 *   m' = b1 m + o1 g;   v' = b2 v + (o2 g) g;   r = (m'/bc1) / (sqrt(v'/bc2) + eps);
 *   r += weight_decay * p (skipped when 0);   u = lr r;
 *   y = -u - c;   s = p + y;   p' = RNE_BF16(s);   c' = RNE_BF16((p' - p) - y)
 * with b_i = (float)beta_i, o_i = (float)(1 - beta_i), bc_i = (float)(1 - beta_i^t) formed in double.
 * param, comp, grad: device BF16 [n] (comp starts at zero); m, v: device moments [n] in
 * state_dtype = ELMO_BF16 (stored round-to-nearest-even) or ELMO_FP32, starting at zero.
 * t >= 1 counts the steps.  All buffers 16-byte aligned, caller-owned, updated in place (grad is
 * only read).  n = 0 is a no-op.  Errors: -1 bad argument, -2 unsupported state_dtype, -3 HIP. */
int elmo_kahan_adamw(void* param, void* comp, void* m, void* v, const void* grad, int64_t n, int state_dtype,
                     float lr, double beta1, double beta2, float eps, float weight_decay, int64_t t,
                     void* hip_stream);

/* Host-side view of the dropout mask of elmo_head_opts.dropout_p: bit i of the result is 1 iff
 * weight element 16 * block + i is kept at (seed, step) for the threshold T = threshold (0..255). */
uint32_t elmo_dropout_keep16(uint64_t seed, uint64_t step, uint64_t block, uint32_t threshold);

/* Host-side Philox4x32-10 (Salmon et al., SC'11) as used for the rounding fields. */
void elmo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

#ifdef __cplusplus
}
#endif
#endif /* ELMO_HEAD_H */
