/*
 * jfa.h -- C ABI of libjfa.so: Jagged Flash Attention for AMD MI355X (gfx950).
 *
 * The operation (paper Section 2: jagged tensor = one values tensor holding all samples back to
 * back + one offsets tensor marking sample boundaries; Section 2.1: flash attention -- two matrix
 * products and a softmax fused block by block with the online-softmax rescaling -- applied to
 * jagged inputs with no padding; Section 2.2: forward and backward):
 *
 *   sample b owns rows offsets[b] .. offsets[b+1]-1 (L_b rows) of q, k, v, each [sum_B, H, D];
 *   for every sample b and head h, with Q, K, V the L_b x D slices,
 *       out = softmax(Q K^T / sqrt(D)) V            (non-causal, every query sees every key of
 *       lse = logsumexp_j(Q K^T / sqrt(D))           its own sample and nothing else)
 *   and, given dout, the gradients dq, dk, dv of sum(out * dout).
 *   No score matrix is written to memory and no buffer is sized by B * max_len.
 *
 * Conventions common to every call
 *   - Every pointer is a DEVICE pointer (HBM of the current HIP device) unless marked "host".
 *   - Values tensors are row-major contiguous [sum_B, H, D]: element (row, h, d) at
 *     (row * H + h) * D + d.  16-byte alignment of the base pointers is required.
 *   - offsets is int64 [B+1] ON THE DEVICE, offsets[0] = 0, non-decreasing, offsets[B] = sum_B.
 *     It is only read by kernels; the host never dereferences it, so calls do not synchronise.
 *     Zero-length samples are legal and produce nothing.
 *   - lse / delta are fp32 [H, sum_B]: element (h, row) at h * sum_B + row, sum_B = offsets[B].
 *     lse is the natural-log logsumexp of the scaled scores.
 *   - max_len is an upper bound on L_b (a hint that bounds nothing in addressing); results are
 *     correct for any max_len >= max_b L_b.  L_b > max_len is undefined on the hot calls and can
 *     be detected with jfa_check_offsets.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *     and return; outputs are ready when the stream reaches that point.
 *   - Ownership: the caller owns every buffer it passes and must keep it alive until the enqueued
 *     work has run.  The library keeps a small private work table per (device, stream), O(B)
 *     bytes, see jfa_workspace_bytes; it is grown with hipMalloc on the first call that needs a
 *     larger one (never inside later calls of the same or smaller B) and kept until process exit.
 *   - Outputs must not alias inputs.  Rows >= sum_B of any buffer are neither read nor written.
 *   - Supported shapes: D in {32, 64, 128}; H >= 1; 0 <= B < 2^31 / 2; sum over samples of
 *     ceil(L_b / 64) times H below 2^31.
 *   - Return value: JFA_OK or a negative jfa_status; jfa_last_error() describes the most recent
 *     failure on the calling thread.  On error nothing has been enqueued.  B == 0 is JFA_OK.
 */
#ifndef JFA_H_
#define JFA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    JFA_OK = 0,
    JFA_ERR_INVALID_ARG = -1, /* null pointer with B > 0, negative size, misaligned pointer */
    JFA_ERR_UNSUPPORTED = -2, /* D outside {32, 64, 128}, sizes beyond the stated limits */
    JFA_ERR_ALLOC = -3,       /* the private work table could not be allocated */
    JFA_ERR_HIP = -4          /* a HIP runtime call or kernel launch failed */
} jfa_status;

/*
 * Forward, bf16 (Section 2.1).  q, k, v, out: bf16 [sum_B, H, D]; lse: fp32 [H, sum_B].
 * Scores and the P V product run on bf16 MFMA with fp32 accumulation; the softmax is fp32;
 * probabilities are rounded to bf16 before the second product; out is rounded to bf16 once.
 */
int jfa_forward(const void *q, const void *k, const void *v, const int64_t *offsets, int64_t B, int64_t max_len,
                int H, int D, void *out, float *lse, void *stream);

/*
 * jfa_forward for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, kernels and results (bit for bit) as jfa_forward, but the private
 * work table (64 counters and two schedules, 8 (B + 33) bytes up to alignment) lives in a fixed array in device
 * memory instead of a table allocated per (device, stream): about 1 MiB that every GPU the library runs on holds
 * until the process ends.  The call allocates and frees nothing and does not synchronise; the array's address is
 * looked up once per device, on the first call made with that device current.
 *   B > JFA_NOALLOC_MAX_B returns JFA_ERR_UNSUPPORTED (nothing is launched).
 *   All calls on one GPU share the one array: calls that overlap in time on a GPU (two streams, two threads) race
 *   on it and give undefined results; calls that follow each other on one stream are safe (each call's scheduler
 *   kernel rewrites the counters and the schedule it uses before its attention kernel reads them).
 *   jfa_timing_enable has no effect on this call (timing events would have to be created).
 */
#define JFA_NOALLOC_MAX_B 65536
int jfa_forward_noalloc(const void *q, const void *k, const void *v, const int64_t *offsets, int64_t B,
                        int64_t max_len, int H, int D, void *out, float *lse, void *stream);

/* Forward, fp32 end to end (same operation; plain FMA arithmetic, for small-tolerance use). */
int jfa_forward_f32(const float *q, const float *k, const float *v, const int64_t *offsets, int64_t B,
                    int64_t max_len, int H, int D, float *out, float *lse, void *stream);

/*
 * Backward, bf16 (Section 2.2 states that every jagged operator has a backward).
 * Inputs: q, k, v as in the forward; out and lse as produced by jfa_forward; dout bf16 [sum_B, H, D].
 * Outputs: dq, dk, dv bf16 [sum_B, H, D]; delta fp32 [2, H, sum_B], a caller-provided buffer that the call
 * fills and then reads: plane 0 is rowsum(dout * out) (an output), plane 1 is -lse * sqrt(D), minus the log-sum-exp
 * in units of the unscaled dot product q.k, the value the kernels' score accumulators start from (scratch).  These two
 * planes are the only sum_B-sized scratch of the backward.
 */
int jfa_backward(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                 const int64_t *offsets, int64_t B, int64_t max_len, int H, int D, void *dq, void *dk, void *dv,
                 float *delta, void *stream);

/* Backward, fp32 end to end.  Here delta is fp32 [H, sum_B] (one plane: rowsum(dout * out)). */
int jfa_backward_f32(const float *q, const float *k, const float *v, const float *out, const float *dout,
                     const float *lse, const int64_t *offsets, int64_t B, int64_t max_len, int H, int D, float *dq,
                     float *dk, float *dv, float *delta, void *stream);

/*
 * Cross attention on jagged tensors: the queries of sample b are rows offsets_q[b] .. offsets_q[b+1] - 1 of q (and
 * of out, dout, dq; sum_Bq rows in all) and its keys and values are rows offsets_kv[b] .. offsets_kv[b+1] - 1 of k
 * and v (and of dk, dv; sum_Bkv rows).  This is the shape of the paper's feature interaction (Section 2: attention
 * between a sample's feature values and its target items); with offsets_kv equal to offsets_q it is jfa_forward /
 * jfa_backward.  Per sample and head:  out_i = sum_j softmax_j(q_i . k_j / sqrt(D)) v_j  over the sample's keys j.
 *
 *   q, out, dout, dq   [sum_Bq, H, D];  k, v, dk, dv  [sum_Bkv, H, D];  bf16, or fp32 for the _f32 variants
 *   offsets_q, offsets_kv   int64 [B+1] on the device
 *   max_len_q, max_len_kv   upper bounds on the samples' query and key counts
 *   lse     fp32 [H, sum_Bq];  delta as for jfa_backward with sum_B = sum_Bq
 * A sample without keys gives out = 0, lse = -inf and dq = 0 for its queries; a sample without queries gives
 * dk = dv = 0 for its keys.  Everything else (alignment, streams, errors, ownership) as for the calls above.
 * max_len_q also selects kernels: with max_len_q <= 32 (a few target items per sample) and D = 128 the bf16 calls
 * run one kernel each that passes over K and V once (the backward writes dq, dk, dv and delta in that pass), so a
 * tight bound is worth passing; as everywhere, a sample with more queries than max_len_q is undefined (no access
 * leaves the buffers, the results are wrong).
 */
int jfa_forward_cross(const void *q, const void *k, const void *v, const int64_t *offsets_q, const int64_t *offsets_kv,
                      int64_t B, int64_t max_len_q, int64_t max_len_kv, int H, int D, void *out, float *lse, void *stream);
int jfa_forward_cross_f32(const float *q, const float *k, const float *v, const int64_t *offsets_q,
                          const int64_t *offsets_kv, int64_t B, int64_t max_len_q, int64_t max_len_kv, int H, int D,
                          float *out, float *lse, void *stream);
int jfa_backward_cross(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                       const int64_t *offsets_q, const int64_t *offsets_kv, int64_t B, int64_t max_len_q,
                       int64_t max_len_kv, int H, int D, void *dq, void *dk, void *dv, float *delta, void *stream);
int jfa_backward_cross_f32(const float *q, const float *k, const float *v, const float *out, const float *dout,
                           const float *lse, const int64_t *offsets_q, const int64_t *offsets_kv, int64_t B,
                           int64_t max_len_q, int64_t max_len_kv, int H, int D, float *dq, float *dk, float *dv,
                           float *delta, void *stream);

/*
 * Causal self attention on jagged tensors: row i of a sample attends to rows 0 .. i of the same sample (the order
 * of a sample's rows is the order of its sequence), as sequential recommendation models use it.  Arguments, layouts,
 * lse and delta exactly as for jfa_forward / jfa_backward (and their _f32 variants); lse_i is the log-sum-exp over
 * the keys j <= i.
 */
int jfa_forward_causal(const void *q, const void *k, const void *v, const int64_t *offsets, int64_t B, int64_t max_len,
                       int H, int D, void *out, float *lse, void *stream);
int jfa_forward_causal_f32(const float *q, const float *k, const float *v, const int64_t *offsets, int64_t B,
                           int64_t max_len, int H, int D, float *out, float *lse, void *stream);
int jfa_backward_causal(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                        const int64_t *offsets, int64_t B, int64_t max_len, int H, int D, void *dq, void *dk, void *dv,
                        float *delta, void *stream);
int jfa_backward_causal_f32(const float *q, const float *k, const float *v, const float *out, const float *dout,
                            const float *lse, const int64_t *offsets, int64_t B, int64_t max_len, int H, int D, float *dq,
                            float *dk, float *dv, float *delta, void *stream);

/*
 * Unfused jagged attention: the three separate jagged operators of the paper's Table 1 (a jagged x jagged product
 * with a jagged square output, a softmax over that output, and its product with a jagged tensor), which write the
 * score array to memory.  They are the baseline that Section 3 compares the fused kernel with, provided here
 * so that the comparison can be run on the same GPU; jfa_forward is the operator to use.
 *
 *   sq_offsets  int64 [B+1] on the device: offsets of the jagged square array, sq[b] = sum of L_c^2 over c < b;
 *               jfa_square_offsets fills it from offsets (one small kernel).
 *   scores      fp32 [H, sq[B]] on the device, caller-provided (the caller sizes it from its lengths): element
 *               (h, b, i, j) at h * sq[B] + sq[b] + i * L_b + j.
 *   jfa_unfused_scores   scores = q k^T / sqrt(D) per sample and head (q, k bf16 [sum_B, H, D]).
 *   jfa_unfused_softmax  row softmax of every L_b x L_b block, in place.
 *   jfa_unfused_apply    out = P v per sample and head (v, out bf16 [sum_B, H, D]); P is rounded to bf16 for
 *                        the matrix product, as in the fused kernel.
 * The paper builds forward and backward for its jagged operators (Section 2.2); the gradients of the three are
 * products of the same kinds plus the softmax's own backward, on the same array layout:
 *   jfa_unfused_product           out[h, sq[b] + i L_b + j] = scale * a[s_b + i, h, :] . b[s_b + j, h, :]  (a, b bf16
 *                                 [sum_B, H, D]); jfa_unfused_scores is the case scale = 1 / sqrt(D), and
 *                                 dP = product(dout, v, 1).
 *   jfa_unfused_softmax_backward  dprobs <- scale * P o (dprobs - rowsum(P o dprobs)) row by row, in place (dS from dP;
 *                                 with scale = 1 / sqrt(D) the two products below need no further scaling).
 *   jfa_unfused_apply_transposed  out[s_b + j, h, :] = sum_i array[h, sq[b] + i L_b + j] x[s_b + i, h, :]  (x, out bf16):
 *                                 dV = apply_transposed(P, dout), dK = apply_transposed(dS, q); dQ = jfa_unfused_apply(dS, k).
 * Errors, streams and ownership as for the calls above.
 */
int jfa_square_offsets(const int64_t *offsets, int64_t B, int64_t *sq_offsets, void *stream);
int jfa_unfused_scores(const void *q, const void *k, const int64_t *offsets, const int64_t *sq_offsets, int64_t B,
                       int64_t max_len, int H, int D, float *scores, void *stream);
int jfa_unfused_softmax(const int64_t *offsets, const int64_t *sq_offsets, int64_t B, int64_t max_len, int H,
                        float *scores, void *stream);
int jfa_unfused_apply(const float *probs, const void *v, const int64_t *offsets, const int64_t *sq_offsets, int64_t B,
                      int64_t max_len, int H, int D, void *out, void *stream);
int jfa_unfused_product(const void *a, const void *b, const int64_t *offsets, const int64_t *sq_offsets, int64_t B,
                        int64_t max_len, int H, int D, float scale, float *out, void *stream);
int jfa_unfused_softmax_backward(const float *probs, const int64_t *offsets, const int64_t *sq_offsets, int64_t B,
                                 int64_t max_len, int H, float scale, float *dprobs, void *stream);
int jfa_unfused_apply_transposed(const float *array, const void *x, const int64_t *offsets, const int64_t *sq_offsets,
                                 int64_t B, int64_t max_len, int H, int D, void *out, void *stream);

/*
 * Jagged <-> padded-dense conversion (paper Section 2.2: jagged tensors are padded where a dense operator
 * needs them and the padding is stripped afterwards).  Rows are opaque: row_bytes is the size of one row of the
 * jagged tensor (everything after its first dimension, e.g. H * D * 2 for bf16 [sum_B, H, D]), a multiple of 16.
 *
 *   jfa_jagged_to_dense  dense[b, i] = values[offsets[b] + i] for i < L_b, and for L_b <= i < max_len the row is
 *                        filled with the 32-bit pad_pattern (a bf16 pad value twice, or an fp32 value's bits).
 *                        values [sum_B, row_bytes] in, dense [B, max_len, row_bytes] out, both on the device.
 *   jfa_dense_to_jagged  values[offsets[b] + i] = dense[b, i] for i < L_b; other bytes of `values` stay untouched.
 * Precondition L_b <= max_len (jfa_check_offsets tells); longer samples are cut at max_len rows, never read or
 * written out of bounds.  Pointers must be 16-byte aligned.  Errors, streams and ownership as for the calls above.
 */
int jfa_jagged_to_dense(const void *values, const int64_t *offsets, int64_t B, int64_t max_len, int64_t row_bytes,
                        uint32_t pad_pattern, void *dense, void *stream);
int jfa_dense_to_jagged(const void *dense, const int64_t *offsets, int64_t B, int64_t max_len, int64_t row_bytes,
                        void *values, void *stream);

/*
 * The jagged feature operators of the paper's Table 1, on bf16 tensors with fp32 accumulation.  x is a jagged
 * tensor [sum_B, D] with the same offsets array as above (s_b = offsets[b], L_b rows per sample); D and T are each
 * one of 32, 64, 128; all tensors on the device, row-major contiguous, 16-byte aligned.
 *
 *   jfa_jagged_dense_bmm   x [sum_B, D] times w [B, D, T] -> out [sum_B, T]:  out[s_b + i, :] = x[s_b + i, :] w[b]
 *   jfa_jagged_jagged_bmm  x [sum_B, D], y [sum_B, T] -> out [B, D, T]:  out[b] = sum over i < L_b of x[s_b + i, :]^T y[s_b + i, :]
 *                          (a zero block for an empty sample).  It is the gradient of jagged_dense_bmm with respect
 *                          to w; jagged_dense_bmm with w transposed is the gradient with respect to x.
 *   jfa_jagged_softmax     x [sum_B, D] -> y [sum_B, D]: softmax along the rows of each sample, one column at a
 *                          time:  y[s_b + i, d] = exp(x[s_b + i, d]) / sum over j < L_b of exp(x[s_b + j, d])
 *   jfa_jagged_softmax_backward  y, dy [sum_B, D] -> dx = y (dy - sum over j < L_b of dy[s_b + j, :] y[s_b + j, :])
 * Outputs are rounded to bf16 once, from fp32.  Rows at and past offsets[B] are neither read nor written.
 * max_len is an upper bound on L_b as elsewhere.  Errors, streams and ownership as for the calls above.
 */
int jfa_jagged_dense_bmm(const void *x, const void *w, const int64_t *offsets, int64_t B, int64_t max_len, int D, int T,
                         void *out, void *stream);
int jfa_jagged_jagged_bmm(const void *x, const void *y, const int64_t *offsets, int64_t B, int64_t max_len, int D, int T,
                          void *out, void *stream);
int jfa_jagged_softmax(const void *x, const int64_t *offsets, int64_t B, int64_t max_len, int D, void *y, void *stream);
int jfa_jagged_softmax_backward(const void *y, const void *dy, const int64_t *offsets, int64_t B, int64_t max_len, int D,
                                void *dx, void *stream);

/*
 * The offsets-driven work schedule on its own (the first kernel of every call above), for
 * inspection and tests.  For row blocks of block_rows rows it writes, on the device,
 *   order      int32 [B]    sample ids, samples with more row blocks first
 *   tile_start int32 [B+1]  exclusive prefix sum of ceil(L_order[p] / block_rows); tile_start[B] = T
 * A work item w in [0, T*H) is (sample, head, row block): p = the position with
 * tile_start[p]*H <= w < tile_start[p+1]*H, r = w - tile_start[p]*H, n = tile_start[p+1]-tile_start[p],
 * head = r / n, block = r % n.  block_rows must be a positive multiple of 32.
 */
int jfa_build_schedule(const int64_t *offsets, int64_t B, int block_rows, int32_t *order, int32_t *tile_start,
                       void *stream);

/*
 * Debug check of an offsets array; SYNCHRONISES the stream.  *host_flags (host pointer) receives a
 * bit mask: 1 = offsets[0] != 0, 2 = decreasing somewhere, 4 = some L_b > max_len.  0 means valid.
 */
int jfa_check_offsets(const int64_t *offsets, int64_t B, int64_t max_len, void *stream, int *host_flags);

/*
 * Bytes of library-private device memory a call with these sizes uses (pass: 0 = forward,
 * 1 = backward).  It depends on B only -- never on max_len or B * max_len.
 */
size_t jfa_workspace_bytes(int64_t B, int64_t max_len, int H, int D, int pass);

/*
 * Per-kernel timing, a benchmark aid (thread-local; do not use under stream capture).  While enabled,
 * every call above brackets each kernel it enqueues with a pair of HIP events on the call's stream.
 * jfa_timing_read waits for those events and reports, per distinct kernel name, the summed duration in
 * milliseconds and the number of launches since the last read (or enable), then forgets them.
 * names / total_ms / launches are host arrays of `capacity` entries; the return value is the number
 * of entries filled, or a negative jfa_status.  The name strings are static.
 */
int jfa_timing_enable(int on);
int jfa_timing_read(int capacity, const char **names, float *total_ms, int *launches);

/* Description of the last failure on this thread (a static, thread-local string; never freed). */
const char *jfa_last_error(void);

/* major * 10000 + minor * 100 + patch. */
int jfa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* JFA_H_ */
