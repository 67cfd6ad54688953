/*
 * flexq.h -- C ABI of the MI355X (gfx950) library for the decode hot path of
 * FlexQuant's dynamic precision switching (arXiv 2506.12024).
 *
 * What the calls compute is defined by the paper:
 *   fq_quantize     asymmetric uniform quantization, Sec. 2.2 Eq. (2)
 *                   (fq_quantize_sym: the symmetric variant; fq_fake_quantize:
 *                   quantize-dequantize at 2..8 bits as in Sec. 5.1)
 *   fq_linear       the weight-only quantized linear layer of the decode phase
 *                   (Sec. 4.1), weights dequantized on the fly by Eq. (3), the
 *                   bit-width of every layer chosen per generated token from
 *                   copies that all stay resident in HBM (Sec. 4.3)
 *   fq_entropy_kl   entropy of softmax(logits) (Sec. 2.3; PPLE of Sec. 4.2
 *                   Eq. (5) is exp of it) and the KL divergence used to rank
 *                   layers (Sec. 3.1, Sec. 4.3)
 *
 * Conventions.
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, who keeps it
 *     alive until the work enqueued on `stream` has finished.  The library never
 *     allocates, frees or copies tensor memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued in order on it; a call returns without waiting.  Four calls
 *     do wait for `stream`, and say so where they are declared: fq_plan_create and
 *     fq_plan_create_staged (they copy their small tables from host memory and
 *     wait for that copy, so they cannot be called under stream capture: create
 *     plans before capturing), fq_plan_status and fq_sched_peek (they read words
 *     back to the host).
 *   - Every function returns FQ_OK (0) or a negative fq_status.  Arguments are
 *     validated before anything is launched; on an error nothing was enqueued.
 *     fq_last_error() returns a message for the calling thread's last failure.
 *   - Matrices are row-major.  A linear layer has K inputs and N outputs and its
 *     weight is W[N][K]; quantization groups are `group` consecutive k of a row.
 *
 * Packed layout (the one fq_quantize writes, fq_layer_attach expects and the
 * kernels stream directly -- a switch of bit-width never repacks anything):
 *   codes, bits = 8 : u8  [N][K]      byte k of row n is the code of W[n][k]
 *   codes, bits = 4 : u8  [N][K/2]    byte j of row n = code(2j) | code(2j+1) << 4
 *   codes, bits = 2 : u8  [N][K/4]    byte j of row n = code(4j) | code(4j+1) << 2 |
 *                                     code(4j+2) << 4 | code(4j+3) << 6
 *                                     (Table 1's lowest width)
 *   codes, bits = 3 : u8  [N][K/32][12]  a block of 12 bytes holds 32 consecutive codes c(0..31)
 *                                     as three little-endian 32-bit words: word j holds c(10j) ..
 *                                     c(10j+9) whole, c(10j + 5h + p) (h = 0, 1; p = 0 .. 4) in
 *                                     bits 16h + 3p .. 16h + 3p + 2; bit 15 of word t is bit t
 *                                     of c(30), bit 31 of word t is bit t of c(31).  The paper
 *                                     runs 3-bit models (Table 1, Sec. 5.1) without fixing a
 *                                     packing: this one is this library's, chosen so that ten
 *                                     codes of a word unpack with one mask-and-merge and one
 *                                     dot product per pair.  Served at M = 1.
 *   scales          : f32 [N][K/group]
 *   zeros           : u8  [N][K/group]
 *   bits = 16       : the fp16 weights W[N][K] themselves, no scales/zeros
 */
#ifndef FLEXQ_H
#define FLEXQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fq_status {
    FQ_OK = 0,
    FQ_ERR_NULL = -1,         /* a required pointer is NULL */
    FQ_ERR_BITS = -2,         /* bit-width not supported by this call */
    FQ_ERR_SHAPE = -3,        /* a size is out of range or K is not a multiple of group */
    FQ_ERR_NOT_ATTACHED = -4, /* the layer holds no copy at the requested bit-width */
    FQ_ERR_ALIGN = -5,        /* a pointer is not aligned as documented */
    FQ_ERR_HIP = -6           /* the HIP runtime reported an error (see fq_last_error) */
} fq_status;

typedef struct fq_layer fq_layer; /* opaque: borrows the caller's packed buffers */
typedef struct fq_plan fq_plan;   /* opaque: a list of linears run by one launch */

#define FQ_GROUP 128      /* the group size the kernels are built for */
#define FQ_MAX_ROW_GROUP_K 65536 /* longest row of an 8-bit copy with one scale per row (group = K) */
#define FQ_MAX_DECODE_M 32 /* rows of x served by the skinny (decode) kernels */
#define FQ_MAX_DECODE_K 32768 /* longest row they take (a row of x stays in LDS at M = 1) */
#define FQ_MAX_LM_HEAD_M 4 /* rows of x served by fq_lm_head_entropy */
#define FQ_SCRATCH_BANKS 16 /* streams per device with a copy of their own of the library's static
                               scratch (fq_entropy_kl over a few rows, fq_lm_head_entropy) */

/* Message describing the calling thread's most recent error ("" if none).  (Interface only: the
 * paper defines no error model.) */
const char *fq_last_error(void);

/*
 * Bytes of the three packed buffers for an N x K weight at `bits` (2, 3, 4 or 8): what Eq. (2) of
 * Sec. 2.2 produces per weight (an n-bit code) and per group (s, z), in the layout above.
 * Any of the three outputs may be NULL.  Host-only; launches nothing.  group = FQ_GROUP, or, at 8 bits,
 * group = K: one scale and zero point per weight row (see fq_quantize).
 */
int fq_packed_sizes(int N, int K, int bits, int group,
                    size_t *codes_bytes, size_t *scales_bytes, size_t *zeros_bytes);

/*
 * Sec. 2.2 Eq. (2), per (row, group): with lo = min(0, min w), hi = max(0, max w),
 *   s = (hi - lo) / (2^bits - 1),  z = round(-lo / s),  q = clamp(round(w / s + z)),
 * all in binary32 with one rounding per operation and round-half-to-even; an
 * all-zero group gets s = 1, z = 0.  Writes the packed layout above.
 *   w_fp16  device, fp16 [N][K], 16-byte aligned      (read)
 *   codes   device, fq_packed_sizes bytes, 16-byte aligned (written)
 *   scales  device, f32 [N][K/group]                   (written)
 *   zeros   device, u8  [N][K/group]                   (written)
 * bits in {2, 3, 4, 8}; group = FQ_GROUP; K a multiple of group; N, K >= 1.
 * At 8 bits group = K is accepted as well (K a multiple of FQ_GROUP, at most FQ_MAX_ROW_GROUP_K): Xmin and
 * Xmax of Eq. (2) are then taken over the whole row, scales and zeros are [N][1] -- the granularity at
 * which the INT8 copy meets 8-bit activations in the prefill without a fold per group (Sec. 4.1: W8A8
 * is there to use the integer matrix units fully).  Such a copy is served by fq_linear_w8a8 only.
 * Non-finite weights give unspecified codes.
 */
int fq_quantize(const void *w_fp16, int N, int K, int bits, int group,
                void *codes, void *scales, void *zeros, void *stream);

/*
 * The symmetric variant stated after Sec. 2.2 Eq. (3): z = 0, Xmax = -Xmin = max |w| of the
 * group, 2^bits - 2 steps.  Per (row, group): s = (2 max|w|) / (2^bits - 2),
 * q = clamp(round(w / s)) in -(2^(bits-1) - 1) .. 2^(bits-1) - 1, binary32, one rounding per
 * operation, round-half-to-even; an all-zero group gets s = 1.  Written in the packed layout of
 * fq_quantize with stored code = q + 2^(bits-1) and stored zero point = 2^(bits-1) in every group,
 * so that Eq. (3), s * (code - zero), is s * q and fq_layer_attach / fq_linear / fq_plan_* take
 * the result as they take fq_quantize's.  Arguments, alignment and errors as fq_quantize.
 */
int fq_quantize_sym(const void *w_fp16, int N, int K, int bits, int group,
                    void *codes, void *scales, void *zeros, void *stream);

/*
 * Quantize and dequantize in one pass, w_hat = fp16(s * (q - z)) with s, z, q of Eq. (2) exactly
 * as fq_quantize (symmetric = 0) or fq_quantize_sym (symmetric != 0) compute them, at any width
 * from 2 to 8 bits.  This is how the paper evaluates its 2- to 4-bit models (Sec. 5.1: those
 * widths are simulated; Table 1); the result is an fp16 weight for fq_layer_attach(layer, 16, ...).
 *   w_fp16      device, fp16 [N][K], 16-byte aligned   (read)
 *   w_hat_fp16  device, fp16 [N][K], 16-byte aligned   (written; may be w_fp16 itself)
 * bits in 2..8; group = FQ_GROUP; K a multiple of group.  Non-finite weights give unspecified
 * results.
 */
int fq_fake_quantize(const void *w_fp16, int N, int K, int bits, int group, int symmetric,
                     void *w_hat_fp16, void *stream);

/*
 * A layer handle: a small host object naming the resident copies of one
 * linear's weight -- Sec. 4.3: every linear is kept in several formats at once, all resident in
 * HBM, and a switch of precision selects among them.  fq_layer_attach records (does not copy) the buffers for one
 * bit-width; any subset of {2, 3, 4, 8, 16} may be attached, each at most once per
 * value (attaching again replaces the pointers).  For bits = 16 pass the fp16
 * weights as `codes` and NULL scales/zeros.  Buffers must be 16-byte aligned.
 * Launches nothing and takes no stream: the kernels stream the packed layout as it is, so there is
 * nothing to re-tile when a copy is attached.  group = FQ_GROUP; or group = K for a layer that holds
 * nothing but an 8-bit copy with one scale per row: fq_layer_attach then takes bits = 8 only, and
 * fq_linear, the plans and fq_linears_static answer FQ_ERR_SHAPE for it (fq_linear_w8a8 serves it).
 */
int fq_layer_create(fq_layer **out, int N, int K, int group);
int fq_layer_attach(fq_layer *layer, int bits, const void *codes,
                    const void *scales, const void *zeros);
int fq_layer_destroy(fq_layer *layer);

/*
 * Decode-phase linear (Sec. 4.1, Eq. (3)):
 *   y[m][n] = fp16( sum_g s[n][g] * sum_{k in g} x[m][k] * (q[n][k] - z[n][g]) )
 * accumulated in binary32, using the copy attached for `bits` -- chosen at call
 * time, nothing is repacked.  bits = 16 multiplies by the fp16 weights.
 *   x_fp16  device, fp16 [M][K], 16-byte aligned   (read)
 *   y_fp16  device, fp16 [M][N]                    (written)
 * 1 <= M <= FQ_MAX_DECODE_M with K <= FQ_MAX_DECODE_K selects the memory-bound skinny
 * kernels; anything else (prefill-shaped, any M >= 1) runs the MFMA dequant-GEMM -- but for
 * bits = 3, which the GEMM does not unpack: there the small-batch kernel runs the call in slabs of
 * FQ_MAX_DECODE_M rows of x, one launch per slab, reading the weights once per slab.
 */
int fq_linear(const fq_layer *layer, int bits, const void *x_fp16, int M,
              void *y_fp16, void *stream);

/*
 * A plan runs `count` linears with ONE launch: entry i computes
 * ys[i] = linear(layers[i], bits[i], xs[i]) with the same M (1..FQ_MAX_DECODE_M)
 * for all and every K <= FQ_MAX_DECODE_K (FQ_ERR_SHAPE otherwise).  The entries must be independent of each other within one run (no
 * ys[i] may alias an xs[j]).  The bit-width of every entry is read by the kernel
 * from DEVICE memory at run time, so the per-token precision pattern of
 * Sec. 4.4 / Alg. 1 can be written by another kernel or a small copy and the
 * same plan (and a HIP graph holding it) serves every pattern.
 *   workspace  device memory of fq_plan_workspace_bytes(count) bytes, 256-byte
 *              aligned, owned by the caller, must outlive the plan; the
 *              descriptor table is copied into it on `stream` by fq_plan_create, which waits for
 *              that copy (the only work it enqueues).  After the
 *              table come the tile queue of the streaming batch kernel, zeroed by
 *              fq_plan_create and left zeroed by every run, and the list of entries a run
 *              draws up for its bit-widths: runs of one plan must not overlap in time
 *              (they would share these, and they write the same ys)
 *   bits_dev   device, int32 [count], each 2, 3, 4, 8 or 16 and attached to its layer;
 *              an entry whose value is anything else is skipped
 *              by the kernel and its y is left untouched.  Such a run sets bit 0 of the plan's
 *              flags, a word in the workspace that stays set and that fq_plan_status reports
 *              (gave_up is always 0 for these plans)
 */
size_t fq_plan_workspace_bytes(int count);
int fq_plan_create(fq_plan **out, int count, const fq_layer *const *layers,
                   const void *const *xs, void *const *ys, int M,
                   void *workspace, size_t workspace_bytes, void *stream);
int fq_plan_run(const fq_plan *plan, const int32_t *bits_dev, void *stream);
int fq_plan_destroy(fq_plan *plan);

/*
 * A stage-ordered plan: the decode step of Alg. 1 in the order a decoder must issue it (Sec. 4.1:
 * each of these linears is bound by loading its weights, so the step is one long weight stream
 * with dependencies in it).  Entry i belongs to stage `stage[i]`; the entries of a stage are
 * independent of each other, and an entry may read (as x) what an entry of an EARLIER stage writes
 * (as y).  fq_plan_run runs all stages in order with ONE launch of a persistent kernel: a grid-wide
 * barrier stands between two stages, and the weights of the next stage are already being fetched
 * while it is crossed.  Results are bit-identical to the same stages run as separate stage-ordered
 * plans (against fq_plan_create's kernel a row may be summed in a different order).
 *   stage      HOST, int32 [count]: stage[0] = 0, never decreasing, rising by at most 1;
 *              at most FQ_MAX_STAGE_ENTRIES entries per stage
 *   workspace  device, fq_plan_staged_workspace_bytes(count, number of stages) bytes, 256-byte
 *              aligned, owned by the caller, must outlive the plan
 *   M          must be 1; every K <= FQ_MAX_DECODE_K, and the table of stages plus one row of x
 *              must fit the LDS of a compute unit (FQ_ERR_SHAPE otherwise: about 1000 stages at
 *              K = 11008, 1500 at 4096)
 * Everything else as fq_plan_create (which also copies the tables and waits for that copy).
 * The kernel's workgroups wait for each other, so the launch needs the device to itself: while
 * another kernel holds compute units the waits may run out.  A wait is bounded (about a second
 * by default, fq_plan_set_wait_limit sets the number of polls): a launch that gives up leaves y
 * incomplete, every workgroup still exits, the barrier's counters are put back, and the next
 * launch starts clean.  fq_plan_status (for either kind of plan) waits for `stream` and reports
 *   gave_up  launches of this plan that gave up so far (never reset)
 *   flags    bit 0: an entry's bit-width was not 2, 3, 4, 8 or 16 or had no copy attached (its y was
 *            left untouched); bit 1: a workgroup's share of a stage exceeded 4096 rows (skipped)
 * Either output may be NULL.  Runs of one plan must not overlap in time.
 */
#define FQ_MAX_STAGE_ENTRIES 32
size_t fq_plan_staged_workspace_bytes(int count, int n_stages);
int fq_plan_create_staged(fq_plan **out, int count, const fq_layer *const *layers,
                          const void *const *xs, void *const *ys, const int32_t *stage, int M,
                          void *workspace, size_t workspace_bytes, void *stream);
int fq_plan_set_wait_limit(fq_plan *plan, long long polls);
int fq_plan_status(const fq_plan *plan, int32_t *gave_up, int32_t *flags, void *stream);

/*
 * For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): what fq_plan_create + fq_plan_run + fq_plan_destroy do, in one call that
 * takes no workspace, creates no object, copies nothing from host memory and never synchronises.
 * Entry i computes ys[i] = linear(layers[i], bits_dev[i], xs[i]); arguments, limits, alignment and
 * errors as for fq_plan_create and fq_plan_run; count <= FQ_STATIC_MAX_ENTRIES (FQ_ERR_SHAPE
 * beyond).  The descriptor table, the tile queue and the entry lists live in a static device array
 * of the library (about 73 KiB, held on every device the library runs on until the process ends);
 * the table is written there by small kernels that carry it in their arguments, one launch per 24
 * entries, ahead of the launch that computes.  Every call on a device shares that array: calls that
 * overlap in time on one device race (calls on one stream, or ordered by events, do not).  The
 * host-side handles in `layers` are read during the call only.
 */
#define FQ_STATIC_MAX_ENTRIES 512
int fq_linears_static(int count, const fq_layer *const *layers, const void *const *xs, void *const *ys,
                      int M, const int32_t *bits_dev, void *stream);

/*
 * Measurement aid: reads `bytes` bytes (rounded down to a multiple of 16) once, with the access
 * pattern of the decode kernels and nothing else -- the rate a benchmark may set the weight stream
 * of Sec. 4.1 against, next to the published peak.  `sink` receives a word only if the data
 * happen to xor to one particular value.
 *   src   device, 16-byte aligned   (read)
 *   sink  device, u32 [1]           (hardly ever written)
 */
int fq_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream);

/*
 * W8A8 prefill (Sec. 4.1, 4.3, 4.5): the prompt is processed with the resident INT8 weights
 * against 8-bit activations on the integer matrix cores.
 *
 * fq_quantize_act quantizes activations per token with the symmetric form stated after
 * Sec. 2.2 Eq. (3): z = 0, s_x[m] = (2 max_k |x[m][k]|) / 254, xq = round(x / s_x) in
 * [-127, 127]; binary32, one rounding per operation, IEEE division, round-half-to-even; an
 * all-zero row gets s_x = 1.  It also writes xsum[g][m] = sum of xq[m][k] over group g
 * (the GEMM needs it for the weights' zero points).  Non-finite activations are unspecified.
 *   x_fp16  device, fp16 [M][K], 16-byte aligned            (read)
 *   xq      device, int8 [M][K], 16-byte aligned            (written)
 *   sx      device, f32 [M]                                 (written)
 *   xsum    device, int32 [K/128][M]  (group-major)         (written)
 * M >= 0 (M = 0 launches nothing), K a positive multiple of 128.
 *
 * fq_linear_w8a8: y[m][n] = fp16( s_x[m] * sum_g s[n][g] * sum_{k in g} xq[m][k] (q[n][k] - z[n][g]) )
 * with q, s, z the layer's 8-bit copy (FQ_ERR_NOT_ATTACHED without one): the products and the
 * sums inside a group are exact integers, groups are accumulated in binary32.  xq, sx, xsum
 * as written by fq_quantize_act for the same M and the layer's K.  For a layer created with group = K
 * the sum over g is one term: the whole row is summed exactly in int32 and scaled once,
 * y[m][n] = fp16( s_x[m] * (s[n] * float( sum_k xq[m][k] (q[n][k] - z[n]) )) ).
 *   y_fp16  device, fp16 [M][N], 2-byte aligned             (written)
 * M >= 1.
 */
int fq_quantize_act(const void *x_fp16, int M, int K, void *xq, float *sx, int32_t *xsum,
                    void *stream);
int fq_linear_w8a8(const fq_layer *layer, const void *xq, const float *sx, const int32_t *xsum,
                   int M, void *y_fp16, void *stream);

/*
 * Per row r of [R][V] fp32 logits (natural logarithm, 0 log 0 = 0):
 *   entropy_out[r] = - sum_i p_i ln p_i,           p = softmax(logits_p[r])
 *   kl_out[r]      =   sum_i p_i (ln p_i - ln q_i), q = softmax(logits_q[r])
 * logits_q and kl_out may both be NULL (entropy only).  One pass over the
 * inputs.  -inf entries carry no mass; +inf and NaN are unspecified.
 *   logits_p, logits_q  device, f32 [R][V]     (read)
 *   entropy_out, kl_out device, f32 [R]        (written)
 * R >= 0 (R = 0 launches nothing), V >= 1.  Calls with R <= 64 combine per-row
 * partials in a small device-resident scratch of the library, of which every stream
 * gets a copy of its own (FQ_SCRATCH_BANKS per device; further streams take a slower path that
 * needs none): such calls may overlap on different streams.  A launch captured into a
 * graph keeps the copy of the stream it was captured on.
 */
int fq_entropy_kl(const float *logits_p, const float *logits_q, int R, int V,
                  float *entropy_out, float *kl_out, void *stream);

/*
 * The same reduction over binary16 logits (each widened exactly to binary32 first), e.g. the
 * fp16 output rows that fq_linear writes: the offline KL analysis of Sec. 3.1 / 4.3 compares
 * what a layer produces at two bit-widths.
 *   logits_p, logits_q  device, fp16 [R][V]    (read)
 * Everything else as fq_entropy_kl.
 */
int fq_entropy_kl_f16(const void *logits_p, const void *logits_q, int R, int V,
                      float *entropy_out, float *kl_out, void *stream);

/*
 * Replacement order of Sec. 4.3: linear layers with the smaller KL divergence are replaced
 * first.  The key of entry e is the sum of values[e][0..m) in double, in index order (m
 * calibration rows per entry); order[i] = the entry with the i-th smallest key, equal keys
 * in index order, NaN keys last.  `order` is what fq_sched_init takes as ev_entry.
 *   values  device, f32 [n][m]   (read)
 *   order   device, int32 [n]    (written: a permutation of 0 .. n-1)
 * 0 <= n <= FQ_MAX_RANK_ENTRIES (n = 0 launches nothing), 1 <= m <= FQ_MAX_RANK_ROWS.
 * The work grows with n * n: n is the number of linears of a model.
 */
#define FQ_MAX_RANK_ENTRIES 65536
#define FQ_MAX_RANK_ROWS 4096
int fq_rank_ascending(const float *values, int n, int m, int32_t *order, void *stream);

/*
 * The output layer fused with what Alg. 1 takes from its logits in every decode step: the next
 * token (argmax) and the entropy behind PPLE (Sec. 4.2 Eq. (5); softmax as in Sec. 2.3).
 *   logits[m][v] = sum_k x[m][k] * w[v][k]   (fp16 operands, binary32 accumulation)
 *   H[m] = -sum_v p ln p, p = softmax(logits[m]);  argmax[m] = the smallest v with the largest logit
 * The logits do not pass through HBM unless asked for.  Two launches on `stream`: the weight
 * stream with per-workgroup partial results, and a one-workgroup merge.
 *   x_fp16  device, fp16 [M][K], 16-byte aligned      (read)
 *   w_fp16  device, fp16 [V][K], 16-byte aligned      (read; the fp16 output-layer weight)
 *   logits  device, f32 [M][V], or NULL               (written if not NULL)
 *   H       device, f32 [M]                           (written)
 *   argmax  device, int32 [M], or NULL                (written if not NULL)
 * 1 <= M <= FQ_MAX_LM_HEAD_M; K a multiple of 512 with M * K <= 32768; V >= 1.  Two logits that
 * differ by less than the rounding of a binary32 sum of K products may swap places in argmax.
 * Uses a static device array for the partial results of its workgroups, of which every stream
 * gets a copy of its own, so calls may overlap on different streams; a stream beyond the first
 * FQ_SCRATCH_BANKS distinct ones on a device is refused (FQ_ERR_HIP).  A call captured into a graph keeps the copy of the
 * stream it was captured on.
 */
int fq_lm_head_entropy(const void *x_fp16, const void *w_fp16, int M, int V, int K,
                       float *logits, float *H, int32_t *argmax, void *stream);

/*
 * Token-wise precision switching on the device (Sec. 4.4, Alg. 1).  Per generated token:
 * PPLE = exp(entropy) enters a sliding window of `window` tokens (20 in the paper); when
 * the window is full and its average is below `thre`, the next `per_trigger` events of
 * the replacement order are applied -- event i sets bits[ev_entry[i]] = ev_bits[i]
 * (ascending offline KL for INT8 -> INT4, Sec. 4.3; a FP16 -> INT8 -> INT4 ladder is a
 * longer list) -- and the window is emptied, so the next judgement only sees tokens
 * generated at the new precision.  `bits` is the array a plan reads (fq_plan_run), so
 * the decode loop needs no host round trip.  All arithmetic in double.
 *   state      device, fq_sched_state_bytes(window) bytes, 8-byte aligned, owned by the
 *              caller, written by fq_sched_init and updated by every step
 *   ev_entry, ev_bits  device, int32 [n_events]   (read; must outlive the state's use)
 *   bits       device, int32 [entries]            (updated in place)
 *   entries    length of `bits`: an event whose entry is outside 0 .. entries - 1, or whose
 *              bit-width is not 2, 3, 4, 8 or 16, is passed over when its turn comes
 *   ev_token   device, int32 [n_events] or NULL   (written: index of the token at which
 *              each event fired; -2 for an event that was passed over)
 *   entropy    device, f32: one value (fq_sched_step: the entropy of this token's logits, as
 *              written by fq_entropy_kl) or [R] (fq_sched_threshold_from_prefill, which sets
 *              thre to the mean PPLE of the last min(last_n, R) of R prefill positions)
 * 1 <= window <= 1024, per_trigger >= 1, n_events >= 0.  fq_sched_peek waits for `stream`
 * and copies the counters back (any output may be NULL).
 */
size_t fq_sched_state_bytes(int window);
int fq_sched_init(void *state, int window, double thre, int per_trigger,
                  const int32_t *ev_entry, const int32_t *ev_bits, int n_events,
                  int32_t *bits, int entries, int32_t *ev_token, void *stream);
int fq_sched_threshold_from_prefill(void *state, const float *entropy, int R, int last_n,
                                    void *stream);
int fq_sched_step(void *state, const float *entropy, void *stream);
int fq_sched_peek(const void *state, int *next_event, int *tokens, double *thre,
                  double *last_mean, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FLEXQ_H */
