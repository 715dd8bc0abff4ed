/*
 * sste.h -- C ABI of the S-STE 2:4 sparse linear-layer hot path for AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels, the per-layer work of one S-STE training
 * iteration (arXiv 2409.09099):
 *   Sec. 4   S(W) = beta * S_soft(W): the 2:4 soft-threshold projection with a frozen per-tensor scale,
 *   Sec. 5.1 Z = X S(W)^T (forward) and grad_W = MVUE(grad_Z^T) X (weight gradient),
 *   Sec. 5.2 optionally with FP8 (OCP e4m3fn) operands and per-tensor scales.
 *
 * Conventions shared by every entry point
 *   - All matrices are row-major.  W is O x I (out x in), X is T x I, Z and dY are T x O, dW is O x I.
 *     Groups of four lie along the contraction axis: along I for W, along T (tokens) for dY.
 *   - Every data pointer is DEVICE memory owned by the caller (any HIP allocation, e.g. a PyTorch
 *     tensor).  The library never allocates, frees or retains device memory.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call only
 *     enqueues kernels on that stream and returns; it never synchronises.
 *   - The return value is an sste_status.  Arguments are validated on the host before anything is
 *     launched; on error nothing has been enqueued and sste_last_error() describes the reason.
 *   - Leading dimensions (ld*) are in elements.  Base pointers and row starts must be 16-byte
 *     aligned, hence ld* must be a multiple of 8 (bf16, 2-byte) / 16 (e4m3, 1-byte) / 4 (float).
 *   - Inputs must be finite.  The order used by the projection treats the 15-bit magnitude field of a
 *     bf16 as an unsigned integer, so it is total even for NaN patterns; nothing else is specified
 *     for non-finite inputs.
 *
 * Packed 2:4 operand ("vals" + "meta"), the format produced by sste_project_pack and
 * sste_mvue_materialize and consumed by sste_linear_fwd.  For an operand with R rows and K dense
 * columns (groups of 4 along K), each group contributes its two recorded values in ascending position
 * order and one nibble pos0 | pos1 << 2 (pos0 < pos1 in 0..3).  Both are stored blocked, in the order
 * the gfx950 sparse matrix instruction consumes them.  Let KS = 64 (bf16) / 128 (e4m3) dense columns
 * per instruction step, S = K / KS steps, RB = ceil(R / 16) row blocks:
 *   vals : RB * S blocks of 1024 bytes, block (rb, s) at byte offset (rb * S + s) * 1024.  A block holds
 *          64 slots of 16 bytes; slot 16 * q + j (q in 0..3, j in 0..15) holds the recorded values of row
 *          16 * rb + j for dense columns [KS * s + KS/4 * q, KS * s + KS/4 * (q + 1)): 8 bf16 / 16 e4m3.
 *   meta : RB * S blocks of 128 (bf16) / 256 (e4m3) bytes in the same block order; slot 16 * q + j holds
 *          2 / 4 bytes: the nibbles of that slot's 4 / 8 groups, group g at bits 4g.
 * Rows R .. 16 * RB - 1 are padding (sste_project_pack writes them as all-zero rows: values 0, nibbles
 * 0 | 1 << 2).  Buffer sizes:
 * vals 16 * RB * K / 2 elements, meta 16 * RB * K / 8 bytes.
 */
#ifndef SSTE_H
#define SSTE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SSTE_OK = 0,
  SSTE_ERR_NULL = 1,        /* a required pointer is NULL */
  SSTE_ERR_SHAPE = 2,       /* negative size, or a size the method itself does not allow */
  SSTE_ERR_ALIGN = 3,       /* pointer or leading dimension breaks the 16-byte rule */
  SSTE_ERR_DTYPE = 4,       /* unknown or inconsistent element type */
  SSTE_ERR_VALUE = 5,       /* beta / scale not finite or not > 0 */
  SSTE_ERR_WORKSPACE = 6,   /* workspace NULL or too small */
  SSTE_ERR_UNSUPPORTED = 7, /* valid problem, but no kernel covers this shape */
  SSTE_ERR_HIP = 8          /* the HIP runtime refused a launch */
} sste_status;

typedef enum {
  SSTE_BF16 = 0,   /* bfloat16 */
  SSTE_F8E4M3 = 1, /* OCP FP8 e4m3fn: bias 7, max 448, no infinity */
  SSTE_F32 = 2,    /* float32: accepted only where an argument's description says so */
  SSTE_F8E5M2 = 3  /* OCP FP8 e5m2 output gradients (the backward format of Sec. 5.2), accepted as `dtype` by
                      sste_linear_wgrad, sste_linear_dgrad and sste_mvue_materialize only: dY (and the
                      sparsified operand made from it) is e5m2, bias 15, max 57344, inputs finite; the
                      other operand of the call (X, or the packed weight) is SSTE_F8E4M3.  Sizes and
                      alignment follow SSTE_F8E4M3. */
} sste_dtype;

/*
 * Projection + scale + pack (Sec. 4.1 displayed definition of S_soft; Sec. 4.2 fixed scale beta).
 *
 * For every group a of four consecutive elements of a row of W: t = third-largest magnitude;
 * the two largest magnitudes are recorded, each as beta * (a_i - t) or beta * (a_i + t) by its sign.
 * Ties: rank by magnitude descending, then index ascending; ranks 0 and 1 are recorded (the values
 * do not depend on the tie-break, only the recorded positions do).  A recorded element whose
 * magnitude equals t is stored as +0.
 * Rounding: sd = a -/+ t and p = sd * beta are single float32 operations; bf16 values store
 * RNE_bf16(p); e4m3 values store RNE_e4m3(clamp(p / val_scale, +-448)) with a true float32 division.
 *
 *   W         in   device, bf16, O x I, leading dimension ldw (>= I, multiple of 8)
 *   O, I      in   O >= 0; I >= 0, a multiple of 4 (whole groups) and of the step KS of val_dtype
 *   beta      in   frozen per-tensor scale, finite and > 0
 *   val_dtype in   SSTE_BF16 or SSTE_F8E4M3: element type of `vals`
 *   val_scale in   finite and > 0; must be 1 for SSTE_BF16
 *   vals      out  device, packed values: 16 * ceil(O/16) * I/2 elements of val_dtype (format above)
 *   meta      out  device, packed position bits: 16 * ceil(O/16) * I/8 bytes
 *   amax_out  out  device float* or NULL.  If given, receives max |p| over all recorded values
 *                  (before division by val_scale and storage rounding); 0 for an empty matrix.
 * Errors: NULL -> ERR_NULL (W/vals/meta may be NULL only if O*I == 0); bad sizes -> ERR_SHAPE; I not a
 * multiple of KS -> ERR_UNSUPPORTED; misalignment -> ERR_ALIGN; bad beta/scale -> ERR_VALUE; bad dtype ->
 * ERR_DTYPE.
 */
int sste_project_pack(const void* W, int64_t O, int64_t I, int64_t ldw, float beta,
                      int val_dtype, float val_scale,
                      void* vals, void* meta, float* amax_out, void* hip_stream);

/*
 * sste_project_pack with the threshold of Sec. 4.1 "Choosing optimal threshold": any t between the
 * third-largest magnitude m3 and the second-largest m2 of a group is feasible; t = m3 + gamma * (m2 - m3)
 * (three float32 operations; the paper's interpolation with gamma = 0 giving its t = |t_2|, larger gamma
 * moving t towards the second-largest magnitude and shrinking S_soft).  gamma = 0 is the method and is
 * sste_project_pack bit for bit; gamma in (0, 1] reproduces the paper's ablation (its Table 3).  The
 * recorded positions do not depend on gamma.  gamma outside [0, 1] (or NaN) -> ERR_VALUE.
 */
int sste_project_pack_gamma(const void* W, int64_t O, int64_t I, int64_t ldw, float beta, float gamma,
                            int val_dtype, float val_scale,
                            void* vals, void* meta, float* amax_out, void* hip_stream);

/*
 * Projection + scale + pack of MANY weight tensors in one launch (the per-iteration re-projection of
 * every sparse layer of a model, Sec. 4: S(W) is recomputed from the dense weights in every iteration).
 * Single layers are small enough that a launch per tensor is dominated by launch latency; one grid
 * over all tensors streams at memory bandwidth.  The arithmetic, the rounding and the packed format of
 * every tensor are exactly those of sste_project_pack.
 *
 * Two calls, so that the launch itself touches no host memory and allocates nothing:
 *   sste_project_pack_batch_prepare  (host only) validates the items and writes a table of
 *       n_items * SSTE_PACK_TABLE_ITEM_BYTES bytes into HOST memory `table_host`, and the total number
 *       of 16-row x one-step blocks into *total_blocks_out.  The caller copies the table to device
 *       memory (16-byte aligned) once; it stays valid as long as the pointers and shapes do.
 *   sste_project_pack_batch  enqueues one kernel that processes all items of the DEVICE copy of the
 *       table.  n_items, total_blocks and val_dtype must be the values given to / returned by prepare.
 *
 *   items     in   host array; per item: W (device, bf16, O x I, leading dimension ldw), vals and meta
 *                  (device, sized as for sste_project_pack), O, I, ldw, beta, val_scale -- each with the
 *                  meaning and the constraints of the same-named argument of sste_project_pack.
 *                  Items with O * I == 0 are allowed and produce nothing.
 * Errors (prepare): as sste_project_pack, reported for the first offending item; n_items < 0 -> ERR_SHAPE.
 * Errors (launch): NULL table with n_items > 0 -> ERR_NULL; misaligned table -> ERR_ALIGN; negative
 * counts -> ERR_SHAPE; bad dtype -> ERR_DTYPE.  The table's contents are not re-validated.
 */
typedef struct sste_pack_item {
  const void* W;
  void* vals;
  void* meta;
  int64_t O, I, ldw;
  float beta;
  float val_scale;
} sste_pack_item;

#define SSTE_PACK_TABLE_ITEM_BYTES 64

int sste_project_pack_batch_prepare(const sste_pack_item* items, int n_items, int val_dtype,
                                    void* table_host, int64_t* total_blocks_out);
int sste_project_pack_batch(const void* table_device, int n_items, int64_t total_blocks, int val_dtype,
                            void* hip_stream);

/*
 * Dense-weight update fused with the projection of the updated weight (Sec. 2: each iteration prunes
 * the dense weight, takes the gradient at the sparse weight and updates the DENSE weight with it,
 * Eq. (7): w_{k+1} = w_k - alpha_k * g_k; Sec. 4: the pruning is S(w) = beta * S_soft(w)).
 * One pass over W: reads W and G, writes W back in place and writes the packed S(W_{k+1}), instead of
 * an update pass followed by sste_project_pack.
 *
 * Rounding: step = alpha * g and w' = w - step are single float32 operations (no fused multiply-add).
 * w_dtype SSTE_BF16: W stores RNE_bf16(w') and the projection reads that.  w_dtype SSTE_F32: W stores
 * w' and the projection reads RNE_bf16(w').  From there on the arithmetic and the packed format are
 * exactly those of sste_project_pack.
 *
 *   W         in/out device, bf16 or float32 (w_dtype), O x I, leading dimension ldw (>= I; a multiple
 *                    of 8 for bf16, of 4 for float32); updated in place
 *   w_dtype   in     SSTE_BF16 or SSTE_F32
 *   G         in     device, float32, O x I, leading dimension ldg (>= I, multiple of 4): the weight
 *                    gradient as sste_linear_wgrad writes it; must not overlap W
 *   alpha     in     learning rate, finite (any sign; 0 re-projects W unchanged)
 *   beta, val_dtype, val_scale, vals, meta, O, I: as for sste_project_pack
 * Errors: as sste_project_pack; bad w_dtype -> ERR_DTYPE; non-finite alpha -> ERR_VALUE; NULL G with
 * O * I > 0 -> ERR_NULL; G or W not 16-byte aligned, bad ldw / ldg -> ERR_ALIGN / ERR_SHAPE.
 */
int sste_sgd_project_pack(void* W, int w_dtype, int64_t O, int64_t I, int64_t ldw,
                          const float* G, int64_t ldg, float alpha, float beta,
                          int val_dtype, float val_scale, void* vals, void* meta, void* hip_stream);

/*
 * The same update + projection + pack for MANY weight tensors in one launch (every sparse layer of a
 * model once per iteration), arranged like sste_project_pack_batch: prepare validates on the host and
 * writes a table for the caller to copy to the device once; the launch reads only the device table.
 * The learning rate alpha is an argument of the launch, since it changes from iteration to iteration.
 * All tensors of one table share w_dtype and val_dtype.  Per tensor the result is exactly that of
 * sste_sgd_project_pack.
 *
 *   items     in   host array; per item W, G, vals, meta (device), O, I, ldw, ldg, beta, val_scale, each
 *                  as the same-named argument of sste_sgd_project_pack.  Empty items produce nothing.
 *   table_host     HOST memory of n_items * SSTE_UPDATE_TABLE_ITEM_BYTES bytes
 *   table_device   the caller's DEVICE copy of it, 16-byte aligned
 * Errors (prepare): as sste_sgd_project_pack, for the first offending item.  Errors (launch): NULL or
 * misaligned table, negative counts, bad dtypes, non-finite alpha.  The table's contents are not
 * re-validated.
 */
typedef struct sste_update_item {
  void* W;
  const float* G;
  void* vals;
  void* meta;
  int64_t O, I, ldw, ldg;
  float beta;
  float val_scale;
} sste_update_item;

#define SSTE_UPDATE_TABLE_ITEM_BYTES 80

int sste_sgd_project_pack_batch_prepare(const sste_update_item* items, int n_items, int w_dtype, int val_dtype,
                                        void* table_host, int64_t* total_blocks_out);
int sste_sgd_project_pack_batch(const void* table_device, int n_items, int64_t total_blocks, int w_dtype,
                                int val_dtype, float alpha, void* hip_stream);

/*
 * Forward GEMM with a 2:4-sparse weight operand (Sec. 5.1: Z_l = X_l S(W_l)^T).
 *
 *   Z = (x_scale * w_scale) * X * decode(vals, meta)^T,  float32 accumulation, Z stored as bf16 (RNE).
 *
 *   X        in   device, T x I of `dtype`, leading dimension ldx
 *   T, I, O  in   T >= 0; O >= 0 and a multiple of 8; I a multiple of 64 (bf16) / 128 (e4m3)
 *   dtype    in   element type of X and of vals (both operands share it)
 *   x_scale, w_scale  in  finite, > 0: dequantisation scales (1 for bf16 operands in the paper's setting)
 *   vals, meta  in   packed S(W) (R = O rows, K = I columns) as written by sste_project_pack
 *   Z        out  device, T x O bf16, leading dimension ldz (multiple of 8)
 * Metadata nibbles are trusted to be well formed (pos0 != pos1); malformed ones give an unspecified
 * but memory-safe result.
 */
int sste_linear_fwd(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float x_scale,
                    const void* vals, const void* meta, int64_t O, float w_scale,
                    void* Z, int64_t ldz, void* hip_stream);

/*
 * sste_linear_fwd with a choice of output format and the output's largest magnitude (Sec. 5.2: the
 * operands of the FP8 GEMMs are rescaled per tensor before the cast; the output of one layer is an
 * operand of the next, so casting it where it is produced saves a pass over it).
 *
 *   z_dtype SSTE_BF16  : Z = RNE_bf16((x_scale * w_scale) * acc); z_scale must be 1; amax_out optional.
 *   z_dtype SSTE_F8E4M3: Z = RNE_e4m3(clamp(acc * q, +-448)) with q = (x_scale * w_scale) / z_scale formed
 *                        in float32 on the host (one product, one division); the consumer reads Z with
 *                        scale z_scale.  O and ldz multiples of 16.  amax_out is required.
 *   amax_out           : device float* or NULL; receives max |acc| * (x_scale * w_scale), the largest
 *                        magnitude of the unrounded output in real units (0 for an empty output), from
 *                        which the caller derives z_scale of a later iteration (delayed scaling: the
 *                        scale used now comes from earlier iterations, see sste_amax_history_push).
 * acc is the float32 accumulator of the product.  Everything else as sste_linear_fwd.
 */
int sste_linear_fwd_ex(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float x_scale,
                       const void* vals, const void* meta, int64_t O, float w_scale,
                       void* Z, int64_t ldz, int z_dtype, float z_scale, float* amax_out, void* hip_stream);

/*
 * The feed-forward block (Sec. 6: S-STE sparsifies the two linear layers of every FFN block; Appendix
 * "Acceleration" times that block): fc1 -> activation -> fc2.  Two calls fuse the activation into the
 * GEMM that touches its tensor anyway, so neither the activation nor its backward costs a pass over
 * the T x 4d tensor:
 *
 *   sste_linear_fwd_act   H = RNE_bf16((x_scale * w_scale) * acc)   the pre-activation (stored if H != NULL:
 *                                                                    training needs it for the backward pass)
 *                         A = act(H)                                 evaluated in float32 on the bf16 H,
 *                         stored as RNE_bf16(A) (a_dtype SSTE_BF16, a_scale 1, amax_out NULL) or as
 *                         RNE_e4m3(clamp(A * (1 / a_scale), +-448)) with 1 / a_scale one float32 division
 *                         on the host (a_dtype SSTE_F8E4M3; amax_out required, receives max |A|).
 *   sste_linear_dgrad_act dX = RNE_bf16(g * act'(H)),  g = RNE_bf16((dy_scale * w_scale) * acc): the input
 *                         gradient of the layer AFTER the activation, multiplied by the activation's
 *                         derivative at the stored pre-activation H (T x I, bf16, leading dimension ldh).
 *                         act = SSTE_ACT_NONE is sste_linear_dgrad.
 *
 * act: SSTE_ACT_GELU_TANH, 0.5 h (1 + tanh(sqrt(2 / pi) (h + 0.044715 h^3))) -- the paper does not name the
 * activation; this is the one of the GPT-2 models whose layer shapes its experiments use.  Its derivative
 * is the analytic one.  float32 arithmetic with the hardware's exp2 / reciprocal (about 1e-6 absolute).
 * Everything not listed is as in sste_linear_fwd / sste_linear_dgrad (A takes the role of Z: T x O, lda).
 */
enum { SSTE_ACT_NONE = 0, SSTE_ACT_GELU_TANH = 1 };
int sste_linear_fwd_act(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float x_scale,
                        const void* vals, const void* meta, int64_t O, float w_scale,
                        int act, void* H, int64_t ldh, void* A, int64_t lda, int a_dtype, float a_scale,
                        float* amax_out, void* hip_stream);
int sste_linear_dgrad_act(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale,
                          const void* vals, const void* meta, int64_t I, float w_scale,
                          int act, const void* H, int64_t ldh, void* dX, int64_t lddx, void* hip_stream);

/*
 * Delayed scaling (the per-tensor scaling recipe Sec. 5.2 refers to): the scale of an 8-bit tensor in
 * iteration k is derived from the largest magnitudes seen in the last `length` iterations, so no pass
 * over the tensor is needed before it is cast.  Host-only helper; the caller owns the struct.
 *   sste_amax_history_init  empties the window (length clamped to 1 .. SSTE_AMAX_HISTORY_MAX).
 *   sste_amax_history_push  records `amax` (a finite value >= 0 read back from an amax_out; anything else
 *                           is ignored) and returns the scale to use next: max(window) / format_max, or 1
 *                           while the window holds only zeros.  format_max: 448 (e4m3) / 57344 (e5m2).
 */
#define SSTE_AMAX_HISTORY_MAX 64
typedef struct sste_amax_history {
  float window[SSTE_AMAX_HISTORY_MAX];
  int length;
  int next;
} sste_amax_history;
void sste_amax_history_init(sste_amax_history* h, int length);
float sste_amax_history_push(sste_amax_history* h, float amax, float format_max);

/*
 * Weight-gradient GEMM with the output gradient sparsified 2:4 by the minimum-variance unbiased
 * estimator (Sec. 5.1: grad_W = MVUE(grad_Z^T) X).
 *
 * Which kernels run: problems with T >= 2048, O >= 256 and I >= 256 (every layer of the GPT-2 workloads)
 * sparsify dY ONCE into the workspace (a packed 2:4 operand in the format above, rows = channels,
 * columns = tokens), run a sparse GEMM on it that is split over the token axis, and sum the splits in a
 * fixed order.  Smaller problems sparsify inside the GEMM's operand load (one kernel, the workspace only
 * holds split partial sums, if any).  The result is the same function of (dY, X, seed, offset) on
 * either path.
 *
 *   dW (+)= scale * MVUE(dY^T; seed, offset) * X,   scale = dy_scale * x_scale (times 2 for the 8-bit
 *   formats, whose sparsified operand is stored halved), float32 accumulation, dW float32.
 *
 * The estimator works on groups of four consecutive tokens t = 4k..4k+3 of one output channel o.
 * Its uniform number is a pure function of (seed, offset, group id = k * O + o), so the result does
 * not depend on tiling or on how the token axis is split.  See sste_mvue_materialize for the rule.
 *
 *   dtype    in   SSTE_BF16, SSTE_F8E4M3, or SSTE_F8E5M2 (dY e5m2, X e4m3: the formats of Sec. 5.2)
 *   dY       in   device, T x O of `dtype`, leading dimension lddy
 *   X        in   device, T x I of `dtype` (e4m3 when dtype is SSTE_F8E5M2), leading dimension ldx
 *   T, O, I  in   T a multiple of 64 (bf16) / 128 (8-bit); O, I >= 0 and multiples of 8 (bf16) / 16 (8-bit)
 *   seed, offset  in  random stream id (e.g. layer seed, training step)
 *   dW       out  device, O x I float32, leading dimension lddw (multiple of 4)
 *   accumulate in 0: dW is overwritten; 1: the product is added to dW
 *   workspace     device scratch of at least sste_wgrad_workspace_bytes(T, O, I, dtype) bytes, 16-byte
 *                 aligned.  Large problems keep the sparsified operand there (packed, about 0.56 x the
 *                 bytes of dY) next to the partial sums of the token-axis splits, which are reduced in
 *                 a fixed order, so the result is bitwise reproducible from run to run.  May be NULL
 *                 when that size is 0.
 */
int sste_linear_wgrad(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale,
                      const void* X, int64_t I, int64_t ldx, float x_scale,
                      uint64_t seed, uint64_t offset,
                      float* dW, int64_t lddw, int accumulate,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * sste_linear_wgrad for a SHARD of the token axis (data parallelism over tokens: every GPU holds a
 * slice of the batch).  `first_token` is the global index of row 0 of dY and X, a multiple of 4; the
 * estimator's group id becomes ((first_token + t) / 4) * O + o, so the shards of a batch draw exactly
 * the numbers the whole batch would draw and the sum of their results does not depend on how the
 * batch was cut.  first_token = 0 is sste_linear_wgrad.  first_token < 0 or not a multiple of 4 ->
 * ERR_SHAPE; group ids beyond 64 bits -> ERR_UNSUPPORTED.
 */
int sste_linear_wgrad_at(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale,
                         const void* X, int64_t I, int64_t ldx, float x_scale,
                         uint64_t seed, uint64_t offset, int64_t first_token,
                         float* dW, int64_t lddw, int accumulate,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * sste_linear_wgrad for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit-identical results; the scratch that sste_linear_wgrad takes as
 * `workspace` is an array of SSTE_NOALLOC_SCRATCH_BYTES bytes inside the library's own device image
 * (each GPU the library runs on holds its copy until the process ends).  The call allocates nothing and
 * frees nothing; on its first use on a device it asks the runtime once for the array's address there.
 * Problems whose sste_wgrad_workspace_bytes() exceeds SSTE_NOALLOC_SCRATCH_BYTES are refused with
 * SSTE_ERR_WORKSPACE before anything is launched (64 MiB covers the 3072 x 768 layer at 8192 tokens;
 * larger layers need sste_linear_wgrad with a caller-owned workspace).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams, or different threads) race; calls on one stream are ordered and safe.  Nothing in the array
 * has to start at zero (every byte a call reads it has written before), so the previous call's contents,
 * of any size, do no harm.
 */
#define SSTE_NOALLOC_SCRATCH_BYTES (64u << 20)
int sste_linear_wgrad_noalloc(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale,
                              const void* X, int64_t I, int64_t ldx, float x_scale,
                              uint64_t seed, uint64_t offset,
                              float* dW, int64_t lddw, int accumulate, void* hip_stream);

/*
 * Input gradient (Sec. 5.1: grad_X_l = grad_Z_l S(W_l); the paper keeps this product dense).
 *
 *   dX = (dy_scale * w_scale) * dY * decode(vals, meta),  float32 accumulation, dX stored as bf16 (RNE).
 *
 *   dY       in   device, T x O of `dtype`, leading dimension lddy
 *   T, O, I  in   T >= 0; O >= 0 and a multiple of 8 (bf16) / 16 (e4m3); I a multiple of 64 / 128
 *   dtype    in   SSTE_BF16 or SSTE_F8E4M3: element type of dY and of vals (per-tensor scales, Sec. 5.2);
 *                 SSTE_F8E5M2: dY is e5m2, vals e4m3
 *   dy_scale, w_scale  in  finite, > 0
 *   vals, meta  in   packed S(W) (R = O rows, K = I columns) as written by sste_project_pack; rows past O
 *                    up to the next multiple of 16 must be the padding that call writes
 *   dX       out  device, T x I bf16, leading dimension lddx (multiple of 8); O == 0 gives zeros
 * The packed weight is expanded to dense-with-zeros on its way into on-chip memory; nothing is
 * written besides dX.
 * Errors: as sste_linear_fwd, with the roles of X / Z taken by dY / dX.
 */
int sste_linear_dgrad(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale,
                      const void* vals, const void* meta, int64_t I, float w_scale,
                      void* dX, int64_t lddx, void* hip_stream);

/* Bytes of scratch sste_linear_wgrad needs for this problem (0 if it needs none; 0 on bad arguments). */
size_t sste_wgrad_workspace_bytes(int64_t T, int64_t O, int64_t I, int dtype);

/*
 * For tests and tuning: fixes the workgroup tile and the number of token-axis splits of the large-problem
 * weight-gradient GEMM instead of letting the library choose them per problem.  (mi, ni) is one of
 * (8, 4) = 256 channels x 256 features, (6, 3) = 192 x 192, (8, 3) = 256 x 192, or (0, 0) = automatic;
 * splits is 1..32 (capped by the problem), or 0 = automatic.  Process-wide, takes effect for the calls
 * that follow (sste_wgrad_workspace_bytes included, which must be asked again); results stay exact to
 * the same tolerance for every choice.  Other values -> SSTE_ERR_VALUE, nothing changes.
 */
int sste_wgrad_plan_override(int mi, int ni, int splits);

/*
 * The estimator of sste_linear_wgrad written out as a packed 2:4 operand (same device function).
 * Used to check the sparsifier bit for bit; also usable as a stand-alone pre-pass.
 *
 * Rule for a group g (Sec. 5.1 names the estimator; the sampling scheme is this library's):
 *   m_i = |g_i| in float32; Lo = (min(m0,m1) + min(m2,m3)) + min(max(m0,m1), max(m2,m3));
 *   clamp = Lo == 0 ? max m : Lo; l_i = min(m_i, clamp); P0 = l0, P1 = P0 + l1, P2 = P1 + l2,
 *   L = P2 + l3, h = L / 2; u = (x >> 8) * 2^-24 with x the 32-bit draw below; tau0 = u * h,
 *   tau1 = tau0 + h; i(tau) = #{k : P_k <= tau}; pos0 = min(i(tau0), 2), pos1 = min(3, max(i(tau1), pos0 + 1)).
 *   Recorded value at p: g_p itself if m_p > h or m_p == 0, else sign(g_p) * h (h rounded to the
 *   storage type).  e4m3 and e5m2 store half of these values.
 *   Draw: key = mix64(seed ^ mix64(offset + 0x9E3779B97F4A7C15)) (SplitMix64 finalizer), k0 = low,
 *   k1 = high word; x = (gid & 0xFFFFFFFF) ^ k0; x += (gid >> 32) * 0x9E3779B9; x ^= x >> 17;
 *   x *= 0xED5AD4BB; x += k1; x ^= x >> 11; x *= 0xAC4C1B51; x ^= x >> 15; x *= 0x31848BAB; x ^= x >> 14.
 *
 *   dY    in   device, T x O of `dtype` (SSTE_BF16, SSTE_F8E4M3 or SSTE_F8E5M2), leading dimension lddy;
 *              T a multiple of 64 (bf16) / 128 (8-bit)
 *   O     a multiple of 8 (bf16) / 16 (8-bit); lddy likewise; dY 16-byte aligned (the kernel reads whole
 *              16-byte pieces of a token row)
 *   vals, meta  out  device, packed format above with R = O rows and K = T columns.  Rows O .. 16 RB - 1
 *              of the last row block are written as all-zero rows (values 0; their position bits are
 *              those the estimator gives an all-zero group, 2 | 3 << 2)
 */
int sste_mvue_materialize(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype,
                          uint64_t seed, uint64_t offset, void* vals, void* meta, void* hip_stream);

/* sste_mvue_materialize for a shard of the token axis: `first_token` as in sste_linear_wgrad_at. */
int sste_mvue_materialize_at(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype,
                             uint64_t seed, uint64_t offset, int64_t first_token,
                             void* vals, void* meta, void* hip_stream);

/*
 * MSE-optimal scale of Sec. 4.2: beta = <W, S_soft(W)> / ||S_soft(W)||^2, computed once from the
 * initial weights and then frozen by the caller.  Products are formed in float32 and summed in
 * float64 in a fixed order (reproducible).
 *
 *   W          in   device, bf16, O x I, leading dimension ldw
 *   beta_out   out  device float*; receives beta, or NaN if S_soft(W) is identically zero
 *   workspace       device scratch of at least sste_beta_workspace_bytes(O, I) bytes, 16-byte aligned
 */
int sste_compute_beta(const void* W, int64_t O, int64_t I, int64_t ldw, float* beta_out,
                      void* workspace, size_t workspace_bytes, void* hip_stream);
size_t sste_beta_workspace_bytes(int64_t O, int64_t I);

/*
 * The scales Sec. 4.2 compares (its Table 4), for a threshold parameter gamma as in sste_project_pack_gamma:
 *   SSTE_BETA_MSE  beta = <W, S_soft(W)> / ||S_soft(W)||^2      (the method; with gamma = 0 this is sste_compute_beta)
 *   SSTE_BETA_L1   beta = ||W||_1 / ||S_soft(W)||_1             (keeps the total magnitude; the variant the paper rejects)
 * Same arguments, workspace and reproducibility as sste_compute_beta; unknown kind or gamma outside [0, 1]
 * -> ERR_VALUE.
 */
enum { SSTE_BETA_MSE = 0, SSTE_BETA_L1 = 1 };
int sste_compute_beta_ex(const void* W, int64_t O, int64_t I, int64_t ldw, int kind, float gamma, float* beta_out,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Per-tensor rescaling and cast of a bf16 tensor to an 8-bit operand format (Sec. 5.2: the operands of
 * the FP8 GEMMs are rescaled per tensor before they are cast; e4m3 for activations, e5m2 or e4m3 for
 * the output gradient).
 *
 *   Q[r][c] = RNE_fmt(clamp(X[r][c] / scale, +-max_fmt)),   the quotient being the IEEE float32 division
 *             (the kernel forms exactly that value; for 2^-40 <= scale <= 2^40 without a division sequence);
 *   *amax_out = max |X[r][c]| (exact, subnormal values included; 0 for an empty tensor).
 *
 * The GEMM calls then take Q with x_scale / dy_scale = scale.  A caller that scales by the current
 * tensor calls once with Q == NULL (largest magnitude only), sets scale = amax / max_fmt, and calls
 * again; one that uses the previous iteration's amax (delayed scaling) calls once.
 *
 *   X         in   device, bf16, R x C, leading dimension ldx (>= C, multiple of 8); C a multiple of 8
 *   out_dtype in   SSTE_F8E4M3 (max 448) or SSTE_F8E5M2 (max 57344)
 *   scale     in   finite and > 0
 *   Q         out  device, R x C bytes, leading dimension ldq (>= C, multiple of 8), 8-byte aligned; or NULL
 *   amax_out  out  device float* or NULL (not both Q and amax_out NULL)
 * Errors: as the other calls (ERR_SHAPE, ERR_ALIGN, ERR_DTYPE, ERR_VALUE, ERR_NULL).
 */
int sste_cast_fp8(const void* X, int64_t R, int64_t C, int64_t ldx, int out_dtype, float scale,
                  void* Q, int64_t ldq, float* amax_out, void* hip_stream);

/*
 * Flip count of Sec. 3.3 (numerator of the flip rate r_k): number of positions whose recorded /
 * not-recorded state differs between two metadata arrays of the same O x I/8 shape.
 *   count_out  out  device uint64_t*; overwritten
 */
int sste_flip_count(const void* meta_a, const void* meta_b, int64_t O, int64_t I,
                    unsigned long long* count_out, void* hip_stream);

/*
 * Per-kernel timing for benchmarks.  Between sste_timing_begin and sste_timing_end every launch of a
 * hot-path kernel is bracketed by its own pair of HIP events on the launch stream (events are host
 * objects; no device memory is allocated).  sste_timing_end waits for the recorded events, adds up
 * the elapsed milliseconds and the launch counts per kernel into arrays of SSTE_K_COUNT entries
 * (either may be NULL) and releases the events.  At most `max_launches` launches are recorded; later
 * ones run untimed.  Timing is process-wide; do not nest.
 */
typedef enum {
  SSTE_K_PROJECT_PACK = 0,   /* projection + scale + pack */
  SSTE_K_FWD = 1,            /* forward sparse GEMM */
  SSTE_K_WGRAD = 2,          /* weight-gradient sparse GEMM */
  SSTE_K_WGRAD_REDUCE = 3,   /* fixed-order reduction of the token-axis splits */
  SSTE_K_MVUE_PACK = 4,      /* estimator pre-pass of the weight-gradient path (large problems) */
  SSTE_K_DGRAD = 5,          /* input-gradient dense GEMM */
  SSTE_K_SGD_PROJECT_PACK = 6, /* dense-weight update fused with projection + pack */
  SSTE_K_CAST = 7,           /* per-tensor rescale + cast to an 8-bit format */
  SSTE_K_COUNT = 8
} sste_kernel_id;
int sste_timing_begin(int max_launches);
int sste_timing_end(double* total_ms, int* launches);

/* Message for the most recent non-OK status returned on the calling thread ("" if none). */
const char* sste_last_error(void);

/* Library version: major * 10000 + minor * 100 + patch. */
int sste_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SSTE_H */
