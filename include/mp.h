/*
 * mp.h - C ABI of the MI355X (gfx950) mixed-precision training-step library.
 *
 * The calls are the steps of one mixed-precision training iteration as the
 * paper states it (Section 3.1: fp16 maths accumulated in fp32, loss scaling,
 * fp32 master weights; Section 3.2: the optimizer wrapper; Section 3.3:
 * regularisation on the fp32 copy):
 *
 *   forward  : mp_gemm_fwd[_ws] (+ mp_layernorm_fwd, mp_attention_fwd | mp_softmax_fwd,
 *              mp_lstm_cell_fwd | mp_lstm_layer_fwd)
 *   loss     : mp_mse_scaled | mp_softmax_xent_scaled[_db] (seed gradient x loss scale)
 *   backward : mp_gemm_bwd_dx[_ws], mp_gemm_bwd_dw | mp_gemm_bwd_dw_grouped (+ mp_layernorm_bwd,
 *              mp_attention_bwd | mp_softmax_bwd, mp_lstm_cell_bwd | mp_lstm_layer_bwd, mp_colsum)
 *   update   : mp_unscale_check_update   (inspect fp16 gradients, unscale, SGD/Adam on
 *                                         fp32 masters, rewrite the fp16 copies - or skip)
 *              mp_loss_scale_update      (halve / count / grow the loss scale)
 *
 * Conventions (all entry points):
 *   - Every pointer marked "device" is GPU memory owned by the caller; the library
 *     never allocates, frees or retains it.  Pointers marked "host" are read during
 *     the call only.
 *   - fp16 data is IEEE binary16 stored as uint16_t bit patterns (mp_half).  Every
 *     fp32 -> fp16 conversion is round-to-nearest-even and overflows to +-inf (never
 *     saturates): that overflow is what the loss-scale policy detects.
 *   - Matrices are row-major with an explicit leading dimension in elements.
 *   - Every call only enqueues work on `stream` (a hipStream_t passed as void*;
 *     NULL is the default stream) and returns without synchronising.  The skip
 *     decision of an overflowing step is taken on the device, so no call depends on
 *     the host reading device memory; a whole training step can be captured in a HIP
 *     graph.
 *   - Return value: MP_OK or a negative error code; mp_last_error() gives a
 *     thread-local human-readable message for the last failure on this thread.
 *     Argument errors (MP_E_INVAL, MP_E_UNSUPPORTED, MP_E_WORKSPACE) are found before
 *     anything is enqueued.  MP_E_HIP from an entry point that makes several launches
 *     (split contractions, column sums, the update over many tensors) may leave the
 *     earlier launches enqueued: treat the outputs as undefined.
 *   - The library keeps no state between calls, with two documented exceptions that are
 *     measurement aids and not part of a training step: mp_gemm_tuning_override /
 *     mp_gemm_tuning_dtl (process-wide, not thread-safe kernel choices for sweeps and
 *     tests) and mp_mfma_sustained_rate
 *     (the ONE call that blocks: it times its own launch with events).
 *   - Scratch ("workspace") is caller-provided device memory; each call that needs it
 *     has a *_workspace_bytes query.  Contents need not be initialised and are
 *     undefined afterwards.  Calls sharing one workspace must be on one stream.
 */
#ifndef MP_H_
#define MP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t mp_half;   /* IEEE binary16 bit pattern */
typedef void*    mp_stream; /* hipStream_t */

enum {
    MP_OK            = 0,
    MP_E_INVAL       = -1, /* null pointer, negative size, bad enum, misaligned pointer */
    MP_E_UNSUPPORTED = -2, /* valid request this build has no kernel for */
    MP_E_WORKSPACE   = -3, /* workspace missing or smaller than the *_workspace_bytes query */
    MP_E_HIP         = -4  /* the HIP runtime refused a launch; see mp_last_error() */
};

const char* mp_last_error(void);
int         mp_version(void);

/* ------------------------------------------------------------------------------------------
 * Loss-scale state (Section 3.1, item 1).  Lives in device memory; every kernel that needs
 * the scale, the overflow flag or the optimizer step count reads it there.
 * ------------------------------------------------------------------------------------------ */
#define MP_HISTORY 4096 /* ring length of the per-step log */

enum { MP_SCALE_STATIC = 0, MP_SCALE_BACKOFF = 1 };

typedef struct mp_scale_state {
    float   scale;           /* S used by the current iteration                               */
    float   inv_scale;       /* 1.0f / S                                                      */
    float   min_scale;
    float   max_scale;
    int32_t mode;            /* MP_SCALE_STATIC | MP_SCALE_BACKOFF                            */
    int32_t growth_interval; /* N: double S after N consecutive clean steps                   */
    int32_t good_steps;      /* consecutive clean steps since the last change of S            */
    int32_t found_inf;       /* nonzero: an inf/NaN was seen in this iteration's gradients    */
    int32_t opt_step;        /* number of optimizer steps applied (Adam's t)                  */
    int32_t total_steps;     /* iterations seen                                               */
    int32_t skipped_steps;   /* iterations skipped because of overflow                        */
    int32_t reserved;
    float   hist_scale[MP_HISTORY];     /* S used at iteration i (mod MP_HISTORY)             */
    int32_t hist_found_inf[MP_HISTORY]; /* overflow flag of iteration i (mod MP_HISTORY)      */
} mp_scale_state;

/* Fill *st (device) : S = init_scale, counters zero, log cleared.  min_scale <= init_scale <= max_scale,
 * growth_interval >= 1 else MP_E_INVAL. */
int mp_scale_state_init(mp_scale_state* st, int mode, float init_scale, int growth_interval,
                        float min_scale, float max_scale, mp_stream stream);

/* End of an iteration (Section 3.1 item 1: the gradients inspected in this iteration decide the
 * scale of the next one).  Reads st->found_inf and then, on the device:
 *   log (S, found_inf); total_steps++
 *   overflow : skipped_steps++, good_steps = 0, BACKOFF: S = max(S/2, min_scale)
 *   clean    : opt_step++, good_steps++, BACKOFF and good_steps == growth_interval:
 *              S = min(2S, max_scale), good_steps = 0
 *   inv_scale = 1/S; found_inf = 0.
 * STATIC mode never changes S (an overflowing step is still skipped and counted). */
int mp_loss_scale_update(mp_scale_state* st, mp_stream stream);

/* ------------------------------------------------------------------------------------------
 * Dense contractions (Section 3.1: fp16 operands, fp32 accumulation, result stored in fp16).
 * One descriptor serves the three calls of a linear layer  Y[M,N] = X[M,K] W[N,K]^T :
 *     fwd    : Y  = epi(alpha * X W^T)          contraction over K
 *     bwd_dx : dX = epi(alpha * dY W)           contraction over N
 *     bwd_dw : dW = alpha * dY^T X              contraction over M (tokens)
 * With trans_w != 0 the second operand is stored as W[K,N] instead (Y = X W): this is how the
 * attention products Q K^T (trans_w = 0) and P V (trans_w = 1) and their gradients use the same
 * entry points.  Batched use: batch_outer x batch_inner independent problems; operand t of batch
 * (o, i) starts at t + o*s?_outer + i*s?_inner (elements).  Strides of 0 broadcast.
 * Fast (MFMA) path needs 16-byte aligned base pointers and ld / batch strides that are multiples
 * of 8 elements; anything else runs a slow scalar kernel with the same results contract.
 * ------------------------------------------------------------------------------------------ */
enum { MP_EPI_NONE = 0, MP_EPI_BIAS = 1, MP_EPI_BIAS_RELU = 2 };

typedef struct mp_gemm_desc {
    int32_t M, N, K;          /* Y is M x N, X is M x K, W is N x K (K x N when trans_w)          */
    int32_t ldx, ldw, ldy;    /* leading dimensions of X (dX), W (dW), Y (dY), in elements        */
    int32_t batch_outer, batch_inner; /* >= 1                                                    */
    int64_t sx_outer, sx_inner;       /* batch strides of X / dX                                 */
    int64_t sw_outer, sw_inner;       /* batch strides of W / dW                                 */
    int64_t sy_outer, sy_inner;       /* batch strides of Y / dY                                 */
    float   alpha;            /* scales the fp32 accumulator before the epilogue (e.g. 1/sqrt(dk)) */
    int32_t epilogue;         /* fwd only: MP_EPI_*                                              */
    int32_t trans_w;          /* 0: W[N,K];  1: W[K,N]                                           */
    int32_t reserved;
} mp_gemm_desc;

/* Bytes of workspace mp_gemm_bwd_dw needs for this descriptor (split-K partials in fp32 and the
 * column-sum partials of db).  mp_gemm_fwd / mp_gemm_bwd_dx need none. */
size_t mp_gemm_bwd_dw_workspace_bytes(const mp_gemm_desc* desc /* host */, int with_db);

/* Y = RNE16( act( alpha * X W^T + acc_in + bias ) ).
 *   X, W, Y   device fp16.  bias[N] device fp16, required iff epilogue != MP_EPI_NONE.
 *   acc_in    device fp32 [M, N] with leading dimension N, or NULL: added to the accumulator
 *             (lets a contraction be split over two calls without an fp16 rounding between).
 *   y_f32     device fp32 [M, N] ld N, or NULL: if given, the fp32 value alpha*X W^T + acc_in
 *             is stored here instead, Y is not written, and the epilogue must be NONE.
 * Batched problems do not support acc_in / y_f32. */
int mp_gemm_fwd(const mp_gemm_desc* desc /* host */, const mp_half* X, const mp_half* W,
                const mp_half* bias, const float* acc_in, mp_half* Y, float* y_f32,
                mp_stream stream);

/* dX = RNE16( RNE16( alpha * dY W  (.) [relu_src > 0] ) + add ).
 *   relu_src  device fp16 [M, K] ld = ld_aux, or NULL: gradient of a ReLU whose stored output is
 *             relu_src (entries where relu_src <= 0 are zeroed).
 *   add       device fp16 [M, K] ld = ld_aux, or NULL: a second gradient flowing into the same
 *             tensor (residual branch); the sum is rounded once more, as if the two tensors had
 *             been stored and then added.
 * relu_src and add share ld_aux and the batch strides of dX; they may not both be given. */
int mp_gemm_bwd_dx(const mp_gemm_desc* desc /* host */, const mp_half* dY, const mp_half* W,
                   const mp_half* relu_src, const mp_half* add, int32_t ld_aux, mp_half* dX,
                   mp_stream stream);

/* mp_gemm_fwd and mp_gemm_bwd_dx with a workspace (Section 3.1 arithmetic unchanged: fp16 operands, fp32 sums, one
 * rounding).  A product with few output rows (the recurrent products of an LSTM: 32 rows) has too few output tiles
 * to occupy the chip; given a workspace such a product splits its contraction over more workgroups (fp32 partial
 * sums in ws, added in split order by a finish launch that applies scale, bias and the rounding).  Only products
 * whose epilogue is none or bias, unbatched, without relu_src / add / acc_in / y_f32, are split; all others run
 * exactly as without a workspace.  ws: device, 16-byte aligned, mp_gemm_split_workspace_bytes(desc) bytes (0: the
 * plan does not split; NULL is then fine), contents irrelevant before and after.  A workspace that is too small
 * is not an error: the product runs unsplit. */
size_t mp_gemm_split_workspace_bytes(const mp_gemm_desc* desc);
int    mp_gemm_fwd_ws(const mp_gemm_desc* desc, const mp_half* X, const mp_half* W, const mp_half* bias,
                      const float* acc_in, mp_half* Y, float* y_f32, void* ws, size_t ws_bytes, mp_stream stream);
int    mp_gemm_bwd_dx_ws(const mp_gemm_desc* desc, const mp_half* dY, const mp_half* W, const mp_half* relu_src,
                         const mp_half* add, int32_t ld_aux, mp_half* dX, void* ws, size_t ws_bytes, mp_stream stream);

/* dW = RNE16( alpha * dY^T X ) (overwrites; there is no gradient accumulation across calls) and,
 * if db != NULL, db[N] = RNE16( column sums of dY ) (unbatched only).
 *   st        device, or NULL: if given, st->found_inf is set when any value written to dW or db
 *             is inf/NaN (the gradient inspection of Section 3.1 done where the gradient is made).
 *   ws        device workspace of at least mp_gemm_bwd_dw_workspace_bytes(desc, db != NULL). */
int mp_gemm_bwd_dw(const mp_gemm_desc* desc /* host */, const mp_half* dY, const mp_half* X,
                   mp_half* dW, mp_half* db, mp_scale_state* st, void* ws, size_t ws_bytes,
                   mp_stream stream);

/* Several weight-gradient products (Section 3.1: fp16 operands, fp32 accumulation, one rounding) in one launch.
 * Each of a layer's dW = dY^T X alone has too few output tiles to occupy the chip without splitting its
 * contraction; together they do.  items: host array of `count` (1..8) problems, each a descriptor as for
 * mp_gemm_bwd_dw (same meaning of M, N, K, ldx, ldw, ldy, trans_w, alpha; no batches) with its device pointers.
 * The overflow flag of `st` (may be NULL) is set if any stored gradient is non-finite.  An item's db (device, N
 * elements, may be NULL) receives the bias gradient RNE16(fp32 column sums of dY[M, N]) from the same launch: the
 * sums are cut into 128-column strips that are handed to workgroups like tiles, each strip summed in a fixed
 * order (same results contract as mp_colsum, not the same summation order).
 * MP_E_UNSUPPORTED, with nothing launched, if an item is batched, fails the 16-byte / multiple-of-8
 * alignment rules of the fast path, or has a weight shape that is not a multiple of 128 in both dimensions or a
 * row count (M) that is not a multiple of 64: use mp_gemm_bwd_dw for those. */
typedef struct mp_gemm_group_item {
    mp_gemm_desc   desc;
    const mp_half* dY;
    const mp_half* X;
    mp_half*       dW;
    mp_half*       db;   /* may be NULL */
} mp_gemm_group_item;
int mp_gemm_bwd_dw_grouped(const mp_gemm_group_item* items, int count, mp_scale_state* st, mp_stream stream);

/* Tuning aid for sweeps and tests, process-wide and not thread-safe (the one piece of mutable library state;
 * a training step never calls it): force every following contraction onto tile shape `tile`
 * (index into the library's tile table: 0 = 256x256, 1 = 256x128, 2 = 128x256, 3 = 128x128, 4 = 128x64,
 * 5 = 64x128, 6 = 64x64, 7 = 32x128, 8 = 256x192 for products whose operands are both stored
 * contraction-contiguous, else 256x256) and, where splitting the contraction is allowed, onto `splits`
 * (0..16; 0 = 1) splits, reduced until every split owns at least one k-tile.  tile >= the table size or splits
 * outside 0..16: MP_E_INVAL.  tile < 0 restores the built-in choice.  Results do not depend on it beyond fp32
 * summation order.
 * Note that mp_gemm_bwd_dw_workspace_bytes answers for the choice in force when it is called. */
int mp_gemm_tuning_override(int tile, int splits);

/* Tuning aid of the same kind (process-wide, not thread-safe, never called by a training step): which interior,
 * unbatched, unsplit products run on the kernels whose operand tiles go from global memory straight into LDS.
 * 0 = none, 1 = weight-gradient products only (the built-in choice), 2 = every product they are built for (all three
 * operand layouts).  Same results contract either way (fp32 summation order may differ).  Other values: MP_E_INVAL. */
int mp_gemm_tuning_dtl(int mode);

/* db[cols] = RNE16( column sums (fp32) of dY[rows, cols] ); optional overflow flag as above.
 * Workspace: mp_colsum_workspace_bytes(rows, cols). */
size_t mp_colsum_workspace_bytes(int rows, int cols);
int mp_colsum(int rows, int cols, const mp_half* dY, int ld, mp_half* db, mp_scale_state* st,
              void* ws, size_t ws_bytes, mp_stream stream);

/* mp_colsum for callers that cannot allocate device memory or bring a workspace: code under HIP-graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same summation order and therefore the same
 * bits as mp_colsum; the partial sums live in a fixed 1 MiB array inside the library's device image (one copy per
 * GPU, held until the process ends) instead of a caller workspace.  The call allocates nothing (no hipMalloc /
 * hipFree, no allocating library routine); the first call on a device looks the array's device address up.
 * Limit: shapes whose mp_colsum_workspace_bytes(rows, cols) exceeds mp_colsum_static_max_bytes() (1 MiB; every
 * shape with cols <= 262144 fits) return MP_E_WORKSPACE with nothing enqueued.  All calls on one GPU share that
 * GPU's array: calls that may overlap in time on one GPU (different streams, different host threads) race on it
 * and must be serialised by the caller.  Nothing in the array has to start at zero: every partial sum a call reads
 * it has written first, so contents left by an earlier (larger) call are harmless. */
size_t mp_colsum_static_max_bytes(void);
int mp_colsum_static(int rows, int cols, const mp_half* dY, int ld, mp_half* db, mp_scale_state* st, mp_stream stream);

/* ------------------------------------------------------------------------------------------
 * Losses: fp32 loss value (unscaled mean) and the loss-scaled fp16 seed gradient
 * (Section 3.1 item 1).  S is read from st on the device.
 * ------------------------------------------------------------------------------------------ */
size_t mp_loss_workspace_bytes(int rows, int cols);

/* loss = mean (y - target)^2 over rows x cols;  dy = RNE16( float(2 S / (rows cols)) * (y - target) ).
 * y, target, dy: device fp16, common leading dimension ld.  loss: device fp32 scalar. */
int mp_mse_scaled(int rows, int cols, const mp_half* y, const mp_half* target, int ld,
                  const mp_scale_state* st, float* loss, mp_half* dy, void* ws, size_t ws_bytes,
                  mp_stream stream);

/* loss = mean over rows of (logsumexp(z) - z[target]), z = float(logits), max-subtracted, fp32;
 * dlogits = RNE16( float(S / rows) * (softmax(z) - onehot(target)) ).
 * A target outside [0, vocab) gives that row zero loss and zero gradient (the mean still divides
 * by rows).  logits / dlogits share ld; dlogits may alias logits (in-place). */
int mp_softmax_xent_scaled(int rows, int vocab, const mp_half* logits, int ld, const int32_t* targets,
                           const mp_scale_state* st, float* loss, mp_half* dlogits, void* ws,
                           size_t ws_bytes, mp_stream stream);

/* mp_softmax_xent_scaled that also returns the bias gradient of the projection behind the logits (Section 3.2: the
 * gradients are fp16 tensors): db[vocab] = RNE16( fp32 column sums over the rows of the dlogits values as stored ).
 * For vocabularies of more than 16384 classes (multiples of 8, 16-byte aligned rows) the sums are taken in the pass
 * that writes dlogits, so the gradient matrix is not read again; other shapes run the plain call followed by mp_colsum.
 * st is read for S as above; its overflow flag is set if a stored db value is non-finite (dlogits itself is bounded
 * by S / rows and is covered by whoever consumes it).  Workspace: mp_softmax_xent_db_workspace_bytes(rows, vocab),
 * 16-byte aligned.  Same results contract as the two separate calls (fp32 summation order differs). */
size_t mp_softmax_xent_db_workspace_bytes(int rows, int vocab);
int mp_softmax_xent_scaled_db(int rows, int vocab, const mp_half* logits, int ld, const int32_t* targets,
                              mp_scale_state* st, float* loss, mp_half* dlogits, mp_half* db, void* ws,
                              size_t ws_bytes, mp_stream stream);

/* ------------------------------------------------------------------------------------------
 * Bandwidth-bound layer pieces (fp32 arithmetic between fp16 storage points, Section 3.2).
 * ------------------------------------------------------------------------------------------ */
/* y = RNE16( LN(x + a) * gamma + beta ) over the last dimension d; a may be NULL.  The sum, mean,
 * biased variance and 1/sqrt(var + eps) stay fp32; mean[rows], rstd[rows] (device fp32) are kept
 * for the backward pass.  x, a, y contiguous [rows, d]. */
int mp_layernorm_fwd(int rows, int d, const mp_half* x, const mp_half* a, const mp_half* gamma,
                     const mp_half* beta, float eps, mp_half* y, float* mean, float* rstd,
                     mp_stream stream);

/* dz = RNE16( rstd (g - mean_d(g) - xhat mean_d(g xhat)) ), g = dy gamma, xhat = (x + a - mean) rstd;
 * dgamma[d] = RNE16( sum_rows dy xhat ), dbeta[d] = RNE16( sum_rows dy ).  dz is the gradient of both
 * x and a.  If dz_colsum != NULL it also receives RNE16( column sums over rows of the stored dz ): the bias
 * gradient of the linear layer whose output entered this LayerNorm, at no extra pass over memory.
 * Optional overflow flag on dgamma / dbeta / dz_colsum.  Workspace: mp_layernorm_bwd_workspace_bytes. */
size_t mp_layernorm_bwd_workspace_bytes(int rows, int d);
int mp_layernorm_bwd(int rows, int d, const mp_half* dy, const mp_half* x, const mp_half* a,
                     const mp_half* gamma, const float* mean, const float* rstd, mp_half* dz,
                     mp_half* dgamma, mp_half* dbeta, mp_half* dz_colsum, mp_scale_state* st, void* ws,
                     size_t ws_bytes, mp_stream stream);

/* Row softmax of attention scores: p = RNE16( softmax_fp32(s) ), rows x cols, contiguous rows of
 * length cols with leading dimension ld (p may alias s). */
int mp_softmax_fwd(int64_t rows, int cols, const mp_half* s, mp_half* p, int ld, mp_stream stream);
/* ds = RNE16( p (dp - sum_j dp_j p_j) ); ds may alias dp. */
int mp_softmax_bwd(int64_t rows, int cols, const mp_half* p, const mp_half* dp, mp_half* ds, int ld,
                   mp_stream stream);

/* Fused scaled-dot-product self-attention on a fused projection qkv[T, >= 3 d_model] (columns [0, d_model) = q,
 * [d_model, 2 d_model) = k, [2 d_model, 3 d_model) = v; head h owns columns [h d_head, (h+1) d_head) of each;
 * sequence b owns rows [b seq_len, (b+1) seq_len)).  One workgroup per (sequence, head):
 *     s = RNE16(alpha q k^T),  p = RNE16(softmax_fp32(s)),  ctx = RNE16(p v)
 * with the same storage points as the unfused chain mp_gemm_fwd -> mp_softmax_fwd -> mp_gemm_fwd, but s never
 * reaches memory.  p (device fp16 [n_seq, n_heads, seq_len, seq_len]) is kept for the backward pass; ctx has the
 * heads side by side (leading dimension ld_ctx).  No mask, no dropout.
 * Supported: d_head == 64, seq_len a multiple of 8 up to 128; otherwise MP_E_UNSUPPORTED (use the unfused chain). */
int mp_attention_fwd(int n_seq, int n_heads, int seq_len, int d_head, const mp_half* qkv, int ld_qkv, float alpha,
                     mp_half* p, mp_half* ctx, int ld_ctx, mp_stream stream);

/* Backward of the above from the stored p:
 *     dP = RNE16(dctx v^T),  dS = RNE16(p (dP - sum_n dP p)),
 *     dV = RNE16(p^T dctx),  dQ = RNE16(alpha dS k),  dK = RNE16(alpha dS^T q),
 * written into dqkv (same column layout as qkv, leading dimension ld_dqkv). */
int mp_attention_bwd(int n_seq, int n_heads, int seq_len, int d_head, const mp_half* qkv, int ld_qkv, float alpha,
                     const mp_half* p, const mp_half* dctx, int ld_ctx, mp_half* dqkv, int ld_dqkv,
                     mp_stream stream);

/* LSTM cell, gate blocks ordered (i, f, g, o) in gates[B, 4H] (leading dimension ldg):
 *   c = sigma(f) c_prev + sigma(i) tanh(g)   (fp32, never rounded),  h = RNE16( sigma(o) tanh(c) ).
 * c_prev, c: device fp32 [B, H] contiguous.  h is written to h_out (ld ldh) and, if h_out2 != NULL,
 * also to h_out2 (ld ldh2) - the next time step's [x, h] row block and the next layer's input. */
int mp_lstm_cell_fwd(int B, int H, const mp_half* gates, int ldg, const float* c_prev, float* c,
                     mp_half* h_out, int ldh, mp_half* h_out2, int ldh2, mp_stream stream);

/* Backward of the cell for one time step.  dh = float(dh_a) + float(dh_b) (either may be NULL),
 * dc (device fp32 [B,H]) carries the cell-state gradient in and out (in place):
 *   do = dh tanh(c) so(1-so);  dc += dh so (1 - tanh(c)^2)
 *   di = dc tanh(g) si(1-si);  df = dc c_prev sf(1-sf);  dg = dc si (1 - tanh(g)^2);  dc *= sf
 *   dgates = RNE16([di, df, dg, do])   (leading dimension ldg, same as gates). */
int mp_lstm_cell_bwd(int B, int H, const mp_half* gates, int ldg, const float* c_prev, const float* c,
                     const mp_half* dh_a, int ld_a, const mp_half* dh_b, int ld_b, float* dc,
                     mp_half* dgates, mp_stream stream);

/* A whole LSTM layer over all time steps in ONE launch per direction (the recurrent encoder of the Section 2 listing
 * and Section 5.1; arithmetic of Sections 3.1 / 3.2 as in the per-step calls: fp16 operands, fp32 sums, each gate sum
 * and each h_t rounded once to fp16, cell state fp32).  Unrolled step by step a layer is a chain of small dependent
 * launches; here every workgroup keeps its rows of the recurrent weights on chip for all T steps and the steps are
 * separated by a grid-wide barrier inside the kernel.
 *
 *   forward : gates_t = RNE16( gx_t + h_{t-1} W_h^T + b ),   W_h = columns [I, I+H) of w[4H, ldw], gate blocks (i, f, g, o)
 *             c_t = sigma(f) c_{t-1} + sigma(i) tanh(g)  (fp32),   h_t = RNE16( sigma(o) tanh(c_t) )
 *     gx     device fp32 [T*B, 4H] (ld 4H): the input half x_t W_x^T of every step's gate sums, e.g. from ONE
 *            mp_gemm_fwd with y_f32 over all T*B rows; kept fp32 so the gate sum is still rounded once.
 *     gates  device fp16 [T*B, 4H] out (kept for the backward pass).
 *     c      device fp32 [(T+1)*B, H]: rows [0, B) hold c_0 on entry, rows of steps 1..T are written.
 *     xh     device fp16 [T*B, ldxh]: columns [I, I+H) of step 0 hold h_0 on entry; h_t is written into the same
 *            columns of step t+1 (t+1 < T).  Columns [0, I) are not touched (they hold x_t for the weight gradient).
 *     h_up   device fp16 [T*B, ld_up] or NULL: h_t is also written to columns [0, H) of row block t (the next layer's
 *            input, or the output).
 *   backward: per step t = T-1 .. 0, dh = float(dh_above_t) + float(dh_rec),
 *             dgates_t = RNE16(cell backward, see mp_lstm_cell_bwd),  dh_rec = RNE16( dgates_t W_h )  for step t-1.
 *     dh_above device fp16 [T*B, ld_up]: gradient reaching h_t from above (leading dimension d->ld_up).
 *     dgates   device fp16 [T*B, 4H] out.  The input gradient dgates W_x and the weight / bias gradients are ordinary
 *              large products over all T*B rows afterwards (mp_gemm_bwd_dx, mp_gemm_bwd_dw).
 *   status   device int32, must be 0 on entry (the caller clears it; it is never cleared here).  The kernel's step
 *            barrier waits at most wait_limit_us (0: 2 s) for the other workgroups; a wait that runs out sets
 *            *status nonzero, every workgroup then leaves its loop, and the outputs are undefined.  A nonzero status
 *            on entry makes the kernel stop at its first barrier.  Check it wherever the host next synchronises.
 *   ws       device, mp_lstm_layer_workspace_bytes() bytes, 4-byte aligned (step flags; cleared by the call).
 * All H / 16 workgroups must be resident at once: the call returns MP_E_UNSUPPORTED if the device has fewer compute
 * units, and launches of this kind that may run at the same time (other streams) must together fit the device.
 * Supported: B <= 32, H a multiple of 128 up to 1024, I, ldw, ldxh multiples of 8, ld_up even, 16-byte aligned
 * pointers; otherwise MP_E_UNSUPPORTED (run the layer with mp_gemm_fwd_ws / mp_lstm_cell_fwd step by step).
 * debug_extra_participants (0 in production) makes the barrier wait for that many flags nobody raises: with a small
 * wait_limit_us it lets a test drive the time-out path while every wave still exits normally. */
typedef struct mp_lstm_layer_desc {
    int32_t T, B, I, H;       /* time steps, batch rows, input width, hidden units                         */
    int32_t ldw, ldxh, ld_up; /* leading dimensions of w, xh, and of h_up (forward) / dh_above (backward)   */
    int32_t wait_limit_us;    /* bound of one barrier wait; 0 = 2 000 000                                   */
    int32_t debug_extra_participants;
    int32_t reserved;
} mp_lstm_layer_desc;
size_t mp_lstm_layer_workspace_bytes(void);
int mp_lstm_layer_fwd(const mp_lstm_layer_desc* d /* host */, const float* gx, const mp_half* w, const mp_half* bias,
                      mp_half* gates, float* c, mp_half* xh, mp_half* h_up, int32_t* status, void* ws, size_t ws_bytes,
                      mp_stream stream);
int mp_lstm_layer_bwd(const mp_lstm_layer_desc* d /* host */, const mp_half* w, const mp_half* gates, const float* c,
                      const mp_half* dh_above, mp_half* dgates, int32_t* status, void* ws, size_t ws_bytes,
                      mp_stream stream);

/* dst = RNE16(src), n elements (initial fp16 copies of masters and inputs). */
int mp_cast_f32_to_f16(size_t n, const float* src, mp_half* dst, mp_stream stream);
/* Fill n 32-bit words (a kernel, safe inside HIP graph capture). */
int mp_fill_u32(size_t n, uint32_t value, void* dst, mp_stream stream);

/* Measurement support for the half-precision matrix-unit rate that Section 3 builds on: the rate the matrix
 * cores sustain on THIS device with operands held in registers, for the operand values the caller supplies.
 * `workgroups` workgroups of 4 waves each run `iters` iterations of 16 independent 32x32x16 fp16 multiply-
 * accumulates (fp32 accumulators) and nothing else.  operands: device, >= 16384 halves, 16-byte aligned (the 8
 * operand registers of every lane; zeros, or values distributed like the tensors of interest: the clock the chip
 * holds under this load depends on them).  sink: device, >= workgroups * 256 floats, receives the accumulator
 * sums.  tflops: host, receives 2 * 32 * 32 * 16 flops per instruction over the time between two events on
 * `stream`.  Blocks until the timed launch has finished (the only call that does).  Errors: MP_E_INVAL for NULL / short / misaligned
 * buffers or counts out of range. */
int mp_mfma_sustained_rate(const mp_half* operands, size_t n_operands, float* sink, size_t n_sink, int workgroups,
                           int iters, double* tflops, mp_stream stream);

/* ------------------------------------------------------------------------------------------
 * Optimizer wrapper (Section 3.2) with the gradient inspection of Section 3.1 and the fp32-side
 * regulariser of Section 3.3.
 * ------------------------------------------------------------------------------------------ */
enum { MP_OPT_SGD = 0, MP_OPT_ADAM = 1 };
enum { MP_UPDATE_DEFAULT = 0,
       MP_UPDATE_PRECHECKED = 1 /* every gradient was produced by a call given `st`: skip the
                                   separate inspection pass and trust st->found_inf */ };

typedef struct mp_tensor_desc {
    const mp_half* g16; /* device: loss-scaled fp16 gradient                          */
    float*         w32; /* device: fp32 master weights (updated in place)             */
    mp_half*       w16; /* device: fp16 copy used by forward/backward (rewritten)     */
    float*         m;   /* device: Adam first moment  (NULL for SGD)                  */
    float*         v;   /* device: Adam second moment (NULL for SGD)                  */
    size_t         n;   /* elements                                                   */
} mp_tensor_desc;

typedef struct mp_opt_cfg {
    int32_t kind;         /* MP_OPT_SGD | MP_OPT_ADAM */
    int32_t reserved;
    double  lr;           /* hyper-parameters are given in double; the kernel uses their fp32   */
    double  beta1, beta2; /* roundings, except that the bias corrections 1 - beta^t are formed  */
    double  eps;          /* in double from the double betas and then rounded to fp32           */
    double  weight_decay; /* L2 coefficient applied to the fp32 master: g += wd * w32           */
} mp_opt_cfg;

/* One call covers every parameter tensor, because the skip decision is global.
 *   phase A: st->found_inf |= any fp16 gradient element with all exponent bits set (inf or NaN)
 *            (skipped with MP_UPDATE_PRECHECKED);
 *   phase B: if st->found_inf == 0, per element in fp32:
 *            g = float(g16) * st->inv_scale + wd * w32
 *            SGD : w32 -= lr g
 *            Adam: m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;  t = st->opt_step + 1
 *                  w32 -= lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
 *            w16 = RNE16(w32)
 *            else nothing is written.
 * `tensors` is a host array of ntensors descriptors (device pointers inside), copied into kernel
 * arguments during the call.  Does not advance opt_step or clear the flag: mp_loss_scale_update does. */
int mp_unscale_check_update(const mp_tensor_desc* tensors /* host */, int ntensors,
                            const mp_opt_cfg* cfg /* host */, mp_scale_state* st, int flags,
                            mp_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* MP_H_ */
