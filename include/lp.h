/*
 * lp.h -- C ABI of the LayerPipe training hot path on one MI355X (gfx950).
 *
 * The library runs one training iteration of a feed-forward network split into the per-layer tasks
 * of the paper (Sec. I, Sec. II-A, Fig. 1(b)):
 *
 *   F   forward product            Z_l  = A_{l-1} . W_l,  A_l = f(Z_l)        Eq. 1, Eq. 2
 *   dX  activation-gradient product dA_{l-1} = dY_l . W_l^T                    Eq. 4   ("delta")
 *   f'  Hadamard part               dY_l = dA_l (.) f'(Z_l)                    Eq. 3, executed in the
 *                                   stage that owns Z_l (inter-layer split, Sec. III-B)
 *   dW  weight-gradient product     G_l  = A_{l-1}^T . dY_l                    Eq. 5   ("G")
 *   U   delayed update              W_l(n) = W_l(n-1) - eta G_l(n - d_l)       Eq. 6, d_l delay
 *                                   elements per layer (Sec. III-A)
 *
 * Notation.  The paper is column-vector (z = W a, W of shape [out, in]).  This ABI is batched and
 * row-major: activations are [batch, features], and the stored weight is the transpose of the
 * paper's, W_l of shape [in, out], so that Z = A.W, dA = dY.W^T and G = A^T.dY (G has W's shape).
 * Layers are numbered l = 1..L and training steps n = 1, 2, ... as in the paper.
 *
 * Tensors.  All tensor pointers are DEVICE pointers unless a parameter says otherwise; dense,
 * row-major, 16-byte aligned.  "act type" is the context's dtype: LP_F32 -> float, LP_BF16 -> bfloat16
 * (upper 16 bits of an IEEE float, round-to-nearest-even).  Gradients G, master weights and the loss
 * are always float.  Convolution layers (3x3, stride 1, zero pad 1, cross-correlation, no bias) use
 * NHWC activations [batch, H, W, C] and weights [3][3][C_in][C_out]; an optional 2x2 stride-2 max-pool
 * follows the activation (first maximum in (row, column) order wins a tie).  No layer has a bias
 * (Eq. 1 has none).
 *
 * Ownership.  The library allocates NO device memory.  The caller owns every buffer, including the
 * workspace whose size lp_workspace_bytes reports (master weights, working weights, one ring of
 * d_l + 1 gradient slots per layer, and the activation stashes lp_step uses).  The context itself
 * (host memory, HIP events) is owned by the library and freed by lp_destroy.
 *
 * Execution.  Compute entry points validate their arguments synchronously, then enqueue kernels on
 * the given hipStream_t (passed as void*; NULL = the default stream) and return without waiting.
 * Every function returns an lp_status and lp_last_error gives a message.  Shapes, sizes and operand
 * limits are checked by lp_create (an operand of 2 GiB or more is LP_ERR_SHAPE there: the kernels use
 * 32-bit byte offsets), pointers and state by each call before its first launch, so an error of these
 * kinds means nothing has been enqueued; LP_ERR_HIP reports a failure of the HIP runtime itself, after
 * which earlier launches of the same call may already be running.  No C++ exception leaves the
 * library (host memory exhaustion inside it is reported as LP_ERR_STATE) and nothing aborts.  A
 * context is not thread-safe.
 *
 * Timing events per task and the matrix-instruction probe used by the benchmark are declared in
 * lp_measure.h; they are not part of the training path.
 */
#ifndef LAYERPIPE_LP_H
#define LAYERPIPE_LP_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lp_ctx lp_ctx;

typedef enum {
  LP_OK = 0,
  LP_ERR_NULL = 1,      /* a required pointer is NULL */
  LP_ERR_SHAPE = 2,     /* a size or range is impossible (batch <= 0, col range, H/W odd with pool ...) */
  LP_ERR_DTYPE = 3,     /* unknown dtype / loss / activation / layer kind */
  LP_ERR_LAYER = 4,     /* layer index outside 1..L, or consecutive layers do not fit */
  LP_ERR_DELAY = 5,     /* delay negative, above the configured one, or changed on a layer with the retimed update */
  LP_ERR_STATE = 6,     /* call needs a bound workspace or weights that were never set */
  LP_ERR_WORKSPACE = 7, /* workspace too small or misaligned */
  LP_ERR_HIP = 8        /* a HIP runtime call failed (message holds hipGetErrorString) */
} lp_status;

typedef enum { LP_F32 = 0, LP_BF16 = 1 } lp_dtype;
typedef enum { LP_LOSS_SOFTMAX_CE = 0, LP_LOSS_MSE = 1 } lp_loss;
typedef enum { LP_LINEAR = 0, LP_CONV3X3 = 1 } lp_kind;
/* f of Eq. 2.  The paper names sigmoid, tanh and ReLU (Sec. II-A); GELU (exact erf form) is added for the
 * transformer-MLP workload. */
typedef enum { LP_ACT_IDENTITY = 0, LP_ACT_RELU = 1, LP_ACT_GELU = 2, LP_ACT_TANH = 3, LP_ACT_SIGMOID = 4 } lp_act;

/* One layer.  LINEAR: in/out are feature counts, H = W = pool = 0.  CONV3X3: in/out are channel
 * counts, H x W the (input = output) image size, pool 0 or 2.  `delay` = d_l >= 0, the number of
 * delay elements on this layer's gradient->update edge (Sec. III-A: twice the number of pipeline
 * stages after the layer). */
typedef struct {
  int kind;   /* lp_kind */
  int in;
  int out;
  int H;
  int W;
  int act;    /* lp_act; the last layer must be LP_ACT_IDENTITY (its output feeds the loss) */
  int pool;
  int delay;
} lp_layer_desc;

/* Which internal tensor lp_tensor returns. */
typedef enum {
  LP_T_MASTER_W = 0,   /* float [in,out] (conv: [3][3][in][out]), the weights Eq. 6 updates          */
  LP_T_WORK_W = 1,     /* act type, the copy F and dX currently read (same buffer as master for F32) */
  LP_T_A = 2,          /* act type, A_l as written by lp_step (after the pool, if any)                */
  LP_T_Z = 3,          /* act type, Z_l as written by lp_step; NULL if the step does not keep it       */
  LP_T_DA = 4,         /* act type, dA_l = dE/dA_l (shape of A_l); NULL for l = L                      */
  LP_T_DY = 5,         /* act type, dY_l = delta_l (shape of Z_l)                                     */
  LP_T_G_LAST = 6      /* float, ring slot holding the gradient of the most recent finished step     */
} lp_tensor_id;

/* ---- life cycle (host only; touches no device) ---------------------------------------------- */

/* Builds a context for L layers and a fixed batch size.  `layers` is copied.  Checks that layer
 * l's output size equals layer l+1's input size (a conv output feeding a linear layer is flattened
 * in NHWC order).  lr is eta of Eq. 6.  *out is set only on LP_OK. */
int lp_create(const lp_layer_desc* layers, int L, int batch, int dtype, int loss, float lr, lp_ctx** out);
/* Frees the context, its events and its captured graphs.  Work that earlier calls enqueued must have
 * finished (lp_sync, or the caller's own stream synchronisation): the library does not wait here. */
int lp_destroy(lp_ctx* ctx);
/* Message of the last failing call on ctx (owned by ctx; valid until the next call).  ctx == NULL
 * returns the message of the last failing lp_create. */
const char* lp_last_error(const lp_ctx* ctx);

/* Bytes of device workspace this context needs (multiple of 256). */
int lp_workspace_bytes(const lp_ctx* ctx, size_t* bytes);
/* Hands the workspace to the context.  dev_ptr: 256-byte aligned device memory of at least
 * lp_workspace_bytes, owned by the caller, which must outlive the context's use of it.  Contents
 * need not be initialised.  Rebinding resets the step counter and marks all weights unset. */
int lp_bind_workspace(lp_ctx* ctx, void* dev_ptr, size_t bytes);

/* Copies float weights of layer l into the master copy and (BF16) rounds them into the working copy.
 * W: [in,out] or [3][3][in][out]; host pointer if is_device == 0 (copied synchronously), else a
 * device pointer (copied on `stream`). */
int lp_set_weights(lp_ctx* ctx, int l, const float* W, int is_device, void* stream);
/* Copies the master weights of layer l to dst (host: synchronous after draining `stream`). */
int lp_get_weights(lp_ctx* ctx, int l, float* dst, int is_device, void* stream);
/* Converts n floats (device) to the context's act type (device): round-to-nearest-even for LP_BF16, a
 * copy for LP_F32.  This is how an input batch or a regression target given as float becomes a tensor
 * lp_step accepts; the storage rounding of Eq. 1's operands is the library's, not the caller's.
 * src and dst 16-byte aligned, not overlapping.  Asynchronous on `stream`. */
int lp_cast(lp_ctx* ctx, const float* src, void* dst, size_t n, void* stream);

/* ---- the per-layer tasks ------------------------------------------------------------------- */

/* F (Eq. 1, Eq. 2).  X: A_{l-1}, act type, [batch, in] (conv: [batch,H,W,in]).  Writes Z_l (shape
 * [batch,out] / [batch,H,W,out]) and A_l = f(Z_l) (conv with pool: [batch,H/2,W/2,out]); either
 * may be NULL to skip that output, except that a pooled layer needs Z.  A is computed from the
 * stored (rounded) Z.  Reads the current working weights W_l(n-1).
 * Scratch: products with few output tiles and a long reduction are split over K, with fp32 partial
 * sums in the workspace.  A context has three such regions: (a) lp_forward and lp_grad_act calls whose
 * range starts at column 0, (b) lp_grad_act calls whose range starts elsewhere, (c) lp_grad_weight.
 * Calls that use one region must not overlap in time: enqueue them on one stream, or order them. */
int lp_forward(lp_ctx* ctx, int l, const void* X, void* Z, void* A, void* stream);

/* Error at the output and delta of the last layer (the paper only says the error is computed from
 * the ground truth; this library offers two).  ZL: act type [batch, D_L].  SOFTMAX_CE: target =
 * int labels [batch] in [0, D_L); E = -mean_b log softmax(z_b)[y_b]; dYL = (softmax - onehot)/batch.
 * A label outside [0, D_L) is not dereferenced: that row gets dYL = softmax/batch and makes E NaN.
 * MSE: target = act type [batch, D_L]; E = mean (z - t)^2; dYL = 2 (z - t) / (batch * D_L).
 * loss_dev: device float, may be NULL.  Needs a bound workspace (row partials). */
int lp_loss_grad(lp_ctx* ctx, const void* ZL, const void* target, void* dYL, float* loss_dev, void* stream);

/* lp_loss_grad for callers that cannot allocate device memory and have no workspace to hand over (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same kernels, same results bit
 * for bit, but the partial sums of the loss live in a static device array inside the library (65536 floats =
 * 256 KiB, held by every GPU the library runs on until the process ends) instead of the workspace.  No
 * workspace needs to be bound; the call allocates nothing on the device or through any library.
 * Limit: batch <= 65536 rows (SOFTMAX_CE) or batch * D_L <= 536870912 elements (MSE: one partial per 8192
 * elements); larger sizes are LP_ERR_SHAPE.  The first call on a device looks up the array's address there
 * (make that call outside a graph capture).  Every call on one GPU uses the same array: calls that overlap in
 * time on one GPU race (enqueue them on one stream, or order them); nothing in it has to start at zero, every
 * partial that is read has been written by the same call.  The stream is not recorded for lp_sync: synchronise
 * `stream` yourself.  ZL, target, dYL, loss_dev as in lp_loss_grad. */
int lp_loss_grad_static(lp_ctx* ctx, const void* ZL, const void* target, void* dYL, float* loss_dev, void* stream);

/* The Hadamard part of Eq. 3 for layer l, the piece the inter-layer split moves into the stage that
 * holds Z_l:  dY_l = dA_l (.) f'(Z_l).  S is the stashed Z_l; for a ReLU layer without pool the
 * stashed A_l works as well (same sign).  For a pooled layer dA has the pooled shape and is routed
 * to the first maximum of each 2x2 window of S before the mask is applied.  dY may alias dA only if
 * the layer is not pooled.  ReLU'(0) = 0; GELU' = Phi(z) + z phi(z). */
int lp_act_grad(lp_ctx* ctx, int l, const void* dA, const void* S, void* dY, void* stream);

/* dX (Eq. 4): dA_{l-1}[:, col0:col1] = dY_l . W_l[col0:col1, :]^T with the current working weights.
 * dX is the full [batch, in] tensor (conv: [batch,H,W,in]); only columns (channels) [col0, col1)
 * of the previous layer's features are written.  (0, in) computes all of it; two calls with
 * complementary ranges are the delta' / delta'' partition of Sec. III-B and may run concurrently
 * (one range starting at column 0, one not: see the scratch note at lp_forward).  Every element is
 * summed in the same order whatever the range: cutting the columns changes no bits. */
int lp_grad_act(lp_ctx* ctx, int l, const void* dY, void* dX, int col0, int col1, void* stream);

/* dW (Eq. 5): G_l = A_{l-1}^T . dY_l, float, shape of W_l.  G == NULL writes into the ring slot of
 * the step in progress, (n+1) mod (d_l+1), where lp_update will find it d_l steps later. */
int lp_grad_weight(lp_ctx* ctx, int l, const void* X, const void* dY, float* G, void* stream);

/* U (Eq. 6).  G != NULL: W_l <- W_l - eta G.  G == NULL: uses G_l((n+1) - d_l) from the ring; does
 * nothing if (n+1) - d_l < 1 (the delay elements start empty).  Updates the float master and (BF16)
 * writes the rounded working copy into the *other* of two buffers, which becomes current for calls
 * made after this one; kernels already enqueued keep reading the old version (weight stashing,
 * Sec. III-A).  F32 contexts update in place: order the call after the readers of W_l. */
int lp_update(lp_ctx* ctx, int l, const float* G, void* stream);

/* Inter-layer split of the delta product inside lp_step (Sec. III-B): the last `cols` of layer l's D_{l-1}
 * output columns (input channels for a convolution) are computed by a second, independent kernel
 * (delta'', the part the following stage borrows) on streams[1], ahead of that layer's G task, while
 * the first D_{l-1} - cols columns (delta') stay on the critical stream; the moved Hadamard of layer
 * l-1 waits for both.  cols = 0 (default) computes the product in one piece.  Results do not depend
 * on cols.  0 <= cols < D_{l-1}; layer 1 has no delta task. */
int lp_set_delta_split(lp_ctx* ctx, int l, int cols);

/* The moved Hadamard product inside lp_step (Eq. 3, placement of Sec. III-B): in an LP_BF16 context, where layer l-1
 * applies ReLU or GELU element-wise, the dX task of layer l (fully connected or convolution) multiplies by
 * f'(S_{l-1}) in its own epilogue and writes dY_{l-1} directly; where layer l-1 is a 2x2 max-pooled ReLU convolution
 * and layer l a convolution, that epilogue also routes each gradient to the first maximum of its window; dA_{l-1} is
 * then never stored (LP_T_DA of layer l-1 is NULL) and the separate Hadamard kernel is not launched.  The arithmetic
 * is that of lp_grad_act followed by lp_act_grad, element for element: dA is rounded to the act type before the
 * product, so every result is bit-identical with the switch off.  Default: on.  enable = 0 restores the two-kernel
 * form (every dA inspectable).  The per-layer entry points are not affected.  May be called at any time between steps. */
int lp_set_fused_hadamard(lp_ctx* ctx, int enable);

/* Forward run-ahead across steps (Sec. III-A, the schedule of Fig. 6 on one device): with enable != 0,
 * lp_step runs the forward chain and the loss on streams[3] and no longer joins the streams between
 * steps, so F_l(n+1) starts as soon as W_l(n) exists (which needs only G_l(n - d_l)) and overlaps the
 * backward pass of step n.  Each layer then keeps two stashes (A_l, Z_l of steps n and n+1), so the
 * workspace grows: call this after lp_create and before lp_workspace_bytes / lp_bind_workspace
 * (LP_ERR_STATE afterwards).  lp_step then needs n_streams >= 4 handles (LP_ERR_STATE): streams[0] critical
 * backward chain, [1] G tasks, [2] updates, [3] forward chain and loss.  streams[3] must differ from streams[0];
 * [1] and [2] may repeat another handle (tasks that share a stream run in the order they are enqueued: fewer
 * cross-stream waits for the host to enqueue, less overlap on the device).
 * Results are those of the serial order, bit for bit.  X0 and target of a step must stay unchanged
 * until that step has finished, and the loss of step n+1 may be written before step n has finished: give
 * consecutive steps different loss_dev addresses (or read the loss before enqueueing the next step).  No stream
 * is joined into another at the end of a step: call lp_sync before reading weights, tensors or the loss from
 * another stream (lp_get_weights to host memory does so itself).  LP_BF16 contexts only (LP_ERR_DTYPE): F32 updates weights in place. */
int lp_set_run_ahead(lp_ctx* ctx, int enable);

/* Factor ring (for layers whose batch is small next to their width): the delay elements of layer l hold
 * the two factors of the gradient, A_{l-1}(n) and dY_l(n) (batch x (in + out) elements), instead of the
 * product G_l(n) (in x out floats).  The G task of a step then only copies the factors; the delayed
 * update of step n forms G_l(n - d_l) tile by tile with the kernel lp_grad_weight uses and applies each
 * tile to the weights in its epilogue, so G never travels through memory: same arithmetic and same bits
 * as the product ring, less memory and less traffic (per parameter 10 bytes instead of 4 + 14).
 * A layer whose G product lp_grad_weight splits over K ranges (fewer than 256 output tiles of 128 x 128
 * and batch >= 2048), or runs on the short-vector kernels of a layer with a handful of outputs (at most 16
 * outputs, inputs a multiple of 8, batch <= 2048), would be summed in another order by the fused update, so
 * it is excluded:
 * l = 0 selects every linear layer but those (they keep the product ring), l > 0 on such a layer is
 * LP_ERR_LAYER.  Applies to lp_step and to lp_grad_weight / lp_update called with
 * G = NULL; LP_T_G_LAST of such a layer is NULL.  Call after lp_create and before lp_workspace_bytes /
 * lp_bind_workspace (LP_ERR_STATE afterwards).  LP_BF16 contexts (LP_ERR_DTYPE), linear layers
 * (LP_ERR_LAYER). */
int lp_set_factor_ring(lp_ctx* ctx, int l, int enable);

/* Retimed update: Eq. 6 with its d_l delay elements moved from the gradient, in front of the update, to the weights,
 * behind it (the retiming of Sec. III-A, which ends with the delays between W and its readers: weight stashing).
 * The G task of step n applies its gradient at once, in the epilogue of the product (tile by tile, the arithmetic
 * of lp_update; G never travels through memory), to master weights that hold every gradient computed so far, and
 * writes the bf16 copy of the result as weight version n; F and dX of step n read version n - 1 - d_l (version 0 =
 * the weights given to lp_set_weights), held in a ring of d_l + 2 bf16 versions that takes the place of the gradient
 * ring.  There is no update task.  The weights every step reads, and with them every activation, delta and the loss,
 * are bit-identical with the gradient ring (the same gradients are applied in the same order; only the moment of the
 * arithmetic differs); per parameter and step 10 bytes move instead of 4 + 14.  What differs for the caller:
 * lp_get_weights / LP_T_MASTER_W of such a layer are d_l gradients ahead of the weights the next step reads
 * (LP_T_WORK_W is those); LP_T_G_LAST is NULL; lp_grad_weight with G == NULL is the whole G task (it applies the
 * gradient and writes version n + 1: call it once per step) and lp_update is LP_ERR_STATE; lp_step accepts only the layer's own
 * d_l in `delay` (LP_ERR_DELAY); lp_set_weights sets the master weights and every held version.
 * LP_BF16 contexts (LP_ERR_DTYPE).  The update rides in the kernel that finishes G (where K is cut into ranges: the one
 * that adds the partial sums): every linear layer without a factor ring qualifies; a convolution qualifies when its G
 * product is split over K (batch x H x W >= 1024 pixels and fewer than 512 output tiles of 128 x 64).  l = 0 selects every such layer and leaves the others as they are, l > 0 on another
 * layer is LP_ERR_LAYER.  Works with every schedule of lp_step (streams, run-ahead,
 * graph replay, delta split).  Call after lp_create and before lp_workspace_bytes / lp_bind_workspace (LP_ERR_STATE
 * afterwards). */
int lp_set_retimed_update(lp_ctx* ctx, int l, int enable);

/* Graph replay of whole steps: with enable != 0, lp_step captures the tasks of a step into a HIP graph
 * the first time it sees that step's combination of buffers (ring slots, working-weight copies, the
 * caller's X0 / target / loss_dev pointers and streams) and afterwards replays it with one launch on
 * streams[0]; this removes the host cost of the 5-7 launches per layer, which bounds small networks.
 * Gradient rings get a power-of-two number of slots (>= d_l + 1) so that the combinations repeat after
 * max_l ring_l steps: the workspace grows, so call this after lp_create and before lp_workspace_bytes /
 * lp_bind_workspace (LP_ERR_STATE afterwards).  Steps up to max d_l + 2 and steps run under lp_profile
 * are enqueued as usual.  Feed lp_step from a small, repeating set of input buffers: each new pointer
 * combination is a new capture (at most 512 are kept, further ones run uncaptured).  Results are those
 * of the uncaptured step, bit for bit.  Not together with lp_set_run_ahead (LP_ERR_STATE). */
int lp_set_graphs(lp_ctx* ctx, int enable);

/* Counters of lp_step calls since lp_create on a context with graph replay: steps captured (and run),
 * steps replayed from a captured graph, steps enqueued uncaptured.  Any pointer may be NULL. */
int lp_graph_stats(const lp_ctx* ctx, long* captured, long* replayed, long* eager);

/* Ends a step driven through the per-layer calls: n <- n + 1. */
int lp_advance(lp_ctx* ctx);

/* One whole training iteration for one minibatch: F for l = 1..L, the loss, then for l = L..1 the
 * tasks dW_l, dX_l and the moved Hadamard of layer l-1, and every layer's delayed update; n <- n+1.
 * X0: act type input batch.  target: as in lp_loss_grad.  delay: optional int[L] overriding the
 * descriptors' d_l for the rest of the context's life (the rings are sized by lp_create, so
 * delay[l] may not exceed the descriptor's value); NULL keeps them.  loss_dev: device float or NULL.
 * streams[0..n_streams): hipStream_t handles.  With one stream all tasks run in order on it.  With
 * more, the critical chain (F, loss, dX, Hadamard) runs on streams[0], dW on streams[1], updates on
 * streams[2 % n_streams]: the G task is off the critical loop (Sec. III-C) and W_l(n) only has to
 * exist before step n+1.  All side-stream work is joined back into streams[0] before returning, so
 * the caller orders against streams[0] only.  X0 and target must stay unchanged until then.
 * With every delay 0 the result equals the per-layer calls made in textbook order. */
int lp_step(lp_ctx* ctx, const void* X0, const void* target, const int* delay, float* loss_dev,
            void* const* streams, int n_streams);

/* Number of finished steps n. */
int lp_step_index(const lp_ctx* ctx, long* n);
/* Blocks until every stream the context has enqueued work on is idle. */
int lp_sync(lp_ctx* ctx);
/* Device address and size of an internal tensor (see lp_tensor_id) for inspection. */
int lp_tensor(lp_ctx* ctx, int l, int which, void** dev_ptr, size_t* bytes);

/* ---- balanced pipeline partitioning (host only) --------------------------------------------- */

/* Algorithm 1 (Sec. III-C).  t_fix[l]: time of layer l's immovable tasks (forward + weight gradient),
 * t_flex[l]: time of its delta task (Eq. 4), l = 0..L-1, any unit, >= 0.  n_proc >= 1 processors,
 * alpha > 1 the relaxation factor of the target load.  Outputs (host arrays owned by the caller):
 * stage_fix[L]: stage (0 = first layers) of each layer's immovable tasks; borrowed_frac[L]: fraction of
 * layer l's delta task that the stage of layer l+1 executes (delta''; 0 if none);
 * stage_delta_rest[L]: stage that executes the rest (delta'); stage_time[n_proc]: load per stage;
 * *t_p (may be NULL): the final target load.  Touches no device. */
int lp_partition(const double* t_fix, const double* t_flex, int L, int n_proc, double alpha, int* stage_fix,
                 int* stage_delta_rest, double* borrowed_frac, double* stage_time, double* t_p);

#ifdef __cplusplus
}
#endif
#endif /* LAYERPIPE_LP_H */
