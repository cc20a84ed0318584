/*
 * kfac.h -- C ABI of the MI355X (gfx950) K-FAC hot-path library.
 *
 * One K-FAC step of one conv/fc layer, as the per-GPU part of the distributed K-FAC optimizer
 * (Algorithm 1: stages 1, 2, 4 and 5) computes it:
 *
 *   kfac_factor_A         A = E[a a^T]       Kronecker factor from the layer's input    (Sec. 3.2, Eq. 5; stage 1)
 *   kfac_factor_G         G = E[g g^T]       Kronecker factor from the output gradient  (Sec. 3.2, Eq. 5; stage 2)
 *   kfac_ema              S <- rho S + (1-rho) X   running average of a factor (standard K-FAC practice;
 *                                                  the paper is silent on it)
 *   kfac_damped_inverse   (S + lambda I)^-1  damping of Sec. 4.2 applied per factor, inverse of Eq. 6 (stage 4)
 *   kfac_precondition     G^-1 gradW A^-1    = (G^-1 (x) A^-1) grad, Eq. 7                (stage 5)
 *
 * Conventions common to every call
 *   - Every pointer is a DEVICE pointer unless its name ends in `_host`.  The caller owns every
 *     buffer; the library allocates no device memory and frees none, and no result depends on an
 *     earlier call.  The one piece of process-wide state is the measurement aid at the end of this
 *     file (a flag and, while it is on, the list of recorded events); it is off by default.
 *     Scratch memory comes in through `ws` / `ws_bytes`; the *_workspace_bytes functions (pure
 *     host functions) say how much a call needs.  `ws` must be 256-byte aligned.
 *   - Matrices are dense, row-major, with leading dimension = number of columns, float32.
 *     Symmetric outputs are written in full (both triangles) and are exactly symmetric.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work; they do not synchronise.  Buffers must stay valid until the stream has drained.
 *   - Return value: KFAC_OK or a negative kfac_status.  Argument errors are detected on the host
 *     before anything is launched; a batched call with count = 0 returns KFAC_OK and launches
 *     nothing, a negative count is an argument error.  Numerical failure of an inversion (matrix not positive
 *     definite) is reported through the device-side `info` word, LAPACK potrf style.
 *   - Thread safety: calls from different host threads, on different streams, with disjoint buffers
 *     may run concurrently (the measurement aid takes a lock of its own when it is on).
 */
#ifndef KFAC_H_
#define KFAC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum kfac_status {
    KFAC_OK = 0,
    KFAC_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, inconsistent descriptor            */
    KFAC_ERR_UNSUPPORTED = -2,   /* valid request this build has no kernel for                           */
    KFAC_ERR_WORKSPACE = -3,     /* ws is NULL / misaligned / smaller than *_workspace_bytes says         */
    KFAC_ERR_HIP = -4,           /* a HIP runtime call (launch, memset) failed                            */
    KFAC_ERR_TOO_LARGE = -5      /* more work than the fixed scratch of a *_noalloc entry point can hold   */
} kfac_status;

typedef enum kfac_dtype { KFAC_F32 = 0, KFAC_BF16 = 1, KFAC_F16 = 2 } kfac_dtype;

/* Memory layout of activation / output-gradient tensors. Logical index is always (n, c, y, x). */
typedef enum kfac_layout { KFAC_NCHW = 0, KFAC_NHWC = 1 } kfac_layout;

/* Order of the unfolded-patch columns of A (and therefore of the columns of gradW):
 *   KFAC_ORDER_C_KH_KW: column (c,i,j) = (c*kh + i)*kw + j   -- weight.reshape(C_out, -1) of an NCHW weight
 *   KFAC_ORDER_KH_KW_C: column (i,j,c) = (i*kw + j)*C_in + c -- memory order of a channels-last weight; the
 *                                                              fast path for NHWC tensors
 * The bias column, when present, is the last one in both orders. */
typedef enum kfac_col_order { KFAC_ORDER_C_KH_KW = 0, KFAC_ORDER_KH_KW_C = 1 } kfac_col_order;

/* One conv or fully connected layer (fc: H = W = kh = kw = 1, stride 1, pad 0).
 * Output size H_o = floor((H + 2 pad - kh)/stride) + 1, same for W.  R = N * H_o * W_o unfolded rows.
 * d_A = C_in*kh*kw + has_bias, d_G = C_out. */
typedef struct kfac_layer_desc {
    int32_t N, C_in, H, W, C_out, kh, kw, stride, pad;
    int32_t has_bias;   /* 1: append a constant-1 column to every unfolded row                           */
    int32_t layout;     /* kfac_layout of act and gout                                                    */
    int32_t dtype;      /* kfac_dtype of act and gout                                                     */
    int32_t order;      /* kfac_col_order of A's rows/columns                                             */
} kfac_layer_desc;

enum { KFAC_OP_FACTOR_A = 0, KFAC_OP_FACTOR_G = 1 };

const char* kfac_status_string(int status);

/* Workspace a factor build needs (split-K partial tiles), op = KFAC_OP_FACTOR_A / _G.  0 on a bad descriptor. */
size_t kfac_factor_workspace_bytes(int op, const kfac_layer_desc* desc);

/* Stage 1.  A[d_A x d_A] = scale * sum_r abar_r abar_r^T over the R unfolded input patches abar_r of `act`
 * (zero padding outside the image, a trailing 1 if has_bias); scale = 0 selects 1/R, the mini-batch
 * mean of Sec. 3.1.  `act` holds N*C_in*H*W elements of desc->dtype in desc->layout.  Accumulation is fp32. */
int kfac_factor_A(const kfac_layer_desc* desc, const void* act, float scale, float* A,
                  void* ws, size_t ws_bytes, void* stream);

/* Stage 2.  G[d_G x d_G] = scale * sum_r g_r g_r^T over the R = N*H_o*W_o output positions, g_r the C_out-vector
 * of `gout` (N*C_out*H_o*W_o elements, same dtype/layout as act) at that position; scale = 0 selects 1/R. */
int kfac_factor_G(const kfac_layer_desc* desc, const void* gout, float scale, float* G,
                  void* ws, size_t ws_bytes, void* stream);

/* Many factor builds at once (all layers of a network): builds that the matrix-core kernel can serve share a
 * launch, so that the many small ones fill the machine together.  items_host[i] / items_dev[i] describe the same
 * build (device copy uploaded once by the caller); each item's `ws` needs kfac_factor_workspace_bytes(op, &desc)
 * bytes of its own.  Results are identical to the single calls.  An item may instead fold its result into a running
 * average (`running`) or deliver it as a packed upper triangle (`packed`); see the fields. */
typedef struct kfac_factor_item {
    kfac_layer_desc desc;
    const void* x;       /* act (op = KFAC_OP_FACTOR_A) or gout (op = KFAC_OP_FACTOR_G), device */
    float* out;          /* d x d factor, device */
    void* ws;            /* per-build scratch (device, 256-byte aligned) or NULL if none is needed */
    size_t ws_bytes;
    float scale;         /* 0 selects 1/R */
    int32_t op;
    float* running;      /* NULL, or the factor's running average S (d x d, device): the build then ends with
                            S <- decay S + (1 - decay) factor in its own epilogue (S is read and written once; the fresh
                            factor is never stored) and `out` must be NULL.  Same values as kfac_ema on a stored factor. */
    float decay;
    int32_t packed;      /* 1: `out` receives the packed upper triangle, d (d + 1) / 2 floats in the layout of
                            kfac_pack_upper_batched (Sec. 3.4, symmetry-aware communication), instead of the square */
} kfac_factor_item;

int kfac_factor_batched(const kfac_factor_item* items_host, const kfac_factor_item* items_dev, int32_t count,
                        void* stream);

/* running[dim x dim] <- decay * running + (1 - decay) * fresh, in place.  running and fresh must not overlap. */
int kfac_ema(float* running, const float* fresh, int32_t dim, float decay, void* stream);

/* The same update for `count` matrices in as few launches as possible (one per 128 matrices).  The array is
 * read on the host during the call and may be freed afterwards; every pointer in it is a device pointer. */
typedef struct kfac_ema_item {
    float* running;      /* dim x dim, updated in place */
    const float* fresh;  /* dim x dim */
    int32_t dim;
} kfac_ema_item;

int kfac_ema_batched(const kfac_ema_item* items_host, int32_t count, float decay, void* stream);

/* Packed upper triangles (Sec. 3.4, symmetry-aware communication: a symmetric factor travels as its upper triangle).
 * Packed layout: row i contributes full[i][i], full[i][i+1], ..., full[i][dim-1], rows in order: dim (dim + 1) / 2
 * floats.  Only the upper triangle of `full` is read.  One launch per 128 matrices.  The arrays are read on the host
 * during the call; every pointer in them is a device pointer; full and packed must not overlap. */
typedef struct kfac_pack_item {
    const float* full;   /* dim x dim, row-major */
    float* packed;       /* dim (dim + 1) / 2 */
    int32_t dim;
} kfac_pack_item;

int kfac_pack_upper_batched(const kfac_pack_item* items_host, int32_t count, void* stream);

/* running[dim x dim] <- decay * running + (1 - decay) * X, where the fresh symmetric factor X arrives packed (what a
 * layer's owner holds after the reduction of Algorithm 1 stage 3 when factors are sent packed).  Both triangles of
 * `running` are written (the lower one as the mirror image of the upper one); only its upper triangle is read. */
typedef struct kfac_ema_packed_item {
    float* running;            /* dim x dim, updated in place */
    const float* packed_fresh; /* dim (dim + 1) / 2 */
    int32_t dim;
} kfac_ema_packed_item;

int kfac_ema_packed_batched(const kfac_ema_packed_item* items_host, int32_t count, float decay, void* stream);

/* Change rate of a statistic between two refreshes, out[i] = ||x - x_prev||_F / ||x_prev||_F (Sec. 5.4, staleness of
 * the Fisher information), for `count` matrices; out is a device array of `count` floats.  Deterministic (fixed
 * summation order, double accumulation across threads).  ws: device scratch of kfac_factor_diff_workspace_bytes
 * bytes, 256-byte aligned.  The item array is read on the host during the call. */
typedef struct kfac_diff_item {
    const float* x;       /* dim x dim, device */
    const float* x_prev;  /* dim x dim, device */
    int32_t dim;
} kfac_diff_item;

size_t kfac_factor_diff_workspace_bytes(const kfac_diff_item* items_host, int32_t count);
int kfac_factor_diff_batched(const kfac_diff_item* items_host, int32_t count, float* out, void* ws, size_t ws_bytes,
                             void* stream);

/* The same computation for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  The chunk sums go to a fixed 1 MiB array inside the
 * library's device image instead of `ws`; the call allocates and frees nothing.  Limit: the matrices' chunk counts
 * (ceil(dim^2 / 8192) each) may add up to at most 65536, i.e. kfac_factor_diff_noalloc_max_elements() = 2^29 elements
 * when every matrix fills its chunks; beyond it the call returns KFAC_ERR_TOO_LARGE and launches nothing.  All calls on
 * one GPU share the array: calls that overlap in time on one GPU (different streams or threads) race and must be
 * serialised by the caller.  Nothing in it needs clearing between calls (every entry is written before it is read).
 * Results are bit-identical to kfac_factor_diff_batched. */
int kfac_factor_diff_batched_noalloc(const kfac_diff_item* items_host, int32_t count, float* out, void* stream);
size_t kfac_factor_diff_noalloc_max_elements(void);

/* Optimizer tail for `count` layers: w_next = w - eta * precond + momentum * (w - w_prev)  (Sec. 4.3, the update
 * equation), then w_next <- sqrt(2 d_out) * w_next / (||w_next|| + eps)  (Sec. 4.4, weights rescaling; the norm is over
 * all n weights of the layer).  On return w holds the rescaled w_next and w_prev the old w.  The learning rate and
 * momentum of the epoch are the caller's (host scalars).  w, w_prev and precond must not overlap.  ws: device scratch
 * of kfac_weight_update_workspace_bytes bytes, 256-byte aligned.  Deterministic. */
typedef struct kfac_update_item {
    float* w;             /* n weights (d_out x d_A), device, updated in place */
    float* w_prev;        /* n, device, updated in place */
    const float* precond; /* n, device: the preconditioned gradient */
    int32_t n;
    int32_t d_out;
} kfac_update_item;

size_t kfac_weight_update_workspace_bytes(const kfac_update_item* items_host, int32_t count);
int kfac_weight_update_batched(const kfac_update_item* items_host, int32_t count, float eta, float momentum, float eps,
                               void* ws, size_t ws_bytes, void* stream);

/* Batch Normalization layers (Sec. 5.4: their Fisher matrix is not Kronecker-factorised).  Per-sample gradients of a
 * BN layer's parameters theta = (scale_1..scale_C, shift_1..shift_C):
 *     g[n][c] = sum_s gout[n][s][c] * xhat[n][s][c],   g[n][C + c] = sum_s gout[n][s][c],   s = 0..HW-1,
 * from the normalised input xhat and the output gradient gout, both N x HW x C (channels last), dtype kfac_dtype.
 * g: N x 2C floats, device.  ws: kfac_bn_sample_grads_workspace_bytes bytes, 256-byte aligned.  Deterministic.
 * The full Fisher matrix F = (1/N) sum_n g_n g_n^T is kfac_factor_G on g seen as an N x 2C x 1 x 1 fp32 tensor, its
 * damped inverse kfac_damped_inverse, and F^-1 grad kfac_precondition with dG = 1. */
size_t kfac_bn_sample_grads_workspace_bytes(int32_t N, int32_t C, int32_t HW);   /* may be 0: then ws may be NULL */
int kfac_bn_sample_grads(const void* xhat, const void* gout, int32_t N, int32_t C, int32_t HW, int32_t dtype, float* g,
                         void* ws, size_t ws_bytes, void* stream);

/* The same for many layers at once (all BN layers of a network in two or three launches).  items_host: host array,
 * read during the call only; the tensors it names are device memory.  Layers may differ in every field. */
typedef struct {
    const void* xhat;
    const void* gout;
    float* g;
    int32_t N, C, HW;
    int32_t dtype;   /* kfac_dtype */
} kfac_bn_item;

size_t kfac_bn_sample_grads_batched_workspace_bytes(const kfac_bn_item* items_host, int32_t count);
int kfac_bn_sample_grads_batched(const kfac_bn_item* items_host, int32_t count, void* ws, size_t ws_bytes, void* stream);

/* Diagonal approximation (Sec. 5.4): fisher_diag[j] = (1/N) sum_n g[n][j]^2 and out[j] = grad[j] / (fisher_diag[j] +
 * damping), j < C2 = 2C; damping = rho_BN * gamma (Sec. 4.2).  Either output may be NULL (grad may be NULL if out is). */
int kfac_bn_diag_precondition(const float* g, int32_t N, int32_t C2, const float* grad, float damping,
                              float* fisher_diag, float* out, void* stream);

/* Workspace for kfac_damped_inverse of one dim x dim matrix. */
size_t kfac_inverse_workspace_bytes(int32_t dim);

/* Minv[dim x dim] = (S + damping * I)^-1 for symmetric S (only S's lower triangle is read).  Sec. 4.2 / Eq. 6.
 * S and Minv must not overlap.  *info (device int32, may be NULL) is set to 0 on success or to k > 0 when the
 * leading minor of order k of the damped matrix is not positive definite; Minv is then unspecified. */
int kfac_damped_inverse(const float* S, int32_t dim, float damping, float* Minv, int32_t* info,
                        void* ws, size_t ws_bytes, void* stream);

/* A batch of independent inversions advanced together (one launch per elimination stage per step for the whole
 * batch), for the many factors of a network.  items_host is a HOST array, sorted by non-increasing dim; the
 * descriptors travel in the kernel arguments, so nothing has to be uploaded.  Each item's `ws` needs
 * kfac_inverse_workspace_bytes(dim) bytes of its own.  Results are identical to the single calls. */
typedef struct kfac_inverse_item {
    const float* S;     /* dim x dim symmetric input (device)                                             */
    float* Minv;        /* dim x dim output (device)                                                      */
    void* ws;           /* per-matrix scratch (device, 256-byte aligned)                                  */
    int32_t* info;      /* device status word or NULL                                                     */
    int32_t dim;
    float damping;
    const float* damping_dev;  /* NULL, or a device float that replaces `damping` (read when the work runs: the
                                  value may come from kfac_pi_damping_batched enqueued before on the same stream) */
    void* planes;       /* NULL, or kfac_inverse_planes_bytes(dim) bytes (device, 256-byte aligned) that receive
                           the inverse a second time in the form the preconditioning products multiply from: 128 x 128
                           blocks, scaled by one power of two, as two planes of fp16 pieces (see
                           kfac_precond_item.Ginv_planes).  Needs damping > 0 and a positive semidefinite S: the scale
                           is chosen from the bound 1 / damping on the inverse's entries.  Minv is written as always. */
} kfac_inverse_item;

size_t kfac_inverse_planes_bytes(int32_t dim);

int kfac_damped_inverse_batched(const kfac_inverse_item* items_host, int32_t count, void* stream);

/* Damping of Sec. 4.2.
 * The split of a block's damping gamma between its Kronecker factors in proportion to their scale (the factored Tikhonov
 * damping the section names): lam[2 i] = pi_i sqrt(gamma) for A_i and lam[2 i + 1] = sqrt(gamma) / pi_i for G_i, with
 * pi_i = sqrt((tr A_i / dA_i) / (tr G_i / dG_i)); pi_i = 1 if a trace is not positive.  lam: 2 * count device floats,
 * meant to be handed to the inversions through kfac_inverse_item.damping_dev.  One launch per 128 layers; deterministic.
 * The item array is read on the host during the call. */
typedef struct kfac_pi_item {
    const float* A;      /* dA x dA (device): the factor as it will be inverted (the running average) */
    const float* G;      /* dG x dG (device) */
    int32_t dA, dG;
} kfac_pi_item;

int kfac_pi_damping_batched(const kfac_pi_item* items_host, int32_t count, float gamma, float* lam, void* stream);

/* Warm-up damping (Sec. 4.2), host arithmetic on scalars: alpha = 2 log10(gamma0 / gamma_target) / t_warmup (NaN for a
 * non-positive argument) and gamma(t+1) = (1 - alpha) gamma(t) + alpha gamma_target; the damping of the Batch
 * Normalization layers is rho_bn * gamma. */
double kfac_warmup_damping_alpha(double gamma0, double gamma_target, double t_warmup);
double kfac_warmup_damping_next(double gamma, double gamma_target, double alpha);
double kfac_bn_damping(double gamma, double rho_bn);

/* Iterations between two refreshes of the statistics in epoch `epoch` (Sec. 5.4, training with stale statistics):
 * KFAC_REFRESH_GROWING: min(20, 5 floor(epoch / 5) + 1); KFAC_REFRESH_LATE: 1 before epoch 13, 20 from then on.
 * -1 for a negative epoch or an unknown heuristic.  Host function. */
enum { KFAC_REFRESH_GROWING = 0, KFAC_REFRESH_LATE = 1 };
int32_t kfac_refresh_interval(int32_t epoch, int32_t heuristic);

/* Workspace for kfac_precondition (the d_A x d_G intermediate). */
size_t kfac_precondition_workspace_bytes(int32_t dG, int32_t dA);

/* Stage 5.  out[dG x dA] = Ginv[dG x dG] * gradW[dG x dA] * Ainv[dA x dA]  (Eq. 7 written for the weight
 * gradient as a matrix).  Ginv and Ainv are symmetric; out must not overlap the inputs. */
int kfac_precondition(const float* Ginv, const float* Ainv, const float* gradW, int32_t dG, int32_t dA,
                      float* out, void* ws, size_t ws_bytes, void* stream);

/* The preconditioning of many layers as two launches over the tiles of all of them (one per product).
 * items_host[i] / items_dev[i] describe the same layer (device copy uploaded once by the caller); each item's
 * `ws` needs kfac_precondition_workspace_bytes(dG, dA) bytes of its own.  Listing layers with large dA first
 * gives the best load balance. */
typedef struct kfac_precond_item {
    const float* Ginv;   /* dG x dG (device) */
    const float* Ainv;   /* dA x dA (device) */
    const float* gradW;  /* dG x dA (device) */
    float* out;          /* dG x dA (device) */
    void* ws;            /* per-layer scratch (device, 256-byte aligned) */
    int32_t dG, dA;
    const void* Ginv_planes;   /* NULL, or the planes kfac_damped_inverse_batched wrote for Ginv (kfac_inverse_item.planes): */
    const void* Ainv_planes;   /* the call then multiplies from them instead of splitting Ginv / Ainv itself (the fp32
                                  matrices are not read); they must belong to the same inverses */
} kfac_precond_item;

int kfac_precondition_batched(const kfac_precond_item* items_host, const kfac_precond_item* items_dev,
                              int32_t count, void* stream);

/* Measurement aid (for benchmarks; not one of the paper's operations).  While enabled, every kernel the
 * library launches is bracketed by two HIP events on its stream.  kfac_kernel_timing_report waits for them
 * and writes one text line per kernel into the HOST buffer: "<kernel name> <total ms> <launches>\n",
 * NUL-terminated, then forgets them.  Returns KFAC_ERR_WORKSPACE if the buffer is too small.  Process-wide
 * state, off by default; do not enable it inside a throughput measurement. */
int kfac_kernel_timing_enable(int enable);
int kfac_kernel_timing_report(char* buf_host, size_t buf_bytes);

/* Probes of what this GPU can at best deliver, for the rooflines (measurement aids too; the caller times them).
 * kfac_probe_mfma: `workgroups` x 4 wavefronts each issue 4 * iters matrix-core instructions on register-resident
 * operands: v_mfma_f32_32x32x2_f32 (dtype KFAC_F32: 4096 flops each), v_mfma_f32_32x32x16_bf16 / _f16 (KFAC_BF16 /
 * KFAC_F16: 32768 flops each).  out: workgroups * 256 device floats.
 * kfac_probe_copy / kfac_probe_read: a plain streaming copy src -> dst, or read of src, of `bytes` bytes (a multiple
 * of 16, 16-byte aligned buffers) by `workgroups` workgroups; sink: one device float. */
int kfac_probe_mfma(int32_t dtype, int32_t workgroups, int32_t iters, float* out, void* stream);
int kfac_probe_copy(const void* src, void* dst, size_t bytes, int32_t workgroups, void* stream);
int kfac_probe_read(const void* src, float* sink, size_t bytes, int32_t workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KFAC_H_ */
