/* gleam.h - C ABI of the MI355X (gfx950) hot path of one GLEAM module step.
 *
 * One module of an unrolled proximal-gradient network trained greedily (paper: Methods,
 * "Greedy LEarning for Accelerated MRI Reconstruction", Alg. 1):
 *
 *     u     = x_in - alpha * A^H (A x_in - y)        data consistency, Eq. 3 (alpha = 2t)
 *     x_out = f_theta(u)                             learned proximal CNN, Eq. 4-5
 *     loss  = L(x_out, x_ref)                        local greedy objective, Eq. 10
 *     grad  = d loss / d theta   (this module only)  Alg. 1, gradient step
 *
 * with the multi-coil forward model A = Omega F S of Eq. 1-2: coil-sensitivity multiply S, orthonormal
 * uncentred DFT F over the last `ndim_fft` image dimensions, sampling mask Omega.
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library allocates and frees no
 *     device memory, writes no input, and enqueues all work on the caller's stream without synchronising.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Arrays are row-major with the last dimension contiguous; complex numbers are interleaved
 *     (re, im) float32 pairs (gleam_c64):
 *         image   x  [B][T][D][H][W]       coils  S [B][C][D][H][W]  (shared by all T frames)
 *         mask    M  [B][T][D][H][W] uint8 (non-zero = sampled, no coil dimension)
 *         k-space y  [B][C][T][D][H][W]    (values off the mask are ignored)
 *     An image is also the prox network's 2-channel real tensor (channels-last: re, im).
 *   - theta / grad_theta: flat float32, per layer W[cout][kt][kd][kh][kw][cin] then b[cout] if has_bias.
 *   - Return value: 0 (GLEAM_OK) or a negative gleam_status.  Arguments are validated on the host before
 *     anything is launched, in the entry points that run several modules as well: on any error other than
 *     GLEAM_E_LAUNCH nothing has been enqueued and no buffer has been written.
 *   - `ws` is scratch the call may overwrite freely; `saved` carries activations from gleam_module_fwd to
 *     gleam_module_bwd and may be reused for the next module afterwards (activations of a finished module
 *     are discarded, as in Alg. 1).  Both must be 256-byte aligned.  Sizes come from gleam_workspace_bytes.
 *   - Calls that share a workspace must be ordered on one stream.
 */
#ifndef GLEAM_H
#define GLEAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct { float re, im; } gleam_c64;

typedef enum {
    GLEAM_OK = 0,
    GLEAM_E_NULL = -1,              /* a required pointer is NULL                                      */
    GLEAM_E_DIMS = -2,              /* non-positive or inconsistent dimension, ndim_fft not 1, 2 or 3  */
    GLEAM_E_UNSUPPORTED_SIZE = -3,  /* a transformed length has no kernel (see gleam_fft_size_supported) */
    GLEAM_E_WORKSPACE = -4,         /* ws / saved too small or misaligned                              */
    GLEAM_E_DESC = -5,              /* prox description is not a valid / supported network             */
    GLEAM_E_LAUNCH = -6             /* the HIP runtime refused a launch                                */
} gleam_status;

/* Problem geometry.  ndim_fft = 2 transforms (H, W) and batches over D; ndim_fft = 3 transforms (D, H, W).
 * T counts temporal frames that are never transformed (2D+t cine); D = 1 and T = 1 for plain 2D.
 * ndim_fft = 1 transforms W only and batches over D and H: the form a problem takes when its mask does not
 * depend on an axis (line masks of 2D Cartesian sampling, a fully sampled read-out), after the measured k-space
 * has been inverse-transformed along that axis once (gleam_kspace_to_hybrid); the whole operator then runs in a
 * single sweep without the k-space buffer.  Every entry point accepts it.
 * centred = 0: zero frequency and spatial origin at index 0 of every transformed axis (the default reading of `F`
 * in Eq. 1, which the paper leaves open).  centred = 1: both in the middle of the axis (index n/2), i.e. the
 * transform fftshift . F . ifftshift that most MRI data comes in; mask and k-space are then indexed that way.
 * Every transformed length is even, so this costs only sign flips at the loads and stores of the sweeps. */
typedef struct {
    int32_t ndim_fft;
    int32_t centred;
    int64_t B, C, T, D, H, W;
} gleam_geom;

/* One convolution layer of the prox: cross-correlation, zero "same" padding, stride 1, odd extents.
 * With t_0 = u and t_l the output of layer l (1-based):
 *     a   = relu_in  ? max(t_{l-1}, 0) : t_{l-1}
 *     v   = conv(a, W_l) + b_l ;  v = relu_out ? max(v, 0) : v
 *     t_l = skip_src >= 0 ? v + t_{skip_src} : v          (skip_src < l, equal channel counts)
 * Layer 1 has cin = 2, the last layer cout = 2, and cin of layer l equals cout of layer l-1.
 * relu_out together with skip_src >= 0 on one layer is rejected (GLEAM_E_DESC). */
typedef struct {
    int32_t cin, cout, kt, kd, kh, kw;
    int32_t relu_in, relu_out, has_bias;
    int32_t skip_src;               /* -1: none */
} gleam_conv;

typedef struct {
    int32_t n_layers;
    const gleam_conv* layers;       /* host pointer, n_layers entries                                    */
    int32_t dtype;                  /* 0: float32 convolutions; 1: bfloat16 operands, float32 accumulate */
    int32_t loss_kind;              /* 0: mean |z-x|^2 over B*P complex pixels; 1: mean |z-x|            */
} gleam_prox_desc;

/* Bytes of scratch (`ws_bytes`, the maximum any of the three entry points needs for this geometry and
 * prox) and of saved activations (`saved_bytes`).  prox may be NULL: then only gleam_sense_normal's
 * scratch is counted and *saved_bytes = 0.  Host-only. */
int gleam_workspace_bytes(const gleam_geom* geom, const gleam_prox_desc* prox,
                          size_t* ws_bytes, size_t* saved_bytes);

/* Number of float32 parameters of the prox (length of theta and grad_theta).  Host-only. */
int gleam_theta_count(const gleam_prox_desc* prox, size_t* n_floats);

/* Kernel-selection policy.  Several layer shapes have two kernels: the fastest one, which every call uses by
 * default (policy 0), and the kernel it replaced, kept for A/B timing and as a second implementation for the
 * parity tests.  The policy is one process-wide word (the library reads nothing from the environment); it is
 * read when a call plans and enqueues its work, so set it before the first call of a forward / backward pair
 * and leave it alone until that pair is done: `saved` of a forward call is only valid for a backward call made
 * under the same policy (the Winograd and 2D-tile bf16 kernels hand ReLU masks over as sign words), and
 * gleam_workspace_bytes must be asked under the policy the calls will run with.  Not synchronised with calls in
 * flight on other threads.  Unknown bits: GLEAM_E_DESC. */
#define GLEAM_POLICY_NO_WINOGRAD      1u  /* 3x3 and 3x3x3 fp32 layers with wide channel counts: direct MFMA kernels    */
#define GLEAM_POLICY_NO_BF16_2D       2u  /* 3x3 bf16 layers: flattened-pixel kernel instead of the 2D-tile one        */
#define GLEAM_POLICY_NO_THIN_MFMA     4u  /* 2-channel first / last layers: vector-ALU kernels instead of matrix-core   */
#define GLEAM_POLICY_NO_WGRAD_BALANCE 8u  /* 27-tap weight gradient: nine 3-tap jobs instead of the balanced 8-wave split */
#define GLEAM_POLICY_NO_FRAME_WALK    16u /* kernels that walk an axis (3x1x1 fp32 layers along the frames: forward, data and
                                          * weight gradient; 3x3 bf16 weight gradient with 128 input channels down the
                                          * rows): the kernels that stage every tap row instead */
#define GLEAM_POLICY_ALL              31u
int gleam_set_kernel_policy(uint32_t policy);
uint32_t gleam_get_kernel_policy(void);

/* 1 if a transform of length n has a kernel, else 0.  Host-only. */
int gleam_fft_size_supported(int64_t n);

/* out = A^H A x : the normal operator of the forward model A = Omega F S (Eq. 1-2; the operator inside
 * the data-consistency step of Eq. 3).  x, out: image; S: coils; M: mask.  out must not alias x. */
int gleam_sense_normal(const gleam_geom* geom, const gleam_c64* x, const gleam_c64* S, const uint8_t* M,
                       gleam_c64* out, void* ws, size_t ws_bytes, void* stream);

/* gleam_sense_normal for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * results, but the coil k-space buffer is a device array of GLEAM_STATIC_SCRATCH_BYTES that the library holds at
 * file scope (one copy per GPU, resident from the moment the library is loaded on that GPU until the process
 * ends).  The call allocates and frees nothing on the device or through any allocating library routine; the
 * first call on a device looks up the array's address there (a runtime symbol query, not an allocation).
 *   - Geometries whose k-space B*C*T*D*H*W*8 bytes exceeds GLEAM_STATIC_SCRATCH_BYTES return GLEAM_E_WORKSPACE
 *     (ndim_fft = 1 uses no buffer but is held to the same limit).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 *     threads) race; order them on one stream.  Nothing needs clearing between calls: the first sweep of a call
 *     writes every element the later sweeps read.
 *   - With gleam_profile_begin active the per-launch bracketing creates HIP events; leave it off for such callers. */
#define GLEAM_STATIC_SCRATCH_BYTES (64u << 20)
int gleam_sense_normal_static(const gleam_geom* geom, const gleam_c64* x, const gleam_c64* S, const uint8_t* M,
                              gleam_c64* out, void* stream);

/* Forward pass of one module, x_out = f_theta(DC(x_in)) (Eq. 3-5; Alg. 1, forward step).
 *   x_ref  : fully sampled reference image, or NULL for inference (then `loss` and `saved` may be NULL
 *            and no backward pass may follow).
 *   loss   : device float32 scalar, overwritten with L(x_out, x_ref) (Eq. 10).
 *   x_out  : image, overwritten; must not alias x_in.  Passing it as the next module's x_in is the
 *            detached hand-off between modules. */
int gleam_module_fwd(const gleam_geom* geom, const gleam_prox_desc* prox,
                     const gleam_c64* x_in, const gleam_c64* S, const uint8_t* M, const gleam_c64* y,
                     float alpha, const float* theta, const gleam_c64* x_ref,
                     gleam_c64* x_out, float* loss,
                     void* saved, size_t saved_bytes, void* ws, size_t ws_bytes, void* stream);

/* Backward pass of the same module: grad_theta = d loss / d theta (Alg. 1, gradient step), overwritten.
 * Consumes `saved` of the matching gleam_module_fwd call (same geom / prox / theta).  No gradient is
 * produced for x_in, S or y: modules are decoupled and the data-consistency step is not differentiated. */
int gleam_module_bwd(const gleam_geom* geom, const gleam_prox_desc* prox, const float* theta,
                     const void* saved, size_t saved_bytes, float* grad_theta,
                     void* ws, size_t ws_bytes, void* stream);

/* gleam_module_bwd for a learnable step size (Eq. 3, alpha = 2t as a parameter of the module): grad_theta as
 * gleam_module_bwd, and grad_alpha (one float32 on the device) = dL/dalpha = -<dL/du, A^H (A x_in - y)>, the
 * inner product taken over real and imaginary parts.  dL/du is the gradient with respect to the prox input,
 * so the prox must have relu_in = 0 on its first layer and at most one layer taking its skip from the input
 * (else GLEAM_E_DESC); the residual image is recomputed with one more SENSE sweep.  x_in, S, M, y are the
 * arguments the forward call had; `saved` is written (the prox input is replaced by its gradient). */
int gleam_module_bwd_alpha(const gleam_geom* geom, const gleam_prox_desc* prox, const gleam_c64* x_in,
                           const gleam_c64* S, const uint8_t* M, const gleam_c64* y, const float* theta,
                           void* saved, size_t saved_bytes, float* grad_theta, float* grad_alpha, void* ws,
                           size_t ws_bytes, void* stream);

/* A module that holds n_iter = N/M unrolled iterations (GLEAM section, N > M), each with its own parameters:
 *     x_j = f_theta_j(DC(x_{j-1})),  j = 1..n_iter,   loss = L(x_{n_iter}, x_ref)
 * The local loss is backpropagated inside the module, through its prox networks and data-consistency steps
 * (dL/dx_{j-1} = g - alpha A^H A g with g = dL/du_j), and not beyond the module input.
 *   theta / grad_theta : [n_iter][n_theta] float32.
 *   saved              : n_iter equal blocks (saved_bytes / n_iter each), sized by gleam_deep_workspace_bytes;
 *                        written by both calls.  After gleam_deep_module_bwd, block j (0-based, j >= 1) begins
 *                        with dL/du_j, the gradient at the prox input of iteration j+1: B*T*D*H*W complex64
 *                        (float32 at every hand-off between iterations, also with dtype = 1).
 *   x_out, x_tmp       : final image and one image of scratch (must not alias x_in or each other).
 * Requires a prox whose first layer has relu_in = 0 and at most one layer taking its skip from the input
 * when n_iter > 1 (else GLEAM_E_DESC).  n_iter = 1 is gleam_module_fwd / gleam_module_bwd. */
int gleam_deep_workspace_bytes(const gleam_geom* geom, const gleam_prox_desc* prox, int n_iter,
                               size_t* ws_bytes, size_t* saved_bytes);
int gleam_deep_module_fwd(const gleam_geom* geom, const gleam_prox_desc* prox, int n_iter,
                          const gleam_c64* x_in, const gleam_c64* S, const uint8_t* M, const gleam_c64* y,
                          float alpha, const float* theta, const gleam_c64* x_ref, gleam_c64* x_out,
                          gleam_c64* x_tmp, float* loss, void* saved, size_t saved_bytes, void* ws,
                          size_t ws_bytes, void* stream);
int gleam_deep_module_bwd(const gleam_geom* geom, const gleam_prox_desc* prox, int n_iter,
                          const gleam_c64* S, const uint8_t* M, float alpha, const float* theta,
                          void* saved, size_t saved_bytes, float* grad_theta, void* ws, size_t ws_bytes,
                          void* stream);

/* out = A^H y = S^H F^H Omega y (Eq. 2's adjoint; the zero-filled SENSE image the networks start from and the
 * constant term of the MoDL update).  ws as sized by gleam_workspace_bytes(geom, NULL or prox) plus one image
 * (B*T*D*H*W complex64), or simply by gleam_modl_workspace_bytes.  out must not alias y. */
int gleam_sense_adjoint(const gleam_geom* geom, const gleam_c64* S, const uint8_t* M, const gleam_c64* y,
                        gleam_c64* out, void* ws, size_t ws_bytes, void* stream);

/* Measured k-space to hybrid space: y_out = inverse transform of y_in along the OUTERMOST transformed axis of
 * `geom` (H when ndim_fft = 2, D when ndim_fft = 3), every other axis untouched; orthonormal, centred when the
 * geometry is.  When the mask does not depend on that axis (gleam_mask_constant_along_outer_axis), the transform
 * along it cancels in A^H A, and the same problem (same x, S, mask, same results) runs with one transformed axis
 * less on y_out: pass the same sizes with ndim_fft - 1 to every other entry point (the axis becomes a batch
 * axis; two sweeps fewer per operator, a single sweep for ndim_fft = 1).  Done once per scan.
 * y_in, y_out: k-space [B][C][T][D][H][W]; y_out may be y_in (in place), otherwise y_in is not written.
 * ndim_fft = 1 has no such axis: GLEAM_E_DIMS. */
int gleam_kspace_to_hybrid(const gleam_geom* geom, const gleam_c64* y_in, gleam_c64* y_out, void* stream);

/* Host-only check on a HOST copy of the mask [B][T][D][H][W]: *constant = 1 when "sampled / not sampled" does
 * not depend on the index along the outermost transformed axis (H for ndim_fft = 2, D for 3), else 0. */
int gleam_mask_constant_along_outer_axis(const gleam_geom* geom, const uint8_t* M_host, int* constant);

/* One MoDL module (MoDL section, Eq. 6-8):
 *     z = f_theta(x_in)                                   (Eq. 8)
 *     x_out = (A^H A + mu I)^-1 (aty + mu z),  aty = A^H y (Eq. 7)
 * solved by exactly n_cg conjugate-gradient steps from zero, one system per batch sample (all scalars of the
 * recurrence stay on the device; a sample whose residual is exactly zero stops moving).  With x_ref the local
 * loss (device scalar) is produced and `saved` keeps what the backward pass needs.
 * gleam_modl_module_bwd: dL/dtheta; dL/dz = mu (A^H A + mu I)^-1 dL/dx_out is formed by the same n_cg-step
 * solve, then the prox is swept backwards; nothing is propagated to x_in.
 *   mu >= 0, n_cg >= 1 (else GLEAM_E_DIMS).  The last prox layer must not end in a ReLU (GLEAM_E_DESC).
 *   saved : as gleam_workspace_bytes reports (written by the backward pass as well).
 *   ws    : gleam_modl_workspace_bytes; x_out must not alias x_in, aty or x_ref. */
int gleam_modl_workspace_bytes(const gleam_geom* geom, const gleam_prox_desc* prox, size_t* ws_bytes,
                               size_t* saved_bytes);
int gleam_modl_module_fwd(const gleam_geom* geom, const gleam_prox_desc* prox, const gleam_c64* x_in,
                          const gleam_c64* S, const uint8_t* M, const gleam_c64* aty, float mu, int n_cg,
                          const float* theta, const gleam_c64* x_ref, gleam_c64* x_out, float* loss,
                          void* saved, size_t saved_bytes, void* ws, size_t ws_bytes, void* stream);
int gleam_modl_module_bwd(const gleam_geom* geom, const gleam_prox_desc* prox, const gleam_c64* S,
                          const uint8_t* M, float mu, int n_cg, const float* theta, void* saved,
                          size_t saved_bytes, float* grad_theta, void* ws, size_t ws_bytes, void* stream);

/* Adam hyper-parameters (Implementation Details: beta1 = 0.9, beta2 = 0.999; the paper does not state the
 * learning rate or epsilon). */
typedef struct {
    float lr, beta1, beta2, eps;
} gleam_adam;

/* One Adam update of n parameters in place ("Update Parameters" of Alg. 1), step count t >= 1:
 *     m <- beta1 m + (1-beta1) g ;  v <- beta2 v + (1-beta2) g^2
 *     theta <- theta - lr * (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps)
 * theta, grad, m, v: device float32 arrays of n elements; m and v are the optimizer state (zero before the
 * first step).  The bias corrections are evaluated on the host in double. */
int gleam_adam_step(const gleam_adam* hyper, int64_t t, size_t n, float* theta, const float* grad,
                    float* m, float* v, void* stream);

/* One greedy training iteration over a mini-batch (Alg. 1): for module i = 1..n_modules, forward
 * x_i = f_theta_i(DC(x_{i-1})), local loss against x_ref (Eq. 10), gradient of that loss with respect to
 * theta_i only, Adam update of theta_i; the module's activations are then dropped (`saved` and `ws` are
 * reused by the next module) and x_i is handed on without gradient.
 *   x0        : input image of module 1 (e.g. the zero-filled reconstruction A^H y); not written.
 *   theta     : [n_modules][n_theta] float32, updated in place (n_theta = gleam_theta_count).
 *   adam_m/_v : optimizer state, same shape as theta.
 *   t         : Adam step count of this iteration (>= 1), the same for every module.
 *   x_out     : x_{n_modules}, overwritten.  x_tmp: one more image of scratch (the modules alternate between
 *               the two).  Neither may alias x0.
 *   losses    : device float32 [n_modules], loss of every module before its update.
 *   grad      : device scratch of n_theta floats.
 * Every module's output is computed with its parameters BEFORE the update.  All modules share the
 * architecture `prox`.  Other arguments as in gleam_module_fwd. */
int gleam_greedy_iteration(const gleam_geom* geom, const gleam_prox_desc* prox, int n_modules,
                           const gleam_c64* x0, const gleam_c64* S, const uint8_t* M, const gleam_c64* y,
                           float alpha, float* theta, float* adam_m, float* adam_v, const gleam_adam* hyper,
                           int64_t t, const gleam_c64* x_ref, gleam_c64* x_out, gleam_c64* x_tmp,
                           float* losses, float* grad, void* saved, size_t saved_bytes, void* ws,
                           size_t ws_bytes, void* stream);

/* Inference through the first n_modules modules (all of them, or fewer: early exit at depth N_inf),
 * x_i = f_theta_i(DC(x_{i-1})); nothing is saved.  theta: [n_modules][n_theta]; x_out, x_tmp as above. */
int gleam_unrolled_infer(const gleam_geom* geom, const gleam_prox_desc* prox, int n_modules,
                         const gleam_c64* x0, const gleam_c64* S, const uint8_t* M, const gleam_c64* y,
                         float alpha, const float* theta, gleam_c64* x_out, gleam_c64* x_tmp,
                         void* ws, size_t ws_bytes, void* stream);

/* Measurement aid (not part of the method): between gleam_profile_begin and gleam_profile_end every kernel
 * this library launches is bracketed by HIP events on the caller's stream.  gleam_profile_end synchronises
 * the device and copies up to `capacity` per-launch records (launch order) to the HOST array `out`;
 * *n_records receives the number of launches seen.  `flops` / `bytes` are the algorithmic work of the launch
 * (padding and re-reads not counted; a convolution counts 2 * taps * cin * cout per pixel whatever the kernel);
 * `mfma_flops` is what the launch issues on the matrix cores: equal to `flops` for the direct kernels, 4/9 of it
 * for the Winograd F(2x2,3x3) kernels, so mfma_flops / time never exceeds the matrix-core peak.
 * Not thread-safe; leave it off in production. */
typedef struct {
    char name[56];
    double flops;
    double bytes;
    double mfma_flops;
    float ms;
} gleam_kernel_record;
int gleam_profile_begin(void);
int gleam_profile_end(gleam_kernel_record* out, int capacity, int* n_records);

/* Static message for a gleam_status value. */
const char* gleam_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* GLEAM_H */
