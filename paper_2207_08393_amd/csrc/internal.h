// Internal (non-ABI) declarations shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>

#include "../../include/gleam.h"

namespace gleam {

constexpr int kMaxLayers = 32;
constexpr int kMaxChannels = 256;
constexpr int kMaxTaps = 32;  // per-pixel tap validity is kept as one 32-bit mask

bool fft_size_supported(long long n);

// Current kernel-selection policy (GLEAM_POLICY_* bits; see gleam_set_kernel_policy).
unsigned kernel_policy();

// Optional per-launch event bracketing (see gleam_profile_begin).  KernelScope records a start event at
// construction and a stop event at destruction when profiling is on, and does nothing otherwise.
// `mfma_flops`: flops the launch issues on the matrix cores; negative = the same as `flops` (the algorithmic count),
// which holds for every direct kernel.  The Winograd kernels issue 16/36 of the direct convolution's flops.
bool prof_enabled();
void prof_begin(const char* name, double flops, double bytes, double mfma_flops, hipStream_t st);
void prof_end(hipStream_t st);
struct KernelScope {
    hipStream_t st;
    bool on;
    KernelScope(const char* name, double flops, double bytes, hipStream_t s, double mfma_flops = -1.0) : st(s), on(prof_enabled()) {
        if (on) prof_begin(name, flops, bytes, mfma_flops < 0.0 ? flops : mfma_flops, st);
    }
    ~KernelScope() {
        if (on) prof_end(st);
    }
};

// out = xs*x + gs * S^H F^H Omega (F S x - y); y may be null (then y = 0).  kbuf holds B*C*T*D*H*W
// complex values and is overwritten.  Everything is enqueued on `st`.
hipError_t sense_dc(const gleam_geom& g, const float2* x, const float2* S, const unsigned char* M,
                    const float2* y, float xs, float gs, float2* out, float2* kbuf, hipStream_t st);

// y: measured k-space, inverse-transformed in place along the outermost transformed axis (ndim_fft 2 or 3).
hipError_t kspace_to_hybrid(const gleam_geom& g, float2* y, hipStream_t st);

// Byte offsets of everything the prox keeps between and during calls.
//   saved : t_0 (= u, fp32 2 channels), t_1 .. t_{L-1} (fp32), g_z = dL/dz (fp32 2 channels)
//   ws    : [k-space | activations when the caller gave no saved buffer] for forward;
//           [G_1 .. G_{L-1} | split-K partials | loss partials] for backward
struct ProxPlan {
    int L;
    long long Q;                      // pixels B*T*D*H*W
    size_t act_off[kMaxLayers + 1];   // t_l inside saved, l < L
    size_t gz_off;
    size_t sign_off[kMaxLayers + 1];  // sign words of t_l inside saved, or 0 when there are none (see plan_prox)
    size_t saved_bytes;
    size_t grad_off[kMaxLayers + 1];  // G_l inside ws, 1 <= l < L
    size_t partial_off, partial_bytes;
    size_t bias_partial_off;          // [n_split][kMaxChannels] floats
    size_t wimg_off_fwd, wimg_off_bwd;  // re-laid weights of the layer being run (inside ws)
    size_t wino_u_off;                  // behind either of them: transformed weights of all Winograd layers of the pass
    size_t red_off;                   // loss partial sums (doubles)
    size_t k_bytes;                   // coil k-space buffer at the head of ws (forward)
    size_t ws_bytes;
    size_t w_off[kMaxLayers], b_off[kMaxLayers];  // float offsets into theta
    int n_split;                      // split-K workgroups of the weight-gradient kernels
    // t_j is stored after the ReLU of its only consumer (layer j+1 has relu_in, no layer takes t_j as a
    // skip source, and the producing layer adds no skip): the consumer then needs no ReLU on its operand,
    // and "stored value > 0" is the same ReLU mask for the backward pass.
    bool post_relu[kMaxLayers + 1];
};

// LDS bytes the weight-gradient kernel needs for one layer (must stay below the 160 KB of a CU).
size_t wgrad_lds_bytes(const gleam_conv& c);

// Whether prox dtype 1 (bfloat16 operands) has kernels for this network.
bool prox_bf16_supported(const gleam_prox_desc& p);

void plan_prox(const gleam_geom& g, const gleam_prox_desc& p, ProxPlan& plan);

// z = f_theta(u) with u = t_0 already stored at act_base + act_off[0]; writes t_1..t_{L-1} next to it
// and z to x_out.  With x_ref: loss (device scalar) and g_z are produced as well.
hipError_t prox_forward(const gleam_geom& g, const gleam_prox_desc& p, const ProxPlan& plan, const float* theta,
                        unsigned char* act_base, const float2* x_ref, float2* x_out, float* loss, void* ws,
                        hipStream_t st);

// grad_theta = dL/dtheta from the activations and g_z left by prox_forward.  g_in (may be null): receives
// dL/du, the gradient with respect to the prox input, float32 2 channels; it may alias t_0 inside `saved`
// (t_0 is dead once the first layer's weight gradient is done).  Requires layers[0].relu_in == 0 and at
// most one layer taking its skip from t_0.
hipError_t prox_backward(const gleam_geom& g, const gleam_prox_desc& p, const ProxPlan& plan, const float* theta,
                         const unsigned char* saved, float* grad_theta, float2* g_in, void* ws, hipStream_t st);

// loss (device scalar) of x against x_ref and g = dL/dx (2 real channels); `part` holds kLossPartials doubles.
// relu_mask: zero the gradient where x <= 0 (x is the output of a layer that ends in a ReLU).
constexpr int kLossPartials = 512;
hipError_t loss_and_grad(const float2* x, const float2* x_ref, float2* g, long long n, int loss_kind, int relu_mask,
                         double* part, float* loss, hipStream_t st);

// n_cg conjugate-gradient steps from zero on (A^H A + mu I) x = c1*u + c2*v (v may be null), one system per
// batch sample.  x may alias u.  kbuf: coil k-space buffer of sense_dc; scratch: cg_scratch_bytes(g) bytes.
constexpr int kCgBlocksMax = 512;  // workgroups (= partial sums) per batch sample
size_t cg_scratch_bytes(const gleam_geom& g);
hipError_t cg_solve(const gleam_geom& g, const float2* S, const unsigned char* M, float mu, int n_cg, const float2* u,
                    const float2* v, float c1, float c2, float2* x, float2* kbuf, void* scratch, hipStream_t st);
hipError_t fill_zero(float2* x, long long n, hipStream_t st);

// out (device scalar) = scale * sum over all samples of Re <u, v>; n complex values in total; part: kLossPartials doubles
hipError_t real_dot(const float2* u, const float2* v, long long n, double scale, double* part, float* out, hipStream_t st);

// theta <- Adam(theta, grad) in place with state m, v; bias corrections evaluated on the host in double.
hipError_t adam_update(const gleam_adam& h, long long t, size_t n, float* theta, const float* grad, float* m, float* v,
                       hipStream_t st);

}  // namespace gleam
