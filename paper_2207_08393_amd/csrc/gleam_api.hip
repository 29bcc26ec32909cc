// C ABI of the library: host-side validation, workspace carving and kernel sequencing.
// Nothing here touches device memory directly; every step is a kernel of sense.hip / prox.hip
// enqueued on the caller's stream.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "internal.h"

using namespace gleam;

namespace gleam {
namespace {
struct ProfRec {
    char name[56];
    double flops, bytes, mfma_flops;
    hipEvent_t e0, e1;
};
bool g_prof_on = false;
std::vector<ProfRec> g_prof;
}  // namespace
namespace {
std::atomic<unsigned> g_policy{0u};
}
unsigned kernel_policy() { return g_policy.load(std::memory_order_relaxed); }
bool prof_enabled() { return g_prof_on; }
void prof_begin(const char* name, double flops, double bytes, double mfma_flops, hipStream_t st) {
    ProfRec r{};
    snprintf(r.name, sizeof(r.name), "%s", name);
    r.flops = flops;
    r.bytes = bytes;
    r.mfma_flops = mfma_flops;
    if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) return;
    (void)hipEventRecord(r.e0, st);
    g_prof.push_back(r);
}
void prof_end(hipStream_t st) {
    if (!g_prof.empty()) (void)hipEventRecord(g_prof.back().e1, st);
}
}  // namespace gleam

// Coil k-space buffer of gleam_sense_normal_static: file-scope device memory, one copy per GPU, held until the
// process ends.  Host code never uses the array's name as an address; static_scratch() asks the runtime for
// the address of the current device's copy once and hands that pointer to the kernels.
static __device__ __align__(256) unsigned char scratch[GLEAM_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device), or null.
void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline bool aligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) % kAlign) == 0; }

int check_geom(const gleam_geom* g) {
    if (!g) return GLEAM_E_NULL;
    if (g->ndim_fft < 1 || g->ndim_fft > 3) return GLEAM_E_DIMS;
    if (g->centred != 0 && g->centred != 1) return GLEAM_E_DIMS;
    if (g->B < 1 || g->C < 1 || g->T < 1 || g->D < 1 || g->H < 1 || g->W < 1) return GLEAM_E_DIMS;
    const long long lim = 1LL << 40;  // keeps every byte offset far inside int64
    long long e = 1;
    for (long long v : {g->B, g->C, g->T, g->D, g->H, g->W}) {
        if (v > lim / e) return GLEAM_E_DIMS;
        e *= v;
    }
    if (!fft_size_supported(g->W)) return GLEAM_E_UNSUPPORTED_SIZE;
    if (g->ndim_fft >= 2 && !fft_size_supported(g->H)) return GLEAM_E_UNSUPPORTED_SIZE;
    if (g->ndim_fft == 3 && !fft_size_supported(g->D)) return GLEAM_E_UNSUPPORTED_SIZE;
    return GLEAM_OK;
}

inline size_t n_coil_pixels(const gleam_geom& g) { return (size_t)(g.B * g.C * g.T * g.D * g.H * g.W); }
inline size_t n_pixels(const gleam_geom& g) { return (size_t)(g.B * g.T * g.D * g.H * g.W); }

int check_prox(const gleam_prox_desc* p) {
    if (!p) return GLEAM_E_NULL;
    if (p->n_layers < 1 || p->n_layers > kMaxLayers || !p->layers) return GLEAM_E_DESC;
    if (p->dtype != 0 && p->dtype != 1) return GLEAM_E_DESC;
    if (p->loss_kind != 0 && p->loss_kind != 1) return GLEAM_E_DESC;
    int prev = 2;
    std::vector<int> ch(p->n_layers + 1);
    ch[0] = 2;
    for (int l = 0; l < p->n_layers; ++l) {
        const gleam_conv& c = p->layers[l];
        if (c.cin != prev || c.cout < 1 || c.cout > kMaxChannels) return GLEAM_E_DESC;
        for (int k : {c.kt, c.kd, c.kh, c.kw})
            if (k < 1 || k > 5 || (k % 2) == 0) return GLEAM_E_DESC;
        if (c.kt * c.kd * c.kh * c.kw > kMaxTaps) return GLEAM_E_DESC;
        if (c.skip_src < -1 || c.skip_src > l) return GLEAM_E_DESC;
        if (c.skip_src >= 0 && ch[c.skip_src] != c.cout) return GLEAM_E_DESC;
        if (c.skip_src >= 0 && c.relu_out) return GLEAM_E_DESC;
        for (int m = 0; m < l; ++m)  // one consumer per skip source
            if (c.skip_src >= 1 && p->layers[m].skip_src == c.skip_src) return GLEAM_E_DESC;
        if (wgrad_lds_bytes(c) > 150 * 1024) return GLEAM_E_DESC;
        ch[l + 1] = c.cout;
        prev = c.cout;
    }
    if (prev != 2) return GLEAM_E_DESC;
    if (p->dtype == 1 && !prox_bf16_supported(*p)) return GLEAM_E_DESC;
    return GLEAM_OK;
}

// Geometry, prox and buffer sizes of a plain module call, checked together so that callers which run several
// modules can refuse bad arguments before the first launch.  `saved` may be null when need_saved is false.
int check_module_buffers(const gleam_geom* geom, const gleam_prox_desc* prox, const void* ws, size_t ws_bytes,
                         const void* saved, size_t saved_bytes, bool need_saved) {
    int rc = check_geom(geom);
    if (rc) return rc;
    rc = check_prox(prox);
    if (rc) return rc;
    if (!ws || (need_saved && !saved)) return GLEAM_E_NULL;
    ProxPlan plan;
    plan_prox(*geom, *prox, plan);
    if (!aligned(ws) || ws_bytes < plan.ws_bytes) return GLEAM_E_WORKSPACE;
    if (saved && (!aligned(saved) || saved_bytes < plan.saved_bytes)) return GLEAM_E_WORKSPACE;
    return GLEAM_OK;
}

bool adam_args_ok(const gleam_adam* h, int64_t t) {
    return t >= 1 && h->beta1 >= 0.f && h->beta1 < 1.f && h->beta2 >= 0.f && h->beta2 < 1.f && h->eps >= 0.f;
}

}  // namespace

extern "C" {

const char* gleam_strerror(int status) {
    switch (status) {
        case GLEAM_OK: return "ok";
        case GLEAM_E_NULL: return "a required pointer is NULL";
        case GLEAM_E_DIMS: return "invalid geometry";
        case GLEAM_E_UNSUPPORTED_SIZE: return "no transform kernel for one of the Fourier lengths";
        case GLEAM_E_WORKSPACE: return "workspace or saved buffer too small or not 256-byte aligned";
        case GLEAM_E_DESC: return "invalid or unsupported prox description";
        case GLEAM_E_LAUNCH: return "HIP launch failed";
        default: return "unknown gleam status";
    }
}

int gleam_profile_begin(void) {
    for (auto& r : g_prof) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
    g_prof.clear();
    g_prof_on = true;
    return GLEAM_OK;
}

int gleam_profile_end(gleam_kernel_record* out, int capacity, int* n_records) {
    g_prof_on = false;
    if (!n_records || (capacity > 0 && !out)) return GLEAM_E_NULL;
    if (hipDeviceSynchronize() != hipSuccess) return GLEAM_E_LAUNCH;
    *n_records = (int)g_prof.size();
    for (int i = 0; i < (int)g_prof.size(); ++i) {
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, g_prof[i].e0, g_prof[i].e1);
        if (i < capacity) {
            memcpy(out[i].name, g_prof[i].name, sizeof(out[i].name));
            out[i].flops = g_prof[i].flops;
            out[i].bytes = g_prof[i].bytes;
            out[i].mfma_flops = g_prof[i].mfma_flops;
            out[i].ms = ms;
        }
        (void)hipEventDestroy(g_prof[i].e0);
        (void)hipEventDestroy(g_prof[i].e1);
    }
    g_prof.clear();
    return GLEAM_OK;
}

int gleam_set_kernel_policy(uint32_t policy) {
    if (policy & ~(uint32_t)GLEAM_POLICY_ALL) return GLEAM_E_DESC;
    g_policy.store(policy, std::memory_order_relaxed);
    return GLEAM_OK;
}

uint32_t gleam_get_kernel_policy(void) { return kernel_policy(); }

int gleam_fft_size_supported(int64_t n) { return fft_size_supported(n) ? 1 : 0; }

int gleam_theta_count(const gleam_prox_desc* prox, size_t* n_floats) {
    if (!n_floats) return GLEAM_E_NULL;
    int rc = check_prox(prox);
    if (rc) return rc;
    size_t n = 0;
    for (int l = 0; l < prox->n_layers; ++l) {
        const gleam_conv& c = prox->layers[l];
        n += (size_t)c.cout * c.kt * c.kd * c.kh * c.kw * c.cin + (c.has_bias ? c.cout : 0);
    }
    *n_floats = n;
    return GLEAM_OK;
}

int gleam_workspace_bytes(const gleam_geom* geom, const gleam_prox_desc* prox, size_t* ws_bytes,
                          size_t* saved_bytes) {
    if (!ws_bytes || !saved_bytes) return GLEAM_E_NULL;
    int rc = check_geom(geom);
    if (rc) return rc;
    size_t ws = align_up(n_coil_pixels(*geom) * sizeof(float2));
    size_t saved = 0;
    if (prox) {
        rc = check_prox(prox);
        if (rc) return rc;
        ProxPlan plan;
        plan_prox(*geom, *prox, plan);
        if (plan.ws_bytes > ws) ws = plan.ws_bytes;
        saved = plan.saved_bytes;
    }
    *ws_bytes = ws;
    *saved_bytes = saved;
    return GLEAM_OK;
}

int gleam_sense_normal(const gleam_geom* geom, const gleam_c64* x, const gleam_c64* S, const uint8_t* M,
                       gleam_c64* out, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc) return rc;
    if (!x || !S || !M || !out || !ws) return GLEAM_E_NULL;
    if (!aligned(ws) || ws_bytes < n_coil_pixels(*geom) * sizeof(float2)) return GLEAM_E_WORKSPACE;
    hipError_t e = sense_dc(*geom, (const float2*)x, (const float2*)S, M, nullptr, 0.f, 1.f, (float2*)out,
                            (float2*)ws, (hipStream_t)stream);
    return e == hipSuccess ? GLEAM_OK : GLEAM_E_LAUNCH;
}

int gleam_sense_normal_static(const gleam_geom* geom, const gleam_c64* x, const gleam_c64* S, const uint8_t* M,
                              gleam_c64* out, void* stream) {
    int rc = check_geom(geom);
    if (rc) return rc;
    if (!x || !S || !M || !out) return GLEAM_E_NULL;
    if (n_coil_pixels(*geom) * sizeof(float2) > (size_t)GLEAM_STATIC_SCRATCH_BYTES) return GLEAM_E_WORKSPACE;
    void* kbuf = static_scratch();
    if (!kbuf) return GLEAM_E_LAUNCH;
    // every k-space element the later sweeps read is written by the first sweep of the same call, so nothing
    // of the previous call's contents has to be cleared
    hipError_t e = sense_dc(*geom, (const float2*)x, (const float2*)S, M, nullptr, 0.f, 1.f, (float2*)out,
                            (float2*)kbuf, (hipStream_t)stream);
    return e == hipSuccess ? GLEAM_OK : GLEAM_E_LAUNCH;
}

int gleam_module_fwd(const gleam_geom* geom, const gleam_prox_desc* prox, const gleam_c64* x_in,
                     const gleam_c64* S, const uint8_t* M, const gleam_c64* y, float alpha, const float* theta,
                     const gleam_c64* x_ref, gleam_c64* x_out, float* loss, void* saved, size_t saved_bytes,
                     void* ws, size_t ws_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc) return rc;
    rc = check_prox(prox);
    if (rc) return rc;
    if (!x_in || !S || !M || !y || !theta || !x_out || !ws) return GLEAM_E_NULL;
    if (x_ref && (!loss || !saved)) return GLEAM_E_NULL;
    ProxPlan plan;
    plan_prox(*geom, *prox, plan);
    if (!aligned(ws) || ws_bytes < plan.ws_bytes) return GLEAM_E_WORKSPACE;
    if (saved && (!aligned(saved) || saved_bytes < plan.saved_bytes)) return GLEAM_E_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    // Without a saved buffer (inference) the activations live in the workspace, after the k-space buffer.
    unsigned char* act_base = saved ? (unsigned char*)saved : (unsigned char*)ws + plan.k_bytes;
    float2* u = (float2*)(act_base + plan.act_off[0]);
    hipError_t e = sense_dc(*geom, (const float2*)x_in, (const float2*)S, M, (const float2*)y, 1.f, -alpha, u,
                            (float2*)ws, st);
    if (e != hipSuccess) return GLEAM_E_LAUNCH;
    e = prox_forward(*geom, *prox, plan, theta, act_base, (const float2*)x_ref, (float2*)x_out, loss, ws, st);
    return e == hipSuccess ? GLEAM_OK : GLEAM_E_LAUNCH;
}

int gleam_module_bwd(const gleam_geom* geom, const gleam_prox_desc* prox, const float* theta, const void* saved,
                     size_t saved_bytes, float* grad_theta, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc) return rc;
    rc = check_prox(prox);
    if (rc) return rc;
    if (!theta || !saved || !grad_theta || !ws) return GLEAM_E_NULL;
    ProxPlan plan;
    plan_prox(*geom, *prox, plan);
    if (!aligned(ws) || ws_bytes < plan.ws_bytes) return GLEAM_E_WORKSPACE;
    if (!aligned(saved) || saved_bytes < plan.saved_bytes) return GLEAM_E_WORKSPACE;
    hipError_t e = prox_backward(*geom, *prox, plan, theta, (const unsigned char*)saved, grad_theta, nullptr, ws,
                                 (hipStream_t)stream);
    return e == hipSuccess ? GLEAM_OK : GLEAM_E_LAUNCH;
}

static int check_deep(const gleam_prox_desc* prox, int n_iter);

int gleam_module_bwd_alpha(const gleam_geom* geom, const gleam_prox_desc* prox, const gleam_c64* x_in, const gleam_c64* S,
                           const uint8_t* M, const gleam_c64* y, const float* theta, void* saved, size_t saved_bytes,
                           float* grad_theta, float* grad_alpha, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc) return rc;
    rc = check_prox(prox);
    if (rc) return rc;
    rc = check_deep(prox, 2);   // the same conditions as a gradient that crosses the prox input
    if (rc) return rc;
    if (!x_in || !S || !M || !y || !theta || !saved || !grad_theta || !grad_alpha || !ws) return GLEAM_E_NULL;
    ProxPlan plan;
    plan_prox(*geom, *prox, plan);
    if (!aligned(ws) || ws_bytes < plan.ws_bytes) return GLEAM_E_WORKSPACE;
    if (!aligned(saved) || saved_bytes < plan.saved_bytes) return GLEAM_E_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    float2* g_u = (float2*)((unsigned char*)saved + plan.act_off[0]);   // dL/du replaces u, which is dead by then
    hipError_t e = prox_backward(*geom, *prox, plan, theta, (const unsigned char*)saved, grad_theta, g_u, ws, st);
    if (e != hipSuccess) return GLEAM_E_LAUNCH;
    // r = A^H (A x_in - y) into the image slot behind the k-space buffer, then dL/dalpha = -<dL/du, r>
    float2* r = (float2*)((unsigned char*)ws + plan.k_bytes);
    e = sense_dc(*geom, (const float2*)x_in, (const float2*)S, M, (const float2*)y, 0.f, 1.f, r, (float2*)ws, st);
    if (e != hipSuccess) return GLEAM_E_LAUNCH;
    // the partial sums go behind the residual image (the head of the workspace is the k-space buffer)
    double* part = (double*)((unsigned char*)ws + plan.k_bytes + align_up((size_t)plan.Q * sizeof(float2)));
    e = real_dot(g_u, r, plan.Q, -1.0, part, grad_alpha, st);
    return e == hipSuccess ? GLEAM_OK : GLEAM_E_LAUNCH;
}

static int check_deep(const gleam_prox_desc* prox, int n_iter) {
    if (n_iter < 1) return GLEAM_E_DIMS;
    if (n_iter == 1) return GLEAM_OK;
    if (prox->layers[0].relu_in) return GLEAM_E_DESC;
    int from_input = 0;
    for (int l = 0; l < prox->n_layers; ++l) from_input += prox->layers[l].skip_src == 0 ? 1 : 0;
    return from_input <= 1 ? GLEAM_OK : GLEAM_E_DESC;
}

int gleam_deep_workspace_bytes(const gleam_geom* geom, const gleam_prox_desc* prox, int n_iter, size_t* ws_bytes,
                               size_t* saved_bytes) {
    if (!prox) return GLEAM_E_NULL;
    int rc = gleam_workspace_bytes(geom, prox, ws_bytes, saved_bytes);
    if (rc) return rc;
    rc = check_deep(prox, n_iter);
    if (rc) return rc;
    *saved_bytes = align_up(*saved_bytes) * (size_t)n_iter;
    return GLEAM_OK;
}

int gleam_deep_module_fwd(const gleam_geom* geom, const gleam_prox_desc* prox, int n_iter, const gleam_c64* x_in,
                          const gleam_c64* S, const uint8_t* M, const gleam_c64* y, float alpha, const float* theta,
                          const gleam_c64* x_ref, gleam_c64* x_out, gleam_c64* x_tmp, float* loss, void* saved,
                          size_t saved_bytes, void* ws, size_t ws_bytes, void* stream) {
    size_t ws_need = 0, saved_need = 0, n_theta = 0;
    int rc = gleam_deep_workspace_bytes(geom, prox, n_iter, &ws_need, &saved_need);
    if (rc) return rc;
    if (!x_in || !S || !M || !y || !theta || !x_ref || !x_out || !x_tmp || !loss || !saved || !ws) return GLEAM_E_NULL;
    if (x_out == x_in || x_tmp == x_in || x_out == x_tmp) return GLEAM_E_DIMS;
    if (!aligned(ws) || ws_bytes < ws_need) return GLEAM_E_WORKSPACE;   // all of it before the first launch
    if (!aligned(saved) || saved_bytes < saved_need) return GLEAM_E_WORKSPACE;
    rc = gleam_theta_count(prox, &n_theta);
    if (rc) return rc;
    const size_t block = saved_need / (size_t)n_iter;
    const gleam_c64* xi = x_in;
    for (int j = 0; j < n_iter; ++j) {
        const bool last = j == n_iter - 1;
        gleam_c64* xo = ((n_iter - 1 - j) % 2 == 0) ? x_out : x_tmp;   // the last iteration writes x_out
        rc = gleam_module_fwd(geom, prox, xi, S, M, y, alpha, theta + (size_t)j * n_theta, last ? x_ref : nullptr, xo,
                              last ? loss : nullptr, (unsigned char*)saved + (size_t)j * block, block, ws, ws_bytes, stream);
        if (rc) return rc;
        xi = xo;
    }
    return GLEAM_OK;
}

int gleam_deep_module_bwd(const gleam_geom* geom, const gleam_prox_desc* prox, int n_iter, const gleam_c64* S,
                          const uint8_t* M, float alpha, const float* theta, void* saved, size_t saved_bytes,
                          float* grad_theta, void* ws, size_t ws_bytes, void* stream) {
    size_t ws_need = 0, saved_need = 0, n_theta = 0;
    int rc = gleam_deep_workspace_bytes(geom, prox, n_iter, &ws_need, &saved_need);
    if (rc) return rc;
    if (!S || !M || !theta || !saved || !grad_theta || !ws) return GLEAM_E_NULL;
    if (!aligned(ws) || ws_bytes < ws_need) return GLEAM_E_WORKSPACE;
    if (!aligned(saved) || saved_bytes < saved_need) return GLEAM_E_WORKSPACE;
    rc = gleam_theta_count(prox, &n_theta);
    if (rc) return rc;
    ProxPlan plan;
    plan_prox(*geom, *prox, plan);
    const size_t block = saved_need / (size_t)n_iter;
    hipStream_t st = (hipStream_t)stream;
    for (int j = n_iter - 1; j >= 0; --j) {
        unsigned char* sj = (unsigned char*)saved + (size_t)j * block;
        // dL/du_j overwrites u_j = t_0 of this iteration, which is dead once its first layer's weight gradient is done
        float2* g_u = j > 0 ? (float2*)(sj + plan.act_off[0]) : nullptr;
        hipError_t e = prox_backward(*geom, *prox, plan, theta + (size_t)j * n_theta, sj, grad_theta + (size_t)j * n_theta, g_u,
                                     ws, st);
        if (e != hipSuccess) return GLEAM_E_LAUNCH;
        if (j > 0) {
            // through the data-consistency step: dL/dx_{j-1} = g_u - alpha A^H A g_u, the incoming gradient of iteration j-1
            float2* g_prev = (float2*)((unsigned char*)saved + (size_t)(j - 1) * block + plan.gz_off);
            e = sense_dc(*geom, g_u, (const float2*)S, M, nullptr, 1.f, -alpha, g_prev, (float2*)ws, st);
            if (e != hipSuccess) return GLEAM_E_LAUNCH;
        }
    }
    return GLEAM_OK;
}

int gleam_sense_adjoint(const gleam_geom* geom, const gleam_c64* S, const uint8_t* M, const gleam_c64* y, gleam_c64* out,
                        void* ws, size_t ws_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc) return rc;
    if (!S || !M || !y || !out || !ws) return GLEAM_E_NULL;
    if (out == y) return GLEAM_E_DIMS;
    const size_t kb = align_up(n_coil_pixels(*geom) * sizeof(float2));
    const long long n = geom->B * geom->T * geom->D * geom->H * geom->W;
    if (!aligned(ws) || ws_bytes < kb + (size_t)n * sizeof(float2)) return GLEAM_E_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    // A^H y = -(A^H (A 0 - y)): the fused sweep on a zero image
    float2* zero = (float2*)((unsigned char*)ws + kb);
    hipError_t e = fill_zero(zero, n, st);
    if (e != hipSuccess) return GLEAM_E_LAUNCH;
    e = sense_dc(*geom, zero, (const float2*)S, M, (const float2*)y, 0.f, -1.f, (float2*)out, (float2*)ws, st);
    return e == hipSuccess ? GLEAM_OK : GLEAM_E_LAUNCH;
}

int gleam_kspace_to_hybrid(const gleam_geom* geom, const gleam_c64* y_in, gleam_c64* y_out, void* stream) {
    int rc = check_geom(geom);
    if (rc) return rc;
    if (geom->ndim_fft < 2) return GLEAM_E_DIMS;
    if (!y_in || !y_out) return GLEAM_E_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (y_out != y_in &&
        hipMemcpyAsync(y_out, y_in, n_coil_pixels(*geom) * sizeof(float2), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return GLEAM_E_LAUNCH;
    return kspace_to_hybrid(*geom, (float2*)y_out, st) == hipSuccess ? GLEAM_OK : GLEAM_E_LAUNCH;
}

int gleam_mask_constant_along_outer_axis(const gleam_geom* geom, const uint8_t* M_host, int* constant) {
    int rc = check_geom(geom);
    if (rc) return rc;
    if (geom->ndim_fft < 2) return GLEAM_E_DIMS;
    if (!M_host || !constant) return GLEAM_E_NULL;
    // mask viewed as [outer][n][inner] with n the axis in question
    const long long n = geom->ndim_fft == 2 ? geom->H : geom->D;
    const long long inner = geom->ndim_fft == 2 ? geom->W : geom->H * geom->W;
    const long long outer = geom->B * geom->T * (geom->ndim_fft == 2 ? geom->D : 1);
    *constant = 1;
    for (long long o = 0; o < outer; ++o) {
        const uint8_t* first = M_host + o * n * inner;
        for (long long i = 1; i < n; ++i) {
            const uint8_t* row = first + i * inner;
            for (long long j = 0; j < inner; ++j)
                if ((row[j] != 0) != (first[j] != 0)) {
                    *constant = 0;
                    return GLEAM_OK;
                }
        }
    }
    return GLEAM_OK;
}

static int check_modl(const gleam_geom* geom, const gleam_prox_desc* prox, float mu, int n_cg) {
    int rc = check_geom(geom);
    if (rc) return rc;
    rc = check_prox(prox);
    if (rc) return rc;
    if (prox->layers[prox->n_layers - 1].relu_out) return GLEAM_E_DESC;
    if (!(mu >= 0.f) || !(mu < 3.0e38f) || n_cg < 1) return GLEAM_E_DIMS;
    return GLEAM_OK;
}

int gleam_modl_workspace_bytes(const gleam_geom* geom, const gleam_prox_desc* prox, size_t* ws_bytes, size_t* saved_bytes) {
    if (!prox) return GLEAM_E_NULL;
    int rc = gleam_workspace_bytes(geom, prox, ws_bytes, saved_bytes);
    if (rc) return rc;
    if (prox->layers[prox->n_layers - 1].relu_out) return GLEAM_E_DESC;
    *ws_bytes = align_up(*ws_bytes) + cg_scratch_bytes(*geom);
    return GLEAM_OK;
}

int gleam_modl_module_fwd(const gleam_geom* geom, const gleam_prox_desc* prox, const gleam_c64* x_in, const gleam_c64* S,
                          const uint8_t* M, const gleam_c64* aty, float mu, int n_cg, const float* theta,
                          const gleam_c64* x_ref, gleam_c64* x_out, float* loss, void* saved, size_t saved_bytes, void* ws,
                          size_t ws_bytes, void* stream) {
    int rc = check_modl(geom, prox, mu, n_cg);
    if (rc) return rc;
    if (!x_in || !S || !M || !aty || !theta || !x_out || !ws) return GLEAM_E_NULL;
    if (x_ref && (!loss || !saved)) return GLEAM_E_NULL;
    if (x_out == x_in || x_out == aty || (x_ref && x_out == x_ref)) return GLEAM_E_DIMS;
    size_t ws_need = 0, saved_need = 0;
    rc = gleam_modl_workspace_bytes(geom, prox, &ws_need, &saved_need);
    if (rc) return rc;
    if (!aligned(ws) || ws_bytes < ws_need) return GLEAM_E_WORKSPACE;
    if (saved && (!aligned(saved) || saved_bytes < saved_need)) return GLEAM_E_WORKSPACE;
    ProxPlan plan;
    plan_prox(*geom, *prox, plan);
    hipStream_t st = (hipStream_t)stream;
    unsigned char* act_base = saved ? (unsigned char*)saved : (unsigned char*)ws + plan.k_bytes;
    unsigned char* scratch = (unsigned char*)ws + (ws_need - cg_scratch_bytes(*geom));
    const size_t img = (size_t)plan.Q * sizeof(float2);
    // the prox input t_0 is the module input itself
    if (hipMemcpyAsync(act_base + plan.act_off[0], x_in, img, hipMemcpyDeviceToDevice, st) != hipSuccess) return GLEAM_E_LAUNCH;
    // z lands in the solver's third vector, which the first operator application overwrites only after the
    // right-hand side aty + mu z has been formed
    float2* z = (float2*)(scratch + 2 * align_up(img));
    hipError_t e = prox_forward(*geom, *prox, plan, theta, act_base, nullptr, z, nullptr, ws, st);
    if (e != hipSuccess) return GLEAM_E_LAUNCH;
    e = cg_solve(*geom, (const float2*)S, M, mu, n_cg, (const float2*)aty, z, 1.f, mu, (float2*)x_out, (float2*)ws, scratch, st);
    if (e != hipSuccess) return GLEAM_E_LAUNCH;
    if (x_ref) {
        e = loss_and_grad((const float2*)x_out, (const float2*)x_ref, (float2*)(act_base + plan.gz_off), plan.Q, prox->loss_kind,
                          0, (double*)((unsigned char*)ws + plan.red_off), loss, st);
        if (e != hipSuccess) return GLEAM_E_LAUNCH;
    }
    return GLEAM_OK;
}

int gleam_modl_module_bwd(const gleam_geom* geom, const gleam_prox_desc* prox, const gleam_c64* S, const uint8_t* M, float mu,
                          int n_cg, const float* theta, void* saved, size_t saved_bytes, float* grad_theta, void* ws,
                          size_t ws_bytes, void* stream) {
    int rc = check_modl(geom, prox, mu, n_cg);
    if (rc) return rc;
    if (!S || !M || !theta || !saved || !grad_theta || !ws) return GLEAM_E_NULL;
    size_t ws_need = 0, saved_need = 0;
    rc = gleam_modl_workspace_bytes(geom, prox, &ws_need, &saved_need);
    if (rc) return rc;
    if (!aligned(ws) || ws_bytes < ws_need) return GLEAM_E_WORKSPACE;
    if (!aligned(saved) || saved_bytes < saved_need) return GLEAM_E_WORKSPACE;
    ProxPlan plan;
    plan_prox(*geom, *prox, plan);
    hipStream_t st = (hipStream_t)stream;
    unsigned char* scratch = (unsigned char*)ws + (ws_need - cg_scratch_bytes(*geom));
    // dL/dz = mu Q^-1 dL/dx_out, solved in place: the solve is linear in its right-hand side, so the factor mu
    // goes into the right-hand side and the solution replaces the loss gradient where the prox sweep expects it
    float2* g = (float2*)((unsigned char*)saved + plan.gz_off);
    hipError_t e = cg_solve(*geom, (const float2*)S, M, mu, n_cg, g, nullptr, mu, 0.f, g, (float2*)ws, scratch, st);
    if (e != hipSuccess) return GLEAM_E_LAUNCH;
    e = prox_backward(*geom, *prox, plan, theta, (const unsigned char*)saved, grad_theta, nullptr, ws, st);
    return e == hipSuccess ? GLEAM_OK : GLEAM_E_LAUNCH;
}

int gleam_adam_step(const gleam_adam* hyper, int64_t t, size_t n, float* theta, const float* grad, float* m, float* v,
                    void* stream) {
    if (!hyper || !theta || !grad || !m || !v) return GLEAM_E_NULL;
    if (!adam_args_ok(hyper, t)) return GLEAM_E_DESC;
    if (n == 0) return GLEAM_OK;
    const hipError_t e = adam_update(*hyper, (long long)t, n, theta, grad, m, v, (hipStream_t)stream);
    return e == hipSuccess ? GLEAM_OK : GLEAM_E_LAUNCH;
}

int gleam_greedy_iteration(const gleam_geom* geom, const gleam_prox_desc* prox, int n_modules, const gleam_c64* x0,
                           const gleam_c64* S, const uint8_t* M, const gleam_c64* y, float alpha, float* theta,
                           float* adam_m, float* adam_v, const gleam_adam* hyper, int64_t t, const gleam_c64* x_ref,
                           gleam_c64* x_out, gleam_c64* x_tmp, float* losses, float* grad, void* saved,
                           size_t saved_bytes, void* ws, size_t ws_bytes, void* stream) {
    if (n_modules < 1) return GLEAM_E_DIMS;
    if (!x0 || !theta || !adam_m || !adam_v || !hyper || !x_ref || !x_out || !x_tmp || !losses || !grad) return GLEAM_E_NULL;
    if (x_out == x0 || x_tmp == x0 || x_out == x_tmp) return GLEAM_E_DIMS;
    // everything any of the per-module calls below would refuse is refused here, before the first launch
    if (!S || !M || !y) return GLEAM_E_NULL;
    int rc = check_module_buffers(geom, prox, ws, ws_bytes, saved, saved_bytes, true);
    if (rc) return rc;
    if (!adam_args_ok(hyper, t)) return GLEAM_E_DESC;
    size_t n_theta = 0;
    rc = gleam_theta_count(prox, &n_theta);
    if (rc) return rc;
    const gleam_c64* x_in = x0;
    for (int i = 0; i < n_modules; ++i) {
        // alternate the two image buffers so that the last module writes x_out
        gleam_c64* xo = ((n_modules - 1 - i) % 2 == 0) ? x_out : x_tmp;
        float* th = theta + (size_t)i * n_theta;
        rc = gleam_module_fwd(geom, prox, x_in, S, M, y, alpha, th, x_ref, xo, losses + i, saved, saved_bytes, ws, ws_bytes,
                              stream);
        if (rc) return rc;
        rc = gleam_module_bwd(geom, prox, th, saved, saved_bytes, grad, ws, ws_bytes, stream);
        if (rc) return rc;
        rc = gleam_adam_step(hyper, t, n_theta, th, grad, adam_m + (size_t)i * n_theta, adam_v + (size_t)i * n_theta, stream);
        if (rc) return rc;
        x_in = xo;
    }
    return GLEAM_OK;
}

int gleam_unrolled_infer(const gleam_geom* geom, const gleam_prox_desc* prox, int n_modules, const gleam_c64* x0,
                         const gleam_c64* S, const uint8_t* M, const gleam_c64* y, float alpha, const float* theta,
                         gleam_c64* x_out, gleam_c64* x_tmp, void* ws, size_t ws_bytes, void* stream) {
    if (n_modules < 1) return GLEAM_E_DIMS;
    if (!x0 || !theta || !x_out || !x_tmp || !S || !M || !y) return GLEAM_E_NULL;
    if (x_out == x0 || x_tmp == x0 || x_out == x_tmp) return GLEAM_E_DIMS;
    int rc = check_module_buffers(geom, prox, ws, ws_bytes, nullptr, 0, false);   // before the first launch
    if (rc) return rc;
    size_t n_theta = 0;
    rc = gleam_theta_count(prox, &n_theta);
    if (rc) return rc;
    const gleam_c64* x_in = x0;
    for (int i = 0; i < n_modules; ++i) {
        gleam_c64* xo = ((n_modules - 1 - i) % 2 == 0) ? x_out : x_tmp;
        rc = gleam_module_fwd(geom, prox, x_in, S, M, y, alpha, theta + (size_t)i * n_theta, nullptr, xo, nullptr, nullptr, 0,
                              ws, ws_bytes, stream);
        if (rc) return rc;
        x_in = xo;
    }
    return GLEAM_OK;
}

}  // extern "C"
