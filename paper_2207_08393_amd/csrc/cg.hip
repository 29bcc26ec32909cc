// Conjugate-gradient vector kernels of the MoDL module (MoDL section, Eq. 6-8): the solve of
// (A^H A + mu I) x = b by a fixed number of CG steps from zero, one system per batch sample.  The operator
// itself is the fused SENSE sweep (sense_dc with xs = mu, gs = 1, y = 0); the kernels here are the three
// HBM-bound vector updates between two applications.  Every scalar of the recurrence stays on the device:
// a workgroup writes its partial inner product, and each consumer sums the partials of its sample in a fixed
// order, so a solve is a plain sequence of launches with no host synchronisation and a reproducible result.
#include "internal.h"

namespace gleam {

constexpr int kCgThreads = 256;

namespace {

__device__ inline double block_sum(double v, double* red) {
    red[threadIdx.x] = v;
    __syncthreads();
    for (int o = kCgThreads / 2; o > 0; o >>= 1) {
        if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    return red[0];
}

// Sum of a sample's nb partials, the same value in every thread: strided per-thread sums in a fixed order, then
// the block tree.  Ends with a barrier so that red can be used again at once.
__device__ inline double sum_partials(const double* __restrict__ part, int nb, double* red) {
    double s = 0.0;
    for (int i = threadIdx.x; i < nb; i += kCgThreads) s += part[i];
    const double total = block_sum(s, red);
    __syncthreads();
    return total;
}

}  // namespace

// grid (nb, B).  r = c1*u + c2*v (v may be null), p = r, x = 0, rr[b][blk] = partial <r, r>.
// x may alias u (each element is read before it is overwritten by the same lane).
__global__ __launch_bounds__(kCgThreads) void cg_init_kernel(const float2* u, const float2* __restrict__ v, float c1, float c2,
                                                             long long n, float2* x, float2* __restrict__ r,
                                                             float2* __restrict__ p, double* __restrict__ rr) {
    __shared__ double red[kCgThreads];
    const long long base = (long long)blockIdx.y * n;
    double s = 0.0;
    for (long long i = (long long)blockIdx.x * kCgThreads + threadIdx.x; i < n; i += (long long)gridDim.x * kCgThreads) {
        float2 t = u[base + i];
        t.x *= c1; t.y *= c1;
        if (v) {
            const float2 w = v[base + i];
            t.x += c2 * w.x; t.y += c2 * w.y;
        }
        x[base + i] = make_float2(0.f, 0.f);
        r[base + i] = t;
        p[base + i] = t;
        s += (double)t.x * t.x + (double)t.y * t.y;
    }
    s = block_sum(s, red);
    if (threadIdx.x == 0) rr[(size_t)blockIdx.y * gridDim.x + blockIdx.x] = s;
}

// pq[b][blk] = partial Re <p, q>
__global__ __launch_bounds__(kCgThreads) void cg_dot_kernel(const float2* __restrict__ p, const float2* __restrict__ q, long long n,
                                                            double* __restrict__ pq) {
    __shared__ double red[kCgThreads];
    const long long base = (long long)blockIdx.y * n;
    double s = 0.0;
    for (long long i = (long long)blockIdx.x * kCgThreads + threadIdx.x; i < n; i += (long long)gridDim.x * kCgThreads) {
        const float2 a = p[base + i], b = q[base + i];
        s += (double)a.x * b.x + (double)a.y * b.y;
    }
    s = block_sum(s, red);
    if (threadIdx.x == 0) pq[(size_t)blockIdx.y * gridDim.x + blockIdx.x] = s;
}

// a = <r,r> / <p,q> (0 when the denominator is not positive); x += a p; r -= a q; rr_new partials.
__global__ __launch_bounds__(kCgThreads) void cg_update_xr_kernel(float2* __restrict__ x, float2* __restrict__ r,
                                                                  const float2* __restrict__ p, const float2* __restrict__ q,
                                                                  long long n, const double* __restrict__ rr_old,
                                                                  const double* __restrict__ pq, double* __restrict__ rr_new) {
    __shared__ double red[kCgThreads];
    const int nb = gridDim.x;
    const double num = sum_partials(rr_old + (size_t)blockIdx.y * nb, nb, red);
    const double den = sum_partials(pq + (size_t)blockIdx.y * nb, nb, red);
    const float a = den > 0.0 ? (float)(num / den) : 0.f;
    const long long base = (long long)blockIdx.y * n;
    double s = 0.0;
    for (long long i = (long long)blockIdx.x * kCgThreads + threadIdx.x; i < n; i += (long long)gridDim.x * kCgThreads) {
        const float2 pv = p[base + i], qv = q[base + i];
        float2 xv = x[base + i], rv = r[base + i];
        xv.x += a * pv.x; xv.y += a * pv.y;
        rv.x -= a * qv.x; rv.y -= a * qv.y;
        x[base + i] = xv;
        r[base + i] = rv;
        s += (double)rv.x * rv.x + (double)rv.y * rv.y;
    }
    s = block_sum(s, red);
    if (threadIdx.x == 0) rr_new[(size_t)blockIdx.y * nb + blockIdx.x] = s;
}

// beta = <r,r>_new / <r,r>_old (0 when the old one is not positive); p = r + beta p.
__global__ __launch_bounds__(kCgThreads) void cg_update_p_kernel(const float2* __restrict__ r, float2* __restrict__ p, long long n,
                                                                 const double* __restrict__ rr_old,
                                                                 const double* __restrict__ rr_new) {
    const int nb = gridDim.x;
    __shared__ double red[kCgThreads];
    const double den = sum_partials(rr_old + (size_t)blockIdx.y * nb, nb, red);
    const double num = sum_partials(rr_new + (size_t)blockIdx.y * nb, nb, red);
    const float beta = den > 0.0 ? (float)(num / den) : 0.f;
    const long long base = (long long)blockIdx.y * n;
    for (long long i = (long long)blockIdx.x * kCgThreads + threadIdx.x; i < n; i += (long long)gridDim.x * kCgThreads) {
        const float2 rv = r[base + i];
        float2 pv = p[base + i];
        pv.x = rv.x + beta * pv.x;
        pv.y = rv.y + beta * pv.y;
        p[base + i] = pv;
    }
}

__global__ __launch_bounds__(kCgThreads) void fill_zero_kernel(float2* __restrict__ x, long long n) {
    for (long long i = (long long)blockIdx.x * kCgThreads + threadIdx.x; i < n; i += (long long)gridDim.x * kCgThreads)
        x[i] = make_float2(0.f, 0.f);
}

static inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }

static int cg_blocks(long long n) {
    long long nb = (n + 4 * kCgThreads - 1) / (4 * kCgThreads);   // at least four elements per lane
    return (int)(nb < 1 ? 1 : (nb > kCgBlocksMax ? kCgBlocksMax : nb));
}

size_t cg_scratch_bytes(const gleam_geom& g) {
    const size_t img = align256((size_t)g.B * g.T * g.D * g.H * g.W * sizeof(float2));
    return 3 * img + align256((size_t)3 * g.B * kCgBlocksMax * sizeof(double));
}

hipError_t fill_zero(float2* x, long long n, hipStream_t st) {
    long long nb = (n + kCgThreads - 1) / kCgThreads;
    if (nb > 2048) nb = 2048;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)nb), dim3(kCgThreads), 0, st, x, n);
    return hipGetLastError();
}

hipError_t cg_solve(const gleam_geom& g, const float2* S, const unsigned char* M, float mu, int n_cg, const float2* u,
                    const float2* v, float c1, float c2, float2* x, float2* kbuf, void* scratch, hipStream_t st) {
    const long long n = g.T * g.D * g.H * g.W;
    const size_t img = align256((size_t)g.B * n * sizeof(float2));
    unsigned char* base = (unsigned char*)scratch;
    float2* r = (float2*)base;
    float2* p = (float2*)(base + img);
    float2* q = (float2*)(base + 2 * img);
    double* sc = (double*)(base + 3 * img);
    const int nb = cg_blocks(n);
    const size_t per = (size_t)g.B * nb;
    double* rr[2] = {sc, sc + per};
    double* pq = sc + 2 * per;
    const dim3 grid((unsigned)nb, (unsigned)g.B), block(kCgThreads);
    const double vec_bytes = 8.0 * (double)g.B * (double)n;
    {
        KernelScope ks("cg_init", 0.0, (v ? 5.0 : 4.0) * vec_bytes, st);
        hipLaunchKernelGGL(cg_init_kernel, grid, block, 0, st, u, v, c1, c2, n, x, r, p, rr[0]);
    }
    for (int k = 0; k < n_cg; ++k) {
        hipError_t e = sense_dc(g, p, S, M, nullptr, mu, 1.f, q, kbuf, st);   // q = (A^H A + mu I) p
        if (e != hipSuccess) return e;
        double* cur = rr[k & 1];
        double* nxt = rr[(k + 1) & 1];
        {
            KernelScope ks("cg_dot", 0.0, 2.0 * vec_bytes, st);
            hipLaunchKernelGGL(cg_dot_kernel, grid, block, 0, st, (const float2*)p, (const float2*)q, n, pq);
        }
        {
            KernelScope ks("cg_update_xr", 0.0, 6.0 * vec_bytes, st);
            hipLaunchKernelGGL(cg_update_xr_kernel, grid, block, 0, st, x, r, (const float2*)p, (const float2*)q, n,
                               (const double*)cur, (const double*)pq, nxt);
        }
        if (k + 1 < n_cg) {   // the search direction of a step that is never taken is not needed
            KernelScope ks("cg_update_p", 0.0, 3.0 * vec_bytes, st);
            hipLaunchKernelGGL(cg_update_p_kernel, grid, block, 0, st, (const float2*)r, p, n, (const double*)cur,
                               (const double*)nxt);
        }
    }
    return hipGetLastError();
}

}  // namespace gleam
