// SENSE normal operator / data-consistency step on gfx950:
//     out = xs * x + gs * S^H F^H Omega (F S x - y)          (Eq. 1-3; A = Omega F S)
// as 2d-1 sweeps over the coil k-space buffer for a d-dimensional transform:
//   rows_expand  : coil multiply fused into the load of the transform along W (contiguous axis)
//   cols_*       : strided axes, a tile of neighbouring columns per workgroup staged through LDS;
//                  the middle sweep does forward transform, mask / residual and inverse transform of
//                  its axis without leaving LDS
//   rows_reduce  : inverse transform along W with conj(S) multiply, coil sum and the DC update fused
//                  into the store (the per-coil images are never written).
#include <hip/hip_runtime.h>

#include "fft_core.h"
#include "internal.h"

namespace gleam {

constexpr int kNT = 256;  // threads per workgroup of every transform kernel

template <int N> constexpr int rows_lines() {
    int l = 1;
    while (l * 2 * N <= 4096 && l < 64) l *= 2;
    return l;
}
template <int N> constexpr int cols_lines() { return N > 320 ? 8 : 16; }

struct RowsArgs {
    const float2* x;      // image [B][T][DH][W]
    const float2* S;      // coils [B][C][DH][W]
    float2* k;            // k-space [B][C][T][DH][W]
    float2* out;          // image (reduce only)
    long long C, T, DH;   // DH = D*H rows per frame
    long long n_rows;     // expand: B*C*T*DH ; reduce: B*T*DH
    float scale;          // N^-1/2
    float xs, gs;         // reduce: out = xs*x + gs*g
};

// Forward transform along W of S*x, one k-space row per line.
template <int N>
__global__ __launch_bounds__(kNT) void rows_expand_kernel(RowsArgs a) {
    constexpr int L = rows_lines<N>();
    __shared__ float2 buf[N * L], tw[N];
    __shared__ long long xoff[L], soff[L];
    fill_twiddles<N, kNT>(tw);
    const long long n_tiles = (a.n_rows + L - 1) / L;
    for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        __syncthreads();
        if (threadIdx.x < L) {
            const long long row = tile * L + threadIdx.x;   // k-space row (b, c, t, dh)
            long long xo = -1, so = -1;
            if (row < a.n_rows) {
                const long long dh = row % a.DH;
                const long long t = (row / a.DH) % a.T;
                const long long bc = row / (a.DH * a.T);
                xo = (((bc / a.C) * a.T + t) * a.DH + dh) * N;
                so = (bc * a.DH + dh) * N;
            }
            xoff[threadIdx.x] = xo;
            soff[threadIdx.x] = so;
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < N * L; idx += kNT) {
            const int line = idx / N, p = idx % N;
            float2 v = make_float2(0.f, 0.f);
            if (xoff[line] >= 0) v = cmul(a.S[soff[line] + p], a.x[xoff[line] + p]);
            buf[idx] = v;
        }
        __syncthreads();
        fft_lines<N, L, false, false, kNT>(buf, tw);
        for (int idx = threadIdx.x; idx < N * L; idx += kNT) {
            const int line = idx / N;
            if (xoff[line] >= 0) {
                const float2 v = buf[idx];
                a.k[(tile * L + line) * N + idx % N] = make_float2(v.x * a.scale, v.y * a.scale);
            }
        }
    }
}

// Inverse transform along W of every coil's row, then out = xs*x + gs*sum_c conj(S_c) * row_c.
template <int N>
__global__ __launch_bounds__(kNT) void rows_reduce_kernel(RowsArgs a) {
    constexpr int L = rows_lines<N>();
    constexpr int PER = (N * L + kNT - 1) / kNT;
    __shared__ float2 buf[N * L], tw[N];
    __shared__ long long koff[L], soff[L];   // offsets of coil 0; coil strides below
    fill_twiddles<N, kNT>(tw);
    const long long n_tiles = (a.n_rows + L - 1) / L;
    const long long kstride = a.T * a.DH * N, sstride = a.DH * N;
    for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        __syncthreads();
        if (threadIdx.x < L) {
            const long long row = tile * L + threadIdx.x;   // image row (b, t, dh)
            long long ko = -1, so = -1;
            if (row < a.n_rows) {
                const long long dh = row % a.DH;
                const long long bt = row / a.DH;
                const long long t = bt % a.T, b = bt / a.T;
                ko = (((b * a.C) * a.T + t) * a.DH + dh) * N;
                so = ((b * a.C) * a.DH + dh) * N;
            }
            koff[threadIdx.x] = ko;
            soff[threadIdx.x] = so;
        }
        __syncthreads();
        float2 acc[PER];
#pragma unroll
        for (int m = 0; m < PER; ++m) acc[m] = make_float2(0.f, 0.f);
        for (long long c = 0; c < a.C; ++c) {
            for (int idx = threadIdx.x; idx < N * L; idx += kNT) {
                const int line = idx / N, p = idx % N;
                float2 v = make_float2(0.f, 0.f);
                if (koff[line] >= 0) v = a.k[koff[line] + c * kstride + p];
                buf[idx] = v;
            }
            __syncthreads();
            fft_lines<N, L, false, true, kNT>(buf, tw);
#pragma unroll
            for (int m = 0; m < PER; ++m) {
                const int idx = threadIdx.x + m * kNT;
                if (idx < N * L) {
                    const int line = idx / N;
                    if (koff[line] >= 0) {
                        const float2 sv = a.S[soff[line] + c * sstride + idx % N];
                        const float2 pr = cmul_conj(buf[idx], sv);
                        acc[m].x += pr.x;
                        acc[m].y += pr.y;
                    }
                }
            }
            __syncthreads();
        }
#pragma unroll
        for (int m = 0; m < PER; ++m) {
            const int idx = threadIdx.x + m * kNT;
            if (idx < N * L) {
                const int line = idx / N;
                if (koff[line] >= 0) {
                    const long long o = (tile * L + line) * N + idx % N;
                    float2 r = make_float2(a.gs * a.scale * acc[m].x, a.gs * a.scale * acc[m].y);
                    if (a.xs != 0.f) {
                        const float2 xv = a.x[o];
                        r.x = fmaf(a.xs, xv.x, r.x);
                        r.y = fmaf(a.xs, xv.y, r.y);
                    }
                    a.out[o] = r;
                }
            }
        }
    }
}

struct ColsArgs {
    float2* k;             // k-space viewed as [outer][N][inner], transformed in place along N
    const float2* y;       // measured k-space, same view (mid only; may be null)
    const unsigned char* M;  // mask (mid only)
    long long outer, inner;
    long long C, T, Dq;    // outer = ((b*C + c)*T + t)*Dq + dq ; mask row = (b*T + t)*Dq + dq
    float scale;           // N^-1/2, applied at the store (mid applies its forward N^-1/2 in LDS)
};

// MODE 0: forward, 1: inverse, 2: forward -> (mask ? k - y : 0) -> inverse.
template <int N, int MODE>
__global__ __launch_bounds__(kNT) void cols_kernel(ColsArgs a) {
    constexpr int L = cols_lines<N>();
    __shared__ float2 buf[N * L], tw[N];
    fill_twiddles<N, kNT>(tw);
    const long long tiles_per = (a.inner + L - 1) / L;
    const long long n_tiles = a.outer * tiles_per;
    for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const long long o = tile / tiles_per;
        const long long i0 = (tile % tiles_per) * L;
        const long long base = o * N * a.inner + i0;
        const int valid = (int)((a.inner - i0) < L ? (a.inner - i0) : L);
        __syncthreads();
        for (int idx = threadIdx.x; idx < N * L; idx += kNT) {
            const int l = idx % L, p = idx / L;
            float2 v = make_float2(0.f, 0.f);
            if (l < valid) v = a.k[base + (long long)p * a.inner + l];
            buf[idx] = v;
        }
        __syncthreads();
        if constexpr (MODE == 1) {
            fft_lines<N, L, true, true, kNT>(buf, tw);
        } else {
            fft_lines<N, L, true, false, kNT>(buf, tw);
        }
        if constexpr (MODE == 2) {
            const long long dq = o % a.Dq;
            const long long t = (o / a.Dq) % a.T;
            const long long b = o / (a.Dq * a.T * a.C);
            const long long mbase = ((b * a.T + t) * a.Dq + dq) * N * a.inner + i0;
            // the forward transform of this axis carries N^-1/2; apply it before subtracting y
            const float fs = rsqrtf((float)N);
            for (int idx = threadIdx.x; idx < N * L; idx += kNT) {
                const int l = idx % L, p = idx / L;
                float2 r = make_float2(0.f, 0.f);
                if (l < valid) {
                    const long long off = (long long)p * a.inner + l;
                    if (a.M[mbase + off] != 0) {
                        const float2 v = buf[idx];
                        r = make_float2(v.x * fs, v.y * fs);
                        if (a.y != nullptr) {
                            const float2 yv = a.y[base + off];
                            r.x -= yv.x;
                            r.y -= yv.y;
                        }
                    }
                }
                buf[idx] = r;
            }
            __syncthreads();
            fft_lines<N, L, true, true, kNT>(buf, tw);
        }
        for (int idx = threadIdx.x; idx < N * L; idx += kNT) {
            const int l = idx % L, p = idx / L;
            if (l < valid) {
                const float2 v = buf[idx];
                a.k[base + (long long)p * a.inner + l] = make_float2(v.x * a.scale, v.y * a.scale);
            }
        }
    }
}

// ------------------------------------------------------------------ host dispatch
#define GLEAM_FFT_SIZES(X) \
    X(4) X(6) X(8) X(10) X(12) X(16) X(20) X(24) X(32) X(46) X(64) X(96) X(128) X(160) X(192) X(256) X(320) X(368) X(640)

bool fft_size_supported(long long n) {
    switch (n) {
#define X(N) case N:
        GLEAM_FFT_SIZES(X)
#undef X
        return true;
        default: return false;
    }
}

static int grid_for(long long n_tiles) {
    const long long cap = 256LL * 8;
    return (int)(n_tiles < cap ? (n_tiles > 0 ? n_tiles : 1) : cap);
}

static hipError_t launch_rows(bool reduce, int N, const RowsArgs& a, hipStream_t st) {
    switch (N) {
#define X(NN)                                                                                          \
    case NN: {                                                                                         \
        const long long tiles = (a.n_rows + rows_lines<NN>() - 1) / rows_lines<NN>();                  \
        if (reduce) hipLaunchKernelGGL(rows_reduce_kernel<NN>, dim3(grid_for(tiles)), dim3(kNT), 0, st, a); \
        else hipLaunchKernelGGL(rows_expand_kernel<NN>, dim3(grid_for(tiles)), dim3(kNT), 0, st, a);   \
        break;                                                                                         \
    }
        GLEAM_FFT_SIZES(X)
#undef X
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

static hipError_t launch_cols(int mode, int N, const ColsArgs& a, hipStream_t st) {
    switch (N) {
#define X(NN)                                                                                          \
    case NN: {                                                                                         \
        const long long tiles = a.outer * ((a.inner + cols_lines<NN>() - 1) / cols_lines<NN>());       \
        const dim3 g(grid_for(tiles)), b(kNT);                                                         \
        if (mode == 0) hipLaunchKernelGGL((cols_kernel<NN, 0>), g, b, 0, st, a);                       \
        else if (mode == 1) hipLaunchKernelGGL((cols_kernel<NN, 1>), g, b, 0, st, a);                  \
        else hipLaunchKernelGGL((cols_kernel<NN, 2>), g, b, 0, st, a);                                 \
        break;                                                                                         \
    }
        GLEAM_FFT_SIZES(X)
#undef X
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t sense_dc(const gleam_geom& g, const float2* x, const float2* S, const unsigned char* M,
                    const float2* y, float xs, float gs, float2* out, float2* kbuf, hipStream_t st) {
    const long long DH = g.D * g.H;
    RowsArgs ra{};
    ra.x = x; ra.S = S; ra.k = kbuf; ra.out = out;
    ra.C = g.C; ra.T = g.T; ra.DH = DH;
    ra.scale = 1.0f / sqrtf((float)g.W);
    ra.xs = xs; ra.gs = gs;
    ra.n_rows = g.B * g.C * g.T * DH;
    const double E8 = 8.0 * (double)(g.B * g.C * g.T * g.D * g.H * g.W);   // bytes of one k-space sweep
    const double P8 = 8.0 * (double)(g.B * g.T * g.D * g.H * g.W);          // bytes of one image
    const double S8 = E8 / (double)g.T, M1 = P8 / 8.0;
    hipError_t e;
    {
        KernelScope ks("sense_rows_expand", 0.0, S8 + P8 + E8, st);
        e = launch_rows(false, (int)g.W, ra, st);
    }
    if (e != hipSuccess) return e;

    ColsArgs ca{};
    ca.k = kbuf; ca.y = y; ca.M = M; ca.C = g.C; ca.T = g.T;
    if (g.ndim_fft == 2) {
        ca.outer = g.B * g.C * g.T * g.D; ca.inner = g.W; ca.Dq = g.D;
        ca.scale = 1.0f / sqrtf((float)g.H);
        {
            KernelScope ks("sense_cols_mid", 0.0, 2.0 * E8 + (y ? E8 : 0.0) + M1, st);
            e = launch_cols(2, (int)g.H, ca, st);
        }
        if (e != hipSuccess) return e;
    } else {
        ColsArgs ha = ca;  // H axis: [B*C*T*D][H][W]
        ha.outer = g.B * g.C * g.T * g.D; ha.inner = g.W; ha.Dq = g.D;
        ha.scale = 1.0f / sqrtf((float)g.H);
        {
            KernelScope ks("sense_cols_fwd", 0.0, 2.0 * E8, st);
            e = launch_cols(0, (int)g.H, ha, st);
        }
        if (e != hipSuccess) return e;
        ca.outer = g.B * g.C * g.T; ca.inner = g.H * g.W; ca.Dq = 1;  // D axis: [B*C*T][D][H*W]
        ca.scale = 1.0f / sqrtf((float)g.D);
        {
            KernelScope ks("sense_cols_mid", 0.0, 2.0 * E8 + (y ? E8 : 0.0) + M1, st);
            e = launch_cols(2, (int)g.D, ca, st);
        }
        if (e != hipSuccess) return e;
        {
            KernelScope ks("sense_cols_inv", 0.0, 2.0 * E8, st);
            e = launch_cols(1, (int)g.H, ha, st);
        }
        if (e != hipSuccess) return e;
    }
    ra.n_rows = g.B * g.T * DH;
    KernelScope ks("sense_rows_reduce", 0.0, E8 + S8 + P8 + (xs != 0.f ? P8 : 0.0), st);
    return launch_rows(true, (int)g.W, ra, st);
}

}  // namespace gleam
