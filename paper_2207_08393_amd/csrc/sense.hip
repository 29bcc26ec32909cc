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
#include "xcd.h"

namespace gleam {

// Lines (rows or columns) per workgroup tile and threads per workgroup, by transform length.  Tiles hold
// 8 or more lines so that every LDS access of a butterfly stage is conflict free (see Layout).  Chosen by
// measurement on the transform-only sweeps (load, transform, store): e.g. 160 x 32 lines on 512 threads and
// 368 x 16 lines on 256 threads for the contiguous axis, 640 x 8 and 256 x 32 lines on 512 threads for the strided one.
template <int N> constexpr int rows_lines() { return N > 384 ? 8 : (N >= 192 ? 16 : (N >= 96 ? 32 : 64)); }
template <int N> constexpr int rows_threads() { return (N * rows_lines<N>() >= 4096 && N != 368) ? 512 : 256; }
// The coil-reduction kernel transforms the same tiles.
template <int N> constexpr int reduce_lines() { return rows_lines<N>(); }
template <int N> constexpr int reduce_threads() { return rows_threads<N>(); }
template <int N> constexpr int cols_lines() { return N >= 512 ? 8 : (N == 256 ? 32 : 16); }
template <int N> constexpr int cols_threads() { return N >= 192 ? 512 : 256; }
// Waves per SIMD the compiler is asked to leave room for.  The middle sweep of the lengths whose butterflies are at
// most 16 points wide would otherwise take ~140-150 registers (the unrolled mask stage) and drop from two resident
// 512-thread workgroups per CU to one; at 128 registers it keeps two (a handful of spilled values, measured faster).
template <int N, int MODE> constexpr int cols_min_waves() {
    return (MODE >= 2 && (N == 640 || N == 256 || N == 192)) ? 4 : 1;
}

struct RowsArgs {
    const float2* x;      // image [B][T][DH][W]
    const float2* S;      // coils [B][C][DH][W]
    float2* k;            // k-space [B][C][T][DH][W]
    float2* out;          // image (reduce only)
    long long C, T, DH;   // DH = D*H rows per frame
    long long n_rows;     // B*T*DH image rows
    float scale;          // N^-1/2
    float xs, gs;         // reduce: out = xs*x + gs*g
    // Centred transform (frequency and spatial origin in the middle of every transformed axis; all lengths are even):
    // F_c = (-1)^(n/2) D F D per axis with D = diag((-1)^index), so the operator is the uncentred one on D x and
    // (sign) D y, times D.  cen: 0 / 1; par_h, par_d: whether the row index h / d takes part in the parity (the
    // axis is transformed); Hh: H, to split a row index into (d, h); ysign_bit: 1 when the product of the
    // (-1)^(n/2) over the transformed axes is -1.
    int cen, par_h, par_d, ysign_bit;
    long long Hh;
};

// v with its sign flipped when bit is 1 (bit is 0 or 1)
__device__ __forceinline__ float2 flip_sign(float2 v, unsigned bit) {
    return make_float2(__uint_as_float(__float_as_uint(v.x) ^ (bit << 31)), __uint_as_float(__float_as_uint(v.y) ^ (bit << 31)));
}
// parity of the transformed row coordinates of row dh = d*H + h (0 when the transform is not centred)
__device__ __forceinline__ unsigned row_parity(const RowsArgs& a, long long dh) {
    if (!a.cen) return 0u;
    const long long h = dh % a.Hh, d = dh / a.Hh;
    return (unsigned)(((a.par_h ? h : 0) + (a.par_d ? d : 0)) & 1);
}

// Forward transform along W of S*x.  A tile is LR image rows x CG coils (LR*CG <= L lines), so that an image row
// is fetched from memory once and reused from cache for all of its coils (tiles of consecutive k-space rows would
// come back to the same image row once per coil, megabytes later); coil multiply fused into the load, two complex
// values (16 bytes) per global access.
template <int N>
__global__ __launch_bounds__(rows_threads<N>()) void rows_expand_kernel(RowsArgs a) {
    constexpr int L = rows_lines<N>(), NT = rows_threads<N>(), H2 = N / 2;
    using Lay = Layout<N, L, 1>;
    __shared__ float2 buf[Lay::kElems], tw[N];
    __shared__ long long xoff[L], soff[L], koff[L];   // per image row of the tile: image, coil map (coil 0), k-space (coil 0)
    __shared__ unsigned lpar[L];
    fill_twiddles<N, NT>(tw);
    const int CG = a.C < L ? (int)a.C : L;        // coils transformed together
    const int LR = L / CG;                        // image rows per tile
    const long long n_tiles = (a.n_rows + LR - 1) / LR;
    const long long kstride = a.T * a.DH * N, sstride = a.DH * N;
    for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        __syncthreads();
        if (threadIdx.x < LR) {
            const long long row = tile * LR + threadIdx.x;   // image row (b, t, dh)
            long long xo = -1, so = -1, ko = -1;
            unsigned par = 0u;
            if (row < a.n_rows) {
                const long long dh = row % a.DH;
                const long long bt = row / a.DH;
                const long long t = bt % a.T, b = bt / a.T;
                xo = row * N;
                so = ((b * a.C) * a.DH + dh) * N;
                ko = (((b * a.C) * a.T + t) * a.DH + dh) * N;
                par = row_parity(a, dh);
            }
            xoff[threadIdx.x] = xo;
            soff[threadIdx.x] = so;
            koff[threadIdx.x] = ko;
            lpar[threadIdx.x] = par;
        }
        __syncthreads();
        for (int c0 = 0; c0 < a.C; c0 += CG) {
            const int ncg = a.C - c0 < CG ? (int)(a.C - c0) : CG;
            // line l = r*CG + c holds coil c0 + c of image row r; unused lines are zero
            for (int idx = threadIdx.x; idx < H2 * L; idx += NT) {
                const int line = idx / H2, p = 2 * (idx % H2);
                const int r = line / CG, c = line % CG;
                float2 v0 = make_float2(0.f, 0.f), v1 = v0;
                if (r < LR && c < ncg && xoff[r] >= 0) {
                    const float4 sv = *reinterpret_cast<const float4*>(a.S + soff[r] + (c0 + c) * sstride + p);
                    const float4 xv = *reinterpret_cast<const float4*>(a.x + xoff[r] + p);
                    v0 = cmul(make_float2(sv.x, sv.y), make_float2(xv.x, xv.y));
                    v1 = cmul(make_float2(sv.z, sv.w), make_float2(xv.z, xv.w));
                    if (a.cen) {   // D x: p is even, so the pair's signs are the row's parity and its opposite
                        v0 = flip_sign(v0, lpar[r]);
                        v1 = flip_sign(v1, lpar[r] ^ 1u);
                    }
                }
                buf[Lay::at(line, p)] = v0;
                buf[Lay::at(line, p + 1)] = v1;
            }
            __syncthreads();
            fft_lines<N, L, 1, false, NT>(buf, tw);
            for (int idx = threadIdx.x; idx < H2 * L; idx += NT) {
                const int line = idx / H2, p = 2 * (idx % H2);
                const int r = line / CG, c = line % CG;
                if (r < LR && c < ncg && xoff[r] >= 0) {
                    const float2 v0 = buf[Lay::at(line, p)], v1 = buf[Lay::at(line, p + 1)];
                    *reinterpret_cast<float4*>(a.k + koff[r] + (c0 + c) * kstride + p) =
                        make_float4(v0.x * a.scale, v0.y * a.scale, v1.x * a.scale, v1.y * a.scale);
                }
            }
            if (c0 + CG < a.C) __syncthreads();   // the next coil group overwrites the tile
        }
    }
}

// Inverse transform along W and coil reduction.  A tile is LR image rows x CG coils (LR*CG <= L lines)
// transformed together; then out = xs*x + gs * sum_c conj(S_c) * row_c is accumulated in registers,
// looping over coil groups when C > CG.  The per-coil images never leave LDS.  LR is capped so that a thread
// owns at most kRedAcc output pairs (two accumulators keep the register count where three workgroups fit a CU).
constexpr int kRedAcc = 2;
template <int N> constexpr int reduce_rows_max() {
    constexpr int m = kRedAcc * reduce_threads<N>() / (N / 2);
    return m < 1 ? 1 : m;
}
static inline int reduce_rows_per_tile(int L, int LRmax, long long C) {
    const int cg = C < L ? (int)C : L;
    const int lr = L / cg;
    return lr < LRmax ? lr : LRmax;
}

template <int N>
__global__ __launch_bounds__(reduce_threads<N>()) void rows_reduce_kernel(RowsArgs a) {
    constexpr int L = reduce_lines<N>(), NT = reduce_threads<N>(), H2 = N / 2;
    constexpr int PER = kRedAcc;
    static_assert(H2 <= PER * NT, "one image row must fit the accumulators");
    using Lay = Layout<N, L, 1>;
    __shared__ float2 buf[Lay::kElems], tw[N];
    __shared__ long long koff[L], soff[L];        // per image row of the tile, coil 0
    __shared__ unsigned lpar[L];
    fill_twiddles<N, NT>(tw);
    const int CG = a.C < L ? (int)a.C : L;        // coils transformed together
    const int LR = (L / CG) < reduce_rows_max<N>() ? (L / CG) : reduce_rows_max<N>();   // image rows per tile
    const long long n_tiles = (a.n_rows + LR - 1) / LR;
    const long long kstride = a.T * a.DH * N, sstride = a.DH * N;
    for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        __syncthreads();
        if (threadIdx.x < LR) {
            const long long row = tile * LR + threadIdx.x;   // image row (b, t, dh)
            long long ko = -1, so = -1;
            unsigned par = 0u;
            if (row < a.n_rows) {
                const long long dh = row % a.DH;
                const long long bt = row / a.DH;
                const long long t = bt % a.T, b = bt / a.T;
                ko = (((b * a.C) * a.T + t) * a.DH + dh) * N;
                so = ((b * a.C) * a.DH + dh) * N;
                par = row_parity(a, dh);
            }
            koff[threadIdx.x] = ko;
            soff[threadIdx.x] = so;
            lpar[threadIdx.x] = par;
        }
        __syncthreads();
        float4 acc[PER];
#pragma unroll
        for (int m = 0; m < PER; ++m) acc[m] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int c0 = 0; c0 < a.C; c0 += CG) {
            const int ncg = a.C - c0 < CG ? (int)(a.C - c0) : CG;
            // line l = r*CG + c holds coil c0 + c of image row r; unused lines are zero
            for (int idx = threadIdx.x; idx < H2 * L; idx += NT) {
                const int line = idx / H2, p = 2 * (idx % H2);
                const int r = line / CG, c = line % CG;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (r < LR && c < ncg && koff[r] >= 0)
                    v = *reinterpret_cast<const float4*>(a.k + koff[r] + (c0 + c) * kstride + p);
                buf[Lay::at(line, p)] = make_float2(v.x, v.y);
                buf[Lay::at(line, p + 1)] = make_float2(v.z, v.w);
            }
            __syncthreads();
            fft_lines<N, L, 1, true, NT>(buf, tw);
#pragma unroll
            for (int m = 0; m < PER; ++m) {
                const int e = threadIdx.x + m * NT;      // pair index over LR rows
                if (e < H2 * LR) {
                    const int r = e / H2, p = 2 * (e % H2);
                    if (koff[r] >= 0) {
                        const float2* sp = a.S + soff[r] + (long long)c0 * sstride + p;
                        // coil maps four at a time: the loads of a group are in flight together
                        for (int c = 0; c < ncg; c += 4) {
                            float4 sv[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                sv[j] = *reinterpret_cast<const float4*>(sp + (c + j < ncg ? (c + j) * sstride : 0));
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                if (c + j < ncg) {
                                    const float2 v0 = buf[Lay::at(r * CG + c + j, p)], v1 = buf[Lay::at(r * CG + c + j, p + 1)];
                                    const float2 p0 = cmul_conj(v0, make_float2(sv[j].x, sv[j].y));
                                    const float2 p1 = cmul_conj(v1, make_float2(sv[j].z, sv[j].w));
                                    acc[m].x += p0.x; acc[m].y += p0.y; acc[m].z += p1.x; acc[m].w += p1.y;
                                }
                            }
                        }
                    }
                }
            }
            __syncthreads();
        }
        const float gsc = a.gs * a.scale;
#pragma unroll
        for (int m = 0; m < PER; ++m) {
            const int e = threadIdx.x + m * NT;
            if (e < H2 * LR) {
                const int r = e / H2, p = 2 * (e % H2);
                if (koff[r] >= 0) {
                    const long long o = (tile * LR + r) * N + p;
                    const float g0 = (a.cen && lpar[r]) ? -gsc : gsc, g1 = a.cen ? -g0 : g0;   // D g when centred: p is even
                    float4 res = make_float4(g0 * acc[m].x, g0 * acc[m].y, g1 * acc[m].z, g1 * acc[m].w);
                    if (a.xs != 0.f) {
                        const float4 xv = *reinterpret_cast<const float4*>(a.x + o);
                        res.x = fmaf(a.xs, xv.x, res.x); res.y = fmaf(a.xs, xv.y, res.y);
                        res.z = fmaf(a.xs, xv.z, res.z); res.w = fmaf(a.xs, xv.w, res.w);
                    }
                    *reinterpret_cast<float4*>(a.out + o) = res;
                }
            }
        }
    }
}

// One transformed axis only (ndim_fft = 1: the mask does not depend on the other image axes, e.g. line masks of
// 2D Cartesian sampling after the transform along the fully sampled axis has been taken out of the data): the
// whole operator in one sweep, nothing but S, x, y and the mask is read and only the image is written.  A tile is
// LR image rows x CG coils as in rows_reduce_kernel; per coil group: S*x -> forward transform ->
// mask ? k - y : 0 -> inverse transform -> accumulate conj(S)*row.
template <int N>
__global__ __launch_bounds__(reduce_threads<N>()) void rows_fused_kernel(RowsArgs a, const float2* __restrict__ y,
                                                                         const unsigned char* __restrict__ M) {
    constexpr int L = reduce_lines<N>(), NT = reduce_threads<N>(), H2 = N / 2;
    constexpr int PER = kRedAcc;
    using Lay = Layout<N, L, 1>;
    __shared__ float2 buf[Lay::kElems], tw[N];
    __shared__ long long koff[L], soff[L], xoff[L];   // per image row of the tile: k-space (coil 0), coil map (coil 0), image
    fill_twiddles<N, NT>(tw);
    const int CG = a.C < L ? (int)a.C : L;
    const int LR = (L / CG) < reduce_rows_max<N>() ? (L / CG) : reduce_rows_max<N>();
    const long long n_tiles = (a.n_rows + LR - 1) / LR;
    const long long kstride = a.T * a.DH * N, sstride = a.DH * N;
    for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        __syncthreads();
        if (threadIdx.x < LR) {
            const long long row = tile * LR + threadIdx.x;   // image row (b, t, dh)
            long long ko = -1, so = -1, xo = -1;
            if (row < a.n_rows) {
                const long long dh = row % a.DH;
                const long long bt = row / a.DH;
                const long long t = bt % a.T, b = bt / a.T;
                ko = (((b * a.C) * a.T + t) * a.DH + dh) * N;
                so = ((b * a.C) * a.DH + dh) * N;
                xo = row * N;
            }
            koff[threadIdx.x] = ko;
            soff[threadIdx.x] = so;
            xoff[threadIdx.x] = xo;
        }
        __syncthreads();
        float4 acc[PER];
#pragma unroll
        for (int m = 0; m < PER; ++m) acc[m] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int c0 = 0; c0 < a.C; c0 += CG) {
            const int ncg = a.C - c0 < CG ? (int)(a.C - c0) : CG;
            // line l = r*CG + c holds coil c0 + c of image row r; unused lines are zero
            for (int idx = threadIdx.x; idx < H2 * L; idx += NT) {
                const int line = idx / H2, p = 2 * (idx % H2);
                const int r = line / CG, c = line % CG;
                float2 v0 = make_float2(0.f, 0.f), v1 = v0;
                if (r < LR && c < ncg && xoff[r] >= 0) {
                    const float4 sv = *reinterpret_cast<const float4*>(a.S + soff[r] + (c0 + c) * sstride + p);
                    const float4 xv = *reinterpret_cast<const float4*>(a.x + xoff[r] + p);
                    v0 = cmul(make_float2(sv.x, sv.y), make_float2(xv.x, xv.y));
                    v1 = cmul(make_float2(sv.z, sv.w), make_float2(xv.z, xv.w));
                    if (a.cen) v1 = flip_sign(v1, 1u);   // D x along the one transformed axis: p is even
                }
                buf[Lay::at(line, p)] = v0;
                buf[Lay::at(line, p + 1)] = v1;
            }
            __syncthreads();
            fft_lines<N, L, 1, false, NT>(buf, tw);
            for (int idx = threadIdx.x; idx < H2 * L; idx += NT) {
                const int line = idx / H2, p = 2 * (idx % H2);
                const int r = line / CG, c = line % CG;
                if (r < LR && c < ncg && xoff[r] >= 0) {
                    const unsigned short mm = *reinterpret_cast<const unsigned short*>(M + xoff[r] + p);
                    float4 yv = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (y) yv = *reinterpret_cast<const float4*>(y + koff[r] + (c0 + c) * kstride + p);
                    if (a.cen) {   // (-1)^(N/2) D y
                        const float s0 = a.ysign_bit ? -1.f : 1.f;
                        yv.x *= s0; yv.y *= s0; yv.z *= -s0; yv.w *= -s0;
                    }
                    const float2 k0 = buf[Lay::at(line, p)], k1 = buf[Lay::at(line, p + 1)];
                    buf[Lay::at(line, p)] = (mm & 0xff) ? make_float2(k0.x * a.scale - yv.x, k0.y * a.scale - yv.y) : make_float2(0.f, 0.f);
                    buf[Lay::at(line, p + 1)] = (mm >> 8) ? make_float2(k1.x * a.scale - yv.z, k1.y * a.scale - yv.w) : make_float2(0.f, 0.f);
                }
            }
            __syncthreads();
            fft_lines<N, L, 1, true, NT>(buf, tw);
#pragma unroll
            for (int m = 0; m < PER; ++m) {
                const int e = threadIdx.x + m * NT;      // pair index over LR rows
                if (e < H2 * LR) {
                    const int r = e / H2, p = 2 * (e % H2);
                    if (xoff[r] >= 0) {
                        for (int c = 0; c < ncg; ++c) {
                            const float4 sv = *reinterpret_cast<const float4*>(a.S + soff[r] + (c0 + c) * sstride + p);
                            const float2 v0 = buf[Lay::at(r * CG + c, p)], v1 = buf[Lay::at(r * CG + c, p + 1)];
                            const float2 p0 = cmul_conj(v0, make_float2(sv.x, sv.y));
                            const float2 p1 = cmul_conj(v1, make_float2(sv.z, sv.w));
                            acc[m].x += p0.x; acc[m].y += p0.y; acc[m].z += p1.x; acc[m].w += p1.y;
                        }
                    }
                }
            }
            __syncthreads();
        }
        const float gsc = a.gs * a.scale;
#pragma unroll
        for (int m = 0; m < PER; ++m) {
            const int e = threadIdx.x + m * NT;
            if (e < H2 * LR) {
                const int r = e / H2, p = 2 * (e % H2);
                if (xoff[r] >= 0) {
                    const long long o = xoff[r] + p;
                    float4 res = make_float4(gsc * acc[m].x, gsc * acc[m].y, gsc * acc[m].z, gsc * acc[m].w);
                    if (a.cen) { res.z = -res.z; res.w = -res.w; }   // D g: p is even
                    if (a.xs != 0.f) {
                        const float4 xv = *reinterpret_cast<const float4*>(a.x + o);
                        res.x = fmaf(a.xs, xv.x, res.x); res.y = fmaf(a.xs, xv.y, res.y);
                        res.z = fmaf(a.xs, xv.z, res.z); res.w = fmaf(a.xs, xv.w, res.w);
                    }
                    *reinterpret_cast<float4*>(a.out + o) = res;
                }
            }
        }
    }
}

struct ColsArgs {
    float2* k;             // k-space viewed as [outer][N][inner], transformed in place along N
    const float2* y;       // measured k-space, same view (mid only; may be null)
    const unsigned char* M;  // mask (mid only)
    long long outer, inner;  // inner is even (it is a product of transform lengths, all even)
    long long C, T, Dq;    // outer = ((b*C + c)*T + t)*Dq + dq ; mask row = (b*T + t)*Dq + dq
    float scale;           // N^-1/2, applied at the store (mid applies its forward N^-1/2 in LDS)
    // Centred transform.  cen_y (mid sweep): the measured k-space enters as (sign) D y, where the parity of an
    // element is p + (column / Wrow) + (column % Wrow) (the inner index is h*W + w when three axes are transformed,
    // w alone otherwise: then column / Wrow is 0) and ysign_bit is 1 when the product of (-1)^(n/2) over the
    // transformed axes is -1.  cen_io (MODE 1 on its own, k-space to hybrid space): the centred inverse transform
    // of this axis, (-1)^(N/2) D F^H D: input and output signs by the parity of p.
    int cen_y, ysign_bit, cen_io;
    long long Wrow;
    // Walk the tiles from the last to the first.  The k-space buffer of the 3D workload (419 MB) is larger than the
    // Infinity Cache (256 MB), which holds what the previous sweep wrote last: a sweep that starts where the previous
    // one ended finds that part there.
    int rev;
};

// Mask bytes of a column tile ([N rows][L columns], row p at mb + p*L) into LDS.  One thread fetches a whole row
// segment with a single 8- or 16-byte load where the addresses allow it (2-byte loads per element pair would issue as
// many memory requests as the k-space tile itself); columns past `valid` read as 0.
template <int N, int L, int NT>
__device__ __forceinline__ void load_mask_tile(const unsigned char* __restrict__ M, long long mbase, long long inner, int valid,
                                               unsigned char* mb) {
    const bool vec = valid == L && (inner % L) == 0 && ((reinterpret_cast<unsigned long long>(M) + (unsigned long long)mbase) % L) == 0;
    if (vec) {
        if constexpr (L == 8) {
            for (int p = threadIdx.x; p < N; p += NT)
                *reinterpret_cast<uint2*>(mb + p * L) = *reinterpret_cast<const uint2*>(M + mbase + (long long)p * inner);
        } else {
            constexpr int Q = L / 16;
            for (int i = threadIdx.x; i < N * Q; i += NT) {
                const int p = i / Q, q = i % Q;
                *reinterpret_cast<uint4*>(mb + p * L + 16 * q) = *reinterpret_cast<const uint4*>(M + mbase + (long long)p * inner + 16 * q);
            }
        }
    } else {
        for (int i = threadIdx.x; i < N * (L / 2); i += NT) {
            const int l = 2 * (i % (L / 2)), p = i / (L / 2);
            unsigned short v = 0;
            if (l < valid) v = *reinterpret_cast<const unsigned short*>(M + mbase + (long long)p * inner + l);
            *reinterpret_cast<unsigned short*>(mb + p * L + l) = v;
        }
    }
}

// Strided axis: a tile is 16 neighbouring columns (128 contiguous bytes per row) of one [N][inner] plane.
// MODE 0: forward, 1: inverse, 2: forward -> (mask ? k : 0) -> inverse, 3: forward -> (mask ? k - y : 0) -> inverse
// (a kernel of its own: with the y path merely compiled in, the sweep without y ran 20-30 % slower).  In MODE 2 the measured
// k-space and the mask bytes of the tile are fetched into registers before the forward transform.
template <int N, int MODE>
__global__ __launch_bounds__(cols_threads<N>(), (cols_min_waves<N, MODE>())) void cols_kernel(ColsArgs a) {
    constexpr int L = cols_lines<N>(), NT = cols_threads<N>(), L2 = L / 2;
    constexpr int PER = (N * L2 + NT - 1) / NT;
    constexpr int kMaskUnroll = PER > 4 ? 4 : PER;   // y loads in flight per thread at the mask stage
    using Lay = Layout<N, L, 0>;
    __shared__ __attribute__((aligned(16))) float2 buf[Lay::kElems];
    __shared__ float2 tw[N];
    __shared__ __attribute__((aligned(16))) unsigned char mb[MODE >= 2 ? N * L : 16];
    fill_twiddles<N, NT>(tw);
    const long long tiles_per = (a.inner + L - 1) / L;
    const long long n_tiles = a.outer * tiles_per;
    // neighbouring column tiles share 128-byte lines: keep them on one XCD (one L2)
    const XcdRange xr = xcd_range(n_tiles);
    for (long long it = xr.first; it < xr.end; it += xr.stride) {
        const long long tile = a.rev ? n_tiles - 1 - it : it;
        const long long o = tile / tiles_per;
        const long long i0 = (tile % tiles_per) * L;
        const long long base = o * N * a.inner + i0;
        const int valid = (int)((a.inner - i0) < L ? (a.inner - i0) : L);   // even
        long long mbase = 0;
        if constexpr (MODE >= 2) {
            const long long dq = o % a.Dq;
            const long long t = (o / a.Dq) % a.T;
            const long long b = o / (a.Dq * a.T * a.C);
            mbase = ((b * a.T + t) * a.Dq + dq) * N * a.inner + i0;
        }
        __syncthreads();
        if constexpr (MODE >= 2) load_mask_tile<N, L, NT>(a.M, mbase, a.inner, valid, mb);
        // an element pair (lines l, l+1 of position p) is 16 contiguous bytes in memory and in the LDS tile
#pragma unroll
        for (int m = 0; m < PER; ++m) {
            const int idx = threadIdx.x + m * NT;
            if (idx < N * L2) {
                const int l = 2 * (idx % L2), p = idx / L2;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (l < valid) v = *reinterpret_cast<const float4*>(a.k + base + (long long)p * a.inner + l);
                if constexpr (MODE == 1) {
                    if (a.cen_io && (p & 1)) v = make_float4(-v.x, -v.y, -v.z, -v.w);
                }
                *reinterpret_cast<float4*>(&buf[Lay::at(l, p)]) = v;
            }
        }
        __syncthreads();
        if constexpr (MODE == 1) {
            fft_lines<N, L, 0, true, NT>(buf, tw);
        } else {
            fft_lines<N, L, 0, false, NT>(buf, tw);
        }
        if constexpr (MODE >= 2) {
            // the forward transform of this axis carries N^-1/2; apply it before subtracting y
            const float fs = rsqrtf((float)N);
            // Centred transform: y enters as (sign) D y.  A thread's elements of one tile share the parity of p (the
            // thread count is an even multiple of the column pairs) and its column pair starts at an even column of
            // an even-length row, so the pair's signs are (p + row of the column + sign bit) and the opposite.
            static_assert((NT / L2) % 2 == 0, "parity of p must not depend on m");
            float ysgn = 1.f, ysgn1 = 1.f;
            if constexpr (MODE == 3) {
                if (a.cen_y) {
                    const long long col = i0 + 2 * (threadIdx.x % L2);
                    ysgn = (((threadIdx.x / L2) + col / a.Wrow + a.ysign_bit) & 1) ? -1.f : 1.f;
                    ysgn1 = -ysgn;
                }
            }
            // The measured k-space is fetched here, a few loads in flight per thread: other resident workgroups cover
            // the latency, and the registers of a full prefetch would cost one of them.
#pragma unroll kMaskUnroll
            for (int m = 0; m < PER; ++m) {
                const int idx = threadIdx.x + m * NT;
                if (idx < N * L2) {
                    const int l = 2 * (idx % L2), p = idx / L2;
                    float4 yy = make_float4(0.f, 0.f, 0.f, 0.f);
                    if constexpr (MODE == 3) {
                        if (l < valid) yy = *reinterpret_cast<const float4*>(a.y + base + (long long)p * a.inner + l);
                    }
                    const unsigned mm = *reinterpret_cast<const unsigned short*>(mb + p * L + l);
                    const float4 v = *reinterpret_cast<const float4*>(&buf[Lay::at(l, p)]);
                    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (mm & 0x00ffu) { r.x = v.x * fs - ysgn * yy.x; r.y = v.y * fs - ysgn * yy.y; }
                    if (mm & 0xff00u) { r.z = v.z * fs - ysgn1 * yy.z; r.w = v.w * fs - ysgn1 * yy.w; }
                    *reinterpret_cast<float4*>(&buf[Lay::at(l, p)]) = r;
                }
            }
            __syncthreads();
            fft_lines<N, L, 0, true, NT>(buf, tw);
        }
#pragma unroll
        for (int m = 0; m < PER; ++m) {
            const int idx = threadIdx.x + m * NT;
            if (idx < N * L2) {
                const int l = 2 * (idx % L2), p = idx / L2;
                if (l < valid) {
                    const float4 v = *reinterpret_cast<const float4*>(&buf[Lay::at(l, p)]);
                    float sc = a.scale;
                    if constexpr (MODE == 1) {
                        if (a.cen_io && ((p + N / 2) & 1)) sc = -sc;
                    }
                    *reinterpret_cast<float4*>(a.k + base + (long long)p * a.inner + l) =
                        make_float4(v.x * sc, v.y * sc, v.z * sc, v.w * sc);
                }
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
    const long long g = n_tiles < cap ? (n_tiles > 0 ? n_tiles : 1) : cap;
    return (int)((g + 7) / 8 * 8);   // multiple of 8 for the XCD-aware split of the column kernels
}

static hipError_t launch_rows(bool reduce, int N, const RowsArgs& a, hipStream_t st) {
    switch (N) {
#define X(NN)                                                                                          \
    case NN: {                                                                                         \
        constexpr int L_ = rows_lines<NN>(), LR_ = reduce_lines<NN>();                                 \
        const long long per = reduce ? reduce_rows_per_tile(LR_, reduce_rows_max<NN>(), a.C)           \
                                     : reduce_rows_per_tile(L_, L_, a.C);                              \
        const long long tiles = (a.n_rows + per - 1) / per;                                            \
        if (reduce) hipLaunchKernelGGL(rows_reduce_kernel<NN>, dim3(grid_for(tiles)), dim3(reduce_threads<NN>()), 0, st, a); \
        else hipLaunchKernelGGL(rows_expand_kernel<NN>, dim3(grid_for(tiles)), dim3(rows_threads<NN>()), 0, st, a);   \
        break;                                                                                         \
    }
        GLEAM_FFT_SIZES(X)
#undef X
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

static hipError_t launch_rows_fused(int N, const RowsArgs& a, const float2* y, const unsigned char* M, hipStream_t st) {
    switch (N) {
#define X(NN)                                                                                          \
    case NN: {                                                                                         \
        constexpr int LR_ = reduce_lines<NN>();                                                        \
        const long long per = reduce_rows_per_tile(LR_, reduce_rows_max<NN>(), a.C);                   \
        const long long tiles = (a.n_rows + per - 1) / per;                                            \
        hipLaunchKernelGGL(rows_fused_kernel<NN>, dim3(grid_for(tiles)), dim3(reduce_threads<NN>()), 0, st, a, y, M); \
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
        const dim3 g(grid_for(tiles)), b(cols_threads<NN>());                                                         \
        if (mode == 0) hipLaunchKernelGGL((cols_kernel<NN, 0>), g, b, 0, st, a);                       \
        else if (mode == 1) hipLaunchKernelGGL((cols_kernel<NN, 1>), g, b, 0, st, a);                  \
        else if (a.y == nullptr) hipLaunchKernelGGL((cols_kernel<NN, 2>), g, b, 0, st, a);             \
        else hipLaunchKernelGGL((cols_kernel<NN, 3>), g, b, 0, st, a);                                 \
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
    ra.cen = g.centred ? 1 : 0; ra.par_h = g.ndim_fft >= 2; ra.par_d = g.ndim_fft >= 3; ra.Hh = g.H;
    {
        long long half = g.W / 2 + (g.ndim_fft >= 2 ? g.H / 2 : 0) + (g.ndim_fft >= 3 ? g.D / 2 : 0);
        ra.ysign_bit = (int)(half & 1);
    }
    ra.n_rows = g.B * g.T * DH;   // image rows: both row sweeps tile over (image row, coil)
    const double E8 = 8.0 * (double)(g.B * g.C * g.T * g.D * g.H * g.W);   // bytes of one k-space sweep
    const double P8 = 8.0 * (double)(g.B * g.T * g.D * g.H * g.W);          // bytes of one image
    const double S8 = E8 / (double)g.T, M1 = P8 / 8.0;
    hipError_t e;
    if (g.ndim_fft == 1) {   // one transformed axis: the whole operator in one sweep, no k-space buffer
        ra.n_rows = g.B * g.T * DH;
        KernelScope ks("sense_rows_fused", 0.0, S8 + P8 + (y ? E8 : 0.0) + M1 + P8 + (xs != 0.f ? P8 : 0.0), st);
        return launch_rows_fused((int)g.W, ra, y, M, st);
    }
    {
        KernelScope ks("sense_rows_expand", 0.0, S8 + P8 + E8, st);
        e = launch_rows(false, (int)g.W, ra, st);
    }
    if (e != hipSuccess) return e;

    ColsArgs ca{};
    ca.k = kbuf; ca.y = y; ca.M = M; ca.C = g.C; ca.T = g.T;
    ca.cen_y = (g.centred && y) ? 1 : 0; ca.ysign_bit = ra.ysign_bit; ca.cen_io = 0; ca.Wrow = g.W;
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
        ha.cen_y = 0;
        ha.rev = 1;
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

// Measured k-space to hybrid space: the inverse transform (centred when the geometry says so) along the outermost
// transformed axis, in place: H for two transformed axes, D for three.
hipError_t kspace_to_hybrid(const gleam_geom& g, float2* y, hipStream_t st) {
    ColsArgs ca{};
    ca.k = y; ca.C = g.C; ca.T = g.T; ca.Wrow = g.W;
    ca.cen_io = g.centred ? 1 : 0;
    int n;
    if (g.ndim_fft == 2) {
        ca.outer = g.B * g.C * g.T * g.D; ca.inner = g.W; ca.Dq = g.D; n = (int)g.H;
    } else {
        ca.outer = g.B * g.C * g.T; ca.inner = g.H * g.W; ca.Dq = 1; n = (int)g.D;
    }
    ca.scale = 1.0f / sqrtf((float)n);
    const double E8 = 8.0 * (double)(g.B * g.C * g.T * g.D * g.H * g.W);
    KernelScope ks("kspace_to_hybrid", 0.0, 2.0 * E8, st);
    return launch_cols(1, n, ca, st);
}

}  // namespace gleam
