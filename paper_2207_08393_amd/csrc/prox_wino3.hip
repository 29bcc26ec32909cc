// 3x3x3 convolution (forward and data gradient, float32): Winograd minimal filtering F(2x2, 3x3) of
// Lavin & Gray inside every slice, the three depth taps as a plain sum in the transformed domain:
//     Y(d) = A^T [ sum_{kd} sum_k (G g_{kd,k} G^T) .* (B^T x_k(d + kd - 1) B) ] A
// so a 2x2 block of outputs costs 3 * 16 multiplications per channel pair instead of 3 * 36, and the products are
// 16 independent matrix products over (depth tap, input channel) on the matrix cores.  The transformed input never
// exists in memory.  (B, G, A as in prox_wino.hip.)
//
// Work split.  A workgroup of 4 waves owns 8 x 32 output pixels of one slice (two groups of 2 x 16 blocks of 2x2,
// "tiles") and 32 output channels.  Wave xi owns row xi of the 4x4 product grid for both tile groups: 4 positions x
// 2 groups x (32 tiles x 32 channels) = 8 MFMA accumulators of 32x32; a transformed-weight operand read from LDS
// serves both groups.  A chunk is one depth tap x 8 input channels: the raw 10 x 34-pixel region of the tapped
// slice (zero outside the volume) and that tap's transformed weights, both copied global -> LDS by direct loads
// into the second of two buffers while the MFMAs of the current chunk run.  After the last chunk the 16 products of
// a tile are spread over the four waves; they are combined through LDS (A^T . A), one tile group per pass, and stored
// with the fused epilogue (bias, ReLU, ReLU mask, skip / gradient add).  Workgroups are persistent; blocks are
// numbered with the slice index fastest, so the workgroups of an XCD work on neighbouring slices of the same
// columns at the same time and the three reads of every slice (as tap -1, 0, +1) meet in its L2.
#include <type_traits>

#include "prox_common.h"

namespace gleam {

namespace {

constexpr int kRawSlots = 704;     // 10 rows x 34 columns x 2 channel quads = 680 quads, rounded up to whole wave loads
constexpr int kRawLoads = kRawSlots / 64;
constexpr int kUSlots = 1024;      // 16 positions x 2 channel quads x 32 output channels
constexpr int kExFloats = 4 * 2 * 32 * 8 * 4;   // per pass: 4 waves x 2 output columns x 32 tiles x 8 channel quads
constexpr int kBufFloats = (kRawSlots + kUSlots) * 4 > kExFloats ? (kRawSlots + kUSlots) * 4 : kExFloats;

// Exchange element (wave, column jj, tile, quad cq): the quad index is XOR-ed with bits of the tile index so that both
// the writers (16 lanes = 16 tiles, one quad) and the readers (16 lanes = 2 tiles x 8 quads) touch 16 different
// 16-byte bank groups.
__device__ __forceinline__ int ex_off(int wave, int jj, int tile, int cq) {
    return ((((wave * 2 + jj) * 32 + tile) * 8) + (cq ^ ((tile >> 1) & 7))) * 4;
}

__device__ __forceinline__ void dma16(const float* g, float* l) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)l, 16, 0, 0);
}
__device__ __forceinline__ void dma16_off(const float* base, unsigned byte_off, float* l) {
    dma16(reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + byte_off), l);
}

__device__ __forceinline__ float4 relu4(float4 v) {   // on the bit patterns: negative floats are negative integers
    int x0 = __float_as_int(v.x), x1 = __float_as_int(v.y), x2 = __float_as_int(v.z), x3 = __float_as_int(v.w);
    x0 = x0 > 0 ? x0 : 0; x1 = x1 > 0 ? x1 : 0; x2 = x2 > 0 ? x2 : 0; x3 = x3 > 0 ? x3 : 0;
    return make_float4(__int_as_float(x0), __int_as_float(x1), __int_as_float(x2), __int_as_float(x3));
}
__device__ __forceinline__ float4 fma4(float s, float4 a, float4 b) {   // s*a + b
    return make_float4(fmaf(s, a.x, b.x), fmaf(s, a.y, b.y), fmaf(s, a.z, b.z), fmaf(s, a.w, b.w));
}
__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ __forceinline__ float4 sub4(float4 a, float4 b) { return make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w); }

}  // namespace

template <bool RELU>
__global__ __launch_bounds__(256, 2) void conv_wino3_kernel(WinoArgs a) {
    // Separate LDS objects: reads of one chunk buffer then do not wait for direct loads into the other.
    __shared__ __attribute__((aligned(16))) float bufA[kBufFloats];
    __shared__ __attribute__((aligned(16))) float bufB[kBufFloats];
    float* const ex = bufB;   // the exchange of the output transform reuses the second chunk buffer
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, h = lane >> 5, xi = wave;
    const int trl = m >> 4, tc = m & 15;

    const XcdRange xr = xcd_range(a.n_blocks);
    const int ny = blockIdx.y, n0 = ny * 32;
    const int n_kc = a.K / 8;          // even (K is a multiple of 16)
    const int n_ch = 3 * n_kc;         // chunks per block
    const long long plane = (long long)a.H * a.W * a.K;   // floats per slice

    // Direct-load sources of this lane: three quads of the raw region (a zero quad outside the slice).
    int s_row[3], s_col[3], s_quad[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int s = tid + i * 256;
        // slot = ((row*2 + column parity)*17 + column/2)*2 + quad: the two quads of a pixel are neighbouring lanes
        // (one 32-byte request), even columns before odd ones
        const int rp = s / 34, rem = s - rp * 34;
        s_col[i] = 2 * (rem >> 1) + (rp & 1);
        s_row[i] = s < 680 ? (rp >> 1) : -100000;            // slots past the region always read the zero quad
        s_quad[i] = rem & 1;
    }
    struct Block {
        int x0, y0, d;
        long long img;
        const float* gp[3];   // this lane's quads in the block's own slice, channel 0 (the zero quad when outside)
        int in_img;           // bit i: quad i lies inside the slice
    };
    auto setup = [&](long long item) {
        Block b;
        b.d = (int)(item % a.D);
        long long rest = item / a.D;
        const int bx = (int)(rest % a.bx_n);
        rest /= a.bx_n;
        const int by = (int)(rest % a.by_n);
        b.img = (rest / a.by_n) * a.D + b.d;
        b.x0 = bx * 32;
        b.y0 = by * 8;
        b.in_img = 0;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int yy = b.y0 - 1 + s_row[i], xx = b.x0 - 1 + s_col[i];
            const bool ok = yy >= 0 && yy < a.H && xx >= 0 && xx < a.W;
            b.gp[i] = ok ? a.in + ((b.img * a.H + yy) * a.W + xx) * a.K + s_quad[i] * 4 : a.zero;
            b.in_img |= ok ? (1 << i) : 0;
        }
        return b;
    };
    const float* ubase = a.u + (size_t)ny * n_ch * (kUSlots * 4);   // uniform; lanes add a 32-bit offset
    const unsigned uoff = 16u * (unsigned)tid;   // bytes

    // chunk c = kd * n_kc + kc
    auto issue = [&](const Block& b, int c, float* dst) {
        const int kd = c >= 2 * n_kc ? 2 : (c >= n_kc ? 1 : 0);
        const int kc = c - kd * n_kc;
        const int dz = b.d + kd - 1;
        const bool slice_ok = dz >= 0 && dz < a.D;          // uniform
        const long long shift = (long long)(kd - 1) * plane + kc * 8;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int o = wave + i * 4;
            if (o < kRawLoads) {
                const float* p = (slice_ok && ((b.in_img >> i) & 1)) ? b.gp[i] + shift : a.zero;
                dma16(p, dst + o * 256);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int o = wave + i * 4;
            const float* ub = ubase + ((size_t)c * (kUSlots * 4) + 1024 * i);   // scalar address
            dma16_off(ub, uoff, dst + kRawSlots * 4 + o * 256);
        }
    };

    // row xi of B^T: d[ra] + sg * d[rb]
    const int ra = xi == 0 ? 0 : (xi == 2 ? 2 : 1);
    const int rb = xi == 3 ? 3 : (xi == 2 ? 1 : 2);
    const float sg = xi == 1 ? 1.f : -1.f;
    // Region quad (row, column, quad) sits at slot ((row*2 + (column & 1))*17 + column/2)*2 + quad; tile group g
    // starts four region rows further down.
    const int offA = (((2 * trl + ra) * 2) * 17 + tc) * 8 + 4 * h;
    const int offB = (((2 * trl + rb) * 2) * 17 + tc) * 8 + 4 * h;
    constexpr int kGroupFloats = 4 * 2 * 17 * 8;
    // U quad (position, channel quad hq, output channel n) at slot ((pos*2 + hq)*32 + n)
    const int offU = kRawSlots * 4 + (((xi * 4) * 2 + h) * 32 + m) * 4;

    floatx16 acc[4][2];

    auto compute = [&](const float* buf, auto first_c) {
        constexpr bool FIRST = decltype(first_c)::value;   // first chunk of a block: accumulators start from zero
        float4 v[2][4];
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            float4 t[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float4 da = *reinterpret_cast<const float4*>(buf + offA + g * kGroupFloats + ((c & 1) * 17 + (c >> 1)) * 8);
                float4 db = *reinterpret_cast<const float4*>(buf + offB + g * kGroupFloats + ((c & 1) * 17 + (c >> 1)) * 8);
                if (RELU) {
                    da = relu4(da);
                    db = relu4(db);
                }
                t[c] = fma4(sg, db, da);
            }
            v[g][0] = sub4(t[0], t[2]);
            v[g][1] = add4(t[1], t[2]);
            v[g][2] = sub4(t[2], t[1]);
            v[g][3] = sub4(t[1], t[3]);
        }
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) {
            const float4 u = *reinterpret_cast<const float4*>(buf + offU + (nu * 2 * 32) * 4);
            if (FIRST) {
                floatx16 z;
#pragma unroll
                for (int r = 0; r < 16; ++r) z[r] = 0.f;
                acc[nu][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(u.x, v[0][nu].x, z, 0, 0, 0);
                acc[nu][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(u.x, v[1][nu].x, z, 0, 0, 0);
            } else {
                acc[nu][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(u.x, v[0][nu].x, acc[nu][0], 0, 0, 0);
                acc[nu][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(u.x, v[1][nu].x, acc[nu][1], 0, 0, 0);
            }
            acc[nu][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(u.y, v[0][nu].y, acc[nu][0], 0, 0, 0);
            acc[nu][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(u.y, v[1][nu].y, acc[nu][1], 0, 0, 0);
            acc[nu][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(u.z, v[0][nu].z, acc[nu][0], 0, 0, 0);
            acc[nu][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(u.z, v[1][nu].z, acc[nu][1], 0, 0, 0);
            acc[nu][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(u.w, v[0][nu].w, acc[nu][0], 0, 0, 0);
            acc[nu][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(u.w, v[1][nu].w, acc[nu][1], 0, 0, 0);
        }
    };

    if (xr.first >= xr.end) return;   // uniform for the workgroup
    Block cur = setup(xr.first);
    issue(cur, 0, bufA);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    const float4 bias_r = a.bias ? *reinterpret_cast<const float4*>(a.bias + n0 + 4 * (tid & 7)) : make_float4(0.f, 0.f, 0.f, 0.f);
    for (long long item = xr.first; item < xr.end; item += xr.stride) {
        const bool has_next = item + xr.stride < xr.end;
        const Block nxt = setup(has_next ? item + xr.stride : item);
        const int x0 = cur.x0, y0 = cur.y0;
        const long long img = cur.img;
        // n_ch is even: chunks alternate between the two buffers
        issue(cur, 1, bufB);
        __builtin_amdgcn_sched_barrier(0);   // keep the direct loads ahead of the MFMAs they overlap with
        compute(bufA, std::true_type{});
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        for (int c = 1; c < n_ch; c += 2) {
            // the first chunk of the next block is fetched under the last MFMAs of this one
            if (c + 1 < n_ch) issue(cur, c + 1, bufA);
            else if (has_next) issue(nxt, 0, bufA);
            __builtin_amdgcn_sched_barrier(0);
            compute(bufB, std::false_type{});
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            if (c + 1 >= n_ch) break;
            issue(cur, c + 2, bufB);
            __builtin_amdgcn_sched_barrier(0);
            compute(bufA, std::false_type{});
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        }

        // Output transform.  In registers over nu: R_0 = M_0 + M_1 + M_2, R_1 = M_1 - M_2 - M_3; across the four waves
        // through LDS: Y_0 = R[xi=0] + R[1] + R[2], Y_1 = R[1] - R[2] - R[3].  One pass per tile group.  A thread
        // finishes the 2x2 pixels of one tile for one channel quad; what the fused epilogue reads from memory (ReLU
        // mask source, tensor to add) is requested for all four pixels before the exchange, from a clamped address
        // where the pixel is outside the slice.
        const int e_cq = tid & 7, e_tile = (tid >> 3) & 31;
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            if (g) __syncthreads();
            const int ey = y0 + 4 * g + 2 * (e_tile >> 4), ex_ = x0 + 2 * (e_tile & 15);
            bool okp[2][2];
            long long op[2][2];
            float4 refv[2][2], addv[2][2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    okp[i][jj] = ey + i < a.H && ex_ + jj < a.W;
                    op[i][jj] = okp[i][jj] ? ((img * a.H + ey + i) * a.W + ex_ + jj) * a.Nn + n0 + 4 * e_cq : (long long)(n0 + 4 * e_cq);
                    refv[i][jj] = make_float4(1.f, 1.f, 1.f, 1.f);
                    addv[i][jj] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (a.mask_ref) refv[i][jj] = *reinterpret_cast<const float4*>(a.mask_ref + op[i][jj]);
                    if (a.add) addv[i][jj] = *reinterpret_cast<const float4*>(a.add + op[i][jj]);
                }
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                float r0[4], r1[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float m0 = acc[0][g][4 * rg + i], m1 = acc[1][g][4 * rg + i];
                    const float m2 = acc[2][g][4 * rg + i], m3 = acc[3][g][4 * rg + i];
                    r0[i] = m0 + m1 + m2;
                    r1[i] = m1 - m2 - m3;
                }
                const int cq = 2 * rg + h;
                *reinterpret_cast<float4*>(ex + ex_off(wave, 0, m, cq)) = make_float4(r0[0], r0[1], r0[2], r0[3]);
                *reinterpret_cast<float4*>(ex + ex_off(wave, 1, m, cq)) = make_float4(r1[0], r1[1], r1[2], r1[3]);
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 2; ++i) {          // output row inside the tile
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {   // output column inside the tile
                    auto rd = [&](int x_i) { return *reinterpret_cast<const float4*>(ex + ex_off(x_i, jj, e_tile, e_cq)); };
                    float4 yv;
                    if (i == 0) yv = add4(add4(rd(0), rd(1)), rd(2));
                    else yv = sub4(sub4(rd(1), rd(2)), rd(3));
                    float v[4] = {yv.x + bias_r.x, yv.y + bias_r.y, yv.z + bias_r.z, yv.w + bias_r.w};
                    if (a.relu_out) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
                    }
                    const float rr[4] = {refv[i][jj].x, refv[i][jj].y, refv[i][jj].z, refv[i][jj].w};
                    const float aa[4] = {addv[i][jj].x, addv[i][jj].y, addv[i][jj].z, addv[i][jj].w};
                    if (a.mask_acc) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = rr[e] > 0.f ? v[e] : 0.f;
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += (a.mask_add && !(rr[e] > 0.f)) ? 0.f : aa[e];
                    if (okp[i][jj]) *reinterpret_cast<float4*>(a.out + op[i][jj]) = make_float4(v[0], v[1], v[2], v[3]);
                }
            }
        }
        __syncthreads();   // the exchange lived in the second chunk buffer, which the next block loads into first
        cur = nxt;
    }
}

// U = G g G^T for every (depth tap, output channel n, input channel k), laid out as the kernel's LDS images:
// u[(((((ny*3 + kd)*n_kc + kc)*16 + pos)*2 + hq)*32 + nn)*4 + kk], n = 32*ny + nn, k = 8*kc + 4*hq + kk, pos = 4*xi + nu;
// one zero quad follows.  Source weight (n, tap, k) at w[n*sn + tapidx*st + k*sk], tap = (kd*3 + kh)*3 + kw, taps
// mirrored for the data gradient.
__global__ __launch_bounds__(256) void wino3_weights_kernel(const float* __restrict__ w, long long sn, long long st_, long long sk,
                                                            int flip, int K, int Nn, float* __restrict__ u) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx == 0) {
        float* z = u + (size_t)48 * K * Nn;
        z[0] = z[1] = z[2] = z[3] = 0.f;
    }
    if (idx >= K * Nn) return;
    const int k = idx % K, n = idx / K;
    const int ny = n / 32, nn = n % 32, kc = k / 8, hq = (k % 8) / 4, kk = k % 4, n_kc = K / 8;
    for (int kd = 0; kd < 3; ++kd) {
        float g[3][3];
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int tap = kd * 9 + t;
            g[t / 3][t % 3] = w[n * sn + (flip ? 26 - tap : tap) * st_ + k * sk];
        }
        float gg[4][3];   // G g
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            gg[0][b] = g[0][b];
            gg[1][b] = 0.5f * (g[0][b] + g[1][b] + g[2][b]);
            gg[2][b] = 0.5f * (g[0][b] - g[1][b] + g[2][b]);
            gg[3][b] = g[2][b];
        }
        float* dst = u + (((((size_t)(ny * 3 + kd) * n_kc + kc) * 16) * 2 + hq) * 32 + nn) * 4 + kk;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const float uu[4] = {gg[x][0], 0.5f * (gg[x][0] + gg[x][1] + gg[x][2]), 0.5f * (gg[x][0] - gg[x][1] + gg[x][2]), gg[x][2]};
#pragma unroll
            for (int nu = 0; nu < 4; ++nu) dst[(size_t)(4 * x + nu) * 2 * 32 * 4] = uu[nu];
        }
    }
}

bool conv_wino3_applies(const PixDims& d, int K, int Nn) {
    return d.kt == 1 && d.kd == 3 && d.kh == 3 && d.kw == 3 && K % 16 == 0 && Nn % 32 == 0 &&
           (long long)d.H * d.W * K < (1LL << 30);
}

size_t conv_wino3_weight_floats(int K, int Nn) { return (size_t)48 * K * Nn + 4; }

hipError_t launch_conv_wino3(WinoArgs a, const float* w, long long sn, long long st_, long long sk, int flip, int relu_in,
                             float* u_scratch, const char* name, hipStream_t st) {
    {
        KernelScope ks("weights_image", 0.0, 4.0 * (27 + 48) * a.K * a.Nn, st);
        hipLaunchKernelGGL(wino3_weights_kernel, dim3((unsigned)((a.K * a.Nn + 255) / 256)), dim3(256), 0, st, w, sn, st_, sk, flip,
                           a.K, a.Nn, u_scratch);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    a.u = u_scratch;
    a.zero = u_scratch + (size_t)48 * a.K * a.Nn;
    a.bx_n = (a.W + 31) / 32;
    a.by_n = (a.H + 7) / 8;
    a.n_blocks = a.NI * (long long)a.bx_n * a.by_n;
    const long long cap = 512 / (a.Nn / 32) > 8 ? 512 / (a.Nn / 32) : 8;   // two workgroups per CU in total
    const long long gx = ((a.n_blocks < cap ? a.n_blocks : cap) + 7) / 8 * 8;
    dim3 grid((unsigned)gx, (unsigned)(a.Nn / 32));
    const double Q = (double)a.NI * a.H * a.W;
    // 16 multiplications per 2x2 outputs, depth tap and channel pair on the matrix cores instead of the 36 of the definition
    KernelScope ks(name, 2.0 * Q * a.K * a.Nn * 27, 4.0 * Q * (a.K + a.Nn), st, 2.0 * Q * a.K * a.Nn * 12);
    if (relu_in) hipLaunchKernelGGL((conv_wino3_kernel<true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((conv_wino3_kernel<false>), grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace gleam
