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
// while the MFMAs of earlier chunks run.  After the last chunk the 16 products of
// a tile are spread over the four waves; they are combined through LDS (A^T . A), one tile group per pass, and stored
// with the fused epilogue (bias, ReLU, ReLU mask, skip / gradient add).  Workgroups are persistent; blocks are
// numbered with the slice index fastest, so the workgroups of an XCD work on neighbouring slices of the same
// columns at the same time and the three reads of every slice (as tap -1, 0, +1) meet in its L2.
#include <type_traits>

#include "prox_common.h"

namespace gleam {

namespace {

constexpr int kUSlots = 1024;      // 16 positions x 2 channel quads x 32 output channels

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

// Staging.  The raw regions are staged 16 input channels at a time (64 contiguous bytes per pixel and request; with 8
// channels, i.e. 32 bytes, the same bytes took twice the memory requests and the kernel 5 % longer) while the
// transformed weights come in 8-channel chunks: a raw half serves two chunks and is requested two chunks ahead, a
// weight chunk one chunk ahead.  Four LDS objects (two raw halves, two weight chunks) and the chunk loop written out
// over its period of four, so that the compiler knows which buffer a read touches and does not make it wait for
// loads in flight into another.  Inside a pixel the four channel quads are XOR-ed with bits 2..3 of the half-column
// index, so that the 16 lanes a 128-bit read serves together (16 neighbouring tiles, one quad) fall on 16 different
// bank groups.  K must be a multiple of 32 (an even number of halves per depth tap keeps the rotation aligned).
constexpr int kRHSlots = 1408;     // 10 rows x 2 column parities x 17 half-columns x 4 quads = 1360, rounded up to whole wave loads
constexpr int kRHLoads = kRHSlots / 64;
constexpr int kExHalfFloats = 4 * 32 * 8 * 4;   // per output column: 4 waves x 32 tiles x 8 channel quads
static_assert(kExHalfFloats <= kUSlots * 4 && kExHalfFloats <= kRHSlots * 4, "the exchange reuses a weight and a raw buffer");
// Exchange element (wave, tile, quad cq) of an output column: the quad index is XOR-ed with bits of the tile index so
// that both the writers (16 lanes = 16 tiles, one quad) and the readers (16 lanes = 2 tiles x 8 quads) touch 16
// different 16-byte bank groups.
__device__ __forceinline__ int exh_off(int wave, int tile, int cq) { return (((wave * 32 + tile) * 8) + (cq ^ ((tile >> 1) & 7))) * 4; }

template <bool RELU, bool EPI>   // EPI: the call has a ReLU mask source or a tensor to add
__global__ __launch_bounds__(256, 2) void conv_wino3_kernel(WinoArgs a) {
    __shared__ __attribute__((aligned(16))) float R0[kRHSlots * 4];
    __shared__ __attribute__((aligned(16))) float R1[kRHSlots * 4];
    __shared__ __attribute__((aligned(16))) float U0[kUSlots * 4];
    __shared__ __attribute__((aligned(16))) float U1[kUSlots * 4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, h = lane >> 5, xi = wave;
    const int trl = m >> 4, tc = m & 15;

    const XcdRange xr = xcd_range(a.n_blocks);
    const int ny = blockIdx.y, n0 = ny * 32;
    const int n_kc = a.K / 8, n_hf = a.K / 16;   // chunks and raw halves per depth tap
    const int n_ch = 3 * n_kc;                   // chunks per block: a multiple of 4
    const long long plane = (long long)a.H * a.W * a.K;   // floats per slice

    // Direct loads of the raw halves: slot s = tid + 256*i holds (row*2 + column parity, half-column, position) =
    // (s / 68, (s % 68) / 4, s % 4); the channel quad at a position is position ^ ((half-column >> 2) & 3).
    unsigned r_off[6];     // byte offset of the slot's quad from the region origin (pixel (y0-1, x0-1), first channel of the half)
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        const int s = tid + 256 * i;
        const int rp = s / 68, rem = s - rp * 68;
        const int colh = rem >> 2, quad = (rem & 3) ^ ((colh >> 2) & 3);
        const int row = rp >> 1, col = 2 * colh + (rp & 1);
        r_off[i] = s < 1360 ? 4u * (unsigned)((row * a.W + col) * a.K + 4 * quad) : 0u;
    }
    struct Block {
        int x0, y0, d;
        long long img;
        unsigned in_img;      // bit i: slot i lies inside the slice
        bool interior;        // the whole region lies inside the slice (uniform)
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
        b.interior = b.y0 >= 1 && b.y0 + 8 < a.H && b.x0 >= 1 && b.x0 + 32 < a.W;
        b.in_img = 0u;
        if (!b.interior) {   // the slots' pixels again (once per border block; not worth six registers)
            int t = tid;
            asm volatile("" : "+v"(t));
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                const int s = t + 256 * i;
                const int rp = s / 68, rem = s - rp * 68;
                const int yy = b.y0 - 1 + (rp >> 1), xx = b.x0 - 1 + 2 * (rem >> 2) + (rp & 1);
                const bool ok = s < 1360 && yy >= 0 && yy < a.H && xx >= 0 && xx < a.W;
                b.in_img |= ok ? (1u << i) : 0u;
            }
        }
        return b;
    };
    // raw half hidx = kd * n_hf + hf of block b
    auto issue_raw = [&](const Block& b, int hidx, float* dst) {
        const int kd = hidx >= 2 * n_hf ? 2 : (hidx >= n_hf ? 1 : 0);
        const int hf = hidx - kd * n_hf;
        const int dz = b.d + kd - 1;
        const bool slice_ok = dz >= 0 && dz < a.D;          // uniform
        // region origin; only dereferenced through lanes whose pixel lies inside the slice
        const float* base = a.in + (b.img + kd - 1) * plane + ((long long)(b.y0 - 1) * a.W + (b.x0 - 1)) * a.K + 16 * hf;
        if (slice_ok && b.interior) {
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                const int o = wave + 4 * i;
                if (o < kRHLoads) dma16_off(base, r_off[i], dst + o * 256);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                const int o = wave + 4 * i;
                if (o < kRHLoads) {
                    const bool ok = slice_ok && ((b.in_img >> i) & 1u);
                    const float* p = ok ? reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + r_off[i]) : a.zero;
                    dma16(p, dst + o * 256);
                }
            }
        }
    };
    const float* ubase = a.u + (size_t)ny * n_ch * (kUSlots * 4);   // uniform; lanes add a 32-bit offset
    const unsigned uoff = 16u * (unsigned)tid;   // bytes
    auto issue_u = [&](int c, float* dst) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int o = wave + i * 4;
            const float* ub = ubase + ((size_t)c * (kUSlots * 4) + 1024 * i);   // scalar address
            dma16_off(ub, uoff, dst + o * 256);
        }
    };

    // row xi of B^T: d[ra] + sg * d[rb]
    const int ra = xi == 0 ? 0 : (xi == 2 ? 2 : 1);
    const int rb = xi == 3 ? 3 : (xi == 2 ? 1 : 2);
    const float sg = xi == 1 ? 1.f : -1.f;
    // float offset of this lane's quad: region row r, column 2*tc + c, channel quad 2*sub + h of the half ->
    // ((r*2 + (c & 1))*17 + tc + (c >> 1))*16 + 4*((2*sub + h) ^ (((tc + (c >> 1)) >> 2) & 3)); tile group g starts four rows down
    int pa[2][2], pb[2][2];   // [c >> 1][sub]
#pragma unroll
    for (int cs = 0; cs < 2; ++cs)
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int colh = tc + cs;
            const int lanepart = colh * 16 + 4 * ((2 * sub + h) ^ ((colh >> 2) & 3));
            pa[cs][sub] = (2 * trl + ra) * 2 * 17 * 16 + lanepart;
            pb[cs][sub] = (2 * trl + rb) * 2 * 17 * 16 + lanepart;
        }
    constexpr int kParFloats = 17 * 16, kGroupFloats = 4 * 2 * 17 * 16;
    // U quad (position, channel quad hq, output channel n) at slot ((pos*2 + hq)*32 + n)
    const int offU = (((xi * 4) * 2 + h) * 32 + m) * 4;

    floatx16 acc[4][2];

    auto compute = [&](const float* raw, const float* u_, auto sub_c, auto first_c) __attribute__((always_inline)) {
        constexpr int SUB = decltype(sub_c)::value;
        constexpr bool FIRST = decltype(first_c)::value;   // first chunk of a block: accumulators start from zero
        float4 v[2][4];
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            float4 t[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float4 da = *reinterpret_cast<const float4*>(raw + pa[c >> 1][SUB] + g * kGroupFloats + (c & 1) * kParFloats);
                float4 db = *reinterpret_cast<const float4*>(raw + pb[c >> 1][SUB] + g * kGroupFloats + (c & 1) * kParFloats);
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
            const float4 u = *reinterpret_cast<const float4*>(u_ + offU + (nu * 2 * 32) * 4);
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
    auto sync = [&]() {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };

    if (xr.first >= xr.end) return;   // uniform for the workgroup
    Block cur = setup(xr.first);
    issue_raw(cur, 0, R0);
    issue_u(0, U0);
    sync();
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    for (long long item = xr.first; item < xr.end; item += xr.stride) {
        const bool has_next = item + xr.stride < xr.end;
        const Block nxt = setup(has_next ? item + xr.stride : item);
        const int x0 = cur.x0, y0 = cur.y0;
        const long long img = cur.img;
        // chunk c reads raw half c / 2 (R0, R0, R1, R1, ...) and weight chunk c (U0, U1, U0, U1, ...); a raw half is
        // requested two chunks before its first use, a weight chunk one chunk before
        for (int c = 0; c < n_ch; c += 4) {
            const bool last4 = c + 4 >= n_ch;
            issue_u(c + 1, U1);
            issue_raw(cur, c / 2 + 1, R1);
            __builtin_amdgcn_sched_barrier(0);   // keep the direct loads ahead of the MFMAs they overlap with
            if (c == 0) compute(R0, U0, I0{}, std::true_type{});
            else compute(R0, U0, I0{}, std::false_type{});
            sync();
            issue_u(c + 2, U0);
            __builtin_amdgcn_sched_barrier(0);
            compute(R0, U1, I1{}, std::false_type{});
            sync();
            issue_u(c + 3, U1);
            if (!last4) issue_raw(cur, c / 2 + 2, R0);
            else if (has_next) issue_raw(nxt, 0, R0);
            __builtin_amdgcn_sched_barrier(0);
            compute(R1, U0, I0{}, std::false_type{});
            sync();
            if (!last4) issue_u(c + 4, U0);
            else if (has_next) issue_u(0, U0);
            __builtin_amdgcn_sched_barrier(0);
            compute(R1, U1, I1{}, std::false_type{});
            sync();
        }

        // Output transform.  In registers over nu: R_0 = M_0 + M_1 + M_2, R_1 = M_1 - M_2 - M_3; across the four waves
        // through LDS: Y_0 = R[xi=0] + R[1] + R[2], Y_1 = R[1] - R[2] - R[3].  One pass per tile group; the exchange goes
        // through the weight and the raw buffer that the loads of the next block do not use, one output column each.
        // A thread finishes the 2x2 pixels of one tile for one channel quad; what the fused epilogue reads from memory
        // (ReLU mask source, tensor to add) is requested for all four pixels before the exchange, from a clamped
        // address where the pixel is outside the slice.
        const int e_cq = tid & 7, e_tile = (tid >> 3) & 31;
        const float4 bias_r = a.bias ? *reinterpret_cast<const float4*>(a.bias + n0 + 4 * e_cq) : make_float4(0.f, 0.f, 0.f, 0.f);
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
                    if constexpr (EPI) {
                        if (a.mask_ref) refv[i][jj] = *reinterpret_cast<const float4*>(a.mask_ref + op[i][jj]);
                        if (a.add) addv[i][jj] = *reinterpret_cast<const float4*>(a.add + op[i][jj]);
                    }
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
                *reinterpret_cast<float4*>(U1 + exh_off(wave, m, cq)) = make_float4(r0[0], r0[1], r0[2], r0[3]);
                *reinterpret_cast<float4*>(R1 + exh_off(wave, m, cq)) = make_float4(r1[0], r1[1], r1[2], r1[3]);
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 2; ++i) {          // output row inside the tile
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {   // output column inside the tile
                    const float* exj = jj ? R1 : U1;
                    auto rd = [&](int x_i) { return *reinterpret_cast<const float4*>(exj + exh_off(x_i, e_tile, e_cq)); };
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
                    if constexpr (EPI) {
                        if (a.mask_acc) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = rr[e] > 0.f ? v[e] : 0.f;
                        }
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += (a.mask_add && !(rr[e] > 0.f)) ? 0.f : aa[e];
                    }
                    if (okp[i][jj]) *reinterpret_cast<float4*>(a.out + op[i][jj]) = make_float4(v[0], v[1], v[2], v[3]);
                }
            }
        }
        __syncthreads();   // the exchange lived in buffers that the first chunk of the next block loads into
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

// ------------------------------------------------------------------ weight gradient
// dL/dg_kd = G^T [ sum over slices d and tiles of (A dY(d) A^T) .* (B^T x(d + kd - 1) B) ] G: per depth tap and position
// of the 4x4 grid a [cout x tiles] . [tiles x cin] matrix product, 16 multiplications per tile, depth tap and channel
// pair instead of 36.  A workgroup of 4 waves owns a 32 x 32 channel block; wave xi owns row xi of the grid for all
// three depth taps: 3 x 4 accumulators of 32x32.  A chunk is 16 tiles (2 x 32 output pixels) of one column of the
// volume at input slice tau: the transformed input operand is formed once and multiplied with the transformed
// gradients of slices tau + 1, tau and tau - 1 (depth taps 0, 1, 2).  A workgroup walks a run of consecutive slices
// of its column, so every chunk needs one new input region (4 x 34 pixels) and one new gradient region (2 x 32
// pixels): the input regions alternate between two LDS buffers and the gradient regions rotate through four, all
// filled by direct global -> LDS loads one chunk ahead.  The six buffers are separate LDS objects and the loop is
// written out over the four rotations, so that the compiler knows which buffer every read touches and does not
// make the reads wait for the loads in flight.  Both MFMA operands are formed on the fly as in the 2D kernel
// (a lane holds one channel and one of the two tiles of a contraction step).  Every workgroup writes its partial
// sums once; a fixed-order reduction and G^T . G follow.
constexpr int k3XSlots = 4 * 34 * 8;   // input region: 4 rows x 34 columns x 8 channel quads
constexpr int k3GSlots = 2 * 32 * 8;   // gradient region
constexpr int k3XLoads = k3XSlots / 64, k3GLoads = k3GSlots / 64;
static_assert(k3XSlots % 64 == 0 && k3GSlots % 64 == 0, "regions are whole wave loads");

template <bool RELU>
__global__ __launch_bounds__(256, 2) void wgrad_wino3_kernel(Wino3WgradArgs a) {
    // element (pixel, channel) of a region sits at (pixel >> 1)*64 + (((pixel & 1) ^ ((pixel >> 1) & 1))*32 + channel:
    // the two lane halves of a 4-byte operand read (pixels two apart) then use different banks
    __shared__ __attribute__((aligned(16))) float X0[k3XSlots * 4];
    __shared__ __attribute__((aligned(16))) float X1[k3XSlots * 4];
    __shared__ __attribute__((aligned(16))) float G0[k3GSlots * 4];
    __shared__ __attribute__((aligned(16))) float G1[k3GSlots * 4];
    __shared__ __attribute__((aligned(16))) float G2[k3GSlots * 4];
    __shared__ __attribute__((aligned(16))) float G3[k3GSlots * 4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int xi = wave;
    const int m = lane & 31, h = lane >> 5;
    const int nci = a.Ci / 32;
    const int co0 = 32 * ((int)blockIdx.y / nci), ci0 = 32 * ((int)blockIdx.y % nci);
    const size_t pblock = (size_t)a.Co * a.Ci;
    float* const pout = a.partial + (size_t)blockIdx.x * 48 * pblock;
    const XcdRange xr = xcd_range(a.n_items);
    if (xr.first >= xr.end) {   // nothing to do: the partial of this workgroup is zero
        for (int i = tid; i < 48 * 32 * 32; i += 256) {
            const int pos = i >> 10, co = (i >> 5) & 31, ci = i & 31;
            pout[((size_t)pos * a.Co + co0 + co) * a.Ci + ci0 + ci] = 0.f;
        }
        if (a.bias_partial && ci0 == 0 && tid < 32) a.bias_partial[(size_t)blockIdx.x * a.Co + co0 + tid] = 0.f;
        return;
    }

    // Direct loads.  Slot s of a region (16 bytes at float offset 4*s) holds channel quad s & 7 of pixel
    // 2*(s >> 4) + (((s >> 3) ^ (s >> 4)) & 1).  A thread's seven slots (five of the input region, two of the gradient
    // region) do not change along a run of slices, so their byte offsets inside a slice - or an offset outside every
    // slice when the pixel lies outside the image - are worked out once per run and kept in a thread-private column
    // of an LDS table (registers are what this kernel is short of).  A chunk's loads then go through a buffer
    // resource that spans the slice (of size 0 for a slice outside the volume): out-of-image pixels arrive as zeros
    // with the data, without bounds checks, selects or zero stores in the loop.
    __shared__ unsigned slot_tab[7 * 256];
    constexpr unsigned kOutside = 0x80000000u;   // (a slice is below 2^31 bytes: checked by wgrad_wino3_applies)
    auto slots_of_run = [&](int y0, int x0) {
#pragma unroll
        for (int i = 0; i < 7; ++i) {
            const bool is_x = i < 5;
            const int s = tid + 256 * (is_x ? i : i - 5);
            const int pp = s >> 4, qd = s & 7;
            const int px = 2 * pp + (((s >> 3) ^ pp) & 1);
            const int cols = is_x ? 34 : 32, C = is_x ? a.Ci : a.Co, c0 = is_x ? ci0 : co0;
            const int row = px / cols, col = px - row * cols;
            const int yy = (is_x ? y0 - 1 : y0) + row, xx = (is_x ? x0 - 1 : x0) + col;
            const bool ok = row < (is_x ? 4 : 2) && yy >= 0 && yy < a.H && xx >= 0 && xx < a.W;
            slot_tab[i * 256 + tid] = ok ? (unsigned)(((yy * a.W + xx) * C + c0 + 4 * qd) * 4) : kOutside;
        }
    };
    // FIRST / LOADS: first table row and wave-wide loads of the region (17 for the input, 8 for the gradient);
    // plane: the slice of the tensor (C channels per pixel), or null if it lies outside the volume
    auto fill = [&](const float* plane, int C, auto first_c, auto loads_c, float* dst) {
        constexpr int FIRST = decltype(first_c)::value, LOADS = decltype(loads_c)::value, N = (LOADS + 3) / 4;
        const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(plane ? plane : a.a), 0, plane ? (unsigned)(a.H * a.W * C * 4) : 0u, 0x00020000);
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int o = wave + 4 * i;
            if (o < LOADS)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)(dst + o * 256), 16,
                                                         slot_tab[(FIRST + i) * 256 + tid], 0, 0, 0);
        }
    };

    // row xi of A dY (coefficients of the two gradient rows) and of B^T d (two of the four input rows)
    const float ca = xi == 3 ? 0.f : 1.f, cb = xi == 0 ? 0.f : (xi == 1 ? 1.f : -1.f);
    const int ra = xi == 0 ? 0 : (xi == 2 ? 2 : 1), rb = xi == 3 ? 3 : (xi == 2 ? 1 : 2);
    const float sg = xi == 1 ? 1.f : -1.f;
    // LDS float offsets of this lane: input pixel (row r, column 4q + 2h + 2cp + e) sits at xo[rs][cp] ^ (32*e), + 128*q;
    // gradient pixel (row, column 4q + 2h + e) at go[e] + 1024*row + 128*q
    int xo[2][2], go[2];
#pragma unroll
    for (int rs = 0; rs < 2; ++rs)
#pragma unroll
        for (int cp = 0; cp < 2; ++cp) {
            const int r = rs ? rb : ra;
            xo[rs][cp] = (17 * r + h + cp) * 64 + ((r + h + cp) & 1) * 32 + m;
        }
#pragma unroll
    for (int e = 0; e < 2; ++e) go[e] = h * 64 + (e ^ h) * 32 + m;

    floatx16 acc[3][4];   // [depth tap][column nu of the product grid]
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
#pragma unroll
        for (int nu = 0; nu < 4; ++nu)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[kd][nu][r] = 0.f;
    float bsum = 0.f;

    // One chunk: 8 contraction steps (tiles 2q and 2q+1 on the two lane halves), 12 MFMAs each.
    // gp / gz / gm: gradient regions of slices tau + 1, tau, tau - 1 (depth taps 0, 1, 2).
    auto run = [&](const float* x, const float* gp, const float* gz, const float* gm) __attribute__((always_inline)) {
        float rg[3][4], rd[2][4];   // raw pixels of one step: gradient [depth tap][row*2 + column], input [row a/b][column]
        auto load = [&](int q) {
#pragma unroll
            for (int kd = 0; kd < 3; ++kd) {
                const float* g = kd == 0 ? gp : (kd == 1 ? gz : gm);
                rg[kd][0] = g[go[0] + 128 * q];
                rg[kd][1] = g[go[1] + 128 * q];
                rg[kd][2] = g[go[0] + 1024 + 128 * q];
                rg[kd][3] = g[go[1] + 1024 + 128 * q];
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                rd[0][c] = x[(xo[0][c >> 1] ^ (32 * (c & 1))) + 128 * q];
                rd[1][c] = x[(xo[1][c >> 1] ^ (32 * (c & 1))) + 128 * q];
            }
        };
        load(0);
#pragma unroll 1
        for (int q = 0; q < 8; ++q) {
            float v[4], z[3][4];
            {
                float t[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float da = rd[0][c], dbv = rd[1][c];
                    if (RELU) {
                        da = __int_as_float(__float_as_int(da) > 0 ? __float_as_int(da) : 0);
                        dbv = __int_as_float(__float_as_int(dbv) > 0 ? __float_as_int(dbv) : 0);
                    }
                    t[c] = fmaf(sg, dbv, da);   // row xi of B^T d
                }
                v[0] = t[0] - t[2];
                v[1] = t[1] + t[2];
                v[2] = t[2] - t[1];
                v[3] = t[1] - t[3];
            }
#pragma unroll
            for (int kd = 0; kd < 3; ++kd) {
                const float r0 = fmaf(cb, rg[kd][2], ca * rg[kd][0]), r1 = fmaf(cb, rg[kd][3], ca * rg[kd][1]);   // row xi of A dY
                z[kd][0] = r0;            // (A dY A^T)[xi][nu]: r0, r0 + r1, r0 - r1, -r1; the last one's sign is
                z[kd][1] = r0 + r1;       // applied to the reduced sums instead
                z[kd][2] = r0 - r1;
                z[kd][3] = r1;
            }
            if (xi == 1) bsum += z[1][1];   // position (1,1) of A dY A^T = sum of the 2x2 block
            load(q + 1 < 8 ? q + 1 : 7);    // the next step's pixels are on their way while this step's MFMAs issue
#pragma unroll
            for (int kd = 0; kd < 3; ++kd)
#pragma unroll
                for (int nu = 0; nu < 4; ++nu)
                    acc[kd][nu] = __builtin_amdgcn_mfma_f32_32x32x2f32(z[kd][nu], v[nu], acc[kd][nu], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    for (long long item = xr.first; item < xr.end; item += xr.stride) {
        const int by = (int)(item % a.by_n);
        long long rest = item / a.by_n;
        const int bx = (int)(rest % a.bx_n);
        rest /= a.bx_n;
        const int seg = (int)(rest % a.segs_per_col);
        const long long vol = rest / a.segs_per_col;
        const int y0 = 2 * by, x0 = 32 * bx;
        const int tau0 = seg * a.seg_len, tau1 = tau0 + a.seg_len < a.D ? tau0 + a.seg_len : a.D;
        slots_of_run(y0, x0);
        const long long px_plane = (long long)a.H * a.W;
        const float* const vx = a.a + (vol * a.D) * px_plane * a.Ci;   // slice 0 of this volume
        const float* const vg = a.g + (vol * a.D) * px_plane * a.Co;
        auto load_x = [&](int tau, float* dst) {
            fill(tau >= 0 && tau < a.D ? vx + tau * px_plane * a.Ci : nullptr, a.Ci, std::integral_constant<int, 0>{},
                 std::integral_constant<int, k3XLoads>{}, dst);
        };
        auto load_g = [&](int tau, float* dst) {
            fill(tau >= 0 && tau < a.D ? vg + tau * px_plane * a.Co : nullptr, a.Co, std::integral_constant<int, 5>{},
                 std::integral_constant<int, k3GLoads>{}, dst);
        };
        // the previous chunk ended with a barrier: all buffers are free
        load_x(tau0, X0);
        load_g(tau0 + 1, G0);
        load_g(tau0, G1);
        load_g(tau0 - 1, G2);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        int tau = tau0;
        // chunk tau: input in xc, gradients of slices tau + 1, tau, tau - 1 in gp, gz, gm; the next chunk's input goes to
        // xn and the gradient slice tau + 2 to gn (the buffer that held slice tau - 2)
        auto chunk = [&](const float* xc, float* xn, const float* gp, const float* gz, const float* gm, float* gn)
                         __attribute__((always_inline)) {
            if (tau + 1 < tau1) {
                load_x(tau + 1, xn);
                load_g(tau + 2, gn);
            }
            __builtin_amdgcn_sched_barrier(0);
            run(xc, gp, gz, gm);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            ++tau;
        };
        while (true) {
            chunk(X0, X1, G0, G1, G2, G3);
            if (tau >= tau1) break;
            chunk(X1, X0, G3, G0, G1, G2);
            if (tau >= tau1) break;
            chunk(X0, X1, G2, G3, G0, G1);
            if (tau >= tau1) break;
            chunk(X1, X0, G1, G2, G3, G0);
            if (tau >= tau1) break;
        }
    }

#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) {
            const int pos = kd * 16 + 4 * xi + nu;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int co = co0 + 8 * (r >> 2) + 4 * h + (r & 3), ci = ci0 + m;
                pout[((size_t)pos * a.Co + co) * a.Ci + ci] = acc[kd][nu][r];
            }
        }
    if (a.bias_partial && ci0 == 0 && xi == 1) {
        const float tot = bsum + __shfl_xor(bsum, 32);
        if (h == 0) a.bias_partial[(size_t)blockIdx.x * a.Co + co0 + m] = tot;
    }
}

// grad_w[co][kd*9 + tap][ci] = G^T P_kd G from the reduced sums P[kd*16 + pos][co][ci] (column 3 arrives negated)
__global__ __launch_bounds__(256) void wgrad_wino3_finish_kernel(const float* __restrict__ psum, int Co, int Ci, float* __restrict__ gw) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= 3 * Co * Ci) return;
    const int ci = idx % Ci, co = (idx / Ci) % Co, kd = idx / (Ci * Co);
    float P[4][4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const float v = psum[((size_t)(kd * 16 + 4 * x + n) * Co + co) * Ci + ci];
            P[x][n] = n == 3 ? -v : v;
        }
    float gp[3][4];   // G^T P
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        gp[0][n] = P[0][n] + 0.5f * (P[1][n] + P[2][n]);
        gp[1][n] = 0.5f * (P[1][n] - P[2][n]);
        gp[2][n] = 0.5f * (P[1][n] + P[2][n]) + P[3][n];
    }
#pragma unroll
    for (int t = 0; t < 3; ++t) {
        float* o = gw + ((size_t)co * 27 + kd * 9 + t * 3) * Ci + ci;
        o[0] = gp[t][0] + 0.5f * (gp[t][1] + gp[t][2]);
        o[Ci] = 0.5f * (gp[t][1] - gp[t][2]);
        o[2 * Ci] = 0.5f * (gp[t][1] + gp[t][2]) + gp[t][3];
    }
}

bool wgrad_wino3_applies(const PixDims& d, int Ci, int Co) {
    return d.kt == 1 && d.kd == 3 && d.kh == 3 && d.kw == 3 && Ci % 32 == 0 && Co % 32 == 0 &&
           (double)d.H * d.W * (Ci > Co ? Ci : Co) * 4.0 < 2.0e9;   // byte offsets inside a slice: 31 bits
}

// Workgroups along x and the run of slices one of them walks per column: the choice that minimises
// (runs per workgroup) x (run length + the chunk and a half a run's first loads cost).
static void wgrad_wino3_split(const PixDims& d, int* grid_x, int* seg_len, int* segs_per_col) {
    const long long vols = d.Q / ((long long)d.D * d.H * d.W);
    const long long cols = vols * ((d.H + 1) / 2) * ((d.W + 31) / 32);
    const long long cap = 512;   // two workgroups per CU
    double best = 1e300;
    *seg_len = d.D; *segs_per_col = 1;
    for (int n = 1; n <= 64 && n <= d.D; ++n) {
        const int len = (d.D + n - 1) / n;
        const int nseg = (d.D + len - 1) / len;
        const long long items = cols * nseg;
        const long long wgs = items < cap ? items : cap;
        const double cost = (double)((items + wgs - 1) / wgs) * (len + 1.5);
        if (cost < best) { best = cost; *seg_len = len; *segs_per_col = nseg; }
    }
    const long long items = cols * *segs_per_col;
    *grid_x = (int)(((items < cap ? items : cap) + 7) / 8 * 8);
}

int wgrad_wino3_splits(const PixDims& d) {
    int gx, len, n;
    wgrad_wino3_split(d, &gx, &len, &n);
    return gx;
}

size_t wgrad_wino3_partial_floats(const PixDims& d, int Ci, int Co) { return (size_t)(wgrad_wino3_splits(d) + 1) * 48 * Ci * Co; }

hipError_t launch_wgrad_wino3(Wino3WgradArgs a, const PixDims& d, int relu_in, hipStream_t st) {
    int gx;
    wgrad_wino3_split(d, &gx, &a.seg_len, &a.segs_per_col);
    a.D = d.D; a.H = d.H; a.W = d.W;
    a.bx_n = (a.W + 31) / 32;
    a.by_n = (a.H + 1) / 2;
    const long long vols = d.Q / ((long long)d.D * d.H * d.W);
    a.n_items = vols * a.segs_per_col * (long long)a.bx_n * a.by_n;
    dim3 grid((unsigned)gx, (unsigned)((a.Co / 32) * (a.Ci / 32)));
    if (relu_in) hipLaunchKernelGGL((wgrad_wino3_kernel<true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((wgrad_wino3_kernel<false>), grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t wgrad_wino3_finish(const float* psum, int Co, int Ci, float* grad_w, hipStream_t st) {
    hipLaunchKernelGGL(wgrad_wino3_finish_kernel, dim3((unsigned)((3 * Co * Ci + 255) / 256)), dim3(256), 0, st, psum, Co, Ci, grad_w);
    return hipGetLastError();
}

bool conv_wino3_applies(const PixDims& d, int K, int Nn) {
    return d.kt == 1 && d.kd == 3 && d.kh == 3 && d.kw == 3 && K % 32 == 0 && Nn % 32 == 0 &&
           40.0 * d.W * K < 2.0e9;   // 32-bit lane byte offsets within the ten rows of a region
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
    const bool epi = a.mask_ref || a.add;
    if (relu_in) {
        if (epi) hipLaunchKernelGGL((conv_wino3_kernel<true, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((conv_wino3_kernel<true, false>), grid, dim3(256), 0, st, a);
    } else {
        if (epi) hipLaunchKernelGGL((conv_wino3_kernel<false, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((conv_wino3_kernel<false, false>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace gleam
