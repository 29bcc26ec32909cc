// 3x3 convolution (forward and data gradient, float32) by the Winograd minimal-filtering algorithm
// F(2x2, 3x3) of Lavin & Gray on gfx950: every 2x2 block of outputs comes from 16 multiplications per
// (input channel, output channel) pair instead of 36, and the 16 element-wise products over all channels
// are 16 independent matrix products that run on the matrix cores:
//     Y = A^T [ sum_k (G g_k G^T) .* (B^T d_k B) ] A
// with d the 4x4 input patch around the 2x2 output block, g the 3x3 kernel, and the constant matrices
//     B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1],  G = [1 0 0; .5 .5 .5; .5 -.5 .5; 0 0 1],
//     A^T = [1 1 1 0; 0 1 -1 -1].
// Everything is fused: the transformed input never exists in memory.
//
// Work split.  A workgroup of 4 waves owns 4 x 32 output pixels (2 x 16 blocks of 2x2, "tiles") and 64 output
// channels; two workgroups share a CU (LDS and registers allow exactly that), so the output transform of one
// overlaps the matrix work of the other.  Wave xi owns row xi of the 4x4 product grid (positions (xi, nu),
// nu = 0..3): 4 positions x (32 tiles x 64 channels) = 8 MFMA accumulators of 32x32.  A wave thus needs only
// row xi of B^T d: two of the four input rows, which it reads from the LDS copy of the raw input region
// (6 x 34 pixels x 8 channels per chunk, filled by direct global->LDS loads, zero outside the image), turns
// into its four B operands with 8 additions per channel, and multiplies with the transformed weights U (also
// staged by direct loads).  After the last channel chunk the 16 products of a tile are spread over the four
// waves; they are combined through LDS (A^T . A) and stored with the usual fused epilogue (bias, ReLU, ReLU
// mask, skip / gradient add).  Workgroups are persistent and fetch the first chunk of their next block under
// the last MFMAs of the current one.
#include <type_traits>

#include "prox_common.h"

namespace gleam {

namespace {

constexpr int kWRawSlots = 448;    // 6 rows x 2 channel quads x 34 columns = 408 quads, rounded up to whole wave loads
constexpr int kWUSlots = 2048;     // 16 positions x 64 output channels x 2 channel quads
constexpr int kWBufFloats = (kWRawSlots + kWUSlots) * 4;
constexpr int kWExFloats = 4 * 2 * 32 * 8 * 4;   // per pass: 4 waves x 2 output columns x 32 tiles x 8 channel quads
static_assert(kWExFloats <= kWBufFloats, "the exchange reuses a chunk buffer");
// Exchange element (wave, column jj, tile, quad cq): the quad index is XOR-ed with bits of the tile index so that
// both the writers (16 lanes = 16 tiles, one quad) and the readers (16 lanes = 2 tiles x 8 quads) touch 16
// different 16-byte bank groups: LDS serves 128-bit accesses 16 lanes at a time out of 64 banks.
__device__ __forceinline__ int ex_off(int wave, int jj, int tile, int cq) {
    return ((((wave * 2 + jj) * 32 + tile) * 8) + (cq ^ ((tile >> 1) & 7))) * 4;
}

__device__ __forceinline__ void dma16(const float* g, float* l) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)l, 16, 0, 0);
}

// uniform base + per-lane unsigned byte offset: the form the compiler turns into a scalar-base direct load
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

template <bool RELU, bool EPI>   // EPI: the call has a ReLU mask (source tensor or sign words) or a tensor to add
__global__ __launch_bounds__(256, 2) void conv_wino_kernel(WinoArgs a) {
    // Separate LDS objects: reads of one chunk buffer then do not wait for direct loads into the other.
    __shared__ __attribute__((aligned(16))) float bufA[kWBufFloats];
    __shared__ __attribute__((aligned(16))) float bufB[kWBufFloats];
    float* const ex = bufB;   // the exchange of the output transform reuses the second chunk buffer
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, h = lane >> 5, xi = wave;
    const int trl = m >> 4, tc = m & 15;

    // Persistent workgroups, XCD-aware order: each XCD owns a contiguous eighth of the blocks (neighbours share
    // halo rows in its L2) and its workgroups walk that range with a fixed stride.
    const XcdRange xr = xcd_range(a.n_blocks);
    const int ny = blockIdx.y, n0 = ny * 64;
    const int n_kc = a.K / 8;

    // Direct-load sources of this lane: two quads of the raw region (a zero quad outside the image) and four
    // of U.  The position of a quad inside the region does not depend on the block.
    int s_row[2], s_col[2], s_quad[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int s = tid + i * 256;
        // slot = ((row*2 + column parity)*17 + column/2)*2 + quad: the two quads of a pixel are neighbouring lanes
        // (one 32-byte request), even columns before odd ones
        const int rp = s / 34, rem = s - rp * 34;
        s_col[i] = 2 * (rem >> 1) + (rp & 1);
        s_row[i] = s < 408 ? (rp >> 1) : -100000;            // slots past the region always read the zero quad
        s_quad[i] = rem & 1;
    }
    struct Block {
        int x0, y0;
        long long img;
        const float* gp[2];
        int gstep[2];
    };
    auto setup = [&](long long item) {
        Block b;
        const int bx = (int)(item % a.bx_n);
        const long long rest = item / a.bx_n;
        const int by = (int)(rest % a.by_n);
        b.img = rest / a.by_n;
        b.x0 = bx * 32;
        b.y0 = by * 4;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int yy = b.y0 - 1 + s_row[i], xx = b.x0 - 1 + s_col[i];
            const bool ok = yy >= 0 && yy < a.H && xx >= 0 && xx < a.W;
            b.gp[i] = ok ? a.in + ((b.img * a.H + yy) * a.W + xx) * a.K + s_quad[i] * 4 : a.zero;
            b.gstep[i] = ok ? 8 : 0;
        }
        return b;
    };
    const float* ubase = a.u + (size_t)ny * n_kc * (kWUSlots * 4);   // uniform; lanes add a 32-bit offset
    const unsigned uoff = 16u * (unsigned)tid;   // bytes

    auto issue = [&](const Block& b, int kc, float* dst) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int o = wave + i * 4;
            if (o < kWRawSlots / 64) dma16(b.gp[i] + kc * b.gstep[i], dst + o * 256);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int o = wave + i * 4;
            const float* ub = ubase + ((size_t)kc * (kWUSlots * 4) + 1024 * i);   // scalar address
            dma16_off(ub, uoff, dst + kWRawSlots * 4 + o * 256);
        }
    };

    // row xi of B^T: d[ra] + sg * d[rb]
    const int ra = xi == 0 ? 0 : (xi == 2 ? 2 : 1);
    const int rb = xi == 3 ? 3 : (xi == 2 ? 1 : 2);
    const float sg = xi == 1 ? 1.f : -1.f;
    // Region quad (row, channel quad, column) sits at slot (row*2 + quad)*34 + (column & 1)*17 + column/2: the 16
    // tiles of a row then read 16 neighbouring slots for each of their four columns (no bank conflicts).
    const int offA = (((2 * trl + ra) * 2) * 17 + tc) * 8 + 4 * h;
    const int offB = (((2 * trl + rb) * 2) * 17 + tc) * 8 + 4 * h;
    // U quad (position, channel quad hq, output channel n) at slot ((pos*2 + hq)*64 + n)
    const int offU = kWRawSlots * 4 + (((xi * 4) * 2 + h) * 64 + m) * 4;

    floatx16 acc[4][2];

    auto compute = [&](const float* buf, auto first_c) {
        constexpr bool FIRST = decltype(first_c)::value;   // first chunk of a block: accumulators start from zero
        float4 t[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float4 da = *reinterpret_cast<const float4*>(buf + offA + ((c & 1) * 17 + (c >> 1)) * 8);
            float4 db = *reinterpret_cast<const float4*>(buf + offB + ((c & 1) * 17 + (c >> 1)) * 8);
            if (RELU) {
                da = relu4(da);
                db = relu4(db);
            }
            t[c] = fma4(sg, db, da);
        }
        float4 v[4];
        v[0] = sub4(t[0], t[2]);
        v[1] = add4(t[1], t[2]);
        v[2] = sub4(t[2], t[1]);
        v[3] = sub4(t[1], t[3]);
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) {
            const float4 u0 = *reinterpret_cast<const float4*>(buf + offU + (nu * 2 * 64) * 4);
            const float4 u1 = *reinterpret_cast<const float4*>(buf + offU + (nu * 2 * 64 + 32) * 4);
            if (FIRST) {
                floatx16 z;
#pragma unroll
                for (int r = 0; r < 16; ++r) z[r] = 0.f;
                acc[nu][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(u0.x, v[nu].x, z, 0, 0, 0);
                acc[nu][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(u1.x, v[nu].x, z, 0, 0, 0);
            } else {
                acc[nu][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(u0.x, v[nu].x, acc[nu][0], 0, 0, 0);
                acc[nu][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(u1.x, v[nu].x, acc[nu][1], 0, 0, 0);
            }
            acc[nu][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(u0.y, v[nu].y, acc[nu][0], 0, 0, 0);
            acc[nu][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(u1.y, v[nu].y, acc[nu][1], 0, 0, 0);
            acc[nu][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(u0.z, v[nu].z, acc[nu][0], 0, 0, 0);
            acc[nu][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(u1.z, v[nu].z, acc[nu][1], 0, 0, 0);
            acc[nu][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(u0.w, v[nu].w, acc[nu][0], 0, 0, 0);
            acc[nu][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(u1.w, v[nu].w, acc[nu][1], 0, 0, 0);
        }
    };

    if (xr.first >= xr.end) return;   // uniform for the workgroup
    Block cur = setup(xr.first);
    issue(cur, 0, bufA);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    const int tid_b = tid;
    float4 bias_r[2];
#pragma unroll
    for (int jp = 0; jp < 2; ++jp)
        bias_r[jp] = a.bias ? *reinterpret_cast<const float4*>(a.bias + n0 + 32 * jp + 4 * (tid_b & 7)) : make_float4(0.f, 0.f, 0.f, 0.f);
    for (long long item = xr.first; item < xr.end; item += xr.stride) {
    const bool has_next = item + xr.stride < xr.end;
    const Block nxt = setup(has_next ? item + xr.stride : item);
    const int x0 = cur.x0, y0 = cur.y0;
    const long long img = cur.img;
    // n_kc is even (K is a multiple of 16): chunks alternate between the two buffers
    issue(cur, 1, bufB);
    __builtin_amdgcn_sched_barrier(0);   // keep the direct loads ahead of the MFMAs they overlap with
    compute(bufA, std::true_type{});
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int kc = 1; kc < n_kc; kc += 2) {
        // the first chunk of the next block is fetched under the last MFMAs of this one
        if (kc + 1 < n_kc) issue(cur, kc + 1, bufA);
        else if (has_next) issue(nxt, 0, bufA);
        __builtin_amdgcn_sched_barrier(0);
        compute(bufB, std::false_type{});
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (kc + 1 >= n_kc) break;
        issue(cur, kc + 2, bufB);
        __builtin_amdgcn_sched_barrier(0);
        compute(bufA, std::false_type{});
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }

    // Output transform.  In registers over nu: R_0 = M_0 + M_1 + M_2, R_1 = M_1 - M_2 - M_3; across the four
    // waves of a tile-row pair through LDS: Y_0 = R[xi=0] + R[1] + R[2], Y_1 = R[1] - R[2] - R[3].
    // One pass per 32 output channels.  A thread finishes the 2x2 pixels of one tile for one channel quad; what
    // the fused epilogue reads from memory (ReLU mask source, tensor to add) is requested for all four pixels
    // before the exchange, from a clamped address where the pixel is outside the image.
    const int e_cq = tid_b & 7, e_tile = (tid_b >> 3) & 31;
    const int ey = y0 + 2 * (e_tile >> 4), ex_ = x0 + 2 * (e_tile & 15);
    bool okp[2][2];
    long long op[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            okp[i][jj] = ey + i < a.H && ex_ + jj < a.W;
            op[i][jj] = okp[i][jj] ? ((img * a.H + ey + i) * a.W + ex_ + jj) * a.Nn + n0 + 4 * e_cq : (long long)(n0 + 4 * e_cq);
        }
    // ReLU mask as sign bits: bit 16*jp + 4*(2*i + jj) + e of this thread's word says whether the value of pass jp,
    // tile pixel (i, jj), channel e of its quad is positive.  The forward launch that produces an activation
    // writes the words, the data-gradient launch into the same tensor (same geometry, hence the same thread for
    // the same values) reads them instead of the activation itself.
    const long long word_idx = ((long long)ny * a.n_blocks + item) * 256 + tid_b;
    unsigned sign_in = 0u, sign_out = 0u;
    if constexpr (EPI) {
        if (a.bits_in) sign_in = a.bits_in[word_idx];
    }
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
        if (jp) __syncthreads();
        float4 refv[2][2], addv[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                refv[i][jj] = make_float4(1.f, 1.f, 1.f, 1.f);
                addv[i][jj] = make_float4(0.f, 0.f, 0.f, 0.f);
                if constexpr (EPI) {
                    if (a.mask_ref && !a.bits_in) refv[i][jj] = *reinterpret_cast<const float4*>(a.mask_ref + op[i][jj] + 32 * jp);
                    if (a.add) addv[i][jj] = *reinterpret_cast<const float4*>(a.add + op[i][jj] + 32 * jp);
                }
            }
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            float r0[4], r1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float m0 = acc[0][jp][4 * rg + i], m1 = acc[1][jp][4 * rg + i];
                const float m2 = acc[2][jp][4 * rg + i], m3 = acc[3][jp][4 * rg + i];
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
                float v[4] = {yv.x + bias_r[jp].x, yv.y + bias_r[jp].y, yv.z + bias_r[jp].z, yv.w + bias_r[jp].w};
                if (a.relu_out) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
                }
                const float rr[4] = {refv[i][jj].x, refv[i][jj].y, refv[i][jj].z, refv[i][jj].w};
                const float aa[4] = {addv[i][jj].x, addv[i][jj].y, addv[i][jj].z, addv[i][jj].w};
                const int bit0 = 16 * jp + 4 * (2 * i + jj);
                if constexpr (EPI) {
                    bool pos[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) pos[e] = a.bits_in ? ((sign_in >> (bit0 + e)) & 1u) != 0u : rr[e] > 0.f;
                    if (a.mask_acc) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = pos[e] ? v[e] : 0.f;
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += (a.mask_add && !pos[e]) ? 0.f : aa[e];
                }
                if (a.bits_out) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) sign_out |= (v[e] > 0.f ? 1u : 0u) << (bit0 + e);
                }
                if (okp[i][jj]) *reinterpret_cast<float4*>(a.out + op[i][jj] + 32 * jp) = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    }
    if (a.bits_out) a.bits_out[word_idx] = sign_out;
    __syncthreads();   // the exchange lived in the second chunk buffer, which the next block loads into first
    cur = nxt;
    }
}

// U = G g G^T for every (output channel n, input channel k), laid out as the kernel's LDS image:
// u[((((ny*n_kc + kc)*16 + pos)*2 + hq)*64 + nn)*4 + kk], n = 64*ny + nn, k = 8*kc + 4*hq + kk, pos = 4*xi + nu; one zero
// quad follows.  Source weight (n, tap, k) at w[n*sn + tapidx*st + k*sk], taps mirrored for the data gradient.
__global__ __launch_bounds__(256) void wino_weights_kernel(WinoWeightBatch b) {
    const WinoWeightJob& jb = b.job[blockIdx.y];
    const float* __restrict__ w = jb.w;
    float* __restrict__ u = jb.u;
    const long long sn = jb.sn, st_ = jb.st, sk = jb.sk;
    const int flip = jb.flip, K = jb.K, Nn = jb.Nn;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx == 0) {
        float* z = u + (size_t)16 * K * Nn;
        z[0] = z[1] = z[2] = z[3] = 0.f;
    }
    if (idx >= K * Nn) return;
    const int k = idx % K, n = idx / K;
    float g[3][3];
#pragma unroll
    for (int t = 0; t < 9; ++t) g[t / 3][t % 3] = w[n * sn + (flip ? 8 - t : t) * st_ + k * sk];
    float gg[4][3];   // G g
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        gg[0][b] = g[0][b];
        gg[1][b] = 0.5f * (g[0][b] + g[1][b] + g[2][b]);
        gg[2][b] = 0.5f * (g[0][b] - g[1][b] + g[2][b]);
        gg[3][b] = g[2][b];
    }
    const int ny = n / 64, nn = n % 64, kc = k / 8, hq = (k % 8) / 4, kk = k % 4, n_kc = K / 8;
    float* dst = u + ((((size_t)(ny * n_kc + kc) * 16) * 2 + hq) * 64 + nn) * 4 + kk;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const float uu[4] = {gg[x][0], 0.5f * (gg[x][0] + gg[x][1] + gg[x][2]), 0.5f * (gg[x][0] - gg[x][1] + gg[x][2]), gg[x][2]};
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) dst[(size_t)(4 * x + nu) * 2 * 64 * 4] = uu[nu];
    }
}

// ------------------------------------------------------------------ weight gradient
// dL/dg = G^T [ sum over tiles of (A dY A^T) .* (B^T d B) ] G: per position of the 4x4 grid a
// [cout x tiles] . [tiles x cin] matrix product.  A workgroup of 8 waves keeps all 16 products of a 64 x 64
// channel block in registers (wave = row xi of the grid x one of the two 32-channel input blocks: 4 positions
// x 64 x 32 = 8 accumulators of 32x32), walks chunks of 16 tiles (2 x 32
// output pixels: the raw gradient rows and the raw input rows with halo are staged in LDS by direct loads,
// all channels, double-buffered) and forms both MFMA operands on the fly: a lane holds one channel and one
// of the two tiles of an MFMA's contraction step, reads the few pixels its position needs (4-byte LDS reads,
// lanes = consecutive channels; the two lane halves are kept on different banks by an XOR of the channel
// index with a pixel bit) and combines them with 2-3 additions.  Persistent split over the image: every
// workgroup writes its partial sums once; a fixed-order reduction and G^T . G follow.
constexpr int kGDPix = 4 * 34, kGGPix = 2 * 32;          // staged pixels per chunk: input rows with halo, gradient rows
constexpr int kGBufFloats = (kGDPix + kGGPix) * 64;
constexpr int kGWaveLoads = (kGDPix + kGGPix) * 16 / 64;   // 50 wave-wide direct loads per chunk

template <bool RELU>
__global__ __launch_bounds__(512) void wgrad_wino_kernel(WinoWgradArgs a) {
    __shared__ __attribute__((aligned(16))) float bufs[2 * kGBufFloats];   // two chunk buffers
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int xi = wave >> 1, ji = wave & 1;   // wave = row of the product grid x 32-channel input block
    const int m = lane & 31, h = lane >> 5;
    const int nci = a.Ci / 64;
    const int co0 = 64 * ((int)blockIdx.y / nci), ci0 = 64 * ((int)blockIdx.y % nci);
    const XcdRange xr = xcd_range(a.n_chunks);
    if (xr.first >= xr.end) {   // nothing to do: the partial of this workgroup is zero
        for (int i = tid; i < 16 * 64 * 64; i += 512) {
            const int pos = i >> 12, co = (i >> 6) & 63, ci = i & 63;
            a.partial[(((size_t)blockIdx.x * 16 + pos) * a.Co + co0 + co) * a.Ci + ci0 + ci] = 0.f;
        }
        if (a.bias_partial && ci0 == 0 && tid < 64) a.bias_partial[(size_t)blockIdx.x * a.Co + co0 + tid] = 0.f;
        return;
    }

    // direct-load slots of this lane (7 x 512 >= 3200 quads): byte offset from the chunk origin and position
    constexpr int NS = 7;
    unsigned s_off[NS];
    int s_rc[NS];   // (row + 1) << 8 | (column + 1), relative to the first output pixel of the chunk
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int s = tid + 512 * i;
        if (s < kGDPix * 16) {
            const int px = s >> 4, qd = (s & 15) ^ (8 * ((px >> 1) & 1));
            const int row = px / 34, col = px - row * 34;
            s_rc[i] = (row << 8) | col;
            s_off[i] = 4u * (unsigned)((row * a.W + col) * a.Ci + 4 * qd);
        } else {
            const int s2 = s - kGDPix * 16;
            const int px = s2 >> 4, qd = (s2 & 15) ^ (8 * ((px >> 1) & 1));
            const int row = px >> 5, col = px & 31;
            s_rc[i] = ((row + 1) << 8) | (col + 1);
            s_off[i] = 4u * (unsigned)((row * a.W + col) * a.Co + 4 * qd);
        }
    }
    // slots 0..2175 belong to the input region, the rest to the gradient region: slot = tid + 512*i
    auto is_g = [&](int i) { return i > 4 || (i == 4 && tid >= kGDPix * 16 - 4 * 512); };
    auto issue = [&](long long item, float* dst) {
        const int bx = (int)(item % a.bx_n);
        const long long rest = item / a.bx_n;
        const int by = (int)(rest % a.by_n);
        const long long img = rest / a.by_n;
        const int x0 = 32 * bx, y0 = 2 * by;
        const float* od = a.a + ((img * a.H + y0 - 1) * a.W + x0 - 1) * a.Ci + ci0;   // uniform; never read outside the tensor
        const float* og = a.g + ((img * a.H + y0) * a.W + x0) * a.Co + co0;
        const bool interior = y0 >= 1 && y0 + 2 < a.H && x0 >= 1 && x0 + 32 < a.W;    // uniform
        if (interior) {
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const int o = wave + 8 * i;
                if (o < kGWaveLoads) {
                    if (i < 4) dma16_off(od, s_off[i], dst + o * 256);
                    else if (i > 4) dma16_off(og, s_off[i], dst + o * 256);
                    else dma16(reinterpret_cast<const float*>(reinterpret_cast<const char*>(is_g(i) ? og : od) + s_off[i]), dst + o * 256);
                }
            }
        } else {
            // a chunk at the image border: through buffer resources that span the image, with an offset outside of it for
            // the lanes whose pixel lies outside - those arrive as zeros with the data (LDS stores of zeros into the
            // buffer would have to wait for the direct loads in flight into it)
            const long long img_px = (long long)a.H * a.W;
            const __amdgpu_buffer_rsrc_t r_d = __builtin_amdgcn_make_buffer_rsrc((void*)(a.a + img * img_px * a.Ci), 0, (unsigned)(img_px * a.Ci * 4), 0x00020000);
            const __amdgpu_buffer_rsrc_t r_g = __builtin_amdgcn_make_buffer_rsrc((void*)(a.g + img * img_px * a.Co), 0, (unsigned)(img_px * a.Co * 4), 0x00020000);
            const unsigned od_off = (unsigned)((((y0 - 1) * a.W + x0 - 1) * a.Ci + ci0) * 4);   // (wraps for the row above the image)
            const unsigned og_off = (unsigned)(((y0 * a.W + x0) * a.Co + co0) * 4);
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const int o = wave + 8 * i;
                if (o < kGWaveLoads) {
                    const int yy = y0 - 1 + (s_rc[i] >> 8), xx = x0 - 1 + (s_rc[i] & 255);
                    const bool ok = yy >= 0 && yy < a.H && xx >= 0 && xx < a.W;
                    const bool g = i > 4 || (i == 4 && wave >= 2);   // uniform: slot 4 is an input slot for tid < 128
                    const unsigned voff = ok ? (g ? og_off : od_off) + s_off[i] : 0x80000000u;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(g ? r_g : r_d, (__attribute__((address_space(3))) void*)(dst + o * 256), 16, voff, 0, 0, 0);
                }
            }
        }
    };

    // row xi of A dY (coefficients of the two gradient rows) and of B^T d (two of the four input rows)
    const float ca = xi == 3 ? 0.f : 1.f, cb = xi == 0 ? 0.f : (xi == 1 ? 1.f : -1.f);
    const int ra = xi == 0 ? 0 : (xi == 2 ? 2 : 1), rb = xi == 3 ? 3 : (xi == 2 ? 1 : 2);
    const float sg = xi == 1 ? 1.f : -1.f;
    // LDS float offsets of this lane inside a chunk buffer: element (pixel, channel) sits at
    // pixel*64 + (channel ^ 32*((pixel>>1)&1))
    int db[2][2];   // input channel 32*ji + m: [row a/b][(column>>1)&1]
#pragma unroll
    for (int rs = 0; rs < 2; ++rs)
#pragma unroll
        for (int cp = 0; cp < 2; ++cp) {
            const int r = rs ? rb : ra;
            db[rs][cp] = (r * 34 + 2 * h) * 64 + m + 32 * (ji ^ ((r + h + cp) & 1));
        }
    int gb[2];      // output channels m and 32 + m
#pragma unroll
    for (int jo = 0; jo < 2; ++jo) gb[jo] = kGDPix * 64 + (2 * h) * 64 + m + 32 * (jo ^ h);

    floatx16 acc[4][2];   // [column nu of the product grid][cout block]
#pragma unroll
    for (int nu = 0; nu < 4; ++nu)
#pragma unroll
        for (int jo = 0; jo < 2; ++jo)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nu][jo][r] = 0.f;
    float bsum[2] = {0.f, 0.f};

    // One chunk: 8 contraction steps (tiles 2q and 2q+1 on the two lane halves), 8 MFMAs each.  One copy of the
    // code serves both chunk buffers (the buffer is a uniform offset added to six lane addresses per chunk); a
    // scheduling fence per step bounds how far the compiler may pull LDS reads forward.
    auto run = [&](int boff) {
        const float* const pd00 = bufs + boff + db[0][0];
        const float* const pd01 = bufs + boff + db[0][1];
        const float* const pd10 = bufs + boff + db[1][0];
        const float* const pd11 = bufs + boff + db[1][1];
        const float* const pg0 = bufs + boff + gb[0];
        const float* const pg1 = bufs + boff + gb[1];
        float rg[2][4], rd[2][4];   // raw pixels of one step: gradient [cout block][row*2 + column], input [row a/b][column]
        auto load = [&](int q) {
#pragma unroll
            for (int jo = 0; jo < 2; ++jo) {
                const float* pg = jo ? pg1 : pg0;
                rg[jo][0] = pg[(4 * q) * 64];
                rg[jo][1] = pg[(4 * q + 1) * 64];
                rg[jo][2] = pg[(32 + 4 * q) * 64];
                rg[jo][3] = pg[(32 + 4 * q + 1) * 64];
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                rd[0][c] = ((c >> 1) & 1 ? pd01 : pd00)[(4 * q + c) * 64];
                rd[1][c] = ((c >> 1) & 1 ? pd11 : pd10)[(4 * q + c) * 64];
            }
        };
        load(0);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float z[4][2], v[4];
#pragma unroll
            for (int jo = 0; jo < 2; ++jo) {
                const float r0 = fmaf(cb, rg[jo][2], ca * rg[jo][0]), r1 = fmaf(cb, rg[jo][3], ca * rg[jo][1]);   // row xi of A dY
                z[0][jo] = r0;                // (A dY A^T)[xi][nu]: r0, r0 + r1, r0 - r1, -r1
                z[1][jo] = r0 + r1;
                z[2][jo] = r0 - r1;
                z[3][jo] = -r1;
            }
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
            if (xi == 1) { bsum[0] += z[1][0]; bsum[1] += z[1][1]; }   // position (1,1) of A dY A^T = sum of the 2x2 block
            if (q + 1 < 8) load(q + 1);      // the next step's pixels are on their way while this step's MFMAs issue
#pragma unroll
            for (int nu = 0; nu < 4; ++nu)
#pragma unroll
                for (int jo = 0; jo < 2; ++jo)
                    acc[nu][jo] = __builtin_amdgcn_mfma_f32_32x32x2f32(z[nu][jo], v[nu], acc[nu][jo], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    issue(xr.first, bufs);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    int cur = 0;
    for (long long item = xr.first; item < xr.end; item += xr.stride) {
        if (item + xr.stride < xr.end) issue(item + xr.stride, bufs + (cur ^ 1) * kGBufFloats);
        __builtin_amdgcn_sched_barrier(0);
        run(cur * kGBufFloats);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        cur ^= 1;
    }

#pragma unroll
    for (int nu = 0; nu < 4; ++nu) {
        const int pos = 4 * xi + nu;
#pragma unroll
        for (int jo = 0; jo < 2; ++jo)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int co = co0 + 32 * jo + 8 * (r >> 2) + 4 * h + (r & 3), ci = ci0 + 32 * ji + m;
                a.partial[(((size_t)blockIdx.x * 16 + pos) * a.Co + co) * a.Ci + ci] = acc[nu][jo][r];
            }
    }
    if (a.bias_partial && ci0 == 0 && xi == 1 && ji == 0) {
#pragma unroll
        for (int jo = 0; jo < 2; ++jo) {
            const float tot = bsum[jo] + __shfl_xor(bsum[jo], 32);
            if (h == 0) a.bias_partial[(size_t)blockIdx.x * a.Co + co0 + 32 * jo + m] = tot;
        }
    }
}

// grad_w[co][tap][ci] = G^T P G from the reduced sums P[pos][co][ci]
__global__ __launch_bounds__(256) void wgrad_wino_finish_kernel(const float* __restrict__ psum, int Co, int Ci, float* __restrict__ gw) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= Co * Ci) return;
    const int ci = idx % Ci, co = idx / Ci;
    float P[4][4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int n = 0; n < 4; ++n) P[x][n] = psum[((size_t)(4 * x + n) * Co + co) * Ci + ci];
    float gp[3][4];   // G^T P
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        gp[0][n] = P[0][n] + 0.5f * (P[1][n] + P[2][n]);
        gp[1][n] = 0.5f * (P[1][n] - P[2][n]);
        gp[2][n] = 0.5f * (P[1][n] + P[2][n]) + P[3][n];
    }
#pragma unroll
    for (int t = 0; t < 3; ++t) {
        float* o = gw + ((size_t)co * 9 + t * 3) * Ci + ci;
        o[0] = gp[t][0] + 0.5f * (gp[t][1] + gp[t][2]);
        o[Ci] = 0.5f * (gp[t][1] - gp[t][2]);
        o[2 * Ci] = 0.5f * (gp[t][1] + gp[t][2]) + gp[t][3];
    }
}

bool wgrad_wino_applies(const PixDims& d, int Ci, int Co) {
    return d.kt == 1 && d.kd == 1 && d.kh == 3 && d.kw == 3 && Ci % 64 == 0 && Co % 64 == 0 &&
           4.0 * d.W * (Ci > Co ? Ci : Co) < 5.0e8 &&   // 32-bit lane byte offsets within four image rows
           4.0 * d.H * d.W * (Ci > Co ? Ci : Co) < 2.0e9;   // ... and within an image (chunks at the border)
}

size_t wgrad_wino_partial_floats(int Ci, int Co, int n_split) { return (size_t)(n_split + 1) * 16 * Ci * Co; }

hipError_t launch_wgrad_wino(WinoWgradArgs a, int relu_in, int n_split, hipStream_t st) {
    a.bx_n = (a.W + 31) / 32;
    a.by_n = (a.H + 1) / 2;
    a.n_chunks = a.NI * (long long)a.bx_n * a.by_n;
    dim3 grid((unsigned)n_split, (unsigned)((a.Co / 64) * (a.Ci / 64)));
    if (relu_in) hipLaunchKernelGGL((wgrad_wino_kernel<true>), grid, dim3(512), 0, st, a);
    else hipLaunchKernelGGL((wgrad_wino_kernel<false>), grid, dim3(512), 0, st, a);
    return hipGetLastError();
}

hipError_t wgrad_wino_finish(const float* psum, int Co, int Ci, float* grad_w, hipStream_t st) {
    hipLaunchKernelGGL(wgrad_wino_finish_kernel, dim3((unsigned)((Co * Ci + 255) / 256)), dim3(256), 0, st, psum, Co, Ci, grad_w);
    return hipGetLastError();
}

bool conv_wino_applies(const PixDims& d, int K, int Nn) {
    return d.kt == 1 && d.kd == 1 && d.kh == 3 && d.kw == 3 && K % 16 == 0 && Nn % 64 == 0;
}

size_t conv_wino_weight_floats(int K, int Nn) { return (size_t)16 * K * Nn + 4; }

size_t conv_wino_sign_words(const PixDims& d, int Nn) {   // one word per thread, block and group of 64 channels
    const size_t n_img = (size_t)d.Q / ((size_t)d.H * d.W);
    return n_img * ((d.W + 31) / 32) * ((d.H + 3) / 4) * 256 * (size_t)(Nn / 64);
}

hipError_t wino_weights_batch(const WinoWeightBatch& b, hipStream_t st) {
    if (b.n < 1) return hipSuccess;
    int most = 0;
    double bytes = 0.0;
    for (int i = 0; i < b.n; ++i) {
        const int kn = b.job[i].K * b.job[i].Nn;
        most = kn > most ? kn : most;
        bytes += 4.0 * (9 + 16) * kn;
    }
    KernelScope ks("weights_image", 0.0, bytes, st);
    hipLaunchKernelGGL(wino_weights_kernel, dim3((unsigned)((most + 255) / 256), (unsigned)b.n), dim3(256), 0, st, b);
    return hipGetLastError();
}

hipError_t launch_conv_wino(WinoArgs a, const float* w, long long sn, long long st_, long long sk, int flip, int relu_in,
                            float* u_scratch, const float* u_ready, const char* name, hipStream_t st) {
    if (!u_ready) {
        WinoWeightBatch one{};
        one.n = 1;
        one.job[0] = WinoWeightJob{w, sn, st_, sk, flip, a.K, a.Nn, u_scratch};
        const hipError_t e = wino_weights_batch(one, st);
        if (e != hipSuccess) return e;
        u_ready = u_scratch;
    }
    a.u = u_ready;
    a.zero = u_ready + (size_t)16 * a.K * a.Nn;
    a.bx_n = (a.W + 31) / 32;
    a.by_n = (a.H + 3) / 4;
    a.n_blocks = a.NI * (long long)a.bx_n * a.by_n;
    const long long cap = 512 / (a.Nn / 64) > 8 ? 512 / (a.Nn / 64) : 8;   // two workgroups per CU in total
    const long long gx = ((a.n_blocks < cap ? a.n_blocks : cap) + 7) / 8 * 8;
    dim3 grid((unsigned)gx, (unsigned)(a.Nn / 64));
    const double Q = (double)a.NI * a.H * a.W;
    // F(2x2, 3x3): 16 multiplications per 2x2 outputs and channel pair on the matrix cores instead of the 36 of the definition
    KernelScope ks(name, 2.0 * Q * a.K * a.Nn * 9, 4.0 * Q * (a.K + a.Nn), st, 2.0 * Q * a.K * a.Nn * 4);
    const bool epi = a.mask_ref || a.add || a.bits_in;
    if (relu_in) {
        if (epi) hipLaunchKernelGGL((conv_wino_kernel<true, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((conv_wino_kernel<true, false>), grid, dim3(256), 0, st, a);
    } else {
        if (epi) hipLaunchKernelGGL((conv_wino_kernel<false, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((conv_wino_kernel<false, false>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace gleam
