// Prox CNN f_theta (Eq. 4-5) forward, local loss (Eq. 10) and the module-confined backward pass
// (Alg. 1, gradient step) on gfx950, float32 with the 32x32x2 fp32 MFMA.
//
// Activations are channels-last [pixels][channels] with pixels flattened over (B,T,D,H,W); a complex
// image is its own 2-channel activation.  Convolutions are implicit GEMMs:
//   conv_mfma_kernel : out[q][n] = sum_{tap,k} in[q + off(tap)][k] * w(n, tap, k)
//                      forward (n = cout, k = cin) and data gradient (n = cin, k = cout, taps flipped)
//                      share it; bias / ReLU / ReLU-mask / residual add are fused into the store.
//   wgrad_mfma_kernel: dw[co][tap][ci] = sum_q g[q][co] * a[q + off(tap)][ci], split over pixel chunks,
//                      partial sums reduced in a fixed order (deterministic).
// Zero padding is a per-pixel 32-bit tap-validity mask, so pixel tiles are plain runs of the flattened
// index and never ragged except at the very end of the tensor.
// 3x3 layers in the plane whose channel counts are multiples of 64 take the Winograd F(2x2, 3x3) kernels of
// prox_wino.hip instead (forward, data gradient and weight gradient); this file keeps the direct kernels for
// every other shape, the two-channel first / last layers, the loss, the reductions and the host side.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <type_traits>

#include "prox_common.h"

namespace gleam {

// ------------------------------------------------------------------ forward / data-gradient conv
struct ConvArgs {
    const float* in;        // [Q][K]
    float* out;             // [Q][Nn]
    const float* wt;        // weights re-laid as LDS images, see weights_image_kernel
    const float* bias;      // [Nn] or null
    const float* mask_ref;  // [Q][Nn] or null: ReLU mask source (value > 0 passes)
    const float* add;       // [Q][Nn] or null: added to the result
    const unsigned* bits_in;   // Winograd launches only, or null: sign words that stand in for mask_ref
    unsigned* bits_out;        // Winograd launches only, or null: sign words of the output
    int K, Nn;              // input / output channels of this GEMM
    int flip;               // 1: data gradient (only used for naming)
    int relu_in, relu_out, mask_acc, mask_add;
    PixDims d;
};

// Software pipeline: while the MFMAs of chunk i (one row-tap x CK input channels) run out of LDS, the
// pixel slab and the weight image of chunk i+1 - of the next tile when the tile ends - are already in
// flight into registers; they are written to LDS between two barriers once the MFMAs are issued.
// Prefetch loads are unconditional: a uniform base pointer plus a per-thread 32-bit offset that never
// changes; slabs that cross the start or the end of the tensor take a clamped-address path and validity
// is applied at the LDS store.  A workgroup owns 256 pixels x NB output channels; each of its four
// waves 64 pixels x NB channels (2 x NB/32 MFMA tiles).
template <int NB, int CK, int KWMAX, bool VEC>
__global__ __launch_bounds__(kConvThreads) void conv_mfma_kernel(ConvArgs a) {
    constexpr int TM = kConvTM, RS = CK + 4, G = CK / 8, NJ = NB / 32, PJ = 2, Q4 = CK / 4;
    constexpr int PS = ((TM + KWMAX - 1) * Q4 + kConvThreads - 1) / kConvThreads;   // slab quads per thread
    constexpr int PW = (KWMAX * CK * NB / 4 + kConvThreads - 1) / kConvThreads;     // weight float4 per thread
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const PixDims d = a.d;
    const int n_pix = TM + d.kw - 1;
    float* slab = smem;             // [n_pix][RS]
    float* wl = smem + n_pix * RS;  // [kw][G][2][NB][4]
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, m = lane & 31, h = lane >> 5;
    const int n0 = blockIdx.y * NB;
    const int rowtaps = d.kt * d.kd * d.kh;
    const int n_kc = (a.K + CK - 1) / CK;
    const int nck = rowtaps * n_kc;                      // chunks per tile
    const int w4 = d.kw * CK * NB / 4;                   // float4 per weight image
    const long long n_tiles = (d.Q + TM - 1) / TM;
    const bool vec_out = (a.Nn % 4) == 0;
    const bool k_full = (a.K % CK) == 0;                 // no channel padding inside a chunk

    // slots this thread moves for every chunk: quad (4 channels) s_ch of slab pixel s_pp
    int s_lds[PS], s_pp[PS], s_ch[PS];
    unsigned s_off[PS];                                  // element offset of the quad from the slab origin
#pragma unroll
    for (int i = 0; i < PS; ++i) {
        const int v = tid + i * kConvThreads;
        const bool used = v < n_pix * Q4;
        s_pp[i] = used ? v / Q4 : 0;
        s_ch[i] = used ? 4 * (v % Q4) : 0;
        s_lds[i] = used ? s_pp[i] * RS + s_ch[i] : -1;
        s_off[i] = (unsigned)(s_pp[i] * a.K + s_ch[i]);
    }
    unsigned w_off[PW];
#pragma unroll
    for (int i = 0; i < PW; ++i) {
        const int idx = tid + i * kConvThreads;
        w_off[i] = idx < w4 ? idx : 0;
    }
    float4 rs[PS], rw[PW];
    unsigned okb = 0u;   // VEC: bit i = quad i valid; scalar: bit 4i+e per element
    bool interior = true;

    auto fetch = [&](long long tile, int c) {
        const int rt = c / n_kc, kc = c % n_kc;
        const long long qs = tile * TM + rowtap_offset(rt, d) - d.kw / 2;
        interior = k_full && qs >= 0 && qs + n_pix <= d.Q;          // uniform
        if (interior) {
            const float* base = a.in + qs * a.K + kc * CK;           // uniform
            if (VEC) {
#pragma unroll
                for (int i = 0; i < PS; ++i) rs[i] = *reinterpret_cast<const float4*>(base + s_off[i]);
            } else {
#pragma unroll
                for (int i = 0; i < PS; ++i)
                    rs[i] = make_float4(base[s_off[i]], base[s_off[i] + 1], base[s_off[i] + 2], base[s_off[i] + 3]);
            }
        } else {
            okb = 0u;
#pragma unroll
            for (int i = 0; i < PS; ++i) {
                const long long qq = qs + s_pp[i];
                const int ch = kc * CK + s_ch[i];
                const bool okp = qq >= 0 && qq < d.Q;
                if (VEC) {
                    const bool ok = okp && ch < a.K;
                    rs[i] = *reinterpret_cast<const float4*>(a.in + (ok ? qq * a.K + ch : 0));
                    okb |= (ok ? 1u : 0u) << i;
                } else {
                    float e4[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool ok = okp && ch + e < a.K;
                        e4[e] = a.in[ok ? qq * a.K + ch + e : 0];
                        okb |= (ok ? 1u : 0u) << (4 * i + e);
                    }
                    rs[i] = make_float4(e4[0], e4[1], e4[2], e4[3]);
                }
            }
        }
        const float4* src = reinterpret_cast<const float4*>(
            a.wt + ((size_t)(rt * n_kc + kc) * gridDim.y + blockIdx.y) * (size_t)(d.kw * CK * NB));
#pragma unroll
        for (int i = 0; i < PW; ++i) rw[i] = src[w_off[i]];
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < PS; ++i) {
            float4 v = rs[i];
            if (!interior) {
                if (VEC) {
                    const unsigned mk = ((okb >> i) & 1u) ? 0xffffffffu : 0u;
                    v.x = __uint_as_float(__float_as_uint(v.x) & mk); v.y = __uint_as_float(__float_as_uint(v.y) & mk);
                    v.z = __uint_as_float(__float_as_uint(v.z) & mk); v.w = __uint_as_float(__float_as_uint(v.w) & mk);
                } else {
                    v.x = ((okb >> (4 * i)) & 1u) ? v.x : 0.f; v.y = ((okb >> (4 * i + 1)) & 1u) ? v.y : 0.f;
                    v.z = ((okb >> (4 * i + 2)) & 1u) ? v.z : 0.f; v.w = ((okb >> (4 * i + 3)) & 1u) ? v.w : 0.f;
                }
            }
            if (a.relu_in) {
                v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f);
            }
            if (s_lds[i] >= 0) *reinterpret_cast<float4*>(slab + s_lds[i]) = v;
        }
#pragma unroll
        for (int i = 0; i < PW; ++i)
            if (tid + i * kConvThreads < w4) reinterpret_cast<float4*>(wl)[tid + i * kConvThreads] = rw[i];
    };

    long long tile = blockIdx.x;
    if (tile < n_tiles) {
        fetch(tile, 0);
        stash();
    }
    __syncthreads();
    for (; tile < n_tiles; tile += gridDim.x) {
        const long long q0 = tile * TM + wave * 64 + m;   // this lane's pixels: q0 and q0 + 32
        unsigned vbits[PJ];
#pragma unroll
        for (int pj = 0; pj < PJ; ++pj) vbits[pj] = tap_validity(q0 + 32 * pj, d);
        floatx16 acc[PJ][NJ];
#pragma unroll
        for (int pj = 0; pj < PJ; ++pj)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[pj][j][r] = 0.f;

        for (int c = 0; c < nck; ++c) {
            const bool last = c + 1 == nck;
            const long long ntile = last ? tile + gridDim.x : tile;
            const bool has_next = ntile < n_tiles;
            if (has_next) fetch(ntile, last ? 0 : c + 1);
            // ---- MFMA: A = weights (rows = output channels), B = pixels (columns)
            const int rt = c / n_kc;
            for (int dw = 0; dw < d.kw; ++dw) {
                unsigned okm[PJ];
#pragma unroll
                for (int pj = 0; pj < PJ; ++pj) okm[pj] = ((vbits[pj] >> (rt * d.kw + dw)) & 1u) ? 0xffffffffu : 0u;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float4 pb[PJ], wa[NJ];
#pragma unroll
                    for (int pj = 0; pj < PJ; ++pj) {
                        pb[pj] = *reinterpret_cast<const float4*>(slab + (wave * 64 + 32 * pj + m + dw) * RS + 8 * g + 4 * h);
                        pb[pj].x = __uint_as_float(__float_as_uint(pb[pj].x) & okm[pj]);  // zero padding
                        pb[pj].y = __uint_as_float(__float_as_uint(pb[pj].y) & okm[pj]);
                        pb[pj].z = __uint_as_float(__float_as_uint(pb[pj].z) & okm[pj]);
                        pb[pj].w = __uint_as_float(__float_as_uint(pb[pj].w) & okm[pj]);
                    }
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        wa[j] = *reinterpret_cast<const float4*>(wl + (((dw * G + g) * 2 + h) * NB + 32 * j + m) * 4);
#pragma unroll
                    for (int pj = 0; pj < PJ; ++pj)
#pragma unroll
                        for (int j = 0; j < NJ; ++j) {
                            acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[j].x, pb[pj].x, acc[pj][j], 0, 0, 0);
                            acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[j].y, pb[pj].y, acc[pj][j], 0, 0, 0);
                            acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[j].z, pb[pj].z, acc[pj][j], 0, 0, 0);
                            acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[j].w, pb[pj].w, acc[pj][j], 0, 0, 0);
                        }
                }
            }
            if (last) {
                // ---- epilogue: lane holds pixels q0 + 32*pj and 4 consecutive output channels per register group
#pragma unroll
                for (int pj = 0; pj < PJ; ++pj) {
                    const long long q = q0 + 32 * pj;
                    if (q >= d.Q) continue;
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg) {
                            const int co0 = n0 + 32 * j + 8 * rg + 4 * h;
                            if (co0 >= a.Nn) continue;
                            float v[4] = {acc[pj][j][4 * rg], acc[pj][j][4 * rg + 1], acc[pj][j][4 * rg + 2], acc[pj][j][4 * rg + 3]};
                            const long long o = q * a.Nn + co0;
                            if (vec_out) {
                                if (a.bias) {
                                    const float4 bv = *reinterpret_cast<const float4*>(a.bias + co0);
                                    v[0] += bv.x; v[1] += bv.y; v[2] += bv.z; v[3] += bv.w;
                                }
                                if (a.relu_out) {
#pragma unroll
                                    for (int i = 0; i < 4; ++i) v[i] = fmaxf(v[i], 0.f);
                                }
                                float4 ref = make_float4(1.f, 1.f, 1.f, 1.f);
                                if (a.mask_ref) ref = *reinterpret_cast<const float4*>(a.mask_ref + o);
                                const float rr[4] = {ref.x, ref.y, ref.z, ref.w};
                                if (a.mask_acc) {
#pragma unroll
                                    for (int i = 0; i < 4; ++i) v[i] = rr[i] > 0.f ? v[i] : 0.f;
                                }
                                if (a.add) {
                                    const float4 av = *reinterpret_cast<const float4*>(a.add + o);
                                    const float aa[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
                                    for (int i = 0; i < 4; ++i) v[i] += (a.mask_add && !(rr[i] > 0.f)) ? 0.f : aa[i];
                                }
                                *reinterpret_cast<float4*>(a.out + o) = make_float4(v[0], v[1], v[2], v[3]);
                            } else {
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    if (co0 + i >= a.Nn) break;
                                    float x = v[i];
                                    if (a.bias) x += a.bias[co0 + i];
                                    if (a.relu_out) x = fmaxf(x, 0.f);
                                    const float ref = a.mask_ref ? a.mask_ref[o + i] : 1.f;
                                    if (a.mask_acc) x = ref > 0.f ? x : 0.f;
                                    if (a.add) x += (a.mask_add && !(ref > 0.f)) ? 0.f : a.add[o + i];
                                    a.out[o + i] = x;
                                }
                            }
                        }
                }
            }
            __syncthreads();
            if (has_next) stash();
            __syncthreads();
        }
    }
}

// Forward / data-gradient convolution with global -> LDS direct loads (no register staging, so few
// VGPRs and three workgroups per CU).  Chunks (row-tap x CK input channels) alternate between two LDS
// buffers: the direct loads of the next chunk - next tile at a tile end - are issued before the MFMAs
// of the current one, one barrier per chunk.  The compiler still waits for a wave's own outstanding
// direct loads before that wave's LDS reads, so most of the overlap comes from the co-resident
// workgroups rather than from within a wave.
// A direct load writes lane l's 16 bytes at (uniform LDS base) + 16*l, so a wave fills 64 consecutive
// quad slots (quad = 4 channels of one slab pixel).  Rows cannot be padded in that scheme; instead the
// quad position inside a pixel row is XOR-swizzled with the pixel index, chosen by picking each lane's
// GLOBAL address, which keeps the 128-bit operand reads bank-conflict free.  Pixels or channels past
// the tensor are read from a clamped address: they only ever meet masked taps or zero weights.
// Requires K % 4 == 0 (16-byte alignment of every quad).
// KW > 0 fixes the kernel extent along W at compile time (all LDS operand offsets become immediates);
// KW == 0 reads it from the arguments.
template <int NB, int CK, int PJ, int NW, int KW, bool RELU>
__global__ __launch_bounds__(NW * 64, 2) void conv_dlds_kernel(ConvArgs a) {
    constexpr int TM = NW * 32 * PJ, G = CK / 8, NJ = NB / 32, Q4 = CK / 4;
    // Swizzle period: LDS serves 128-bit accesses 16 lanes at a time out of 64 banks (256 bytes), so 16 consecutive
    // pixels must land on 16 different 16-byte slots: pixel rows per 256 bytes of LDS.
    constexpr int RP = Q4 >= 16 ? 1 : 16 / Q4;
    constexpr int KWM = KW > 0 ? KW : 5;       // most taps along W
    constexpr int MAXS = ((TM + KWM - 1) * Q4 + 63) / 64 / NW + 1;   // slab loads per wave and chunk
    constexpr int MAXW = (KWM * CK * NB / 4 + 63) / 64 / NW + 1;     // weight loads per wave and chunk
    // The two chunk buffers are separate LDS objects on purpose: the compiler can then tell that an LDS
    // read of one buffer does not depend on direct loads still in flight into the other, and does not
    // make a wave wait for its own prefetch before its MFMAs.
    constexpr int kBufFloats = (((TM + KWM - 1) * Q4 + 63) / 64 + (KWM * CK * NB / 4 + 63) / 64) * 256;
    __shared__ float bufA[kBufFloats];
    __shared__ float bufB[kBufFloats];
    const PixDims d = a.d;
    const int kw = KW > 0 ? KW : d.kw;
    const int n_pix = TM + kw - 1;
    const int slab_ops = (n_pix * Q4 + 63) / 64;          // wave-wide loads per slab
    const int w4 = kw * CK * NB / 4;
    const int w_ops = (w4 + 63) / 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), m = lane & 31, h = lane >> 5;
    const int n0 = blockIdx.y * NB;
    const int rowtaps = d.kt * d.kd * d.kh;
    const int n_kc = (a.K + CK - 1) / CK;
    const int nck = rowtaps * n_kc;
    const long long n_tiles = (d.Q + TM - 1) / TM;
    const bool vec_out = (a.Nn % 4) == 0;
    const bool k_full = (a.K % CK) == 0;
    const long long last_quad = d.Q * a.K - 4;            // highest legal quad start

    // Per-lane constants of the direct loads: element offset of this lane's quad from the slab origin
    // (pixel qs, channel kc*CK) and float offset of its weight quad inside an image.
    unsigned s_off[MAXS], w_off[MAXW];
    int s_pp[MAXS], s_c4[MAXS];
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
        const int v = (wave + i * NW) * 64 + lane;
        s_pp[i] = v / Q4;
        s_c4[i] = (v % Q4) ^ ((s_pp[i] / RP) % Q4);
        s_off[i] = (unsigned)(s_pp[i] * a.K + 4 * s_c4[i]);
    }
#pragma unroll
    for (int i = 0; i < MAXW; ++i) {
        const int v = (wave + i * NW) * 64 + lane;
        w_off[i] = 4u * (unsigned)(v < w4 ? v : 0);
    }

    auto issue = [&](long long tile, const ChunkIter& ci, float* dst) {
        const int rt = ci.rt, kc = ci.kc;
        const long long qs = tile * TM + ci.off - kw / 2;
        const bool interior = k_full && qs >= 0 && qs + (long long)slab_ops * 64 / Q4 <= d.Q;   // uniform
        if (interior) {
            const float* base = a.in + qs * a.K + kc * CK;                                       // uniform
#pragma unroll
            for (int i = 0; i < MAXS; ++i) {
                const int o = wave + i * NW;
                if (o < slab_ops)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + s_off[i]),
                                                     (__attribute__((address_space(3))) void*)(dst + o * 256), 16, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < MAXS; ++i) {
                const int o = wave + i * NW;
                if (o < slab_ops) {
                    long long off = (qs + s_pp[i]) * a.K + kc * CK + 4 * s_c4[i];
                    off = off < 0 ? 0 : (off > last_quad ? last_quad : off);
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(a.in + off),
                                                     (__attribute__((address_space(3))) void*)(dst + o * 256), 16, 0, 0);
                }
            }
        }
        const float* src = a.wt + ((size_t)(rt * n_kc + kc) * gridDim.y + blockIdx.y) * (size_t)(kw * CK * NB);
        float* wdst = dst + slab_ops * 256;
#pragma unroll
        for (int i = 0; i < MAXW; ++i) {
            const int o = wave + i * NW;
            if (o < w_ops)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + w_off[i]),
                                                 (__attribute__((address_space(3))) void*)(wdst + o * 256), 16, 0, 0);
        }
    };

    // LDS float offsets of this lane's pixel operand for every (pixel block, tap along W, 8-channel group)
    int p_off[PJ][KWM][G];
#pragma unroll
    for (int pj = 0; pj < PJ; ++pj)
#pragma unroll
        for (int dw = 0; dw < KWM; ++dw) {
            const int pix = wave * (32 * PJ) + 32 * pj + m + dw;
            const int key = (pix / RP) % Q4;
#pragma unroll
            for (int g = 0; g < G; ++g) p_off[pj][dw][g] = pix * CK + 4 * ((2 * g + h) ^ key);
        }
    const int wa_lane = (h * NB + m) * 4;

    const XcdRange xr = xcd_range(n_tiles);
    long long tile = xr.first;
    ChunkIter ci = chunk_first(d);
    if (tile < xr.end) issue(tile, ci, bufA);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // this lane's pixels of the current tile, tracked by coordinates (no divisions per tile)
    long long q0 = (tile < xr.end ? tile : 0) * TM + wave * (32 * PJ) + m;
    PixCoord qc[PJ];
#pragma unroll
    for (int pj = 0; pj < PJ; ++pj) qc[pj] = pix_coord(q0 + 32 * pj < d.Q ? q0 + 32 * pj : 0, d);
    const PixCoord qstep = pix_coord(xr.stride * TM, d);
    unsigned vbits[PJ];
    floatx16 acc[PJ][NJ];
    // One chunk: prefetch the following chunk into `nxt`, run the MFMAs of the current one out of `slab`.
    // Called alternately with (bufA, bufB) and (bufB, bufA) so that each call site names its buffers.
    auto step = [&](const float* slab, float* nxt) {
        if (ci.c == 0) {
#pragma unroll
            for (int pj = 0; pj < PJ; ++pj) vbits[pj] = q0 + 32 * pj < d.Q ? tap_validity_at(qc[pj], d) : 0u;
#pragma unroll
            for (int pj = 0; pj < PJ; ++pj)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[pj][j][r] = 0.f;
        }
        const bool last = ci.c + 1 == nck;
        const long long ntile = last ? tile + xr.stride : tile;
        const ChunkIter nci = chunk_next(ci, n_kc, nck, d);
        if (ntile < xr.end) issue(ntile, nci, nxt);
        {
            const float* wl = slab + slab_ops * 256 + wa_lane;
            const int rt = ci.rt;
            if constexpr (KW > 0) {
                // Operands of unit u + 1 (one tap along W x 8 input channels) are read from LDS before the
                // MFMAs of unit u are issued, and consecutive MFMAs alternate between accumulators.
                constexpr int U = KW * G;
                float4 pb[2][PJ], wa[2][NJ];
                auto load_unit = [&](int u, int slot) {
                    const int dw = u / G, g = u % G;
#pragma unroll
                    for (int pj = 0; pj < PJ; ++pj) pb[slot][pj] = *reinterpret_cast<const float4*>(slab + p_off[pj][dw][g]);
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        wa[slot][j] = *reinterpret_cast<const float4*>(wl + ((dw * G + g) * 2 * NB + 32 * j) * 4);
                };
                load_unit(0, 0);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int cur = u & 1, dw = u / G;
                    if (u + 1 < U) load_unit(u + 1, cur ^ 1);
                    // Ordinary vector instructions take issue slots from the MFMAs, so ReLU and the zero
                    // padding are done on the bit patterns: max with 0 as a signed integer is ReLU (negative
                    // floats have the sign bit set), and the padding mask is one AND.
#pragma unroll
                    for (int pj = 0; pj < PJ; ++pj) {
                        const int okm = -(int)((vbits[pj] >> (rt * kw + dw)) & 1u);   // all ones: tap inside the grid
                        float4& v = pb[cur][pj];
                        int x0 = __float_as_int(v.x), x1 = __float_as_int(v.y), x2 = __float_as_int(v.z), x3 = __float_as_int(v.w);
                        if (RELU) {
                            x0 = x0 > 0 ? x0 : 0; x1 = x1 > 0 ? x1 : 0; x2 = x2 > 0 ? x2 : 0; x3 = x3 > 0 ? x3 : 0;
                        }
                        v.x = __int_as_float(x0 & okm); v.y = __int_as_float(x1 & okm);
                        v.z = __int_as_float(x2 & okm); v.w = __int_as_float(x3 & okm);
                    }
#pragma unroll
                    for (int pj = 0; pj < PJ; ++pj) {
#pragma unroll
                        for (int j = 0; j < NJ; ++j)
                            acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[cur][j].x, pb[cur][pj].x, acc[pj][j], 0, 0, 0);
#pragma unroll
                        for (int j = 0; j < NJ; ++j)
                            acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[cur][j].y, pb[cur][pj].y, acc[pj][j], 0, 0, 0);
#pragma unroll
                        for (int j = 0; j < NJ; ++j)
                            acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[cur][j].z, pb[cur][pj].z, acc[pj][j], 0, 0, 0);
#pragma unroll
                        for (int j = 0; j < NJ; ++j)
                            acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[cur][j].w, pb[cur][pj].w, acc[pj][j], 0, 0, 0);
                    }
                }
            } else {
#pragma unroll
                for (int dw = 0; dw < KWM; ++dw) {
                    if (KW == 0 && dw >= kw) continue;
                    unsigned okm[PJ];
    #pragma unroll
                    for (int pj = 0; pj < PJ; ++pj) okm[pj] = ((vbits[pj] >> (rt * kw + dw)) & 1u) ? 0xffffffffu : 0u;
    #pragma unroll
                    for (int g = 0; g < G; ++g) {
                        float4 pb[PJ], wa[NJ];
    #pragma unroll
                        for (int pj = 0; pj < PJ; ++pj) {
                            pb[pj] = *reinterpret_cast<const float4*>(slab + p_off[pj][dw][g]);
                            if (a.relu_in) {
                                pb[pj].x = fmaxf(pb[pj].x, 0.f); pb[pj].y = fmaxf(pb[pj].y, 0.f);
                                pb[pj].z = fmaxf(pb[pj].z, 0.f); pb[pj].w = fmaxf(pb[pj].w, 0.f);
                            }
                            pb[pj].x = __uint_as_float(__float_as_uint(pb[pj].x) & okm[pj]);  // zero padding
                            pb[pj].y = __uint_as_float(__float_as_uint(pb[pj].y) & okm[pj]);
                            pb[pj].z = __uint_as_float(__float_as_uint(pb[pj].z) & okm[pj]);
                            pb[pj].w = __uint_as_float(__float_as_uint(pb[pj].w) & okm[pj]);
                        }
    #pragma unroll
                        for (int j = 0; j < NJ; ++j)
                            wa[j] = *reinterpret_cast<const float4*>(wl + ((dw * G + g) * 2 * NB + 32 * j) * 4);
    #pragma unroll
                        for (int pj = 0; pj < PJ; ++pj)
    #pragma unroll
                            for (int j = 0; j < NJ; ++j) {
                                acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[j].x, pb[pj].x, acc[pj][j], 0, 0, 0);
                                acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[j].y, pb[pj].y, acc[pj][j], 0, 0, 0);
                                acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[j].z, pb[pj].z, acc[pj][j], 0, 0, 0);
                                acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[j].w, pb[pj].w, acc[pj][j], 0, 0, 0);
                            }
                    }
                }
}
            if (last) {
#pragma unroll
                for (int pj = 0; pj < PJ; ++pj) {
                    const long long q = q0 + 32 * pj;
                    if (q >= d.Q) continue;
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg) {
                            const int co0 = n0 + 32 * j + 8 * rg + 4 * h;
                            if (co0 >= a.Nn) continue;
                            float v[4] = {acc[pj][j][4 * rg], acc[pj][j][4 * rg + 1], acc[pj][j][4 * rg + 2], acc[pj][j][4 * rg + 3]};
                            const long long o = q * a.Nn + co0;
                            if (vec_out) {
                                if (a.bias) {
                                    const float4 bv = *reinterpret_cast<const float4*>(a.bias + co0);
                                    v[0] += bv.x; v[1] += bv.y; v[2] += bv.z; v[3] += bv.w;
                                }
                                if (a.relu_out) {
#pragma unroll
                                    for (int i = 0; i < 4; ++i) v[i] = fmaxf(v[i], 0.f);
                                }
                                float4 ref = make_float4(1.f, 1.f, 1.f, 1.f);
                                if (a.mask_ref) ref = *reinterpret_cast<const float4*>(a.mask_ref + o);
                                const float rr[4] = {ref.x, ref.y, ref.z, ref.w};
                                if (a.mask_acc) {
#pragma unroll
                                    for (int i = 0; i < 4; ++i) v[i] = rr[i] > 0.f ? v[i] : 0.f;
                                }
                                if (a.add) {
                                    const float4 av = *reinterpret_cast<const float4*>(a.add + o);
                                    const float aa[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
                                    for (int i = 0; i < 4; ++i) v[i] += (a.mask_add && !(rr[i] > 0.f)) ? 0.f : aa[i];
                                }
                                *reinterpret_cast<float4*>(a.out + o) = make_float4(v[0], v[1], v[2], v[3]);
                            } else {
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    if (co0 + i >= a.Nn) break;
                                    float x = v[i];
                                    if (a.bias) x += a.bias[co0 + i];
                                    if (a.relu_out) x = fmaxf(x, 0.f);
                                    const float ref = a.mask_ref ? a.mask_ref[o + i] : 1.f;
                                    if (a.mask_acc) x = ref > 0.f ? x : 0.f;
                                    if (a.add) x += (a.mask_add && !(ref > 0.f)) ? 0.f : a.add[o + i];
                                    a.out[o + i] = x;
                                }
                            }
                        }
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0);   // the next chunk's direct loads have landed in LDS
        __syncthreads();                 // ... and every wave is done reading the current buffer
        if (last) {
            q0 += xr.stride * TM;
#pragma unroll
            for (int pj = 0; pj < PJ; ++pj) pix_advance(qc[pj], qstep, d);
        }
        tile = ntile;
        ci = nci;
    };
    while (tile < xr.end) {
        step(bufA, bufB);
        if (tile >= xr.end) break;
        step(bufB, bufA);
    }
}

// Convolution whose INPUT has two channels (first layer forward; data gradient of a layer whose output
// is the 2-channel image): K = 2 -> Nn wide.  HBM-bound on the output, so no MFMA: lanes index the
// output channel and keep their 2*taps weights in registers; the 2-channel input rows around the current
// image row sit in LDS, zero-filled outside the grid, and are read as wave-wide broadcasts.  Same fused
// epilogue as conv_dlds_kernel.  Source weight (n, tap, e) at w[n*sn + tapidx*st + e*sk].
struct ConvThinInArgs {
    ConvArgs c;          // in = [Q][2]; wt unused
    const float* w;
    long long sn, st, sk;
};

template <int KT, int KD, int KH, int KW, bool BF>
__global__ __launch_bounds__(256) void conv_thin_in_kernel(ConvThinInArgs ta) {
    constexpr int RT = KT * KD * KH, TAPS = RT * KW, TH = 2, PX = 4;   // PX pixels per lane and step
    constexpr int NC4 = (PX + KW - 1 + 1) / 2;                          // float4 (2 pixels x 2 channels) per row tap
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const ConvArgs& a = ta.c;
    const PixDims d = a.d;
    const int WS = (d.W + PX - 1) / PX * PX + 2 * NC4 - PX;   // slab row: columns -KW/2 .. , zero past the row
    float* slab = smem;   // [RT][WS][2]
    const int WCr = a.Nn <= 32 ? 32 : (a.Nn <= 64 ? 64 : (a.Nn <= 128 ? 128 : 256));
    const int groups = 256 / WCr;
    const int n = threadIdx.x % WCr;
    const int pg = threadIdx.x / WCr;
    const bool n_ok = n < a.Nn;
    const int nc = n_ok ? n : 0;
    float wreg[TAPS][TH];
#pragma unroll
    for (int t = 0; t < TAPS; ++t) {
        const int tapidx = a.flip ? TAPS - 1 - t : t;
#pragma unroll
        for (int e = 0; e < TH; ++e) wreg[t][e] = ta.w[nc * ta.sn + tapidx * ta.st + e * ta.sk];
    }
    const float bias = (a.bias && n_ok) ? a.bias[n] : 0.f;
    const long long n_rows = d.Q / d.W;
    for (long long row = blockIdx.x; row < n_rows; row += gridDim.x) {
        long long r = row;
        const int hh = (int)(r % d.H);
        r /= d.H;
        const int dd = (int)(r % d.D);
        r /= d.D;
        const int tt = (int)(r % d.T);
        __syncthreads();
        // stage the RT input rows: all loads of a pass are issued (clamped addresses) before any LDS store
        for (int j0 = 0; j0 < WS; j0 += 256) {
            const int j = j0 + threadIdx.x, col = j - KW / 2;
            float2 v[RT];
            bool ok[RT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const int ih = rt % KH, id = (rt / KH) % KD, it = rt / (KH * KD);
                const int ot = it - KT / 2, od = id - KD / 2, oh = ih - KH / 2;
                const bool row_ok = tt + ot >= 0 && tt + ot < d.T && dd + od >= 0 && dd + od < d.D && hh + oh >= 0 && hh + oh < d.H;
                const long long src_row = row + ((long long)ot * d.D + od) * d.H + oh;
                ok[rt] = row_ok && col >= 0 && col < d.W;
                v[rt] = *reinterpret_cast<const float2*>(a.in + (ok[rt] ? (src_row * d.W + col) * TH : 0));
            }
            if (j < WS) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    float2 x = make_float2(ok[rt] ? v[rt].x : 0.f, ok[rt] ? v[rt].y : 0.f);
                    if (a.relu_in) x = make_float2(fmaxf(x.x, 0.f), fmaxf(x.y, 0.f));
                    *reinterpret_cast<float2*>(slab + (rt * WS + j) * TH) = x;
                }
            }
        }
        __syncthreads();
        // each lane: one output channel, PX consecutive pixels; the input columns of a row tap come as
        // 16-byte reads (two pixels x two channels), the same address for all lanes of a channel group
        for (int w = pg * PX; w < d.W; w += groups * PX) {
            float acc[PX];
#pragma unroll
            for (int p = 0; p < PX; ++p) acc[p] = bias;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                float col[2 * NC4][TH];
#pragma unroll
                for (int c4 = 0; c4 < NC4; ++c4) {
                    const float4 v = *reinterpret_cast<const float4*>(slab + (rt * WS + w + 2 * c4) * TH);
                    col[2 * c4][0] = v.x; col[2 * c4][1] = v.y; col[2 * c4 + 1][0] = v.z; col[2 * c4 + 1][1] = v.w;
                }
#pragma unroll
                for (int iw = 0; iw < KW; ++iw)
#pragma unroll
                    for (int p = 0; p < PX; ++p) {
                        acc[p] = fmaf(wreg[rt * KW + iw][0], col[p + iw][0], acc[p]);
                        acc[p] = fmaf(wreg[rt * KW + iw][1], col[p + iw][1], acc[p]);
                    }
            }
            if (n_ok) {
                // reference / skip values of the PX outputs are requested together, then combined and stored
                const long long o0 = (row * d.W + w) * a.Nn + n;
                float ref[PX], add[PX];
#pragma unroll
                for (int p = 0; p < PX; ++p) {
                    const long long o = w + p < d.W ? o0 + (long long)p * a.Nn : o0;
                    ref[p] = 1.f;
                    add[p] = 0.f;
                    if (BF) {   // wide tensors (out, mask_ref, add) are bfloat16
                        if (a.mask_ref) ref[p] = bf16_to_f32(reinterpret_cast<const unsigned short*>(a.mask_ref)[o]);
                        if (a.add) add[p] = bf16_to_f32(reinterpret_cast<const unsigned short*>(a.add)[o]);
                    } else {
                        if (a.mask_ref) ref[p] = a.mask_ref[o];
                        if (a.add) add[p] = a.add[o];
                    }
                }
#pragma unroll
                for (int p = 0; p < PX; ++p) {
                    float x = acc[p];
                    if (a.relu_out) x = fmaxf(x, 0.f);
                    if (a.mask_acc) x = ref[p] > 0.f ? x : 0.f;
                    x += (a.mask_add && !(ref[p] > 0.f)) ? 0.f : add[p];
                    if (w + p < d.W) {
                        const long long o = o0 + (long long)p * a.Nn;
                        if (BF) reinterpret_cast<unsigned short*>(a.out)[o] = f32_to_bf16(x);
                        else a.out[o] = x;
                    }
                }
            }
        }
    }
}

// Convolution whose OUTPUT has two channels (last layer forward): K wide -> 2, for the shapes the matrix-core
// kernels of prox_thin.hip do not cover.  HBM-bound on its input, vector ALUs only.  A tile is 64 neighbouring pixels of one image row, one lane each.  The input rows of every
// row tap are staged in LDS (KC channels per round, zero outside the grid, ReLU applied), pixel stride
// KC + 4 floats so that 16-byte reads of neighbouring lanes do not collide.  Work items (row tap,
// 16-channel chunk) are dealt to the four waves; the two output channels' weights of an item are
// wave-uniform, read straight from theta (a restrict kernel argument, so they come as scalar loads).  Partial sums of the waves meet in LDS, where bias and the
// skip tensor are added.  Input is float32 or (BF) bfloat16; output, skip and weights are float32.
struct ConvThinOutArgs {
    const void* in;       // [Q][K]
    const float* bias;    // [2] or null
    const float* add;     // [Q][2] or null
    float* out;           // [Q][2]
    int K, KC, relu_in, relu_out;
    PixDims d;
};

constexpr int kThinOutPx = 64;

__device__ __forceinline__ float4 zero_unless(bool ok, float4 v) {
    return make_float4(ok ? v.x : 0.f, ok ? v.y : 0.f, ok ? v.z : 0.f, ok ? v.w : 0.f);
}

template <int KT, int KD, int KH, int KW, bool BF, int KC>
__global__ __launch_bounds__(256) void conv_thin_out_kernel(ConvThinOutArgs a, const float* __restrict__ wts) {
    constexpr int RT = KT * KD * KH, TAPS = RT * KW, PXS = kThinOutPx + KW - 1, EPG = BF ? 8 : 4;
    constexpr int RS = KC + 4, GPN = KC / EPG;   // pixel stride in floats; 16-byte groups per pixel and round
    constexpr int PER_ROW = PXS * GPN, TOTAL = RT * PER_ROW, ITER = (TOTAL + 255) / 256;
    constexpr int NCH = KC / 16;
    static_assert(ITER <= 32, "validity bits of one staging round must fit a 32-bit mask");
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const PixDims d = a.d;
    float* slab = smem;                        // [RT][PXS][RS]
    float* red = smem + RT * PXS * RS;         // [4][64][2]
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
    const int n_rounds = a.K / KC;
    const int segs = (d.W + kThinOutPx - 1) / kThinOutPx;
    const long long n_tiles = (d.Q / d.W) * segs;
    const XcdRange xr = xcd_range(n_tiles);

    // Per-thread staging slots, the same for every tile: slot `it` moves one 16-byte group from element
    // offset rel[it] (relative to the tile's first pixel, channel 0 of the round) to LDS offset dst[it].
    int rel[ITER], dst[ITER], pxo[ITER];
    unsigned rtm[ITER];
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int idx = threadIdx.x + it * 256;
        const int rt = idx / PER_ROW, rem = idx % PER_ROW, px = rem / GPN, gi = rem % GPN;
        const int ih = rt % KH, id = (rt / KH) % KD, itp = rt / (KH * KD);
        const int ot = itp - KT / 2, od = id - KD / 2, oh = ih - KH / 2;
        rel[it] = ((((ot * d.D + od) * d.H + oh) * d.W) + px - KW / 2) * a.K + gi * EPG;
        dst[it] = (rt * PXS + px) * RS + gi * EPG;
        pxo[it] = px - KW / 2;
        rtm[it] = idx < TOTAL ? 1u << rt : 0u;
    }
    // Staging registers of the NEXT (tile, round): fetched while the current one is being computed.
    uint4 stg[ITER];
    unsigned okm = 0u;
    auto fetch = [&](long long tile, int rd) {
        const long long row = tile / segs;
        const int w0 = (int)(tile % segs) * kThinOutPx;
        long long r = row;
        const int hh = (int)(r % d.H);
        r /= d.H;
        const int dd = (int)(r % d.D);
        r /= d.D;
        const int tt = (int)(r % d.T);
        unsigned rows_ok = 0u;   // bit rt: the input row of row tap rt lies inside the grid
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const int ih = rt % KH, id = (rt / KH) % KD, itp = rt / (KH * KD);
            const bool v = (unsigned)(tt + itp - KT / 2) < (unsigned)d.T && (unsigned)(dd + id - KD / 2) < (unsigned)d.D &&
                           (unsigned)(hh + ih - KH / 2) < (unsigned)d.H;
            rows_ok |= (v ? 1u : 0u) << rt;
        }
        const char* base = reinterpret_cast<const char*>(a.in) + ((row * d.W + w0) * a.K + rd * KC) * (BF ? 2 : 4);
        okm = 0u;
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            const bool ok = (rows_ok & rtm[it]) != 0u && (unsigned)(w0 + pxo[it]) < (unsigned)d.W;
            const char* src = ok ? base + (long long)rel[it] * (BF ? 2 : 4) : reinterpret_cast<const char*>(a.in);
            stg[it] = *reinterpret_cast<const uint4*>(src);   // clamped, always readable
            okm |= (ok ? 1u : 0u) << it;
        }
    };

    const float biasv = a.bias ? a.bias[threadIdx.x & 1] : 0.f;
    long long tile = xr.first;
    int rd = 0;
    if (tile < xr.end) fetch(tile, 0);
    float acc0 = 0.f, acc1 = 0.f;
    while (tile < xr.end) {
        __syncthreads();   // the previous round's readers are done with the slab
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            if (rtm[it] != 0u) {
                const bool ok = (okm >> it) & 1u;
                float* dp = slab + dst[it];
                const uint4 u = stg[it];
                if constexpr (BF) {
                    float4 lo = make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                                            __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u));
                    float4 hi = make_float4(__uint_as_float(u.z << 16), __uint_as_float(u.z & 0xffff0000u),
                                            __uint_as_float(u.w << 16), __uint_as_float(u.w & 0xffff0000u));
                    if (a.relu_in) {
                        lo = make_float4(fmaxf(lo.x, 0.f), fmaxf(lo.y, 0.f), fmaxf(lo.z, 0.f), fmaxf(lo.w, 0.f));
                        hi = make_float4(fmaxf(hi.x, 0.f), fmaxf(hi.y, 0.f), fmaxf(hi.z, 0.f), fmaxf(hi.w, 0.f));
                    }
                    *reinterpret_cast<float4*>(dp) = zero_unless(ok, lo);
                    *reinterpret_cast<float4*>(dp + 4) = zero_unless(ok, hi);
                } else {
                    float4 v = make_float4(__uint_as_float(u.x), __uint_as_float(u.y), __uint_as_float(u.z), __uint_as_float(u.w));
                    if (a.relu_in) v = make_float4(fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f));
                    *reinterpret_cast<float4*>(dp) = zero_unless(ok, v);
                }
            }
        }
        __syncthreads();
        const int k0 = rd * KC;
        const bool last_round = rd + 1 == n_rounds;
        const long long ntile = last_round ? tile + xr.stride : tile;
        const int nrd = last_round ? 0 : rd + 1;
        // the skip value of this thread's output is requested ahead of the next tile's fetch, so that
        // waiting for it later does not wait for that fetch as well (loads complete in order)
        float addv = 0.f;
        if (last_round && a.add && threadIdx.x < 2 * kThinOutPx) {
            const int w0 = (int)(tile % segs) * kThinOutPx, px = threadIdx.x >> 1;
            if (w0 + px < d.W) addv = a.add[((tile / segs) * d.W + w0 + px) * 2 + (threadIdx.x & 1)];
        }
        if (ntile < xr.end) fetch(ntile, nrd);
#pragma unroll
        for (int i = 0; i < (RT * NCH + 3) / 4; ++i) {
            const int item = wave + 4 * i;
            if ((RT * NCH) % 4 != 0 && item >= RT * NCH) break;
            const int rt = item / NCH, ch = item % NCH;
#pragma unroll
            for (int dw = 0; dw < KW; ++dw) {
                const float* __restrict__ wp0 = wts + (long long)(rt * KW + dw) * a.K + k0 + ch * 16;
                const float* __restrict__ wp1 = wp0 + (long long)TAPS * a.K;
                const float* sp = slab + (rt * PXS + lane + dw) * RS + ch * 16;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float4 x = *reinterpret_cast<const float4*>(sp + 4 * j);
                    acc0 = fmaf(x.x, wp0[4 * j + 0], acc0); acc1 = fmaf(x.x, wp1[4 * j + 0], acc1);
                    acc0 = fmaf(x.y, wp0[4 * j + 1], acc0); acc1 = fmaf(x.y, wp1[4 * j + 1], acc1);
                    acc0 = fmaf(x.z, wp0[4 * j + 2], acc0); acc1 = fmaf(x.z, wp1[4 * j + 2], acc1);
                    acc0 = fmaf(x.w, wp0[4 * j + 3], acc0); acc1 = fmaf(x.w, wp1[4 * j + 3], acc1);
                }
            }
        }
        if (last_round) {
            const long long row = tile / segs;
            const int w0 = (int)(tile % segs) * kThinOutPx;
            *reinterpret_cast<float2*>(red + (wave * kThinOutPx + lane) * 2) = make_float2(acc0, acc1);
            acc0 = 0.f;
            acc1 = 0.f;
            __syncthreads();
            if (threadIdx.x < 2 * kThinOutPx) {
                const int px = threadIdx.x >> 1, co = threadIdx.x & 1;
                if (w0 + px < d.W) {
                    float v = red[threadIdx.x] + red[2 * kThinOutPx + threadIdx.x] + red[4 * kThinOutPx + threadIdx.x] +
                              red[6 * kThinOutPx + threadIdx.x];
                    v += biasv;
                    if (a.relu_out) v = fmaxf(v, 0.f);
                    a.out[(row * d.W + w0 + px) * 2 + co] = v + addv;
                }
            }
        }
        tile = ntile;
        rd = nrd;
    }
}

// Re-lays one layer's weights as the LDS images conv_mfma_kernel<NB, CK> copies verbatim.  Image
// (rt, kc, nb) holds row-tap rt, input-channel chunk kc and output-channel block nb as
// [kw][CK/8][2][NB][4]: element (dw, k = 8g + 4h + s, n) at (((dw*G + g)*2 + h)*NB + n)*4 + s, zero
// where k or n runs past the layer.  Source element (n, tap, k) is w[n*sn + tapidx*st + k*sk] with
// tapidx = flip ? taps-1-tap : tap, which covers the forward pass (n = cout, k = cin) and the data
// gradient (n = cin, k = cout, taps mirrored).
struct WimgArgs {
    const float* w;
    float* wt;
    long long sn, st, sk;
    int K, Nn, flip, taps, kw, CK, NB, n_kc, n_nb;
    long long total;
};
__global__ void weights_image_kernel(WimgArgs a) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.total) return;
    const int img_elems = a.kw * a.CK * a.NB;
    const long long img = i / img_elems;
    const int e = (int)(i % img_elems);
    const int s = e & 3, n = (e >> 2) % a.NB, hg = (e >> 2) / a.NB;   // hg = (dw*G + g)*2 + h
    const int h = hg & 1, g = (hg >> 1) % (a.CK / 8), dw = (hg >> 1) / (a.CK / 8);
    const int nb = (int)(img % a.n_nb), kc = (int)((img / a.n_nb) % a.n_kc), rt = (int)(img / ((long long)a.n_nb * a.n_kc));
    const int k = kc * a.CK + 8 * g + 4 * h + s, nn = nb * a.NB + n;
    const int tap = rt * a.kw + dw;
    const int tapidx = a.flip ? a.taps - 1 - tap : tap;
    float v = 0.f;
    if (k < a.K && nn < a.Nn) v = a.w[nn * a.sn + tapidx * a.st + k * a.sk];
    a.wt[i] = v;
}

static int conv_grid_x(long long n_tiles) {
    const long long cap = 256LL * 2;   // persistent: two workgroups per CU fit (LDS), each loops over tiles
    return (int)(n_tiles < cap ? n_tiles : cap);
}

template <int NB, int CK, int KWMAX, bool VEC>
static void launch_conv_k(const ConvArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    static bool once = false;
    if (!once) {
        (void)hipFuncSetAttribute((const void*)conv_mfma_kernel<NB, CK, KWMAX, VEC>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        once = true;
    }
    hipLaunchKernelGGL((conv_mfma_kernel<NB, CK, KWMAX, VEC>), grid, dim3(kConvThreads), lds, st, a);
}

template <int NB, int CK, int PJ, int NW, int KW>
static void launch_conv_dlds_k(const ConvArgs& a, hipStream_t st) {
    constexpr int TM = NW * 32 * PJ, Q4 = CK / 4, KWM = KW > 0 ? KW : 5;
    constexpr size_t lds = (size_t)2 * (((TM + KWM - 1) * Q4 + 63) / 64 + (KWM * CK * NB / 4 + 63) / 64) * 1024;   // static in the kernel
    const long long n_tiles = (a.d.Q + TM - 1) / TM;
    int per_cu = (int)(160 * 1024 / lds);
    if (per_cu * NW > 16) per_cu = 16 / NW;
    if (per_cu < 1) per_cu = 1;
    const long long cap = 256LL * per_cu;
    const long long gx = ((n_tiles < cap ? n_tiles : cap) + 7) / 8 * 8;   // XCD-aware split needs a multiple of 8
    dim3 grid((unsigned)gx, (a.Nn + NB - 1) / NB);
    if (a.relu_in) hipLaunchKernelGGL((conv_dlds_kernel<NB, CK, PJ, NW, KW, true>), grid, dim3(NW * 64), 0, st, a);
    else hipLaunchKernelGGL((conv_dlds_kernel<NB, CK, PJ, NW, KW, false>), grid, dim3(NW * 64), 0, st, a);
}

template <int NB, int CK, int PJ, int NW>
static void launch_conv_dlds(const ConvArgs& a, hipStream_t st) {
    if (a.d.kw == 3) launch_conv_dlds_k<NB, CK, PJ, NW, 3>(a, st);
    else if (a.d.kw == 1) launch_conv_dlds_k<NB, CK, PJ, NW, 1>(a, st);
    else launch_conv_dlds_k<NB, CK, PJ, NW, 0>(a, st);
}

template <int NB, int CK>
static hipError_t launch_conv_t(const ConvArgs& a, hipStream_t st) {
    if ((a.K % 4) == 0) {
        launch_conv_dlds<NB, CK, 1, 4>(a, st);
        return hipGetLastError();
    }
    const long long n_tiles = (a.d.Q + kConvTM - 1) / kConvTM;
    const size_t lds = ((size_t)(kConvTM + a.d.kw - 1) * (CK + 4) + (size_t)a.d.kw * CK * NB) * sizeof(float);
    dim3 grid(conv_grid_x(n_tiles), (a.Nn + NB - 1) / NB);
    if (a.d.kw > 3) launch_conv_k<NB, CK, 5, false>(a, grid, lds, st);
    else launch_conv_k<NB, CK, 3, false>(a, grid, lds, st);
    return hipGetLastError();
}

struct ConvWeights {
    const float* w;
    long long sn, st, sk;
};

// Input channels per staged chunk: 16 keeps a double-buffered workgroup near 42 KB of LDS, so three
// workgroups share a CU (measured faster than 32-channel chunks at one workgroup per CU).
static inline int conv_ck(int K) { return K <= 8 ? 8 : 16; }
static inline int conv_nb(int Nn) { return Nn <= 32 ? 32 : 64; }

// Floats of scratch the re-laid weights of a (K -> Nn, taps) convolution need.
static size_t conv_wimg_floats(int K, int Nn, int taps) {
    const int ck = conv_ck(K), nb = conv_nb(Nn);
    return (size_t)taps * ((K + ck - 1) / ck) * ck * ((Nn + nb - 1) / nb) * nb;
}

// The Winograd path can be switched off (GLEAM_POLICY_NO_WINOGRAD) to run the direct kernels instead.
static bool wino_enabled() { return !(kernel_policy() & GLEAM_POLICY_NO_WINOGRAD); }

template <int KT, int KD, int KH, int KW>
static void launch_conv_thin_in_t(const ConvArgs& a, const ConvWeights& cw, bool bf, hipStream_t st) {
    ConvThinInArgs t{a, cw.w, cw.sn, cw.st, cw.sk};
    const long long n_rows = a.d.Q / a.d.W;
    constexpr int PX = 4, NC4 = (PX + KW - 1 + 1) / 2;
    const size_t lds = (size_t)KT * KD * KH * ((a.d.W + PX - 1) / PX * PX + 2 * NC4 - PX) * 2 * sizeof(float);
    const long long cap = 256LL * 8;
    const dim3 grid((unsigned)(n_rows < cap ? n_rows : cap));
    if (bf) hipLaunchKernelGGL((conv_thin_in_kernel<KT, KD, KH, KW, true>), grid, dim3(256), lds, st, t);
    else hipLaunchKernelGGL((conv_thin_in_kernel<KT, KD, KH, KW, false>), grid, dim3(256), lds, st, t);
}

static bool conv_thin_in_applies(const PixDims& d, int K, int Nn) {
    if (!(K == 2 && Nn >= 8 && Nn <= 256)) return false;
    const bool k2 = d.kt == 1 && d.kd == 1 && d.kh == 3 && d.kw == 3, k3 = d.kt == 1 && d.kd == 3 && d.kh == 3 && d.kw == 3;
    const bool kt3 = d.kt == 3 && d.kd == 1 && d.kh == 1 && d.kw == 1;
    return k2 || k3 || kt3;
}

// Launches the two-channel-input kernel when the layer fits it; *hit tells whether it did.
static hipError_t launch_conv_thin_in(const ConvArgs& a, const ConvWeights& cw, bool bf, bool* hit, hipStream_t st) {
    *hit = false;
    const int taps_ = a.d.kt * a.d.kd * a.d.kh * a.d.kw;
    if (!conv_thin_in_applies(a.d, a.K, a.Nn)) return hipSuccess;
    const PixDims& d = a.d;
    const bool k2 = d.kt == 1 && d.kd == 1 && d.kh == 3 && d.kw == 3, k3 = d.kt == 1 && d.kd == 3 && d.kh == 3 && d.kw == 3;
    char name[56];
    snprintf(name, sizeof(name), "conv_%s_%dto%d_t%d", a.flip ? "dgrad" : "fwd", a.K, a.Nn, taps_);
    KernelScope ks(name, 2.0 * (double)a.d.Q * a.K * a.Nn * taps_, (bf ? 2.0 : 4.0) * (double)a.d.Q * a.Nn + 8.0 * (double)a.d.Q, st);
    if (conv_thin_in_mfma_applies(d, a.Nn)) {   // 3x3x3: one MFMA of depth two per tap and 32 output channels
        ThinInMfmaArgs t{};
        t.in = a.in; t.out = a.out; t.bias = a.bias; t.mask_ref = a.mask_ref; t.add = a.add;
        t.w = cw.w; t.sn = cw.sn; t.st = cw.st; t.sk = cw.sk;
        t.Nn = a.Nn; t.flip = a.flip; t.relu_in = a.relu_in; t.relu_out = a.relu_out; t.mask_acc = a.mask_acc; t.mask_add = a.mask_add;
        t.d = d;
        *hit = true;
        return launch_conv_thin_in_mfma(t, bf, st);
    }
    if (k2) launch_conv_thin_in_t<1, 1, 3, 3>(a, cw, bf, st);
    else if (k3) launch_conv_thin_in_t<1, 3, 3, 3>(a, cw, bf, st);
    else launch_conv_thin_in_t<3, 1, 1, 1>(a, cw, bf, st);
    *hit = true;
    return hipGetLastError();
}

template <int KT, int KD, int KH, int KW, int KC>
static void launch_conv_thin_out_k(const ConvThinOutArgs& t, const float* w, bool bf, hipStream_t st) {
    constexpr int RT = KT * KD * KH, PXS = kThinOutPx + KW - 1;
    constexpr size_t lds = ((size_t)RT * PXS * (KC + 4) + 4 * kThinOutPx * 2) * sizeof(float);
    const long long n_tiles = (t.d.Q / t.d.W) * ((t.d.W + kThinOutPx - 1) / kThinOutPx);
    const long long cap = 256LL * (lds > 53 * 1024 ? 2 : 3);
    const dim3 grid((unsigned)(((n_tiles < cap ? n_tiles : cap) + 7) / 8 * 8));
    if (bf) hipLaunchKernelGGL((conv_thin_out_kernel<KT, KD, KH, KW, true, KC>), grid, dim3(256), lds, st, t, w);
    else hipLaunchKernelGGL((conv_thin_out_kernel<KT, KD, KH, KW, false, KC>), grid, dim3(256), lds, st, t, w);
}
template <int KT, int KD, int KH, int KW>
static void launch_conv_thin_out_t(const ConvThinOutArgs& t, const float* w, bool bf, hipStream_t st) {
    constexpr int RT = KT * KD * KH;
    if constexpr (RT <= 3) {   // slab of at most 56 KB: 64, 32 or 16 channels per round
        if (t.KC == 64) return launch_conv_thin_out_k<KT, KD, KH, KW, 64>(t, w, bf, st);
        if (t.KC == 32) return launch_conv_thin_out_k<KT, KD, KH, KW, 32>(t, w, bf, st);
    }
    launch_conv_thin_out_k<KT, KD, KH, KW, 16>(t, w, bf, st);
}

// wt[n][tap][k] = w[n*sn + tapidx*st + k*sk] (tapidx mirrored when flip), n < 2: the layout the
// two-channel-output kernel reads, for the data gradient of a layer whose INPUT is the 2-channel image.
// round_bf: the values are rounded to bfloat16 (kept as float32), for the kernels that multiply bfloat16 data
// with float32 arithmetic: weights that meet bfloat16 data are bfloat16 values in every kernel.
__global__ void thin_out_weights_kernel(const float* __restrict__ w, long long sn, long long st_, long long sk, int flip,
                                        int taps, int K, int round_bf, float* __restrict__ wt) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= 2 * taps * K) return;
    const int k = i % K, tap = (i / K) % taps, n = i / (K * taps);
    const int tapidx = flip ? taps - 1 - tap : tap;
    const float v = w[n * sn + tapidx * st_ + k * sk];
    wt[i] = round_bf ? bf16_to_f32(f32_to_bf16(v)) : v;
}

// Launches the two-channel-output kernel when the layer fits it; *hit tells whether it did.  The forward
// pass reads theta's own layout; other weight layouts (the data gradient into the image) are re-laid into
// wt_scratch first.  `in` is bfloat16 when bf.
static hipError_t launch_conv_thin_out(const ConvArgs& a, const ConvWeights& cw, bool bf, float* wt_scratch, bool* hit,
                                       hipStream_t st) {
    *hit = false;
    const PixDims& d = a.d;
    const int taps_ = d.kt * d.kd * d.kh * d.kw;
    if (!(a.Nn == 2 && a.K >= 16 && a.K % 16 == 0 && !a.mask_ref)) return hipSuccess;
    const bool in_place = !a.flip && cw.sk == 1 && cw.st == a.K && cw.sn == (long long)taps_ * a.K;
    // bfloat16 data: the matrix-core kernel packs its weights to bfloat16 itself; the lane-per-pixel kernel computes
    // in float32 and gets a rounded copy, so that the result does not depend on which of the two runs
    const bool round_copy = bf && !conv_thin_out_mfma_applies(a.d, a.K, bf);
    const bool direct = in_place && !round_copy;
    if (!direct && wt_scratch == nullptr) return hipSuccess;
    const bool k2 = d.kt == 1 && d.kd == 1 && d.kh == 3 && d.kw == 3, k3 = d.kt == 1 && d.kd == 3 && d.kh == 3 && d.kw == 3;
    const bool kt3 = d.kt == 3 && d.kd == 1 && d.kh == 1 && d.kw == 1;
    if (!k2 && !k3 && !kt3) return hipSuccess;
    const int rt = taps_ / d.kw;
    if ((double)(d.kt / 2 + 1) * d.D * d.H * d.W * a.K * 4.0 >= 2147483648.0) return hipSuccess;   // 32-bit tap offsets
    const int kc = rt > 3 ? 16 : (a.K % 64 == 0 ? 64 : (a.K % 32 == 0 ? 32 : 16));   // channels per round
    ConvThinOutArgs t{};
    t.in = a.in; t.bias = a.bias; t.add = a.add; t.out = a.out;
    t.K = a.K; t.KC = kc; t.relu_in = a.relu_in; t.relu_out = a.relu_out; t.d = d;
    const float* wts = cw.w;
    if (!direct) {
        const int n = 2 * taps_ * a.K;
        hipLaunchKernelGGL(thin_out_weights_kernel, dim3((n + 255) / 256), dim3(256), 0, st, cw.w, cw.sn, cw.st, cw.sk, a.flip,
                           taps_, a.K, round_copy ? 1 : 0, wt_scratch);
        wts = wt_scratch;
    }
    char name[56];
    snprintf(name, sizeof(name), "conv_%s_%dto%d_t%d", a.flip ? "dgrad" : "fwd", a.K, a.Nn, taps_);
    KernelScope ks(name, 2.0 * (double)d.Q * a.K * a.Nn * taps_, (bf ? 2.0 : 4.0) * (double)d.Q * a.K + 8.0 * (double)d.Q, st);
    if (conv_thin_out_mfma_applies(d, a.K, bf)) {   // 3x3 in the plane: dense product on the matrix cores + shifted sum
        *hit = true;
        return launch_conv_thin_out_mfma(a.in, wts, a.bias, a.add, a.out, a.K, a.relu_in, a.relu_out, d, bf, st);
    }
    if (k2) launch_conv_thin_out_t<1, 1, 3, 3>(t, wts, bf, st);
    else if (k3) launch_conv_thin_out_t<1, 3, 3, 3>(t, wts, bf, st);
    else launch_conv_thin_out_t<3, 1, 1, 1>(t, wts, bf, st);
    *hit = true;
    return hipGetLastError();
}

static hipError_t launch_conv(ConvArgs a, const ConvWeights& cw, float* wt_scratch, hipStream_t st, const float* wino_u = nullptr) {
    const int taps_ = a.d.kt * a.d.kd * a.d.kh * a.d.kw;
    {   // two input channels and a wide output: HBM-bound kernels (matrix cores for 3x3x3 taps, vector ALUs otherwise)
        bool hit = false;
        const hipError_t e = launch_conv_thin_in(a, cw, false, &hit, st);
        if (hit || e != hipSuccess) return e;
    }
    {   // two output channels and a wide input (forward): HBM-bound kernels (prox_thin.hip where it has the shape)
        bool hit = false;
        const hipError_t e = launch_conv_thin_out(a, cw, false, wt_scratch, &hit, st);
        if (hit || e != hipSuccess) return e;
    }
    if (wino_enabled() && conv_wino_applies(a.d, a.K, a.Nn)) {   // 3x3 in the plane: Winograd F(2x2, 3x3)
        WinoArgs wa{};
        wa.in = a.in; wa.out = a.out; wa.bias = a.bias; wa.mask_ref = a.mask_ref; wa.add = a.add;
        wa.bits_in = a.bits_in; wa.bits_out = a.bits_out;
        wa.K = a.K; wa.Nn = a.Nn; wa.relu_out = a.relu_out; wa.mask_acc = a.mask_acc; wa.mask_add = a.mask_add;
        wa.H = a.d.H; wa.W = a.d.W; wa.NI = a.d.Q / ((long long)a.d.H * a.d.W);
        char name[56];
        snprintf(name, sizeof(name), "conv_%s_%dto%d_t%d", a.flip ? "dgrad" : "fwd", a.K, a.Nn, taps_);
        return launch_conv_wino(wa, cw.w, cw.sn, cw.st, cw.sk, a.flip, a.relu_in, wt_scratch, wino_u, name, st);
    }
    if (wino_enabled() && conv_wino3_applies(a.d, a.K, a.Nn)) {   // 3x3x3: Winograd in the slice, depth taps summed
        WinoArgs wa{};
        wa.in = a.in; wa.out = a.out; wa.bias = a.bias; wa.mask_ref = a.mask_ref; wa.add = a.add;
        wa.K = a.K; wa.Nn = a.Nn; wa.relu_out = a.relu_out; wa.mask_acc = a.mask_acc; wa.mask_add = a.mask_add;
        wa.H = a.d.H; wa.W = a.d.W; wa.D = a.d.D; wa.NI = a.d.Q / ((long long)a.d.H * a.d.W);
        char name[56];
        snprintf(name, sizeof(name), "conv_%s_%dto%d_t%d", a.flip ? "dgrad" : "fwd", a.K, a.Nn, taps_);
        return launch_conv_wino3(wa, cw.w, cw.sn, cw.st, cw.sk, a.flip, a.relu_in, wt_scratch, name, st);
    }
    if (!(kernel_policy() & GLEAM_POLICY_NO_FRAME_WALK) && conv_time_applies(a.d, a.K, a.Nn)) {   // temporal 3x1x1: walk along the frames
        TimeConvArgs t{};
        t.in = a.in; t.out = a.out; t.bias = a.bias; t.mask_ref = a.mask_ref; t.add = a.add;
        t.w = cw.w; t.sn = cw.sn; t.st = cw.st; t.sk = cw.sk; t.flip = a.flip;
        t.Nn = a.Nn; t.relu_in = a.relu_in; t.relu_out = a.relu_out; t.mask_acc = a.mask_acc; t.mask_add = a.mask_add;
        char name[56];
        snprintf(name, sizeof(name), "conv_%s_%dto%d_t%d", a.flip ? "dgrad" : "fwd", a.K, a.Nn, taps_);
        KernelScope ks(name, 2.0 * (double)a.d.Q * a.K * a.Nn * taps_, 4.0 * (double)a.d.Q * (a.K + a.Nn), st);
        return launch_conv_time(t, a.d, st);
    }
    const int ck = conv_ck(a.K), nb = conv_nb(a.Nn);
    {
        WimgArgs t{};
        t.w = cw.w; t.wt = wt_scratch; t.sn = cw.sn; t.st = cw.st; t.sk = cw.sk;
        t.K = a.K; t.Nn = a.Nn; t.flip = a.flip; t.taps = taps_; t.kw = a.d.kw; t.CK = ck; t.NB = nb;
        t.n_kc = (a.K + ck - 1) / ck; t.n_nb = (a.Nn + nb - 1) / nb;
        t.total = (long long)conv_wimg_floats(a.K, a.Nn, taps_);
        KernelScope ks("weights_image", 0.0, 8.0 * (double)t.total, st);
        hipLaunchKernelGGL(weights_image_kernel, dim3((unsigned)((t.total + 255) / 256)), dim3(256), 0, st, t);
    }
    a.wt = wt_scratch;
    char name[56];
    snprintf(name, sizeof(name), "conv_%s_%dto%d_t%d", a.flip ? "dgrad" : "fwd", a.K, a.Nn, taps_);
    KernelScope ks(name, 2.0 * (double)a.d.Q * a.K * a.Nn * taps_, 4.0 * (double)a.d.Q * (a.K + a.Nn), st);
    if (nb == 32) return ck == 8 ? launch_conv_t<32, 8>(a, st) : launch_conv_t<32, 16>(a, st);
    return ck == 8 ? launch_conv_t<64, 8>(a, st) : launch_conv_t<64, 16>(a, st);
}

// ------------------------------------------------------------------ weight gradient
struct WgradArgs {
    const float* g;    // [Q][Co]  gradient at the conv output (already ReLU-masked)
    const float* a;    // [Q][Ci]  conv input before its optional ReLU
    float* partial;    // [n_split][Co][taps][Ci]
    int Co, Ci, relu_in;
    PixDims d;
};

constexpr int kWgTM = 32;  // pixels per staged chunk
constexpr int kThinSplit = 1024;  // most partial sums the thin weight-gradient kernel writes

template <int JT>
__global__ __launch_bounds__(kConvThreads) void wgrad_mfma_kernel(WgradArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const PixDims d = a.d;
    const int RSg = (a.Co + 3) / 4 * 4 + 1, RSa = (a.Ci + 3) / 4 * 4 + 1;
    const int rowtaps = d.kt * d.kd * d.kh, taps = rowtaps * d.kw;
    const int n_pa = kWgTM + d.kw - 1;
    float* gs = smem;                          // [kWgTM][RSg]
    float* as = gs + kWgTM * RSg;              // [rowtaps][n_pa][RSa]
    unsigned* vmask = reinterpret_cast<unsigned*>(as + rowtaps * n_pa * RSa);  // [kWgTM]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, m = lane & 31, h = lane >> 5;
    const int ncb = (a.Co + 31) / 32, nib = (a.Ci + 31) / 32, tapgroups = (taps + JT - 1) / JT;
    const int job = blockIdx.y * 4 + wave;
    const bool active = job < ncb * nib * tapgroups;
    const int tg = job % tapgroups, pair = job / tapgroups;
    const int cb = pair / nib, ib = pair % nib;
    const int tap0 = tg * JT;

    floatx16 acc[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    const long long n_chunks = (d.Q + kWgTM - 1) / kWgTM;
    for (long long chunk = blockIdx.x; chunk < n_chunks; chunk += gridDim.x) {
        const long long q0 = chunk * kWgTM;
        __syncthreads();
        for (int v = threadIdx.x; v < kWgTM * a.Co; v += kConvThreads) {
            const int p = v / a.Co, c = v % a.Co;
            const long long qq = q0 + p;
            gs[p * RSg + c] = qq < d.Q ? a.g[qq * a.Co + c] : 0.f;
        }
        for (int rt = 0; rt < rowtaps; ++rt) {
            const long long qs = q0 + rowtap_offset(rt, d) - d.kw / 2;
            float* dst = as + rt * n_pa * RSa;
            for (int v = threadIdx.x; v < n_pa * a.Ci; v += kConvThreads) {
                const int p = v / a.Ci, c = v % a.Ci;
                const long long qq = qs + p;
                float val = (qq >= 0 && qq < d.Q) ? a.a[qq * a.Ci + c] : 0.f;
                if (a.relu_in) val = fmaxf(val, 0.f);
                dst[p * RSa + c] = val;
            }
        }
        if (threadIdx.x < kWgTM) vmask[threadIdx.x] = tap_validity(q0 + threadIdx.x, d);
        __syncthreads();
        if (active) {
            // channels / taps beyond the layer read a clamped address; their sums are never stored
            const int co_c = cb * 32 + m < a.Co ? cb * 32 + m : a.Co - 1;
            const int ci_c = ib * 32 + m < a.Ci ? ib * 32 + m : a.Ci - 1;
#pragma unroll 4
            for (int s = 0; s < kWgTM / 2; ++s) {
                const int p = 2 * s + h;
                const float av = gs[p * RSg + co_c];
                const unsigned vm = vmask[p];
                float bv[JT];
#pragma unroll
                for (int j = 0; j < JT; ++j) {
                    const int tap = tap0 + j < taps ? tap0 + j : taps - 1;
                    const int rt = tap / d.kw, dw = tap % d.kw;
                    bv[j] = as[(rt * n_pa + p + dw) * RSa + ci_c];
                }
#pragma unroll
                for (int j = 0; j < JT; ++j) {
                    const int tap = tap0 + j < taps ? tap0 + j : taps - 1;
                    const float b = ((vm >> tap) & 1u) ? bv[j] : 0.f;
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b, acc[j], 0, 0, 0);
                }
            }
        }
    }
    if (active) {
        float* dst = a.partial + (size_t)blockIdx.x * a.Co * taps * a.Ci;
        const int ci = ib * 32 + m;
#pragma unroll
        for (int j = 0; j < JT; ++j) {
            const int tap = tap0 + j;
            if (tap >= taps || ci >= a.Ci) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int co = cb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (co < a.Co) dst[((size_t)co * taps + tap) * a.Ci + ci] = acc[j][r];
            }
        }
    }
}

// Pipelined weight gradient for channel counts that are multiples of 4: the next 32-pixel chunk is
// fetched into registers (float4) while the MFMAs of the current chunk run from LDS, so global latency
// hides behind the matrix pipe.  Same job layout as wgrad_mfma_kernel.  Optionally accumulates the bias
// gradient (column sums of g) from the values it stages anyway.
struct WgradPipeArgs {
    WgradArgs w;
    float* bias_partial;  // [n_split][Co] or null
};

// BAL (one 32x32 channel block, more taps than waves): the taps are dealt to all NW waves in runs whose lengths
// differ by at most one, longest first, so that the waves sharing a SIMD (w and w + 4) carry nearly the same
// number of MFMAs; JT is then the longest run.
template <int JT, int PG, int PA, int NW, bool BAL = false>
__global__ __launch_bounds__(NW * 64) void wgrad_pipe_kernel(WgradPipeArgs pa) {
    constexpr int NT = NW * 64;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const WgradArgs& a = pa.w;
    const PixDims d = a.d;
    const int Co4 = a.Co / 4, Ci4 = a.Ci / 4;
    const int RSg = a.Co + 4, RSa = a.Ci + 4;
    const int rowtaps = d.kt * d.kd * d.kh, taps = rowtaps * d.kw;
    const int n_pa = kWgTM + d.kw - 1;
    float* gs = smem;                          // [kWgTM][RSg]
    float* as = gs + kWgTM * RSg;              // [rowtaps][n_pa][RSa]
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, m = lane & 31, h = lane >> 5;
    const int ncb = (a.Co + 31) / 32, nib = (a.Ci + 31) / 32, tapgroups = (taps + JT - 1) / JT;
    const int job = blockIdx.y * NW + wave;
    const bool active = BAL || job < ncb * nib * tapgroups;
    const int tg = job % tapgroups, pair = job / tapgroups;
    const int cb = BAL ? 0 : pair / nib, ib = BAL ? 0 : pair % nib;
    const int bal_base = taps / NW, bal_extra = taps % NW;
    const int tap0 = BAL ? wave * bal_base + (wave < bal_extra ? wave : bal_extra) : tg * JT;
    const int n_my = BAL ? bal_base + (wave < bal_extra ? 1 : 0) : JT;   // taps of this wave (uniform per wave)
    const int n_g4 = kWgTM * Co4, n_a4 = rowtaps * n_pa * Ci4;

    // Per-thread staging descriptors: the float4 slots this thread moves are the same for every chunk.
    int g_lds[PG], g_dq[PG], g_c[PG];
    int a_lds[PA], a_dq[PA], a_c[PA], a_px[PA];
    unsigned a_rt[PA];
#pragma unroll
    for (int i = 0; i < PG; ++i) {
        const int v = tid + i * NT;
        const int p = v / Co4, c4 = v % Co4;
        g_lds[i] = v < n_g4 ? p * RSg + 4 * c4 : -1;
        g_dq[i] = p;
        g_c[i] = p * a.Co + 4 * c4;   // element offset from the chunk's first pixel
    }
#pragma unroll
    for (int i = 0; i < PA; ++i) {
        const int v = tid + i * NT;
        const int rt = v / (n_pa * Ci4), r = v % (n_pa * Ci4);
        const int p = r / Ci4, c4 = r % Ci4;
        a_lds[i] = v < n_a4 ? (rt * n_pa + p) * RSa + 4 * c4 : -1;
        a_dq[i] = v < n_a4 ? (int)rowtap_offset(rt, d) - d.kw / 2 + p : 0;
        a_c[i] = a_dq[i] * a.Ci + 4 * c4;   // element offset from the chunk's first pixel (may be negative)
        a_px[i] = p - d.kw / 2;
        a_rt[i] = v < n_a4 ? 1u << rt : 0u;
    }
    float4 rg[PG], ra[PA], bsum[PG];
#pragma unroll
    for (int i = 0; i < PG; ++i) bsum[i] = make_float4(0.f, 0.f, 0.f, 0.f);

    // Prefetch loads are unconditional (clamped addresses); validity and ReLU are applied at the LDS
    // store, so nothing between the loads waits on memory.
    unsigned g_okb = 0u, a_okb = 0u;
    // A chunk is a 32-pixel segment of one image row (the last segment of a row may be ragged).  Pixels
    // past the end of the row get g = 0, and slab entries outside the grid (row taps above / below the
    // image, the halo columns left / right of it) are stored as 0, so the MFMA loop needs no masks.
    const int segs = (d.W + kWgTM - 1) / kWgTM;
    // (segment, row, slice, frame) of the chunk to fetch, advanced chunk by chunk without divisions
    PixDims cd = d;
    cd.W = segs;
    PixCoord cc{0, 0, 0, 0}, cstep{0, 0, 0, 0};
    long long crow = 0, rstep = 0;   // image row of that chunk, whole rows per step
    auto fetch = [&]() {
        const long long row = crow;
        const int w0 = cc.w * kWgTM;
        const int hh = cc.h, dd = cc.dd, tt = cc.t;
        unsigned rows_ok = 0u;
        {
            int rt = 0;
            for (int it = 0; it < d.kt; ++it)
                for (int id = 0; id < d.kd; ++id)
                    for (int ih = 0; ih < d.kh; ++ih, ++rt) {
                        const bool v = (unsigned)(tt + it - d.kt / 2) < (unsigned)d.T && (unsigned)(dd + id - d.kd / 2) < (unsigned)d.D &&
                                       (unsigned)(hh + ih - d.kh / 2) < (unsigned)d.H;
                        rows_ok |= (v ? 1u : 0u) << rt;
                    }
        }
        crow += rstep + (cc.w + cstep.w >= segs ? 1 : 0);
        pix_advance(cc, cstep, cd);
        const long long q0 = row * d.W + w0;
        const float* gbase = a.g + q0 * a.Co;   // uniform; per-slot offsets are 32-bit constants
        const float* abase = a.a + q0 * a.Ci;
        g_okb = 0u;
        a_okb = 0u;
#pragma unroll
        for (int i = 0; i < PG; ++i) {
            const bool ok = g_lds[i] >= 0 && w0 + g_dq[i] < d.W;
            rg[i] = *reinterpret_cast<const float4*>(ok ? gbase + g_c[i] : a.g);
            g_okb |= (ok ? 1u : 0u) << i;
        }
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const bool ok = (rows_ok & a_rt[i]) != 0u && (unsigned)(w0 + a_px[i]) < (unsigned)d.W;
            ra[i] = *reinterpret_cast<const float4*>(ok ? abase + a_c[i] : a.a);
            a_okb |= (ok ? 1u : 0u) << i;
        }
    };
    // masks and ReLU work on the bit patterns (integer max with 0 is ReLU): every ordinary vector
    // instruction saved here is an issue slot returned to the MFMAs
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < PG; ++i) {
            const int mk = -(int)((g_okb >> i) & 1u);
            float4 v = rg[i];
            v.x = __int_as_float(__float_as_int(v.x) & mk); v.y = __int_as_float(__float_as_int(v.y) & mk);
            v.z = __int_as_float(__float_as_int(v.z) & mk); v.w = __int_as_float(__float_as_int(v.w) & mk);
            if (g_lds[i] >= 0) *reinterpret_cast<float4*>(gs + g_lds[i]) = v;
            if (pa.bias_partial != nullptr) {
                bsum[i].x += v.x; bsum[i].y += v.y; bsum[i].z += v.z; bsum[i].w += v.w;
            }
        }
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const int mk = -(int)((a_okb >> i) & 1u);
            int x0 = __float_as_int(ra[i].x), x1 = __float_as_int(ra[i].y), x2 = __float_as_int(ra[i].z), x3 = __float_as_int(ra[i].w);
            if (a.relu_in) {
                x0 = x0 > 0 ? x0 : 0; x1 = x1 > 0 ? x1 : 0; x2 = x2 > 0 ? x2 : 0; x3 = x3 > 0 ? x3 : 0;
            }
            if (a_lds[i] >= 0)
                *reinterpret_cast<float4*>(as + a_lds[i]) = make_float4(__int_as_float(x0 & mk), __int_as_float(x1 & mk),
                                                                        __int_as_float(x2 & mk), __int_as_float(x3 & mk));
        }
    };

    floatx16 acc[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    // Per-lane LDS read bases.  Channels and taps beyond the layer are clamped to a valid address:
    // what they accumulate lands in rows / columns / taps that are never stored, so no value masking
    // (and no branch) is needed in the loop.
    const int co = cb * 32 + m, ci = ib * 32 + m;
    const int co_c = co < a.Co ? co : a.Co - 1, ci_c = ci < a.Ci ? ci : a.Ci - 1;
    int b_off[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j) {
        const int tap = tap0 + j < taps ? tap0 + j : taps - 1;
        const int rt = tap / d.kw, dw = tap % d.kw;
        b_off[j] = (rt * n_pa + dw + h) * RSa + ci_c;
    }
    const int a_off = h * RSg + co_c;

    const long long n_chunks = (d.Q / d.W) * segs;
    const XcdRange xr = xcd_range(n_chunks);
    long long chunk = xr.first;
    if (chunk < xr.end) {
        cc = pix_coord(chunk, cd);
        cstep = pix_coord(xr.stride, cd);
        crow = chunk / segs;
        rstep = xr.stride / segs;
        fetch();
        stash();
    }
    __syncthreads();
    for (; chunk < xr.end; chunk += xr.stride) {
        const long long next = chunk + xr.stride;
        if (next < xr.end) fetch();
        if (active) {
            // software pipeline over the 2-pixel K-steps: operands of step s+1 are read from LDS
            // before the MFMAs of step s are issued
            float av = gs[a_off];
            float bv[JT];
#pragma unroll
            for (int j = 0; j < JT; ++j) bv[j] = as[b_off[j]];
#pragma unroll 2
            for (int s = 0; s < kWgTM / 2; ++s) {
                const int sn = s + 1 < kWgTM / 2 ? s + 1 : s;
                const float av_n = gs[a_off + 2 * sn * RSg];
                float bv_n[JT];
#pragma unroll
                for (int j = 0; j < JT; ++j) bv_n[j] = as[b_off[j] + 2 * sn * RSa];
#pragma unroll
                for (int j = 0; j < JT; ++j)
                    if (!BAL || j < JT - 1 || n_my == JT) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[j], acc[j], 0, 0, 0);
                av = av_n;
#pragma unroll
                for (int j = 0; j < JT; ++j) bv[j] = bv_n[j];
            }
        }
        __syncthreads();
        if (next < xr.end) stash();
        __syncthreads();
    }
    if (active) {
        float* dst = a.partial + (size_t)blockIdx.x * a.Co * taps * a.Ci;
#pragma unroll
        for (int j = 0; j < JT; ++j) {
            const int tap = tap0 + j;
            if (tap >= taps || j >= n_my || ci >= a.Ci) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int cc = cb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (cc < a.Co) dst[((size_t)cc * taps + tap) * a.Ci + ci] = acc[j][r];
            }
        }
    }
    if (pa.bias_partial != nullptr && blockIdx.y == 0) {
        // thread (tid, i) summed channels g_c[i]..+3 over its pixels; fold the pixel lanes through LDS
        __syncthreads();
        float4* red = reinterpret_cast<float4*>(smem);  // [PG*256] float4 <= staging area
#pragma unroll
        for (int i = 0; i < PG; ++i) red[tid + i * NT] = g_lds[i] >= 0 ? bsum[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        __syncthreads();
        if (tid < a.Co) {
            const int c4 = tid / 4, e = tid % 4;
            float t = 0.f;
            for (int v = c4; v < PG * NT; v += Co4) {
                const float4 x = red[v];
                t += e == 0 ? x.x : (e == 1 ? x.y : (e == 2 ? x.z : x.w));
            }
            pa.bias_partial[(size_t)blockIdx.x * a.Co + tid] = t;
        }
    }
}

// Weight gradient of a layer whose input OR output has very few channels (the 2-channel image side):
// HBM-bound, so no MFMA.  Lanes index the wide channel dimension; the wide tensor is read once per
// pixel (coalesced); the thin tensor's rows around the current image row sit in LDS, zero-filled where
// a tap falls outside the grid, and are read as wave-wide broadcasts - no validity test in the loop.
//   THIN_IN  (cin thin):  dw[co][tap][ci] += g[q][co] * a[q + off(tap)][ci]          lanes = co
//   !THIN_IN (cout thin): dw[co][tap][ci] += a[q'][ci] * g[q' - off(tap)][co]        lanes = ci
struct WgradThinArgs {
    const float* wide;   // [Q][WC]
    const float* thin;   // [Q][TH]
    float* partial;      // [gridDim.x][Co][taps][Ci]
    float* bias_partial; // [gridDim.x][Co] or null
    int WC;              // wide channels (<= 256)
    int relu_in;
    PixDims d;
};

template <int KT, int KD, int KH, int KW, int TH, bool THIN_IN, bool BF>
__global__ __launch_bounds__(256) void wgrad_thin_kernel(WgradThinArgs a) {
    static_assert(TH == 2, "the thin side is the 2-channel image");
    constexpr int RT = KT * KD * KH, TAPS = RT * KW, PX = 4;   // PX pixels per lane and step
    constexpr int NC4 = (PX + KW - 1 + 1) / 2;                  // float4 (2 pixels x 2 channels) per row tap
    constexpr int sgn = THIN_IN ? 1 : -1;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const PixDims d = a.d;
    const int WS = (d.W + PX - 1) / PX * PX + 2 * NC4 - PX;   // slab columns: image columns -KW/2 .., zero past the row
    float* slab = smem;                     // [RT][WS][TH]
    float* red = smem + RT * WS * TH;       // [256]
    const int WCr = a.WC <= 32 ? 32 : (a.WC <= 64 ? 64 : (a.WC <= 128 ? 128 : 256));
    const int groups = 256 / WCr;
    const int c = threadIdx.x % WCr;
    const int pg = threadIdx.x / WCr;
    const bool c_ok = c < a.WC;
    const long long n_rows = d.Q / d.W;

    float acc[TAPS][TH];
    float bs[THIN_IN ? 1 : TH];
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int e = 0; e < TH; ++e) acc[t][e] = 0.f;
#pragma unroll
    for (int e = 0; e < (THIN_IN ? 1 : TH); ++e) bs[e] = 0.f;

    for (long long row = blockIdx.x; row < n_rows; row += gridDim.x) {
        long long r = row;
        const int hh = (int)(r % d.H);
        r /= d.H;
        const int dd = (int)(r % d.D);
        r /= d.D;
        const int tt = (int)(r % d.T);
        __syncthreads();
        // stage the RT thin rows: all loads of a pass are issued (clamped addresses) before any LDS store
        for (int j0 = 0; j0 < WS; j0 += 256) {
            const int j = j0 + threadIdx.x, col = j - KW / 2;
            float2 v[RT];
            bool ok[RT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const int ih = rt % KH, id = (rt / KH) % KD, it = rt / (KH * KD);
                const int ot = sgn * (it - KT / 2), od = sgn * (id - KD / 2), oh = sgn * (ih - KH / 2);
                const bool row_ok = tt + ot >= 0 && tt + ot < d.T && dd + od >= 0 && dd + od < d.D && hh + oh >= 0 && hh + oh < d.H;
                const long long src_row = row + ((long long)ot * d.D + od) * d.H + oh;
                ok[rt] = row_ok && col >= 0 && col < d.W;
                v[rt] = *reinterpret_cast<const float2*>(a.thin + (ok[rt] ? (src_row * d.W + col) * TH : 0));
            }
            if (j < WS) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    float2 x = make_float2(ok[rt] ? v[rt].x : 0.f, ok[rt] ? v[rt].y : 0.f);
                    if (THIN_IN && a.relu_in) x = make_float2(fmaxf(x.x, 0.f), fmaxf(x.y, 0.f));
                    *reinterpret_cast<float2*>(slab + (rt * WS + j) * TH) = x;
                }
            }
        }
        __syncthreads();
        // each lane: one wide channel, PX consecutive pixels per step (their loads are issued together)
        for (int w = pg * PX; w < d.W; w += groups * PX) {
            float wv[PX];
#pragma unroll
            for (int p = 0; p < PX; ++p) {
                const bool ok = c_ok && w + p < d.W;
                const long long o = ok ? (row * d.W + w + p) * a.WC + c : 0;
                const float x = BF ? bf16_to_f32(reinterpret_cast<const unsigned short*>(a.wide)[o]) : a.wide[o];
                wv[p] = ok ? x : 0.f;
            }
            if (!THIN_IN && a.relu_in) {
#pragma unroll
                for (int p = 0; p < PX; ++p) wv[p] = fmaxf(wv[p], 0.f);
            }
            if (THIN_IN) {
#pragma unroll
                for (int p = 0; p < PX; ++p) bs[0] += wv[p];
            }
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                float col[2 * NC4][TH];
#pragma unroll
                for (int c4 = 0; c4 < NC4; ++c4) {
                    const float4 v = *reinterpret_cast<const float4*>(slab + (rt * WS + w + 2 * c4) * TH);
                    col[2 * c4][0] = v.x; col[2 * c4][1] = v.y; col[2 * c4 + 1][0] = v.z; col[2 * c4 + 1][1] = v.w;
                }
#pragma unroll
                for (int iw = 0; iw < KW; ++iw)
#pragma unroll
                    for (int p = 0; p < PX; ++p)
#pragma unroll
                        for (int e = 0; e < TH; ++e)
                            acc[rt * KW + iw][e] = fmaf(wv[p], col[p + (THIN_IN ? iw : KW - 1 - iw)][e], acc[rt * KW + iw][e]);
                if (!THIN_IN && rt == RT / 2) {   // centre tap = the pixel itself: bias gradient of the thin side
#pragma unroll
                    for (int p = 0; p < PX; ++p)
#pragma unroll
                        for (int e = 0; e < TH; ++e) bs[e] += col[p + KW / 2][e];
                }
            }
        }
    }
    // fold the pixel groups of this workgroup, then write the partial in dw layout
    const int Co = THIN_IN ? a.WC : TH, Ci = THIN_IN ? TH : a.WC;
    float* dst = a.partial + (size_t)blockIdx.x * Co * TAPS * Ci;
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int e = 0; e < TH; ++e) {
            __syncthreads();
            red[threadIdx.x] = acc[t][e];
            __syncthreads();
            if (pg == 0 && c_ok) {
                float sum = 0.f;
                for (int g2 = 0; g2 < groups; ++g2) sum += red[g2 * WCr + c];
                const size_t o = THIN_IN ? ((size_t)c * TAPS + t) * Ci + e : ((size_t)e * TAPS + t) * Ci + c;
                dst[o] = sum;
            }
        }
    if (a.bias_partial != nullptr) {
#pragma unroll
        for (int e = 0; e < (THIN_IN ? 1 : TH); ++e) {
            __syncthreads();
            red[threadIdx.x] = bs[e];
            __syncthreads();
            if (THIN_IN) {
                if (pg == 0 && c_ok) {
                    float sum = 0.f;
                    for (int g2 = 0; g2 < groups; ++g2) sum += red[g2 * WCr + c];
                    a.bias_partial[(size_t)blockIdx.x * Co + c] = sum;
                }
            } else if (threadIdx.x == 0) {
                float sum = 0.f;
                for (int g2 = 0; g2 < groups; ++g2) sum += red[g2 * WCr];
                a.bias_partial[(size_t)blockIdx.x * Co + e] = sum;
            }
        }
    }
}

// out[i] = sum_s partial[s][i] in a fixed order (run-to-run identical bits).  Two segments in one launch:
// the weight-gradient partials (n elements, blocks [0, nbw)) and, when n2 > 0, the bias-gradient partials.
// A block of 256 threads is 16 split groups x 16 lanes: group g sums its contiguous sixteenth of the
// partials (several loads in flight per thread), the 16 group sums are then added in ascending order.
// VEC = 4 (weights only, when n % 4 == 0 and `out` is 16-byte aligned) moves float4 per lane.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, int n_split, long long n,
                                                              float* __restrict__ out, int vec, int nbw,
                                                              const float* __restrict__ partial2, long long n2,
                                                              float* __restrict__ out2) {
    __shared__ float4 red[16][16];
    const int lane = threadIdx.x & 15, sg = threadIdx.x >> 4;
    const int per = (n_split + 15) / 16;
    const int k0 = sg * per, k1 = k0 + per < n_split ? k0 + per : n_split;
    const bool first = (int)blockIdx.x < nbw;
    const float* src = first ? partial : partial2;
    float* dst = first ? out : out2;
    const long long stride = first ? n : n2;
    const int width = (first && vec) ? 4 : 1;
    const long long i = ((long long)(first ? blockIdx.x : blockIdx.x - nbw) * 16 + lane) * width;
    const bool ok = i < stride;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (ok) {
        if (width == 4) {
            int k = k0;
            for (; k + 4 <= k1; k += 4) {
                float4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(src + (size_t)(k + u) * stride + i);
#pragma unroll
                for (int u = 0; u < 4; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
            }
            for (; k < k1; ++k) {
                const float4 v = *reinterpret_cast<const float4*>(src + (size_t)k * stride + i);
                s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
            }
        } else {
            int k = k0;
            for (; k + 4 <= k1; k += 4) {
                float v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = src[(size_t)(k + u) * stride + i];
#pragma unroll
                for (int u = 0; u < 4; ++u) s.x += v[u];
            }
            for (; k < k1; ++k) s.x += src[(size_t)k * stride + i];
        }
    }
    red[sg][lane] = s;
    __syncthreads();
    if (sg == 0 && ok) {
        float4 t = red[0][lane];
#pragma unroll
        for (int g2 = 1; g2 < 16; ++g2) {
            const float4 v = red[g2][lane];
            t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
        }
        if (width == 4) *reinterpret_cast<float4*>(dst + i) = t;
        else dst[i] = t.x;
    }
}

// partial[blk][c] = sum over this workgroup's pixels of g[q][c]  (bias gradient).
__global__ __launch_bounds__(256) void colsum_kernel(const float* __restrict__ g, long long Q, int C, float* __restrict__ partial) {
    __shared__ float red[256];
    const int per = 256 / C > 0 ? 256 / C : 1;  // pixel lanes per channel (C <= 256 here)
    const int c = threadIdx.x % C, lane = threadIdx.x / C;
    float s = 0.f;
    if (lane < per) {
        for (long long q = (long long)blockIdx.x * per + lane; q < Q; q += (long long)gridDim.x * per) s += g[q * C + c];
    }
    red[threadIdx.x] = (lane < per) ? s : 0.f;
    __syncthreads();
    if (threadIdx.x < C) {
        float t = 0.f;
        for (int l = 0; l < per; ++l) t += red[l * C + threadIdx.x];
        partial[(size_t)blockIdx.x * C + threadIdx.x] = t;
    }
}

// ------------------------------------------------------------------ loss
// part[blk] = sum over this workgroup's pixels of |z-x|^2 (kind 0) or |z-x| (kind 1); gz = dL/dz.
__global__ __launch_bounds__(256) void loss_kernel(const float2* __restrict__ z, const float2* __restrict__ xr, float2* __restrict__ gz,
                                                   long long n, int kind, float inv_n, int relu_mask, double* __restrict__ part) {
    __shared__ double red[256];
    double s = 0.0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
        const float2 zv = z[i], xv = xr[i];
        const float dx = zv.x - xv.x, dy = zv.y - xv.y;
        float2 g;
        if (kind == 0) {
            s += (double)dx * dx + (double)dy * dy;
            g = make_float2(2.f * dx * inv_n, 2.f * dy * inv_n);
        } else {
            const float mag = sqrtf(dx * dx + dy * dy);
            s += (double)mag;
            g = mag > 0.f ? make_float2(dx / mag * inv_n, dy / mag * inv_n) : make_float2(0.f, 0.f);
        }
        if (relu_mask) {  // last layer ended in a ReLU: gradient passes where its output is positive
            g.x = zv.x > 0.f ? g.x : 0.f;
            g.y = zv.y > 0.f ? g.y : 0.f;
        }
        gz[i] = g;
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = red[0];
}

__global__ void loss_final_kernel(const double* __restrict__ part, int n_part, double inv_n, float* __restrict__ loss) {
    __shared__ double red[64];
    double s = 0.0;
    for (int i = threadIdx.x; i < n_part; i += 64) s += part[i];
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int i = 0; i < 64; ++i) t += red[i];
        *loss = (float)(t * inv_n);
    }
}

// part[blk] = partial sum of Re <u, v> (complex values as two reals)
__global__ __launch_bounds__(256) void real_dot_kernel(const float2* __restrict__ u, const float2* __restrict__ v, long long n,
                                                       double* __restrict__ part) {
    __shared__ double red[256];
    double s = 0.0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
        const float2 a = u[i], b = v[i];
        s += (double)a.x * b.x + (double)a.y * b.y;
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = red[0];
}

// ------------------------------------------------------------------ host side
static inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }
constexpr int kLossBlocks = kLossPartials;

hipError_t loss_and_grad(const float2* x, const float2* x_ref, float2* g, long long n, int loss_kind, int relu_mask,
                         double* part, float* loss, hipStream_t st) {
    KernelScope ks("loss", 0.0, 24.0 * (double)n, st);
    hipLaunchKernelGGL(loss_kernel, dim3(kLossBlocks), dim3(256), 0, st, x, x_ref, g, n, loss_kind, (float)(1.0 / (double)n),
                       relu_mask, part);
    hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(64), 0, st, (const double*)part, kLossBlocks, 1.0 / (double)n, loss);
    return hipGetLastError();
}

hipError_t real_dot(const float2* u, const float2* v, long long n, double scale, double* part, float* out, hipStream_t st) {
    KernelScope ks("real_dot", 0.0, 16.0 * (double)n, st);
    hipLaunchKernelGGL(real_dot_kernel, dim3(kLossBlocks), dim3(256), 0, st, u, v, n, part);
    hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(64), 0, st, (const double*)part, kLossBlocks, scale, out);
    return hipGetLastError();
}

static PixDims pix_dims(const gleam_geom& g, const gleam_conv& c) {
    PixDims d;
    d.T = (int)g.T; d.D = (int)g.D; d.H = (int)g.H; d.W = (int)g.W;
    d.kt = c.kt; d.kd = c.kd; d.kh = c.kh; d.kw = c.kw;
    d.Q = g.B * g.T * g.D * g.H * g.W;
    return d;
}

// Whether the bfloat16 operand mode has kernels for this network: 2-channel first input and last output
// handled by the thin kernels, every interior channel count a multiple of 8, kernel extent 1 or 3 along W.
bool prox_bf16_supported(const gleam_prox_desc& p) {
    const int L = p.n_layers;
    if (L < 2) return false;
    auto thin_shape = [](const gleam_conv& c) {
        return (c.kt == 1 && c.kd == 1 && c.kh == 3 && c.kw == 3) || (c.kt == 1 && c.kd == 3 && c.kh == 3 && c.kw == 3) ||
               (c.kt == 3 && c.kd == 1 && c.kh == 1 && c.kw == 1);
    };
    auto wide_ok = [](int ch) { return ch >= 8 && ch % 8 == 0 && ch <= 256; };
    for (int l = 0; l < L; ++l) {
        const gleam_conv& c = p.layers[l];
        if (c.kw != 1 && c.kw != 3) return false;
        if (l == 0) {
            if (c.cin != 2 || !wide_ok(c.cout) || !thin_shape(c)) return false;
        } else if (l == L - 1) {
            if (c.cout != 2 || !wide_ok(c.cin) || !thin_shape(c)) return false;
            if (c.skip_src > 0) return false;
        } else {
            if (c.cin % 8 || c.cout % 8) return false;
            if (wgrad_bf16_lds_bytes(c.cout, c.cin, c.kt, c.kd, c.kh, c.kw) > 150 * 1024) return false;
            const int rowtaps = c.kt * c.kd * c.kh;
            if (32 * (c.cout / 8) > 2 * 512 || rowtaps * (32 + c.kw - 1) * (c.cin / 8) > 8 * 512) return false;
        }
    }
    return true;
}

void plan_prox(const gleam_geom& g, const gleam_prox_desc& p, ProxPlan& plan) {
    for (int t = 0; t <= kMaxLayers; ++t) plan.post_relu[t] = false;
    for (int t = 1; t < p.n_layers; ++t) {
        bool ok = p.layers[t].relu_in != 0 && p.layers[t - 1].skip_src < 0;
        for (int l = 0; l < p.n_layers; ++l) ok = ok && p.layers[l].skip_src != t;
        plan.post_relu[t] = ok;
    }
    const int L = p.n_layers;
    plan.L = L;
    plan.Q = g.B * g.T * g.D * g.H * g.W;
    const size_t Q = (size_t)plan.Q;
    const size_t es = p.dtype == 1 ? 2 : 4;   // bytes per element of the interior activations / gradients
    size_t off = 0, th = 0, max_w = 0;
    for (int l = 0; l < L; ++l) {
        const gleam_conv& c = p.layers[l];
        plan.act_off[l] = off;
        off += align256(Q * c.cin * (l == 0 ? sizeof(float) : es));   // t_0 = u is always float32
        plan.w_off[l] = th;
        const size_t nw = (size_t)c.cout * c.kt * c.kd * c.kh * c.kw * c.cin;
        th += nw;
        plan.b_off[l] = th;
        if (c.has_bias) th += c.cout;
        if (nw > max_w) max_w = nw;
    }
    plan.gz_off = off;
    off += align256(Q * 2 * sizeof(float));
    // ReLU masks as sign bits: where both the layer that produces t_l and the data gradient that flows back into
    // it run on the Winograd kernel, the forward launch leaves one bit per value and the backward launch reads
    // those (1/32 of the bytes of t_l)
    for (int l = 0; l <= kMaxLayers; ++l) plan.sign_off[l] = 0;
    if (p.dtype == 1)   // the same between two launches of the two-dimensional-tile bfloat16 kernel
        for (int l = 2; l + 1 < L; ++l) {   // t_1 comes from, and the gradient into t_{L-1} goes through, the thin kernels
            const gleam_conv& below = p.layers[l - 1];
            const gleam_conv& above = p.layers[l];
            if (!(above.relu_in || below.relu_out)) continue;
            PixDims db{}, da{};
            db.T = da.T = (int)g.T; db.D = da.D = (int)g.D; db.H = da.H = (int)g.H; db.W = da.W = (int)g.W;
            db.Q = da.Q = plan.Q;
            db.kt = below.kt; db.kd = below.kd; db.kh = below.kh; db.kw = below.kw;
            da.kt = above.kt; da.kd = above.kd; da.kh = above.kh; da.kw = above.kw;
            // the launch that writes the words and the one that reads them must be the same kernel (same tile geometry)
            const int variant = conv_bf16_takes_sign_words(db, below.cin, below.cout);
            if (variant == 0 || variant != conv_bf16_takes_sign_words(da, above.cout, above.cin)) continue;
            plan.sign_off[l] = off;
            off += align256(conv_bf16_sign_words(db, below.cout, variant) * sizeof(unsigned));
        }
    if (p.dtype == 0)
        for (int l = 1; l < L; ++l) {
            const gleam_conv& below = p.layers[l - 1];
            const gleam_conv& above = p.layers[l];
            if (!(above.relu_in || below.relu_out)) continue;
            PixDims db{}, da{};
            db.T = da.T = (int)g.T; db.D = da.D = (int)g.D; db.H = da.H = (int)g.H; db.W = da.W = (int)g.W;
            db.Q = da.Q = plan.Q;
            db.kt = below.kt; db.kd = below.kd; db.kh = below.kh; db.kw = below.kw;
            da.kt = above.kt; da.kd = above.kd; da.kh = above.kh; da.kw = above.kw;
            if (!conv_wino_applies(db, below.cin, below.cout) || !conv_wino_applies(da, above.cout, above.cin)) continue;
            plan.sign_off[l] = off;
            off += align256(conv_wino_sign_words(db, below.cout) * sizeof(unsigned));
        }
    plan.saved_bytes = off;

    // split-K: enough workgroups to fill the chip, never more than there are pixel chunks
    const long long chunks = (plan.Q + kWgTM - 1) / kWgTM;
    plan.n_split = (int)(chunks < 256 ? (chunks + 7) / 8 * 8 : 256);   // multiple of 8: XCD-aware split

    size_t w = 0;
    plan.grad_off[0] = 0;
    for (int l = 1; l < L; ++l) {
        plan.grad_off[l] = w;
        w += align256(Q * p.layers[l].cin * es);
    }
    plan.grad_off[L] = 0;  // G_L = g_z lives in saved
    plan.partial_off = w;
    plan.partial_bytes = align256((size_t)plan.n_split * max_w * sizeof(float));
    for (int l = 0; l < L; ++l) {   // Winograd weight gradient: 16 products per channel pair, per split, plus their sum
        const gleam_conv& c = p.layers[l];
        PixDims dd{};
        dd.T = (int)g.T; dd.D = (int)g.D; dd.H = (int)g.H; dd.W = (int)g.W;
        dd.kt = c.kt; dd.kd = c.kd; dd.kh = c.kh; dd.kw = c.kw;
        if (p.dtype == 0 && wgrad_wino_applies(dd, c.cin, c.cout)) {
            const size_t need = align256(wgrad_wino_partial_floats(c.cin, c.cout, plan.n_split) * sizeof(float));
            if (need > plan.partial_bytes) plan.partial_bytes = need;
        }
        if (p.dtype == 0 && wgrad_time_applies(dd, c.cin, c.cout)) {
            dd.Q = plan.Q;
            const size_t need = align256(wgrad_time_partial_floats(dd, c.cin, c.cout) * sizeof(float));
            if (need > plan.partial_bytes) plan.partial_bytes = need;
        }
        if (p.dtype == 0 && wgrad_wino3_applies(dd, c.cin, c.cout)) {
            dd.Q = plan.Q;
            const size_t need = align256(wgrad_wino3_partial_floats(dd, c.cin, c.cout) * sizeof(float));
            if (need > plan.partial_bytes) plan.partial_bytes = need;
        }
        if (p.dtype == 1 && wgrad_bf16_walk_applies(dd, c.cin, c.cout)) {
            dd.Q = plan.Q;
            const size_t need = align256(wgrad_bf16_walk_partial_floats(dd, c.cin, c.cout) * sizeof(float));
            if (need > plan.partial_bytes) plan.partial_bytes = need;
        }
    }
    w += plan.partial_bytes;
    plan.bias_partial_off = w;
    w += align256((size_t)kThinSplit * kMaxChannels * sizeof(float));
    size_t max_img = 0;
    for (int l = 0; l < L; ++l) {
        const gleam_conv& c = p.layers[l];
        const int taps = c.kt * c.kd * c.kh * c.kw;
        const size_t f = conv_wimg_floats(c.cin, c.cout, taps), b = conv_wimg_floats(c.cout, c.cin, taps);
        max_img = f > max_img ? f : max_img;
        max_img = b > max_img ? b : max_img;
        if (taps == 9) {      // transformed weights of the Winograd path (16 values per channel pair)
            const size_t wn = conv_wino_weight_floats(c.cin, c.cout);
            max_img = wn > max_img ? wn : max_img;
        }
        if (taps == 27) {     // ... and of its 3x3x3 form (16 values per depth tap)
            const size_t wn = conv_wino3_weight_floats(c.cin, c.cout);
            max_img = wn > max_img ? wn : max_img;
        }
        if (p.dtype == 1) {   // bf16 images are half the bytes per element, but chunked by 32 channels
            const size_t fb = (conv_bf16_wimg_elems(c.cin, c.cout, taps) + 1) / 2, bb = (conv_bf16_wimg_elems(c.cout, c.cin, taps) + 1) / 2;
            max_img = fb > max_img ? fb : max_img;
            max_img = bb > max_img ? bb : max_img;
        }
    }
    // behind the per-layer scratch: the transformed weights of all Winograd layers of one pass, made in one launch
    size_t wino_floats = 0;
    if (p.dtype == 0)
        for (int l = 0; l < L; ++l) {
            const gleam_conv& c = p.layers[l];
            PixDims dd{};
            dd.T = (int)g.T; dd.D = (int)g.D; dd.H = (int)g.H; dd.W = (int)g.W;
            dd.kt = c.kt; dd.kd = c.kd; dd.kh = c.kh; dd.kw = c.kw;
            if (conv_wino_applies(dd, c.cin, c.cout) || conv_wino_applies(dd, c.cout, c.cin))
                wino_floats += (conv_wino_weight_floats(c.cin, c.cout) + 63) / 64 * 64;
        }
    plan.wino_u_off = align256(max_img * sizeof(float));
    const size_t img_bytes = plan.wino_u_off + align256(wino_floats * sizeof(float));
    plan.wimg_off_bwd = w;
    w += img_bytes;
    const size_t bwd_ws = w;

    plan.red_off = 0;  // loss partials reuse the head of the k-space buffer once DC is done
    size_t kbytes = align256((size_t)(g.B * g.C * g.T * g.D * g.H * g.W) * sizeof(float2));
    if (kbytes < align256(kLossBlocks * sizeof(double))) kbytes = align256(kLossBlocks * sizeof(double));
    plan.k_bytes = kbytes;
    plan.wimg_off_fwd = kbytes + plan.saved_bytes;
    const size_t fwd_ws = kbytes + plan.saved_bytes + img_bytes;  // activations live here when no saved buffer is given
    plan.ws_bytes = fwd_ws > bwd_ws ? fwd_ws : bwd_ws;
}

hipError_t prox_forward(const gleam_geom& g, const gleam_prox_desc& p, const ProxPlan& plan, const float* theta,
                        unsigned char* act_base, const float2* x_ref, float2* x_out, float* loss, void* ws,
                        hipStream_t st) {
    const int L = p.n_layers;
    const float* wino_u[kMaxLayers] = {};
    if (p.dtype == 0 && wino_enabled()) {   // transformed weights of every Winograd layer, one launch
        WinoWeightBatch wb{};
        float* up = reinterpret_cast<float*>((unsigned char*)ws + plan.wimg_off_fwd + plan.wino_u_off);
        for (int l = 0; l < L; ++l) {
            const gleam_conv& c = p.layers[l];
            if (!conv_wino_applies(pix_dims(g, c), c.cin, c.cout)) continue;
            wb.job[wb.n++] = WinoWeightJob{theta + plan.w_off[l], (long long)(9 * c.cin), (long long)c.cin, 1, 0, c.cin, c.cout, up};
            wino_u[l] = up;
            up += (conv_wino_weight_floats(c.cin, c.cout) + 63) / 64 * 64;
        }
        const hipError_t e = wino_weights_batch(wb, st);
        if (e != hipSuccess) return e;
    }
    for (int l = 0; l < L; ++l) {
        const gleam_conv& c = p.layers[l];
        const size_t taps = (size_t)c.kt * c.kd * c.kh * c.kw;
        ConvArgs a{};
        a.in = reinterpret_cast<const float*>(act_base + plan.act_off[l]);
        a.out = (l == L - 1) ? reinterpret_cast<float*>(x_out) : reinterpret_cast<float*>(act_base + plan.act_off[l + 1]);
        const ConvWeights cw{theta + plan.w_off[l], (long long)(taps * c.cin), (long long)c.cin, 1};
        a.bias = c.has_bias ? theta + plan.b_off[l] : nullptr;
        a.add = c.skip_src >= 0 ? reinterpret_cast<const float*>(act_base + plan.act_off[c.skip_src]) : nullptr;
        a.K = c.cin; a.Nn = c.cout;
        if (wino_u[l] && l + 1 < L && plan.sign_off[l + 1]) a.bits_out = reinterpret_cast<unsigned*>(act_base + plan.sign_off[l + 1]);
        a.relu_in = (c.relu_in && !plan.post_relu[l]) ? 1 : 0;
        a.relu_out = (c.relu_out || (l + 1 < L && plan.post_relu[l + 1])) ? 1 : 0;
        a.d = pix_dims(g, c);
        hipError_t e;
        if (p.dtype == 1) {
            if (l == 0) {           // float32 image in, bfloat16 features out
                bool hit = false;
                e = launch_conv_thin_in(a, cw, true, &hit, st);
                // cannot miss: prox_bf16_supported (checked before any launch) admits exactly the first-layer
                // shapes conv_thin_in_applies takes, whatever the geometry
                if (e == hipSuccess && !hit) e = hipErrorInvalidValue;
            } else {                // bfloat16 in; the last layer writes the float32 image
                if (l == L - 1) {
                    bool hit = false;
                    e = launch_conv_thin_out(a, cw, true, reinterpret_cast<float*>((unsigned char*)ws + plan.wimg_off_fwd), &hit, st);
                    if (e != hipSuccess) return e;
                    if (hit) continue;
                }
                ConvBf16Args b{};
                b.in = reinterpret_cast<const unsigned short*>(a.in);
                b.out = a.out;
                b.bias = a.bias;
                b.add = a.add;
                b.K = c.cin; b.Nn = c.cout;
                b.out_f32 = (l == L - 1) ? 1 : 0;
                b.relu_in = a.relu_in; b.relu_out = a.relu_out;
                b.d = a.d;
                if (l + 1 < L && plan.sign_off[l + 1]) b.bits_out = reinterpret_cast<unsigned*>(act_base + plan.sign_off[l + 1]);
                e = launch_conv_bf16(b, cw.w, cw.sn, cw.st, cw.sk, 0,
                                     reinterpret_cast<unsigned short*>((unsigned char*)ws + plan.wimg_off_fwd), st);
            }
        } else {
            e = launch_conv(a, cw, reinterpret_cast<float*>((unsigned char*)ws + plan.wimg_off_fwd), st, wino_u[l]);
        }
        if (e != hipSuccess) return e;
    }
    if (x_ref) {
        const long long n = plan.Q;
        double* part = reinterpret_cast<double*>((unsigned char*)ws + plan.red_off);
        float2* gz = reinterpret_cast<float2*>(act_base + plan.gz_off);
        return loss_and_grad((const float2*)x_out, x_ref, gz, n, p.loss_kind, p.layers[L - 1].relu_out, part, loss, st);
    }
    return hipSuccess;
}

template <int JT, int PG, int PA, int NW, bool BAL = false>
static void launch_wgrad_pipe_t(const WgradPipeArgs& pa, dim3 grid, size_t lds, hipStream_t st) {
    static bool once = false;
    if (!once) {
        (void)hipFuncSetAttribute((const void*)wgrad_pipe_kernel<JT, PG, PA, NW, BAL>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        once = true;
    }
    if (lds < (size_t)PG * NW * 64 * sizeof(float4)) lds = (size_t)PG * NW * 64 * sizeof(float4);
    hipLaunchKernelGGL((wgrad_pipe_kernel<JT, PG, PA, NW, BAL>), grid, dim3(NW * 64), lds, st, pa);
}

template <int KT, int KD, int KH, int KW>
static void launch_wgrad_thin_t(const WgradArgs& a, float* bias_partial, int n_split, bool bf, hipStream_t st) {
    WgradThinArgs t{};
    t.partial = a.partial; t.bias_partial = bias_partial; t.relu_in = a.relu_in; t.d = a.d;
    constexpr int PX = 4, NC4 = (PX + KW - 1 + 1) / 2;
    const size_t lds = ((size_t)KT * KD * KH * ((a.d.W + PX - 1) / PX * PX + 2 * NC4 - PX) * 2 + 256) * sizeof(float);
    const dim3 grid(n_split), blk(256);
    if (a.Ci == 2) {   // thin input a (float32), wide output gradient g
        t.wide = a.g; t.thin = a.a; t.WC = a.Co;
        if (bf) hipLaunchKernelGGL((wgrad_thin_kernel<KT, KD, KH, KW, 2, true, true>), grid, blk, lds, st, t);
        else hipLaunchKernelGGL((wgrad_thin_kernel<KT, KD, KH, KW, 2, true, false>), grid, blk, lds, st, t);
    } else {           // thin output gradient g (float32), wide input a
        t.wide = a.a; t.thin = a.g; t.WC = a.Ci;
        if (bf) hipLaunchKernelGGL((wgrad_thin_kernel<KT, KD, KH, KW, 2, false, true>), grid, blk, lds, st, t);
        else hipLaunchKernelGGL((wgrad_thin_kernel<KT, KD, KH, KW, 2, false, false>), grid, blk, lds, st, t);
    }
}

// Thin-layer weight gradient if the layer fits it (*hit).  `bf`: the wide tensor is bfloat16.
static hipError_t launch_wgrad_thin(const WgradArgs& a, float* bias_partial, bool bf, size_t partial_floats, int* used_split,
                                    bool* hit, hipStream_t st) {
    *hit = false;
    const PixDims& d = a.d;
    const int taps = d.kt * d.kd * d.kh * d.kw;
    const int wide = a.Ci == 2 ? a.Co : a.Ci;
    if (!((a.Ci == 2) != (a.Co == 2) && wide >= 8 && wide <= 256)) return hipSuccess;
    const bool k2 = d.kt == 1 && d.kd == 1 && d.kh == 3 && d.kw == 3, k3 = d.kt == 1 && d.kd == 3 && d.kh == 3 && d.kw == 3;
    const bool kt3 = d.kt == 3 && d.kd == 1 && d.kh == 1 && d.kw == 1;
    if (!k2 && !k3 && !kt3) return hipSuccess;
    if (wgrad_thin_walk_applies(d, wide, bf)) {   // 3x3 / 3x3x3 with 32, 64 or 128 wide channels: matrix cores
        WgradThinWalkArgs t{};
        t.partial = a.partial; t.bias_partial = bias_partial; t.relu_in = a.relu_in; t.d = d; t.WC = wide; t.bf = bf ? 1 : 0;
        if (a.Ci == 2) { t.wide = a.g; t.thin = a.a; t.thin_in = 1; }
        else { t.wide = a.a; t.thin = a.g; t.thin_in = 0; }
        *hit = true;
        return launch_wgrad_thin_walk(t, partial_floats, used_split, st);
    }
    // HBM-bound: one workgroup per image row up to kThinSplit partials (as many as the scratch holds)
    long long ts = d.Q / d.W;
    if (ts > kThinSplit) ts = kThinSplit;
    const long long fit = (long long)(partial_floats / ((size_t)a.Co * taps * a.Ci));
    if (ts > fit) ts = fit;
    const int tsplit = (int)(ts < 1 ? 1 : ts);
    if (k2) launch_wgrad_thin_t<1, 1, 3, 3>(a, bias_partial, tsplit, bf, st);
    else if (k3) launch_wgrad_thin_t<1, 3, 3, 3>(a, bias_partial, tsplit, bf, st);
    else launch_wgrad_thin_t<3, 1, 1, 1>(a, bias_partial, tsplit, bf, st);
    *used_split = tsplit;
    *hit = true;
    return hipGetLastError();
}

// Launches the weight-gradient kernel that fits the layer.  *bias_done is set when the kernel also
// wrote the bias-gradient partials (bias_partial non-null on entry).
static hipError_t launch_wgrad(const WgradArgs& a, float* bias_partial, bool* bias_done, int n_split, size_t partial_floats,
                               int* used_split, hipStream_t st) {
    const PixDims& d = a.d;
    const int rowtaps = d.kt * d.kd * d.kh, taps = rowtaps * d.kw;
    char name[56];
    snprintf(name, sizeof(name), "conv_wgrad_%dto%d_t%d", a.Ci, a.Co, taps);
    KernelScope ks(name, 2.0 * (double)d.Q * a.Ci * a.Co * taps, 4.0 * (double)d.Q * (a.Ci + a.Co), st);
    *bias_done = false;
    *used_split = n_split;
    const int ncb = (a.Co + 31) / 32, nib = (a.Ci + 31) / 32;
    const int jt = taps >= 9 ? 9 : 3;
    const int tapgroups = (taps + jt - 1) / jt;
    dim3 grid(n_split, (ncb * nib * tapgroups + 3) / 4);

    // (1) one side is the 2-channel image: HBM-bound kernel without MFMA
    {
        bool hit = false;
        const hipError_t e = launch_wgrad_thin(a, bias_partial, false, partial_floats, used_split, &hit, st);
        if (e != hipSuccess) return e;
        if (hit) {
            *bias_done = bias_partial != nullptr;
            return hipSuccess;
        }
    }
    // (2) channel counts that are multiples of 4: register-prefetch pipelined MFMA kernel
    const double max_off = (double)(d.kt / 2 + 1) * d.D * d.H * d.W * (a.Ci > a.Co ? a.Ci : a.Co);   // 32-bit slot offsets
    if (a.Co % 4 == 0 && a.Ci % 4 == 0 && max_off < 2147483648.0) {
        const int n_pa = kWgTM + d.kw - 1;
        const int need_pg = (kWgTM * (a.Co / 4) + kConvThreads - 1) / kConvThreads;
        const int need_pa = (rowtaps * n_pa * (a.Ci / 4) + kConvThreads - 1) / kConvThreads;
        const size_t lds = ((size_t)kWgTM * (a.Co + 4) + (size_t)rowtaps * n_pa * (a.Ci + 4) + kWgTM) * sizeof(float);
        WgradPipeArgs pa{a, bias_partial};
        bool hit = true;
        bool hit_none = true;
        // Twelve waves when the layer splits into 7..12 jobs of one 32x32 channel block x 3 taps (9 taps on
        // 2x2 blocks, 27 taps on one block) or x 1 tap (3 taps on 2x2 blocks): three waves share a SIMD
        // and cover each other's LDS and issue latencies, and no wave carries a padded tap.
        {
            const int blocks = ncb * nib;
            const int jobs3 = blocks * ((taps + 2) / 3), jobs1 = blocks * taps;
            const int pg12 = (kWgTM * (a.Co / 4) + 767) / 768, pa12 = (rowtaps * n_pa * (a.Ci / 4) + 767) / 768;
            const dim3 g12(n_split, 1);
            const int pg8b = (kWgTM * (a.Co / 4) + 511) / 512, pa8b = (rowtaps * n_pa * (a.Ci / 4) + 511) / 512;
            const bool bal_on = !(kernel_policy() & GLEAM_POLICY_NO_WGRAD_BALANCE);
            if (bal_on && blocks == 1 && taps == 27 && pg8b <= 1 && pa8b <= 5) {
                // 27 taps on one channel block: nine 3-tap jobs would put three on one SIMD and two on the others;
                // eight waves with 4,4,4,3,3,3,3,3 taps load the SIMDs 7,7,7,6
                launch_wgrad_pipe_t<4, 1, 5, 8, true>(pa, g12, lds, st);
                hit_none = false;
            } else if (taps % 3 == 0 && jobs3 >= 7 && jobs3 <= 12 && pg12 <= 1 && pa12 <= 4) {
                if (pa12 <= 3) launch_wgrad_pipe_t<3, 1, 3, 12>(pa, g12, lds, st);
                else launch_wgrad_pipe_t<3, 1, 4, 12>(pa, g12, lds, st);
                hit_none = false;
            } else if (jobs1 >= 7 && jobs1 <= 12 && pg12 <= 1 && pa12 <= 3) {
                launch_wgrad_pipe_t<1, 1, 3, 12>(pa, g12, lds, st);
                hit_none = false;
            } else if (taps == 9 && blocks == 4) {   // wider layers: eight waves, 5 + 4 taps per wave pair
                const int pg8 = (kWgTM * (a.Co / 4) + 511) / 512, pa8 = (rowtaps * n_pa * (a.Ci / 4) + 511) / 512;
                if (pg8 <= 1 && pa8 <= 4) {
                    dim3 g8(n_split, 1);
                    launch_wgrad_pipe_t<5, 1, 4, 8>(pa, g8, lds, st);
                    hit_none = false;
                }
            }
        }
#define GLEAM_WG_TRY(JT_, PG_, PA_)                                             \
    if (hit_none && jt == JT_ && need_pg <= PG_ && need_pa <= PA_) {            \
        launch_wgrad_pipe_t<JT_, PG_, PA_, 4>(pa, grid, lds, st);               \
        hit_none = false;                                                       \
    }
        GLEAM_WG_TRY(9, 1, 4) GLEAM_WG_TRY(9, 2, 8) GLEAM_WG_TRY(9, 1, 16) GLEAM_WG_TRY(9, 4, 16)
        GLEAM_WG_TRY(3, 1, 4) GLEAM_WG_TRY(3, 2, 8) GLEAM_WG_TRY(3, 1, 16) GLEAM_WG_TRY(3, 4, 16)
#undef GLEAM_WG_TRY
        hit = !hit_none;
        if (hit && lds <= 150 * 1024) {
            *bias_done = bias_partial != nullptr;
            return hipGetLastError();
        }
        if (hit) return hipErrorInvalidValue;  // cannot happen: the plan bounds LDS use
    }
    // (3) generic fallback
    const int RSg = (a.Co + 3) / 4 * 4 + 1, RSa = (a.Ci + 3) / 4 * 4 + 1;
    const size_t lds = ((size_t)kWgTM * RSg + (size_t)rowtaps * (kWgTM + d.kw - 1) * RSa + kWgTM) * sizeof(float);
    if (jt == 9) {
        static bool once9 = false;
        if (!once9) { (void)hipFuncSetAttribute((const void*)wgrad_mfma_kernel<9>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); once9 = true; }
        hipLaunchKernelGGL(wgrad_mfma_kernel<9>, grid, dim3(kConvThreads), lds, st, a);
    } else {
        static bool once3 = false;
        if (!once3) { (void)hipFuncSetAttribute((const void*)wgrad_mfma_kernel<3>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); once3 = true; }
        hipLaunchKernelGGL(wgrad_mfma_kernel<3>, grid, dim3(kConvThreads), lds, st, a);
    }
    return hipGetLastError();
}

size_t wgrad_lds_bytes(const gleam_conv& c) {
    const int rowtaps = c.kt * c.kd * c.kh;
    const int RSg = (c.cout + 3) / 4 * 4 + 4, RSa = (c.cin + 3) / 4 * 4 + 4;  // the wider of the two layouts
    return ((size_t)kWgTM * RSg + (size_t)rowtaps * (kWgTM + c.kw - 1) * RSa + kWgTM) * sizeof(float);
}

hipError_t prox_backward(const gleam_geom& g, const gleam_prox_desc& p, const ProxPlan& plan, const float* theta,
                         const unsigned char* saved, float* grad_theta, float2* g_in, void* ws, hipStream_t st) {
    const int L = p.n_layers;
    int skip_from_input = 0;   // layer (1-based) whose output gradient also flows into t_0 = u through its skip
    unsigned char* wsb = (unsigned char*)ws;
    float* partial = reinterpret_cast<float*>(wsb + plan.partial_off);
    // Gradient buffer of tensor t_l (1 <= l <= L); G_L is g_z.
    auto G = [&](int l) -> float* {
        return l == L ? reinterpret_cast<float*>(const_cast<unsigned char*>(saved) + plan.gz_off)
                      : reinterpret_cast<float*>(wsb + plan.grad_off[l]);
    };
    auto act = [&](int l) -> const float* { return reinterpret_cast<const float*>(saved + plan.act_off[l]); };
    // pending[s]: layer (1-based) whose output gradient also flows into t_s through its skip, or 0
    int pending[kMaxLayers + 1] = {0};

    const float* wino_u[kMaxLayers] = {};   // transformed (mirrored, transposed) weights of the data gradients, one launch
    if (p.dtype == 0 && wino_enabled()) {
        WinoWeightBatch wb{};
        float* up = reinterpret_cast<float*>(wsb + plan.wimg_off_bwd + plan.wino_u_off);
        for (int l = 2; l <= L; ++l) {   // the data gradient of layer l maps cout -> cin channels
            const gleam_conv& c = p.layers[l - 1];
            if (!conv_wino_applies(pix_dims(g, c), c.cout, c.cin)) continue;
            wb.job[wb.n++] = WinoWeightJob{theta + plan.w_off[l - 1], 1, (long long)c.cin, (long long)(9 * c.cin), 1, c.cout, c.cin, up};
            wino_u[l - 1] = up;
            up += (conv_wino_weight_floats(c.cout, c.cin) + 63) / 64 * 64;
        }
        const hipError_t e = wino_weights_batch(wb, st);
        if (e != hipSuccess) return e;
    }

    for (int l = L; l >= 1; --l) {  // layer l maps t_{l-1} -> t_l
        const gleam_conv& c = p.layers[l - 1];
        const size_t taps = (size_t)c.kt * c.kd * c.kh * c.kw;
        const PixDims d = pix_dims(g, c);
        if (c.skip_src >= 1) {
            if (pending[c.skip_src] != 0) return hipErrorInvalidValue;  // one consumer per skip source (checked at plan time)
            pending[c.skip_src] = l;
        }
        if (c.skip_src == 0) {
            if (g_in && skip_from_input != 0) return hipErrorInvalidValue;   // checked by the caller
            skip_from_input = l;
        }
        // weight gradient (+ bias gradient)
        WgradArgs wa{};
        wa.g = G(l); wa.a = act(l - 1); wa.partial = partial;
        wa.Co = c.cout; wa.Ci = c.cin; wa.relu_in = (c.relu_in && !plan.post_relu[l - 1]) ? 1 : 0; wa.d = d;
        float* bpart = reinterpret_cast<float*>(wsb + plan.bias_partial_off);
        bool bias_done = false, wino_wgrad_done = false;
        int used_split = plan.n_split;
        hipError_t e;
        if (p.dtype == 1) {
            if (l == 1 || l == L) {   // one side is the float32 2-channel image, the wide side is bfloat16
                bool hit = false;
                KernelScope ks(l == 1 ? "conv_bf16_wgrad_thin_in" : "conv_bf16_wgrad_thin_out", 2.0 * (double)d.Q * c.cin * c.cout * taps,
                               2.0 * (double)d.Q * (c.cin + c.cout), st);
                e = launch_wgrad_thin(wa, c.has_bias ? bpart : nullptr, true, plan.partial_bytes / sizeof(float), &used_split, &hit, st);
                if (e == hipSuccess && !hit) e = hipErrorInvalidValue;
                bias_done = c.has_bias;
            } else {
                WgradBf16Args wb{};
                wb.g = reinterpret_cast<const unsigned short*>(wa.g);
                wb.a = reinterpret_cast<const unsigned short*>(wa.a);
                wb.partial = partial;
                wb.bias_partial = c.has_bias ? bpart : nullptr;
                wb.Co = c.cout; wb.Ci = c.cin; wb.relu_in = wa.relu_in; wb.d = d;
                if (!(kernel_policy() & GLEAM_POLICY_NO_FRAME_WALK) && wgrad_bf16_walk_applies(d, c.cin, c.cout)) {
                    e = launch_wgrad_bf16_walk(wb, st);   // down the rows, every input row segment staged once
                    used_split = wgrad_bf16_walk_splits(d, c.cout);
                } else {
                    e = launch_wgrad_bf16(wb, plan.n_split, st);
                }
                bias_done = c.has_bias;
            }
        } else if (wino_enabled() && wgrad_wino_applies(d, c.cin, c.cout)) {
            // Winograd F(2x2, 3x3): partial sums of the 16 transformed products, fixed-order reduction, back-transform
            WinoWgradArgs ww{};
            ww.g = wa.g; ww.a = wa.a; ww.partial = partial; ww.bias_partial = c.has_bias ? bpart : nullptr;
            ww.Co = c.cout; ww.Ci = c.cin; ww.H = d.H; ww.W = d.W; ww.NI = d.Q / ((long long)d.H * d.W);
            const long long np = 16LL * c.cout * c.cin, nb = c.has_bias ? c.cout : 0;
            {
                char name[56];
                snprintf(name, sizeof(name), "conv_wgrad_%dto%d_t%d", c.cin, c.cout, taps);
                // 16 instead of 36 multiplications per 2x2 pixels and channel pair run on the matrix cores
                KernelScope ks(name, 2.0 * (double)d.Q * c.cin * c.cout * taps, 4.0 * (double)d.Q * (c.cin + c.cout), st,
                               2.0 * (double)d.Q * c.cin * c.cout * 4);
                e = launch_wgrad_wino(ww, wa.relu_in, plan.n_split, st);
                if (e != hipSuccess) return e;
            }
            float* psum = partial + (size_t)plan.n_split * np;
            {
                KernelScope ks("wgrad_reduce", 0.0, 4.0 * (double)(np + nb) * (plan.n_split + 1), st);
                const int nbw = (int)((np + 63) / 64), nbb = (int)((nb + 15) / 16);
                hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)(nbw + nbb)), dim3(256), 0, st, (const float*)partial,
                                   plan.n_split, np, psum, 1, nbw, (const float*)bpart, nb,
                                   c.has_bias ? grad_theta + plan.b_off[l - 1] : nullptr);
                e = wgrad_wino_finish(psum, c.cout, c.cin, grad_theta + plan.w_off[l - 1], st);
                if (e != hipSuccess) return e;
            }
            wino_wgrad_done = true;
        } else if (wino_enabled() && wgrad_wino3_applies(d, c.cin, c.cout)) {
            // 3x3x3: the same scheme inside every slice, one set of 16 products per depth tap
            Wino3WgradArgs ww{};
            ww.g = wa.g; ww.a = wa.a; ww.partial = partial; ww.bias_partial = c.has_bias ? bpart : nullptr;
            ww.Co = c.cout; ww.Ci = c.cin;
            const int n3 = wgrad_wino3_splits(d);
            const long long np = 48LL * c.cout * c.cin, nb = c.has_bias ? c.cout : 0;
            {
                char name[56];
                snprintf(name, sizeof(name), "conv_wgrad_%dto%d_t%d", c.cin, c.cout, taps);
                KernelScope ks(name, 2.0 * (double)d.Q * c.cin * c.cout * taps, 4.0 * (double)d.Q * (c.cin + c.cout), st,
                               2.0 * (double)d.Q * c.cin * c.cout * 12);
                e = launch_wgrad_wino3(ww, d, wa.relu_in, st);
                if (e != hipSuccess) return e;
            }
            float* psum = partial + (size_t)n3 * np;
            {
                KernelScope ks("wgrad_reduce", 0.0, 4.0 * (double)(np + nb) * (n3 + 1), st);
                const int nbw = (int)((np + 63) / 64), nbb = (int)((nb + 15) / 16);
                hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)(nbw + nbb)), dim3(256), 0, st, (const float*)partial,
                                   n3, np, psum, 1, nbw, (const float*)bpart, nb,
                                   c.has_bias ? grad_theta + plan.b_off[l - 1] : nullptr);
                e = wgrad_wino3_finish(psum, c.cout, c.cin, grad_theta + plan.w_off[l - 1], st);
                if (e != hipSuccess) return e;
            }
            wino_wgrad_done = true;
        } else if (!(kernel_policy() & GLEAM_POLICY_NO_FRAME_WALK) && wgrad_time_applies(d, c.cin, c.cout)) {
            // temporal 3x1x1: walk along the frames, every input and gradient read once
            TimeWgradArgs tw{};
            tw.g = wa.g; tw.a = wa.a; tw.partial = partial; tw.bias_partial = c.has_bias ? bpart : nullptr;
            tw.Co = c.cout; tw.Ci = c.cin;
            char name[56];
            snprintf(name, sizeof(name), "conv_wgrad_%dto%d_t%d", c.cin, c.cout, taps);
            KernelScope ks(name, 2.0 * (double)d.Q * c.cin * c.cout * taps, 4.0 * (double)d.Q * (c.cin + c.cout), st);
            e = launch_wgrad_time(tw, d, wa.relu_in, st);
            used_split = wgrad_time_splits(d);
            bias_done = c.has_bias;
        } else {
            e = launch_wgrad(wa, c.has_bias ? bpart : nullptr, &bias_done, plan.n_split,
                             plan.partial_bytes / sizeof(float), &used_split, st);
        }
        if (e != hipSuccess) return e;
        const long long nw = (long long)(c.cout * taps * c.cin);
        if (c.has_bias && !bias_done && !wino_wgrad_done) {
            KernelScope ks("bias_grad", 0.0, 4.0 * (double)plan.Q * c.cout, st);
            hipLaunchKernelGGL(colsum_kernel, dim3(used_split), dim3(256), 0, st, (const float*)G(l), plan.Q, c.cout, bpart);
        }
        if (!wino_wgrad_done) {
            const long long nb = c.has_bias ? c.cout : 0;
            KernelScope ks("wgrad_reduce", 0.0, 4.0 * (double)(nw + nb) * (used_split + 1), st);
            float* gw = grad_theta + plan.w_off[l - 1];
            const int vec = (nw % 4 == 0 && (reinterpret_cast<uintptr_t>(gw) & 15) == 0) ? 1 : 0;
            const int nbw = (int)((nw + 16 * (vec ? 4 : 1) - 1) / (16 * (vec ? 4 : 1))), nbb = (int)((nb + 15) / 16);
            hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)(nbw + nbb)), dim3(256), 0, st,
                               (const float*)partial, used_split, nw, gw, vec, nbw,
                               (const float*)bpart, nb, c.has_bias ? grad_theta + plan.b_off[l - 1] : nullptr);
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (l == 1) {
            if (!g_in) break;   // nothing flows into t_0 = u: the module input is detached
            // a module of several unrolled iterations: gradient with respect to this iteration's input u,
            // dL/du = conv_1^T(G_1) + (gradient of a skip taken from u), float32 2 channels
            ConvArgs a{};
            a.in = G(1); a.out = reinterpret_cast<float*>(g_in);
            const ConvWeights cw{theta + plan.w_off[0], 1, (long long)c.cin, (long long)(taps * c.cin)};
            a.flip = 1;
            a.K = c.cout; a.Nn = c.cin;
            a.add = skip_from_input ? G(skip_from_input) : nullptr;
            a.d = d;
            float* scratch = reinterpret_cast<float*>(wsb + plan.wimg_off_bwd);
            if (p.dtype == 1) {
                bool hit = false;
                e = launch_conv_thin_out(a, cw, true, scratch, &hit, st);
                if (e == hipSuccess && !hit) {
                    ConvBf16Args b{};
                    b.in = reinterpret_cast<const unsigned short*>(a.in);
                    b.out = a.out; b.add = a.add; b.out_f32 = 1;
                    b.K = a.K; b.Nn = a.Nn; b.d = d;
                    e = launch_conv_bf16(b, cw.w, cw.sn, cw.st, cw.sk, 1, reinterpret_cast<unsigned short*>(scratch), st);
                }
            } else {
                e = launch_conv(a, cw, scratch, st);
            }
            if (e != hipSuccess) return e;
            break;
        }
        // data gradient into t_{l-1}, fused with the ReLU masks and the pending skip gradient
        const gleam_conv& below = p.layers[l - 2];  // layer that produced t_{l-1}
        ConvArgs a{};
        a.in = G(l); a.out = G(l - 1);
        const ConvWeights cw{theta + plan.w_off[l - 1], 1, (long long)c.cin, (long long)(taps * c.cin)};
        a.flip = 1;
        a.K = c.cout; a.Nn = c.cin;
        a.mask_acc = (c.relu_in || below.relu_out) ? 1 : 0;
        a.mask_add = below.relu_out ? 1 : 0;
        a.mask_ref = (a.mask_acc || a.mask_add) ? act(l - 1) : nullptr;
        a.add = pending[l - 1] ? G(pending[l - 1]) : nullptr;
        if (p.dtype == 0 && wino_enabled() && a.mask_ref && plan.sign_off[l - 1])   // then the forward pass wrote them
            a.bits_in = reinterpret_cast<const unsigned*>(saved + plan.sign_off[l - 1]);
        a.d = d;
        if (p.dtype == 1) {
            if (l == L) {           // float32 loss gradient in, bfloat16 gradient out
                bool hit = false;
                e = launch_conv_thin_in(a, cw, true, &hit, st);
                if (e == hipSuccess && !hit) e = hipErrorInvalidValue;
            } else {
                ConvBf16Args b{};
                b.in = reinterpret_cast<const unsigned short*>(a.in);
                b.out = a.out;
                b.mask_ref = reinterpret_cast<const unsigned short*>(a.mask_ref);
                b.add = a.add;
                b.K = a.K; b.Nn = a.Nn;
                b.mask_acc = a.mask_acc; b.mask_add = a.mask_add;
                b.d = d;
                if (a.mask_ref && plan.sign_off[l - 1]) b.bits_in = reinterpret_cast<const unsigned*>(saved + plan.sign_off[l - 1]);
                e = launch_conv_bf16(b, cw.w, cw.sn, cw.st, cw.sk, 1, reinterpret_cast<unsigned short*>(wsb + plan.wimg_off_bwd), st);
            }
        } else {
            e = launch_conv(a, cw, reinterpret_cast<float*>(wsb + plan.wimg_off_bwd), st, wino_u[l - 1]);
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ------------------------------------------------------------------ Adam ("Update Parameters", Alg. 1)
__global__ __launch_bounds__(256) void adam_kernel(float* __restrict__ theta, const float* __restrict__ grad,
                                                   float* __restrict__ m, float* __restrict__ v, size_t n, float beta1,
                                                   float beta2, float step, float inv_c2, float eps) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float g = grad[i];
    const float mi = beta1 * m[i] + (1.f - beta1) * g;
    const float vi = beta2 * v[i] + (1.f - beta2) * g * g;
    m[i] = mi;
    v[i] = vi;
    // step = lr / (1 - beta1^t), inv_c2 = 1 / (1 - beta2^t)
    theta[i] -= step * mi / (sqrtf(vi * inv_c2) + eps);
}

hipError_t adam_update(const gleam_adam& h, long long t, size_t n, float* theta, const float* grad, float* m, float* v,
                       hipStream_t st) {
    const double c1 = 1.0 - pow((double)h.beta1, (double)t), c2 = 1.0 - pow((double)h.beta2, (double)t);
    KernelScope ks("adam", 0.0, 28.0 * (double)n, st);
    hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, theta, grad, m, v, n, h.beta1, h.beta2,
                       (float)((double)h.lr / c1), (float)(1.0 / c2), h.eps);
    return hipGetLastError();
}

}  // namespace gleam
