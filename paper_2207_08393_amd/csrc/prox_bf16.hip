// Prox convolutions with bfloat16 operands and float32 accumulation on the gfx950 32x32x16 bf16 MFMA
// (prox dtype 1).  Activations and inter-layer gradients are bfloat16 [pixels][channels]; weights are
// rounded from the float32 master copy once per layer and call; bias, loss, residual add into the image
// and every weight gradient stay float32.
//
//   conv_bf16_kernel  : forward and data gradient, same scheme as the float32 direct-to-LDS kernel - two
//                       LDS chunk buffers filled by global->LDS direct loads, XOR-swizzled 16-byte quads
//                       (8 channels), 32 input channels per chunk (two MFMA K-blocks per tap).
//   conv_bf16_2d_kernel : forward and data gradient of 3x3 layers on two-dimensional pixel tiles (zero-filled
//                       halo instead of tap masks, all nine taps per chunk, output through LDS).
//   wgrad_bf16_kernel : weight gradient; the contraction runs over pixels, so g and a are transposed into
//                       LDS ([channel][pixel]) while they are staged and each lane reads its 8 pixels as
//                       one 16-byte word; the three taps along W come from one 20-byte window by shifts.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#include <type_traits>

#include "prox_common.h"

namespace gleam {

constexpr int kBfCK = 32;   // input channels per staged chunk of the forward / data-gradient kernel

// ------------------------------------------------------------------ weights -> bf16 LDS images
// Image (rt, kc, nb) = [kw][kBfCK/16][2][NB][8]: element (dw, k = 16g + 8h + s, n) at
// ((((dw*G + g)*2 + h)*NB + n)*8 + s, zero past the layer; source (n, tap, k) at w[n*sn + tapidx*st + k*sk].
struct WimgBf16Args {
    const float* w;
    unsigned short* wt;
    long long sn, st, sk;
    int K, Nn, flip, taps, kw, NB, n_kc, n_nb;
    long long total;
};
__global__ void weights_image_bf16_kernel(WimgBf16Args a) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.total) return;
    constexpr int G = kBfCK / 16;
    const int img_elems = a.kw * kBfCK * a.NB;
    const long long img = i / img_elems;
    const int e = (int)(i % img_elems);
    const int s = e & 7, n = (e >> 3) % a.NB, hg = (e >> 3) / a.NB;
    const int h = hg & 1, g = (hg >> 1) % G, dw = (hg >> 1) / G;
    const int nb = (int)(img % a.n_nb), kc = (int)((img / a.n_nb) % a.n_kc), rt = (int)(img / ((long long)a.n_nb * a.n_kc));
    const int k = kc * kBfCK + 16 * g + 8 * h + s, nn = nb * a.NB + n;
    const int tap = rt * a.kw + dw;
    const int tapidx = a.flip ? a.taps - 1 - tap : tap;
    float v = 0.f;
    if (k < a.K && nn < a.Nn) v = a.w[nn * a.sn + tapidx * a.st + k * a.sk];
    a.wt[i] = f32_to_bf16(v);
}

static inline int bf_nb(int Nn) { return Nn <= 32 ? 32 : 64; }
size_t conv_bf16_wimg_elems(int K, int Nn, int taps) {
    const int nb = bf_nb(Nn);
    return (size_t)taps * ((K + kBfCK - 1) / kBfCK) * kBfCK * ((Nn + nb - 1) / nb) * nb + 16;   // + a zero quad for the 2D kernel
}

// ------------------------------------------------------------------ forward / data gradient
// A wave owns 32*PJ pixels x NB output channels: every weight operand read from LDS feeds PJ MFMAs and
// every pixel operand NB/32 of them (the kernel is bound by LDS operand bandwidth, not by the MFMA rate).
template <int NB, int KW, bool RELU, int PJ>
__global__ __launch_bounds__(256, 2) void conv_bf16_kernel(ConvBf16Args a) {
    constexpr int NW = 4, TM = NW * 32 * PJ, G = kBfCK / 16, NJ = NB / 32, QP = kBfCK / 8;   // QP quads per pixel row
    constexpr int RP = 16 / QP;                // pixel rows per 256 bytes of LDS: 16 consecutive pixels (the lanes one
                                               // 128-bit LDS access serves together) land on 16 different 16-byte slots
    constexpr int KWM = KW > 0 ? KW : 5;
    constexpr int kSlabOpsMax = ((TM + KWM - 1) * QP + 63) / 64, kWOpsMax = (KWM * kBfCK * NB / 8 + 63) / 64;
    constexpr int MAXS = kSlabOpsMax / NW + 1, MAXW = kWOpsMax / NW + 1;
    constexpr int kBufQuads = (kSlabOpsMax + kWOpsMax) * 64;
    __shared__ uint4 bufA[kBufQuads];
    __shared__ uint4 bufB[kBufQuads];
    const PixDims d = a.d;
    const int kw = KW > 0 ? KW : d.kw;
    const int n_pix = TM + kw - 1;
    const int slab_ops = (n_pix * QP + 63) / 64;
    const int w8 = kw * kBfCK * NB / 8;        // quads per weight image
    const int w_ops = (w8 + 63) / 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), m = lane & 31, h = lane >> 5;
    const int n0 = blockIdx.y * NB;
    const int rowtaps = d.kt * d.kd * d.kh;
    const int n_kc = (a.K + kBfCK - 1) / kBfCK;
    const int nck = rowtaps * n_kc;
    const long long n_tiles = (d.Q + TM - 1) / TM;
    const bool k_full = (a.K % kBfCK) == 0;
    const long long last_quad = d.Q * a.K - 8;   // highest legal quad start (elements)

    unsigned s_off[MAXS], w_off[MAXW];
    int s_pp[MAXS], s_c8[MAXS];
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
        const int v = (wave + i * NW) * 64 + lane;
        s_pp[i] = v / QP;
        s_c8[i] = (v % QP) ^ ((s_pp[i] / RP) % QP);
        s_off[i] = (unsigned)(s_pp[i] * a.K + 8 * s_c8[i]);
    }
#pragma unroll
    for (int i = 0; i < MAXW; ++i) {
        const int v = (wave + i * NW) * 64 + lane;
        w_off[i] = 8u * (unsigned)(v < w8 ? v : 0);
    }
    auto issue = [&](long long tile, const ChunkIter& ci, uint4* dst) {
        const int rt = ci.rt, kc = ci.kc;
        const long long qs = tile * TM + ci.off - kw / 2;
        const bool interior = k_full && qs >= 0 && qs + (long long)slab_ops * 64 / QP <= d.Q;   // uniform
        if (interior) {
            const unsigned short* base = a.in + qs * a.K + kc * kBfCK;
#pragma unroll
            for (int i = 0; i < MAXS; ++i) {
                const int o = wave + i * NW;
                if (o < slab_ops)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + s_off[i]),
                                                     (__attribute__((address_space(3))) void*)(dst + o * 64), 16, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < MAXS; ++i) {
                const int o = wave + i * NW;
                if (o < slab_ops) {
                    long long off = (qs + s_pp[i]) * a.K + kc * kBfCK + 8 * s_c8[i];
                    off = off < 0 ? 0 : (off > last_quad ? last_quad : off);
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(a.in + off),
                                                     (__attribute__((address_space(3))) void*)(dst + o * 64), 16, 0, 0);
                }
            }
        }
        const unsigned short* src = a.wt + ((size_t)(rt * n_kc + kc) * gridDim.y + blockIdx.y) * (size_t)(kw * kBfCK * NB);
        uint4* wdst = dst + slab_ops * 64;
#pragma unroll
        for (int i = 0; i < MAXW; ++i) {
            const int o = wave + i * NW;
            if (o < w_ops)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + w_off[i]),
                                                 (__attribute__((address_space(3))) void*)(wdst + o * 64), 16, 0, 0);
        }
    };

    // quad index of this lane's pixel operand for every (tap along W, 16-channel K-block)
    int p_off[PJ][KWM][G];
#pragma unroll
    for (int pj = 0; pj < PJ; ++pj)
#pragma unroll
        for (int dw = 0; dw < KWM; ++dw) {
            const int pix = wave * (32 * PJ) + 32 * pj + m + dw;
            const int key = (pix / RP) % QP;
#pragma unroll
            for (int g = 0; g < G; ++g) p_off[pj][dw][g] = pix * QP + ((2 * g + h) ^ key);
        }
    const int wa_lane = h * NB + m;

    const XcdRange xr = xcd_range(n_tiles);
    long long tile = xr.first;
    ChunkIter ci = chunk_first(d);
    if (tile < xr.end) issue(tile, ci, bufA);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // this lane's pixel of the current tile, tracked by coordinates (no divisions per tile)
    long long q0 = (tile < xr.end ? tile : 0) * TM + wave * (32 * PJ) + m;   // pixel of pj = 0; pj adds 32
    PixCoord qc[PJ];
#pragma unroll
    for (int pj = 0; pj < PJ; ++pj) qc[pj] = pix_coord(q0 + 32 * pj < d.Q ? q0 + 32 * pj : 0, d);
    const PixCoord qstep = pix_coord(xr.stride * TM, d);
    unsigned vbits[PJ];
    bool tile_masked = true;
    const int n_taps = rowtaps * kw;
    const unsigned all_taps = n_taps >= 32 ? 0xffffffffu : (1u << n_taps) - 1u;
    floatx16 acc[PJ][NJ];
    auto step = [&](const uint4* slab, uint4* nxt) {
        if (ci.c == 0) {
            bool any = false;
#pragma unroll
            for (int pj = 0; pj < PJ; ++pj) {
                vbits[pj] = q0 + 32 * pj < d.Q ? tap_validity_at(qc[pj], d) : 0u;
                any = any || vbits[pj] != all_taps;
            }
            tile_masked = __builtin_amdgcn_ballot_w64(any) != 0ull;   // wave-uniform
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
        const uint4* wl = slab + slab_ops * 64 + wa_lane;
        const int rt = ci.rt;
        // MASKED: some lane of this wave has a tap outside the grid in this tile (zero padding); interior
        // tiles take the path without the per-operand AND (ordinary vector instructions cost MFMA issue slots)
        auto units = [&](auto masked) {
            constexpr bool MASKED = decltype(masked)::value;
#pragma unroll
            for (int dw = 0; dw < KWM; ++dw) {
                if (KW == 0 && dw >= kw) continue;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    bf16x8 pv[PJ];
#pragma unroll
                    for (int pj = 0; pj < PJ; ++pj) {
                        uint4 pb = slab[p_off[pj][dw][g]];
                        if (RELU) {
                            pb.x = relu_bf16x2(pb.x); pb.y = relu_bf16x2(pb.y); pb.z = relu_bf16x2(pb.z); pb.w = relu_bf16x2(pb.w);
                        }
                        if (MASKED) {
                            const unsigned okm = ((vbits[pj] >> (rt * kw + dw)) & 1u) ? 0xffffffffu : 0u;
                            pb.x &= okm; pb.y &= okm; pb.z &= okm; pb.w &= okm;
                        }
                        pv[pj] = __builtin_bit_cast(bf16x8, pb);
                    }
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        const bf16x8 wv = __builtin_bit_cast(bf16x8, wl[(dw * G + g) * 2 * NB + 32 * j]);
#pragma unroll
                        for (int pj = 0; pj < PJ; ++pj)
                            acc[pj][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, pv[pj], acc[pj][j], 0, 0, 0);
                    }
                }
            }
        };
        if (tile_masked) units(std::true_type{});
        else units(std::false_type{});
        if (last) {
            // lane holds pixel q and, per register group, 4 consecutive output channels
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
                    const long long o = q * a.Nn + co0;
                    if (!a.out_f32 && (a.Nn % 4) == 0) {
                        // four consecutive bf16 channels = one 8-byte access
                        float x[4] = {acc[pj][j][4 * rg], acc[pj][j][4 * rg + 1], acc[pj][j][4 * rg + 2], acc[pj][j][4 * rg + 3]};
                        if (a.bias) {
                            const float4 bv = *reinterpret_cast<const float4*>(a.bias + co0);
                            x[0] += bv.x; x[1] += bv.y; x[2] += bv.z; x[3] += bv.w;
                        }
                        if (a.relu_out) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) x[i] = fmaxf(x[i], 0.f);
                        }
                        uint2 rf = make_uint2(0x3f803f80u, 0x3f803f80u);   // 1.0 in every half
                        if (a.mask_ref) rf = *reinterpret_cast<const uint2*>(a.mask_ref + o);
                        const float ref[4] = {bf16_to_f32((unsigned short)rf.x), bf16_to_f32((unsigned short)(rf.x >> 16)),
                                              bf16_to_f32((unsigned short)rf.y), bf16_to_f32((unsigned short)(rf.y >> 16))};
                        if (a.mask_acc) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) x[i] = ref[i] > 0.f ? x[i] : 0.f;
                        }
                        if (a.add) {
                            const uint2 av = *reinterpret_cast<const uint2*>(reinterpret_cast<const unsigned short*>(a.add) + o);
                            const float ad[4] = {bf16_to_f32((unsigned short)av.x), bf16_to_f32((unsigned short)(av.x >> 16)),
                                                 bf16_to_f32((unsigned short)av.y), bf16_to_f32((unsigned short)(av.y >> 16))};
#pragma unroll
                            for (int i = 0; i < 4; ++i) x[i] += (a.mask_add && !(ref[i] > 0.f)) ? 0.f : ad[i];
                        }
                        *reinterpret_cast<uint2*>(reinterpret_cast<unsigned short*>(a.out) + o) =
                            make_uint2(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]));
                        continue;
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (co0 + i >= a.Nn) break;
                        float x = acc[pj][j][4 * rg + i];
                        if (a.bias) x += a.bias[co0 + i];
                        if (a.relu_out) x = fmaxf(x, 0.f);
                        const float ref = a.mask_ref ? bf16_to_f32(a.mask_ref[o + i]) : 1.f;
                        if (a.mask_acc) x = ref > 0.f ? x : 0.f;
                        if (a.add) {
                            const float av = a.out_f32 ? reinterpret_cast<const float*>(a.add)[o + i]
                                                       : bf16_to_f32(reinterpret_cast<const unsigned short*>(a.add)[o + i]);
                            x += (a.mask_add && !(ref > 0.f)) ? 0.f : av;
                        }
                        if (a.out_f32) reinterpret_cast<float*>(a.out)[o + i] = x;
                        else reinterpret_cast<unsigned short*>(a.out)[o + i] = f32_to_bf16(x);
                    }
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
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

template <int NB, int KW, int PJ>
static void launch_conv_bf16_k(const ConvBf16Args& a, hipStream_t st) {
    constexpr int TM = 128 * PJ, QP = kBfCK / 8, KWM = KW > 0 ? KW : 5;
    constexpr size_t lds = (size_t)2 * (((TM + KWM - 1) * QP + 63) / 64 + (KWM * kBfCK * NB / 8 + 63) / 64) * 1024;
    const long long n_tiles = (a.d.Q + TM - 1) / TM;
    int per_cu = (int)(160 * 1024 / lds);
    if (per_cu > 4) per_cu = 4;
    if (per_cu < 1) per_cu = 1;
    const long long cap = 256LL * per_cu;
    const long long gx = ((n_tiles < cap ? n_tiles : cap) + 7) / 8 * 8;
    dim3 grid((unsigned)gx, (a.Nn + NB - 1) / NB);
    if (a.relu_in) hipLaunchKernelGGL((conv_bf16_kernel<NB, KW, true, PJ>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((conv_bf16_kernel<NB, KW, false, PJ>), grid, dim3(256), 0, st, a);
}

// ------------------------------------------------------------------ 3x3 layers: two-dimensional tiles
// Forward / data gradient of 3x3 layers in the plane with cin a multiple of 32 and cout a multiple of 64.  The
// flattened-pixel kernel above re-reads the weights for every 128 pixels and every row tap's slab separately,
// and stores 8-byte pieces 256 bytes apart; it spends more time waiting for staged data and on its stores than
// on the MFMAs.  Here a workgroup of 4 waves owns (4 * kB2Rows) x 32 output pixels x 64 output channels: per
// 16-channel chunk the raw pixel region with its one-pixel halo and all nine taps' weights are staged by direct
// loads into one of two buffers; a wave owns kB2Rows image rows, reads the (kB2Rows + 2) x 3 pixel operands and the
// 18 weight operands of its nine taps and feeds 18 * kB2Rows MFMAs per chunk from them.  Out-of-image quads of the
// region are zeros written once per block (no tap masks, no loads for them).  The output goes through wave-private
// LDS rows so that the fused epilogue reads and writes 64 contiguous bytes per pixel; one barrier per block for it.
// LDS layouts put the 16 lanes a 128-bit access serves together on 16 neighbouring 16-byte slots.  Two workgroups
// per CU.  Measured on the brain workload (128 -> 128, 819 200 pixels, 241.6 GFLOP per launch): 345 us with two
// rows per wave, 350 us with four (half the operand reads and weight traffic per MFMA, but 7 rounds of blocks for
// 6.25 and spilled registers); taking parts out: matrix instructions alone (operands in registers) 134 us, with the
// operand reads 178 us, with the staging loads but no epilogue 257 us, staging loads alone 154 us.
constexpr int kB2Rows = 2;            // image rows per wave
constexpr int kB2TileRows = 4 * kB2Rows;
constexpr int kB2RegUsed = (kB2TileRows + 2) * 2 * 34;          // quads of the region: rows x 2 channel quads x 34 columns
constexpr int kB2RegQuads = (kB2RegUsed + 63) / 64 * 64;       // rounded up to whole wave loads
constexpr int kB2WQuads = 9 * 2 * 64; // nine taps x 2 channel quads x 64 output channels
constexpr int kB2BufQuads = kB2RegQuads + kB2WQuads;
constexpr int kB2StageStride = 34;    // floats per staged output pixel: 32 channels + 2 (bank spread)
constexpr int kB2RegLoads = (kB2RegQuads + 255) / 256;   // direct-load slots per lane: region
constexpr int kB2WLoads = (kB2WQuads + 255) / 256;       // and weights

// weights as LDS images: wt[((((ny*n_kc + kc)*9 + tap)*2 + hq)*64 + nn)*8 + kk], k = 16*kc + 8*hq + kk, n = 64*ny + nn;
// one zero quad follows.  Source (n, tap, k) at w[n*sn + tapidx*st + k*sk], taps mirrored for the data gradient.
__global__ __launch_bounds__(256) void weights_image_bf16_2d_kernel(const float* __restrict__ w, long long sn, long long st_, long long sk,
                                                                    int flip, int K, int Nn, unsigned short* __restrict__ wt) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long total = 9LL * K * Nn;
    if (i < 8) wt[total + i] = 0;
    if (i >= total) return;
    const int kk = (int)(i & 7), nn = (int)((i >> 3) & 63), hq = (int)((i >> 9) & 1);
    const long long rest = i >> 10;
    const int tap = (int)(rest % 9);
    const long long ck = rest / 9;
    const int n_kc = K / 16;
    const int kc = (int)(ck % n_kc), ny = (int)(ck / n_kc);
    const int k = 16 * kc + 8 * hq + kk, n = 64 * ny + nn;
    wt[i] = f32_to_bf16(w[n * sn + (flip ? 8 - tap : tap) * st_ + k * sk]);
}

template <bool RELU>
__global__ __launch_bounds__(256, 2) void conv_bf16_2d_kernel(ConvBf16Args a, int bx_n, int by_n, long long n_blocks) {
    // Two chunk buffers as two arrays, and the chunk loop written out for both: the compiler orders a direct load's
    // LDS write against LDS reads by what it can prove about the addresses, and waits for every pending direct load
    // before any read of the same array (with one array and a computed offset the next chunk's loads were complete
    // before the first operand read of the current chunk, i.e. staging and matrix work ran one after the other).
    __shared__ uint4 bufA[kB2BufQuads];
    __shared__ uint4 bufB[kB2BufQuads];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, h = lane >> 5;
    const int H = a.d.H, W = a.d.W;
    const XcdRange xr = xcd_range(n_blocks);
    if (xr.first >= xr.end) return;   // uniform for the workgroup
    const int ny = blockIdx.y, n0 = 64 * ny, n_kc = a.K / 16;

    // direct-load slots of this lane: quads of the region (slot = (row*2 + channel quad)*34 + column), packed as
    // row << 8 | column << 1 | channel quad; the position of a quad inside the region does not depend on the block.
    // Addresses are formed when a load is issued (a few integer operations per chunk) rather than kept per block:
    // the pointers of two blocks cost more registers than the kernel has, and a spilled pointer is reloaded through
    // the same counter the direct loads use, which serialises them.
    int slot[kB2RegLoads];
#pragma unroll
    for (int i = 0; i < kB2RegLoads; ++i) {
        const int s = tid + 256 * i;
        const int rq = s / 34;
        slot[i] = s < kB2RegUsed ? ((rq >> 1) << 8) | ((s - rq * 34) << 1) | (rq & 1) : -1;   // slots past the region read the zero quad
    }
    struct Block {   // uniform over the workgroup
        int x0, y0;
        long long img;
    };
    auto setup = [&](long long item) {
        Block b;
        const int bx = (int)(item % bx_n);
        const long long rest = item / bx_n;
        const int by = (int)(rest % by_n);
        b.img = rest / by_n;
        b.x0 = bx * 32;
        b.y0 = by * kB2TileRows;
        return b;
    };
    // byte offset of region slot i of block b from a.in (32 bits: the launcher checks the tensor's size), or ~0u for a
    // slot outside the image / past the region
    auto slot_off = [&](const Block& b, int i) -> unsigned {
        const int yy = b.y0 - 1 + (slot[i] >> 8), xx = b.x0 - 1 + ((slot[i] >> 1) & 127);
        const bool ok = slot[i] >= 0 && yy >= 0 && yy < H && xx >= 0 && xx < W;
        return ok ? (unsigned)((((unsigned)(b.img * H + yy) * (unsigned)W + (unsigned)xx) * (unsigned)a.K + 8u * (slot[i] & 1)) * 2u) : ~0u;
    };
    const char* in_bytes = reinterpret_cast<const char*>(a.in);
    const char* w_bytes = reinterpret_cast<const char*>(a.wt) + ((size_t)ny * n_kc * (kB2WQuads * 8) + tid * 8) * 2;
    // Slots outside the image are not loaded; they hold zeros, written by zero_halo when a block touches the border.
    auto issue = [&](const Block& b, int kc, uint4* dst) {
#pragma unroll
        for (int i = 0; i < kB2RegLoads; ++i) {
            const int o = wave + 4 * i;
            if (o < kB2RegQuads / 64) {
                unsigned off = slot_off(b, i);
                if (off != ~0u) {
                    off += kc * 32;
                    asm volatile("" : "+v"(off));   // keeps the 64-bit address out of registers across chunks
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(in_bytes + off),
                                                     (__attribute__((address_space(3))) void*)(dst + o * 64), 16, 0, 0);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < kB2WLoads; ++i) {
            const int o = wave + 4 * i;
            if (o < kB2WQuads / 64) {
                unsigned off = (unsigned)kc * (kB2WQuads * 16) + i * 4096;
                asm volatile("" : "+v"(off));
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(w_bytes + off),
                                                 (__attribute__((address_space(3))) void*)(dst + kB2RegQuads + o * 64), 16, 0, 0);
            }
        }
    };
    auto touches_border = [&](const Block& b) { return b.x0 == 0 || b.y0 == 0 || b.x0 + 32 >= W || b.y0 + kB2TileRows >= H; };
    auto zero_halo = [&](const Block& b, uint4* dst) {
#pragma unroll
        for (int i = 0; i < kB2RegLoads; ++i) {
            const int o = wave + 4 * i;
            if (o < kB2RegQuads / 64 && slot_off(b, i) == ~0u) dst[o * 64 + lane] = make_uint4(0u, 0u, 0u, 0u);
        }
    };

    // this lane's operands: pixel (region row 4*wave + r, column m + dx), channel quad h; weights (tap, quad h, cout m + 32 j)
    const int pb0 = ((kB2Rows * wave) * 2 + h) * 34 + m;
    const int wa0 = kB2RegQuads + h * 64 + m;

    floatx16 acc[kB2Rows][2];   // [image row of the wave][cout block]
    auto compute = [&](const uint4* buf) {
        // the pixel operands of all taps first, then per tap its two weight operands and the matrix instructions that
        // use them (fetching every weight operand up front as well measured the same)
        bf16x8 pv[kB2Rows + 2][3];
#pragma unroll
        for (int r = 0; r < kB2Rows + 2; ++r)
#pragma unroll
            for (int dx = 0; dx < 3; ++dx) {
                uint4 pb = buf[pb0 + r * 68 + dx];
                if (RELU) {
                    pb.x = relu_bf16x2(pb.x); pb.y = relu_bf16x2(pb.y); pb.z = relu_bf16x2(pb.z); pb.w = relu_bf16x2(pb.w);
                }
                pv[r][dx] = __builtin_bit_cast(bf16x8, pb);
            }
#pragma unroll
        for (int dy = 0; dy < 3; ++dy)
#pragma unroll
            for (int dx = 0; dx < 3; ++dx) {
                const bf16x8 w0 = __builtin_bit_cast(bf16x8, buf[wa0 + (dy * 3 + dx) * 128]);
                const bf16x8 w1 = __builtin_bit_cast(bf16x8, buf[wa0 + (dy * 3 + dx) * 128 + 32]);
#pragma unroll
                for (int r = 0; r < kB2Rows; ++r) {
                    acc[r][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0, pv[dy + r][dx], acc[r][0], 0, 0, 0);
                    acc[r][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1, pv[dy + r][dx], acc[r][1], 0, 0, 0);
                }
            }
    };

    // epilogue constants: a lane finishes 4 output channels (one 8-byte bf16 piece) of 4 pixels per pass
    const int e_piece = lane & 7, e_px = lane >> 3;
    Block cur = setup(xr.first);
    issue(cur, 0, bufA);
    for (long long item = xr.first; item < xr.end; item += xr.stride) {
        const bool has_next = item + xr.stride < xr.end;
        const Block nxt = setup(has_next ? item + xr.stride : item);
        // Out-of-image slots of both buffers: zeros, valid for every chunk of this block (the direct loads skip them).
        // The first buffer already holds (or is receiving) this block's first chunk in its other slots; the second
        // was the previous block's staging area.
        if (touches_border(cur)) {
            zero_halo(cur, bufA);
            zero_halo(cur, bufB);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
#pragma unroll
        for (int pj = 0; pj < kB2Rows; ++pj)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[pj][j][r] = 0.f;
        for (int kc = 0; kc < n_kc; kc += 2) {   // n_kc is even
            issue(cur, kc + 1, bufB);
            __builtin_amdgcn_sched_barrier(0);
            compute(bufA);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            // the first chunk of the next block is fetched under the last MFMAs of this one
            if (kc + 2 < n_kc) issue(cur, kc + 2, bufA);
            else if (has_next) issue(nxt, 0, bufA);
            __builtin_amdgcn_sched_barrier(0);
            compute(bufB);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        }
        // Output through LDS, one pass per (image row of the wave, cout block): the wave turns its own float32
        // [32 pixels][32 channels] block through its own staging rows (LDS operations of one wave execute in order,
        // so no barrier separates the passes), then bias / ReLU / ReLU mask / add and 8-byte stores that are
        // contiguous per pixel.  The staging area is the chunk buffer that the prefetch of the next block does not
        // use; the next block's second chunk will be loaded into it, hence the one barrier after the last pass.
        float* stage = reinterpret_cast<float*>(bufB) + wave * 32 * kB2StageStride;   // the prefetch of the next block went into bufA
        // ReLU mask as sign bits: bit 16*j + 4*it + e of this lane's word pj says whether the value of pass (pj, j),
        // pixel e_px + 8*it, channel e of its piece is positive.  The forward launch that produces an activation writes
        // the words, the data-gradient launch into the same tensor (same geometry, so the same lane holds the
        // same values) reads them instead of the activation.
        const long long word_idx = (((long long)ny * n_blocks + item) * 256 + tid) * 4;
        uint4 sign_in4 = make_uint4(0u, 0u, 0u, 0u);
        if (a.bits_in) sign_in4 = *reinterpret_cast<const uint4*>(a.bits_in + word_idx);
        const unsigned sign_in[4] = {sign_in4.x, sign_in4.y, sign_in4.z, sign_in4.w};
        unsigned sign_out[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int pj = 0; pj < kB2Rows; ++pj)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int rg = 0; rg < 4; ++rg)
                    *reinterpret_cast<float4*>(stage + m * kB2StageStride + 8 * rg + 4 * h) =
                        make_float4(acc[pj][j][4 * rg], acc[pj][j][4 * rg + 1], acc[pj][j][4 * rg + 2], acc[pj][j][4 * rg + 3]);
                const int y = cur.y0 + kB2Rows * wave + pj;
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int px = e_px + 8 * it;                  // column of the tile
                    const int x = cur.x0 + px;
                    const float4 v4 = *reinterpret_cast<const float4*>(stage + px * kB2StageStride + 4 * e_piece);
                    if (y < H && x < W) {
                        const int co = n0 + 32 * j + 4 * e_piece;
                        const long long o = ((cur.img * H + y) * W + x) * a.Nn + co;
                        float xv[4] = {v4.x, v4.y, v4.z, v4.w};
                        if (a.bias) {
                            const float4 bv = *reinterpret_cast<const float4*>(a.bias + co);
                            xv[0] += bv.x; xv[1] += bv.y; xv[2] += bv.z; xv[3] += bv.w;
                        }
                        if (a.relu_out) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) xv[e] = fmaxf(xv[e], 0.f);
                        }
                        uint2 rf = make_uint2(0x3f803f80u, 0x3f803f80u);   // 1.0 in every half
                        if (a.mask_ref && !a.bits_in) rf = *reinterpret_cast<const uint2*>(a.mask_ref + o);
                        const float ref[4] = {bf16_to_f32((unsigned short)rf.x), bf16_to_f32((unsigned short)(rf.x >> 16)),
                                              bf16_to_f32((unsigned short)rf.y), bf16_to_f32((unsigned short)(rf.y >> 16))};
                        const int bit0 = 16 * j + 4 * it;
                        const unsigned sw = sign_in[pj];
                        bool pos[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) pos[e] = a.bits_in ? ((sw >> (bit0 + e)) & 1u) != 0u : ref[e] > 0.f;
                        if (a.mask_acc) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) xv[e] = pos[e] ? xv[e] : 0.f;
                        }
                        if (a.add) {
                            const uint2 av = *reinterpret_cast<const uint2*>(reinterpret_cast<const unsigned short*>(a.add) + o);
                            const float ad[4] = {bf16_to_f32((unsigned short)av.x), bf16_to_f32((unsigned short)(av.x >> 16)),
                                                 bf16_to_f32((unsigned short)av.y), bf16_to_f32((unsigned short)(av.y >> 16))};
#pragma unroll
                            for (int e = 0; e < 4; ++e) xv[e] += (a.mask_add && !pos[e]) ? 0.f : ad[e];
                        }
                        const uint2 packed = make_uint2(pack_bf16x2(xv[0], xv[1]), pack_bf16x2(xv[2], xv[3]));
                        *reinterpret_cast<uint2*>(reinterpret_cast<unsigned short*>(a.out) + o) = packed;
                        if (a.bits_out) {   // the sign of what was stored, i.e. of the rounded value: 0x0001 .. 0x7fff
                            const unsigned hv[4] = {packed.x & 0xffffu, packed.x >> 16, packed.y & 0xffffu, packed.y >> 16};
#pragma unroll
                            for (int e = 0; e < 4; ++e) sign_out[pj] |= (hv[e] - 1u < 0x7fffu ? 1u : 0u) << (bit0 + e);
                        }
                    }
                }
            }
        if (a.bits_out) *reinterpret_cast<uint4*>(a.bits_out + word_idx) = make_uint4(sign_out[0], sign_out[1], sign_out[2], sign_out[3]);
        __syncthreads();   // every wave is done with its staging rows: the next block's second chunk lands there
        cur = nxt;
    }
}

// ------------------------------------------------------------------ 3x3 layers: weights resident in registers
// Forward / data gradient of 3x3 layers with up to 128 input channels and a multiple of 128 output channels.  The
// kernels above re-stage the nine taps' weights for every tile (two thirds of what they pull through L2) and are bound
// by that traffic and by LDS operand reads.  Here one workgroup of 4 waves owns a CU (one wave per SIMD, the whole
// 512-register file each): wave w keeps the weights of its 32 output channels - 9 taps x K input channels, 72 MFMA
// A operands = 288 registers for K = 128 - for the life of the kernel, and only pixels stream: the raw 6 x 34-pixel
// region of a 4 x 32-pixel tile with all K channels goes global -> LDS by direct loads into one of two buffers (separate
// LDS objects, tile loop written out for both) while the MFMAs of the previous tile run; all four waves read the
// same pixel operands.  A wave works on two image rows at a time (two independent accumulator chains; a pixel
// operand read from LDS feeds up to two MFMAs).  A pixel takes one 16-byte slot more than its channel quads in LDS, so
// that the 16 lanes a 128-bit read serves together (16 neighbouring pixels, one quad) fall on 16 different bank groups
// while every operand address is one lane register plus a constant (an XOR swizzle needs a register per operand:
// 96 of them, which the compiler spills).  Out-of-image quads and the padding slots are loaded from a zero quad.  Epilogue straight from the accumulators: a lane holds 16 channels
// of its pixel in groups of four, 8-byte stores.
constexpr int kRwStageStride = 36;   // floats per staged output pixel: 32 channels + 4 (bank spread)
template <int NKC> struct RwGeom {
    static constexpr int PIXQ = 2 * NKC;                 // 16-byte quads per pixel (K = 16 * NKC channels)
    static constexpr int PIXS = PIXQ + 1;                // LDS slots per pixel: one unused slot of padding
    static constexpr int ROWS = 6, COLS = 34;            // region of a 4 x 32 tile
    static constexpr int QUADS = ROWS * COLS * PIXS;
    static constexpr int LOADS = (QUADS + 63) / 64;      // wave-wide direct loads per region
    static constexpr int PER_LANE = (LOADS + 3) / 4;
};

// weights as A operands: wt[((((ny*4 + wave)*9 + tap)*NKC + kc)*64 + lane)*8 + s] = W[n = 128*ny + 32*wave + (lane & 31)]
// [tap][k = 16*kc + 8*(lane >> 5) + s]; one zero quad follows.  Source (n, tap, k) at w[n*sn + tapidx*st + k*sk].
__global__ __launch_bounds__(256) void weights_image_bf16_rw_kernel(const float* __restrict__ w, long long sn, long long st_, long long sk,
                                                                    int flip, int K, int Nn, unsigned short* __restrict__ wt) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long total = 9LL * K * Nn;
    if (i < 8) wt[total + i] = 0;
    if (i >= total) return;
    const int nkc = K / 16;
    const int s = (int)(i & 7), lane = (int)((i >> 3) & 63);
    long long rest = i >> 9;
    const int kc = (int)(rest % nkc);
    rest /= nkc;
    const int tap = (int)(rest % 9);
    rest /= 9;
    const int wave = (int)(rest & 3), ny = (int)(rest >> 2);
    const int n = 128 * ny + 32 * wave + (lane & 31), k = 16 * kc + 8 * (lane >> 5) + s;
    wt[i] = f32_to_bf16(w[n * sn + (flip ? 8 - tap : tap) * st_ + k * sk]);
}

// VAR: 0 forward; 1 forward that leaves the ReLU mask of its output as lane masks; 2 data gradient with the ReLU mask
// taken from the activation; 3 data gradient with the mask taken from lane masks.
template <bool RELU, int NKC, int VAR>
__global__ __launch_bounds__(256, 1) void conv_bf16_rw_kernel(ConvBf16Args a, int bx_n, int by_n, long long n_blocks) {
    using G = RwGeom<NKC>;
    constexpr int PIXQ = G::PIXQ, K = 16 * NKC;
    __shared__ uint4 bufA[G::LOADS * 64];
    __shared__ uint4 bufB[G::LOADS * 64];
    __shared__ __attribute__((aligned(16))) float stage_all[4 * 32 * kRwStageStride];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, h = lane >> 5;
    const int H = a.d.H, W = a.d.W;
    const XcdRange xr = xcd_range(n_blocks);
    if (xr.first >= xr.end) return;   // uniform for the workgroup
    const int ny = blockIdx.y, n0 = 128 * ny + 32 * wave;

    // this wave's weights, for the life of the kernel
    bf16x8 wr[9][NKC];
    {
        const uint4* wp = reinterpret_cast<const uint4*>(a.wt) + ((size_t)(ny * 4 + wave) * 9 * NKC) * 64 + lane;
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) wr[t][kc] = __builtin_bit_cast(bf16x8, wp[(t * NKC + kc) * 64]);
    }
    const unsigned short* zero = a.wt + 9LL * K * a.Nn;

    // direct-load slots of this lane: slot s = tid + 256*i is channel quad s % PIXS (the last one: padding) of region
    // pixel s / PIXS; element offset from the region origin (pixel (y0-1, x0-1))
    constexpr int PIXS = G::PIXS;
    unsigned s_off[G::PER_LANE];
#pragma unroll
    for (int i = 0; i < G::PER_LANE; ++i) {
        const int s = tid + 256 * i;
        const int px = s / PIXS, pos = s - px * PIXS;
        const int row = px / G::COLS, col = px - row * G::COLS;
        s_off[i] = (s < G::QUADS && pos < PIXQ) ? (unsigned)((row * W + col) * K + 8 * pos) : 0u;
    }
    struct Block {
        int x0, y0;
        long long img, item;
    };
    auto setup = [&](long long item) {
        Block b;
        b.item = item;
        const int bx = (int)(item % bx_n);
        const long long rest = item / bx_n;
        const int by = (int)(rest % by_n);
        b.img = rest / by_n;
        b.x0 = bx * 32;
        b.y0 = by * 4;
        return b;
    };
    auto issue = [&](const Block& b, uint4* dst) {
        const bool interior = b.y0 >= 1 && b.y0 + 4 < H && b.x0 >= 1 && b.x0 + 32 < W;   // uniform
        const unsigned short* base = a.in + ((b.img * H + b.y0 - 1) * W + b.x0 - 1) * K;   // only dereferenced inside the image
        if (interior) {
            // uniform base + 32-bit lane offset; the padding slots (never read) fetch the region's first quad
#pragma unroll
            for (int i = 0; i < G::PER_LANE; ++i) {
                const int o = wave + 4 * i;
                if (o < G::LOADS)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + s_off[i]),
                                                     (__attribute__((address_space(3))) void*)(dst + o * 64), 16, 0, 0);
            }
        } else {
            int t = tid;
            asm volatile("" : "+v"(t));   // the slots' pixels are recomputed per border tile rather than kept in registers
#pragma unroll
            for (int i = 0; i < G::PER_LANE; ++i) {
                const int o = wave + 4 * i;
                if (o < G::LOADS) {
                    const int s = t + 256 * i;
                    const int px = s / PIXS;
                    const int row = px / G::COLS, col = px - row * G::COLS;
                    const int yy = b.y0 - 1 + row, xx = b.x0 - 1 + col;
                    const bool ok = s < G::QUADS && yy >= 0 && yy < H && xx >= 0 && xx < W;
                    const unsigned short* p = ok ? base + s_off[i] : zero;
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)p,
                                                     (__attribute__((address_space(3))) void*)(dst + o * 64), 16, 0, 0);
                }
            }
        }
    };

    floatx16 acc[4];   // the tile's four image rows
    const int lane_q = m * PIXS + h;   // this lane's pixel column and half of a 16-channel block, in 16-byte slots

    // ---- epilogue, cut into parts that are interleaved with the MFMAs of the next image-row pair.  With one wave per
    // SIMD nothing else hides its instructions (run after the MFMAs it took a third of the kernel's time), and every
    // vector instruction takes an issue slot from the MFMAs, so it is kept short.  It is free of branches, so that the
    // compiler can schedule its parts between the MFMAs: pixels outside the image (and a tile that does not exist) get
    // a buffer offset past the end, which the hardware drops on stores and answers with zeros on loads, and a tensor to
    // add that the call does not have is read through an empty buffer.
    // Accumulator r of lane (m, h): output channel n0 + 8*(r/4) + 4*h + r%4 of pixel (row, x0 + m).  Stored from there a
    // wave store would touch 32 separate 16-byte pieces (the L2 takes as long over those as the MFMAs over the tile), so
    // the wave turns its 32 pixels x 32 channels around in its own LDS rows (LDS operations of one wave execute in
    // order: no barrier) and a lane finishes 8 channels of a pixel: 16-byte stores, 64 contiguous bytes per pixel.
    // ReLU mask as sign bits, in the form the hardware compares and selects with: one 64-bit lane mask per (wave, image
    // row, pass, channel e of a lane's piece), bit l = the value lane l holds is positive.  The forward launch that
    // produces an activation writes the masks (VAR 1), the data-gradient launch into the same tensor (same geometry,
    // so the same lane holds the same values) reads them (VAR 3) instead of the activation (VAR 2); VAR 0: no mask.
    constexpr bool kMasked = VAR >= 2, kWriteBits = VAR == 1, kReadBits = VAR == 3;
    float* stage = stage_all + wave * 32 * kRwStageStride;
    const int e_px = lane >> 2, e_c8 = lane & 3;
    const unsigned out_bytes = (unsigned)(2 * a.d.Q * a.Nn);   // the launcher checks that this fits 32 bits
    const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, out_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t r_mask =
        __builtin_amdgcn_make_buffer_rsrc((void*)(VAR == 2 ? (const void*)a.mask_ref : (const void*)a.out), 0, VAR == 2 ? out_bytes : 0u, 0x00020000);
    const __amdgpu_buffer_rsrc_t r_add =
        __builtin_amdgcn_make_buffer_rsrc((void*)(a.add ? a.add : (const void*)a.out), 0, a.add ? out_bytes : 0u, 0x00020000);
    const unsigned word_bytes = (unsigned)(n_blocks * (a.Nn / 128) * 256 * 8);
    const __amdgpu_buffer_rsrc_t r_bits = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(kReadBits ? (const void*)a.bits_in : (kWriteBits ? (const void*)a.bits_out : (const void*)a.out)), 0,
        (kReadBits || kWriteBits) ? word_bytes : 0u, 0x00020000);
    float bias_r[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) bias_r[e] = a.bias ? a.bias[n0 + 8 * e_c8 + e] : 0.f;
    const float relu_floor = a.relu_out ? 0.f : -__builtin_huge_valf();
    const unsigned long long acc_all = a.mask_acc ? 0ull : ~0ull, add_all = a.mask_add ? 0ull : ~0ull;   // uniform

    typedef unsigned uint4v __attribute__((ext_vector_type(4)));
    typedef unsigned uint2v __attribute__((ext_vector_type(2)));
    struct Slice {   // one piece (image row j, pass it) on its way out
        unsigned off;
        float xv[8];
        uint4v rf, av;
        uint2v mk;
        unsigned long long pos[8];   // uniform: lane masks of the ReLU mask
    };
    Slice sl;
    // byte offset of the eight lane masks of piece (pair q, s = row parity * 2 + pass) of block b: lane e < 8 of a wave holds mask e
    auto mask_off = [&](const Block& b, int q, int s_, bool all_lanes) -> unsigned {
        const bool ok = b.item >= 0 && (all_lanes || lane < 8);
        return ok ? (unsigned)(((((((long long)ny * n_blocks + b.item) * 4 + wave) * 2 + q) * 4 + s_) * 8 + (lane & 7)) * 8) : ~0u;
    };
    // a 16-bit half of w is a positive bfloat16 (0x0001 .. 0x7fff), as a lane mask
    auto positive_lo = [&](unsigned w) { return __builtin_amdgcn_ballot_w64((int)(w << 16) > 0); };
    auto positive_hi = [&](unsigned w) { return __builtin_amdgcn_ballot_w64((int)w > 0xffff); };
    // part 0..5 of piece (j, it) of block b; q = j / 2
    auto epi_part = [&](const Block& b, int j, int it, int part) __attribute__((always_inline)) {
        const int q = j >> 1, s_ = 2 * (j & 1) + it;
        if (part == 0) {
            if (it == 0) {
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<float4*>(stage + m * kRwStageStride + 8 * g + 4 * h) =
                        make_float4(acc[j][4 * g], acc[j][4 * g + 1], acc[j][4 * g + 2], acc[j][4 * g + 3]);
            }
            const int px = e_px + 16 * it, x = b.x0 + px, y = b.y0 + j;
            const bool ok = b.item >= 0 && y < H && x < W;
            sl.off = ok ? ((unsigned)(b.img * H + y) * (unsigned)W + (unsigned)x) * (unsigned)(2 * a.Nn) + 2u * (unsigned)(n0 + 8 * e_c8) : ~0u;
            if (VAR == 2) sl.rf = __builtin_amdgcn_raw_buffer_load_b128(r_mask, sl.off, 0, 0);
            if (kReadBits) sl.mk = __builtin_amdgcn_raw_buffer_load_b64(r_bits, mask_off(b, q, s_, true), 0, 0);
            sl.av = __builtin_amdgcn_raw_buffer_load_b128(r_add, sl.off, 0, 0);
        } else if (part == 1) {
            const int px = e_px + 16 * it;
            const float4 v0 = *reinterpret_cast<const float4*>(stage + px * kRwStageStride + 8 * e_c8);
            const float4 v1 = *reinterpret_cast<const float4*>(stage + px * kRwStageStride + 8 * e_c8 + 4);
            const float t[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) sl.xv[e] = fmaxf(t[e] + bias_r[e], relu_floor);
        } else if (part == 2) {
            if (kMasked) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (kReadBits)
                        sl.pos[e] = (unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)sl.mk[0], e) |   // (the builtin returns int)
                                    ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)sl.mk[1], e) << 32);
                    else
                        sl.pos[e] = (e & 1) ? positive_hi(sl.rf[e >> 1]) : positive_lo(sl.rf[e >> 1]);
                }
            }
        } else if (part == 3) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float x = sl.xv[e];
                const float ad = __uint_as_float((e & 1) ? (sl.av[e >> 1] & 0xffff0000u) : (sl.av[e >> 1] << 16));
                if (kMasked) {
                    x = __builtin_amdgcn_inverse_ballot_w64(sl.pos[e] | acc_all) ? x : 0.f;
                    x += __builtin_amdgcn_inverse_ballot_w64(sl.pos[e] | add_all) ? ad : 0.f;
                } else {
                    x += ad;
                }
                sl.xv[e] = x;
            }
        } else if (part == 4) {
            uint4v packed;
            packed[0] = pack_bf16x2(sl.xv[0], sl.xv[1]); packed[1] = pack_bf16x2(sl.xv[2], sl.xv[3]);
            packed[2] = pack_bf16x2(sl.xv[4], sl.xv[5]); packed[3] = pack_bf16x2(sl.xv[6], sl.xv[7]);
            __builtin_amdgcn_raw_buffer_store_b128(packed, r_out, sl.off, 0, 0);
            sl.rf = packed;   // kept for the sign masks
        } else {
            if (kWriteBits) {
                // the sign of what was stored, i.e. of the rounded value; lanes whose store was dropped report "not positive"
                const unsigned keep = sl.off != ~0u ? 0xffffffffu : 0u;
                uint2v out_m = {0u, 0u};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const unsigned w = sl.rf[e >> 1] & keep;
                    const unsigned long long pm = (e & 1) ? positive_hi(w) : positive_lo(w);
                    out_m[0] = lane == e ? (unsigned)pm : out_m[0];
                    out_m[1] = lane == e ? (unsigned)(pm >> 32) : out_m[1];
                }
                __builtin_amdgcn_raw_buffer_store_b64(out_m, r_bits, mask_off(b, q, s_, false), 0, 0);
            }
        }
    };

    // MFMAs of image rows 2p and 2p + 1 of the tile in `buf`, with the epilogue of rows 2q, 2q + 1 of block eb between them.
    // Pixel operand (region row 2p + rho, column m + dx, channels 16 kc + 8 h ..) feeds tap (rho, dx) of the upper row and
    // tap (rho - 1, dx) of the lower one; operands come in groups of four (one dx of one 16-channel block), the reads of
    // a group are issued before the six MFMAs of the group ahead of it, and every group carries one part of the epilogue
    // (4 pieces x 6 parts = 24 groups).
    auto compute = [&](const uint4* buf, int p, const Block& eb, int q) __attribute__((always_inline)) {
        uint4 bq[2][4];
        auto read_group = [&](int g, uint4* b) {
            const int kc = g / 3, dx = g - 3 * kc;
#pragma unroll
            for (int rho = 0; rho < 4; ++rho) {
                b[rho] = buf[lane_q + ((2 * p + rho) * G::COLS + dx) * PIXS + 2 * kc];
                if (RELU) {
                    b[rho].x = relu_bf16x2(b[rho].x); b[rho].y = relu_bf16x2(b[rho].y);
                    b[rho].z = relu_bf16x2(b[rho].z); b[rho].w = relu_bf16x2(b[rho].w);
                }
            }
        };
        read_group(0, bq[0]);
#pragma unroll
        for (int g = 0; g < 3 * NKC; ++g) {
            const int kc = g / 3, dx = g - 3 * kc;
            if (g + 1 < 3 * NKC) read_group(g + 1, bq[(g + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            epi_part(eb, 2 * q + g / 12, (g / 6) & 1, g % 6);
#pragma unroll
            for (int rho = 0; rho < 4; ++rho) {
                const bf16x8 bv = __builtin_bit_cast(bf16x8, bq[g & 1][rho]);
                if (rho <= 2) {
                    if (g == 0 && rho == 0) {
                        floatx16 z;
#pragma unroll
                        for (int r = 0; r < 16; ++r) z[r] = 0.f;
                        acc[2 * p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[rho * 3 + dx][kc], bv, z, 0, 0, 0);
                    } else {
                        acc[2 * p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[rho * 3 + dx][kc], bv, acc[2 * p], 0, 0, 0);
                    }
                }
                if (rho >= 1) {
                    if (g == 0 && rho == 1) {
                        floatx16 z;
#pragma unroll
                        for (int r = 0; r < 16; ++r) z[r] = 0.f;
                        acc[2 * p + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[(rho - 1) * 3 + dx][kc], bv, z, 0, 0, 0);
                    } else {
                        acc[2 * p + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[(rho - 1) * 3 + dx][kc], bv, acc[2 * p + 1], 0, 0, 0);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    static_assert(NKC == 8, "24 operand groups per row pair carry the 24 epilogue parts");

    // One tile: rows 0, 1 are computed while rows 2, 3 of the previous tile leave, then rows 2, 3 while rows 0, 1 leave.
    auto tile = [&](const Block& cur, const Block& prev, const Block& nxt, bool has_next, const uint4* buf, uint4* other)
                    __attribute__((always_inline)) {
        if (has_next) issue(nxt, other);
        __builtin_amdgcn_sched_barrier(0);
        compute(buf, 0, prev, 1);
        compute(buf, 1, cur, 0);
        // (the counter waited on also counts this tile's stores; they have had the tile to drain)
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };

    Block none;
    none.x0 = none.y0 = 0; none.img = 0; none.item = -1;
    Block cur = setup(xr.first), prev = none;
    issue(cur, bufA);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (long long item = xr.first; item < xr.end; item += 2 * xr.stride) {
        const bool n1 = item + xr.stride < xr.end;
        const Block b1 = setup(n1 ? item + xr.stride : item);
        tile(cur, prev, b1, n1, bufA, bufB);
        prev = cur;
        if (!n1) break;
        const bool n2 = item + 2 * xr.stride < xr.end;
        const Block b2 = setup(n2 ? item + 2 * xr.stride : item);
        tile(b1, prev, b2, n2, bufB, bufA);
        prev = b1;
        cur = b2;
    }
    // rows 2, 3 of the last tile
#pragma unroll
    for (int s_ = 0; s_ < 4; ++s_)
#pragma unroll
        for (int part = 0; part < 6; ++part) epi_part(prev, 2 + s_ / 2, s_ & 1, part);
}

static bool conv_bf16_rw_applies(const ConvBf16Args& a) {
    // byte offsets inside a region are 32 bits in the kernel
    return a.d.kt == 1 && a.d.kd == 1 && a.d.kh == 3 && a.d.kw == 3 && a.K == 128 && a.Nn % 128 == 0 && !a.out_f32 &&
           12.0 * a.d.W * a.K < 2.0e9 && 2.0 * (double)a.d.Q * a.Nn < 4.0e9;
}

static hipError_t launch_conv_bf16_rw(ConvBf16Args a, const float* w, long long sn, long long st_, long long sk, int flip,
                                      unsigned short* wt_scratch, hipStream_t st) {
    {
        const long long total = 9LL * a.K * a.Nn;
        KernelScope ks("weights_image_bf16", 0.0, 6.0 * (double)total, st);
        hipLaunchKernelGGL(weights_image_bf16_rw_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, w, sn, st_, sk, flip,
                           a.K, a.Nn, wt_scratch);
    }
    a.wt = wt_scratch;
    const int bx_n = (a.d.W + 31) / 32, by_n = (a.d.H + 3) / 4;
    const long long n_img = a.d.Q / ((long long)a.d.H * a.d.W);
    const long long n_blocks = n_img * bx_n * by_n;
    const long long cap = 256;   // one workgroup per CU
    const long long gx = ((n_blocks < cap ? n_blocks : cap) + 7) / 8 * 8;
    dim3 grid((unsigned)gx, (unsigned)(a.Nn / 128));
    char name[56];
    snprintf(name, sizeof(name), "conv_bf16_%s_%dto%d_t9", flip ? "dgrad" : "fwd", a.K, a.Nn);
    KernelScope ks(name, 2.0 * (double)a.d.Q * a.K * a.Nn * 9, 2.0 * (double)a.d.Q * (a.K + a.Nn), st);
    const int var = a.mask_ref ? (a.bits_in ? 3 : 2) : (a.bits_out ? 1 : 0);
    auto go = [&](auto kern) { hipLaunchKernelGGL(kern, grid, dim3(256), 0, st, a, bx_n, by_n, n_blocks); };
    if (a.relu_in) {
        if (var == 0) go(conv_bf16_rw_kernel<true, 8, 0>);
        else if (var == 1) go(conv_bf16_rw_kernel<true, 8, 1>);
        else if (var == 2) go(conv_bf16_rw_kernel<true, 8, 2>);
        else go(conv_bf16_rw_kernel<true, 8, 3>);
    } else {
        if (var == 0) go(conv_bf16_rw_kernel<false, 8, 0>);
        else if (var == 1) go(conv_bf16_rw_kernel<false, 8, 1>);
        else if (var == 2) go(conv_bf16_rw_kernel<false, 8, 2>);
        else go(conv_bf16_rw_kernel<false, 8, 3>);
    }
    return hipGetLastError();
}

static bool conv_bf16_2d_applies(const ConvBf16Args& a) {
    // an even number of 16-channel chunks; byte offsets into the input tensor are 32 bits in the kernel
    return a.d.kt == 1 && a.d.kd == 1 && a.d.kh == 3 && a.d.kw == 3 && a.K % 32 == 0 && a.Nn % 64 == 0 && !a.out_f32 &&
           2.0 * (double)a.d.Q * a.K < 4.0e9;
}

// GLEAM_POLICY_NO_BF16_2D keeps the flattened-pixel kernel
static bool bf16_2d_enabled() { return !(kernel_policy() & GLEAM_POLICY_NO_BF16_2D); }

int conv_bf16_takes_sign_words(const PixDims& d, int K, int Nn) {
    ConvBf16Args a{};
    a.d = d; a.K = K; a.Nn = Nn;
    if (!bf16_2d_enabled()) return 0;
    if (conv_bf16_rw_applies(a)) return 2;
    return conv_bf16_2d_applies(a) ? 1 : 0;
}

size_t conv_bf16_sign_words(const PixDims& d, int Nn, int variant) {
    const size_t n_img = (size_t)d.Q / ((size_t)d.H * d.W);
    if (variant == 2)   // two words per thread, 4 x 32 tile and group of 128 channels
        return n_img * ((d.W + 31) / 32) * ((d.H + 3) / 4) * 256 * 2 * (size_t)(Nn / 128);
    // four words per thread, block and group of 64 channels
    return n_img * ((d.W + 31) / 32) * ((d.H + kB2TileRows - 1) / kB2TileRows) * 256 * 4 * (size_t)(Nn / 64);
}

static hipError_t launch_conv_bf16_2d(ConvBf16Args a, const float* w, long long sn, long long st_, long long sk, int flip,
                                      unsigned short* wt_scratch, hipStream_t st) {
    {
        const long long total = 9LL * a.K * a.Nn;
        KernelScope ks("weights_image_bf16", 0.0, 6.0 * (double)total, st);
        hipLaunchKernelGGL(weights_image_bf16_2d_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, w, sn, st_, sk, flip,
                           a.K, a.Nn, wt_scratch);
    }
    a.wt = wt_scratch;
    const int bx_n = (a.d.W + 31) / 32, by_n = (a.d.H + kB2TileRows - 1) / kB2TileRows;
    const long long n_img = a.d.Q / ((long long)a.d.H * a.d.W);
    const long long n_blocks = n_img * bx_n * by_n;
    const long long cap = 512 / (a.Nn / 64) > 8 ? 512 / (a.Nn / 64) : 8;   // two workgroups per CU in total
    const long long gx = ((n_blocks < cap ? n_blocks : cap) + 7) / 8 * 8;
    dim3 grid((unsigned)gx, (unsigned)(a.Nn / 64));
    char name[56];
    snprintf(name, sizeof(name), "conv_bf16_%s_%dto%d_t9", flip ? "dgrad" : "fwd", a.K, a.Nn);
    KernelScope ks(name, 2.0 * (double)a.d.Q * a.K * a.Nn * 9, 2.0 * (double)a.d.Q * (a.K + a.Nn), st);
    if (a.relu_in) hipLaunchKernelGGL((conv_bf16_2d_kernel<true>), grid, dim3(256), 0, st, a, bx_n, by_n, n_blocks);
    else hipLaunchKernelGGL((conv_bf16_2d_kernel<false>), grid, dim3(256), 0, st, a, bx_n, by_n, n_blocks);
    return hipGetLastError();
}

hipError_t launch_conv_bf16(const ConvBf16Args& a_in, const float* w, long long sn, long long st_, long long sk, int flip,
                            unsigned short* wt_scratch, hipStream_t stream) {
    ConvBf16Args a = a_in;
    if (bf16_2d_enabled() && conv_bf16_rw_applies(a)) return launch_conv_bf16_rw(a, w, sn, st_, sk, flip, wt_scratch, stream);
    if (bf16_2d_enabled() && conv_bf16_2d_applies(a)) return launch_conv_bf16_2d(a, w, sn, st_, sk, flip, wt_scratch, stream);
    const int taps = a.d.kt * a.d.kd * a.d.kh * a.d.kw;
    const int nb = bf_nb(a.Nn);
    {
        WimgBf16Args t{};
        t.w = w; t.wt = wt_scratch; t.sn = sn; t.st = st_; t.sk = sk;
        t.K = a.K; t.Nn = a.Nn; t.flip = flip; t.taps = taps; t.kw = a.d.kw; t.NB = nb;
        t.n_kc = (a.K + kBfCK - 1) / kBfCK; t.n_nb = (a.Nn + nb - 1) / nb;
        t.total = (long long)conv_bf16_wimg_elems(a.K, a.Nn, taps);
        KernelScope ks("weights_image_bf16", 0.0, 6.0 * (double)t.total, stream);
        hipLaunchKernelGGL(weights_image_bf16_kernel, dim3((unsigned)((t.total + 255) / 256)), dim3(256), 0, stream, t);
    }
    a.wt = wt_scratch;
    char name[56];
    snprintf(name, sizeof(name), "conv_bf16_%s_%dto%d_t%d", flip ? "dgrad" : "fwd", a.K, a.Nn, taps);
    KernelScope ks(name, 2.0 * (double)a.d.Q * a.K * a.Nn * taps, 2.0 * (double)a.d.Q * (a.K + a.Nn), stream);
    if (nb == 32) {
        if (a.d.kw == 3) launch_conv_bf16_k<32, 3, 1>(a, stream);
        else if (a.d.kw == 1) launch_conv_bf16_k<32, 1, 1>(a, stream);
        else launch_conv_bf16_k<32, 0, 1>(a, stream);
    } else {
        if (a.d.kw == 3) launch_conv_bf16_k<64, 3, 1>(a, stream);
        else if (a.d.kw == 1) launch_conv_bf16_k<64, 1, 1>(a, stream);
        else launch_conv_bf16_k<64, 0, 1>(a, stream);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ weight gradient
constexpr int kBwTM = 32;     // pixels per staged chunk = two MFMA K-blocks of 16
constexpr int kBwSlab = 36;   // slab rows per row tap: 32 + 2 halo, rounded up to the 12-pixel read windows
constexpr size_t kBwLdsMax = 150 * 1024;

// LDS rows are pixels, [pixel][channels rounded up to 32, + 16]: the 32-byte pad puts the four pixel rows
// a 16-lane group touches in one transposing read into different banks.
__host__ __device__ inline int bw_row(int ch) { return (ch + 31) / 32 * 32 + 16; }

size_t wgrad_bf16_lds_bytes(int Co, int Ci, int kt, int kd, int kh, int kw) {
    const int rowtaps = kt * kd * kh, taps = rowtaps * kw;
    const size_t buf = ((size_t)kBwTM * bw_row(Co) + (size_t)rowtaps * kBwSlab * bw_row(Ci) + 7) / 8 * 8;
    const size_t two = 2 * buf * sizeof(unsigned short);
    return two <= kBwLdsMax ? two : two / 2;   // double-buffered when it fits
}

typedef short short4v __attribute__((ext_vector_type(4)));
// gfx950 LDS transposing read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane s passes the
// address of 4 consecutive 16-bit values of row s/4, columns 4*(s%4)..+3 of a 4 x 16 block; lane j gets
// column j of the block, rows 0..3.  (Checked with an index pattern on the device.)
__device__ __forceinline__ uint2 lds_read_tr16(const unsigned short* p) {
    const short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(p));
    return __builtin_bit_cast(uint2, v);
}

// Each wave owns one (32 cout x 32 cin) block and JT consecutive taps starting at a multiple of KW.
// PG / PA: 16-byte staging slots per thread for the gradient chunk and the input slab.
template <int JT, int KW, int NW, int PG, int PA>
__global__ __launch_bounds__(NW * 64) void wgrad_bf16_kernel(WgradBf16Args a) {
    constexpr int NT = NW * 64;
    extern __shared__ __attribute__((aligned(16))) unsigned short smem16[];
    const PixDims d = a.d;
    const int rowtaps = d.kt * d.kd * d.kh, taps = rowtaps * KW;
    const int n_pa = kBwTM + KW - 1;
    const int CoP = bw_row(a.Co), CiP = bw_row(a.Ci);
    // two staging buffers, each: gs [kBwTM][CoP] (chunk pixel p, channel c), as [rowtaps][kBwSlab][CiP]
    // (slab pixel pp = p + dw, channel c).  A chunk is a 32-pixel segment of one image row; pixels past
    // the row end get g = 0 and slab entries outside the grid are stored as 0, so the MFMA loop needs no masks.
    const int as_off = kBwTM * CoP;
    const int buf_elems = (as_off + rowtaps * kBwSlab * CiP + 7) / 8 * 8;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), m = lane & 31, h = lane >> 5;
    const int ncb = (a.Co + 31) / 32, nib = (a.Ci + 31) / 32;
    const int tapgroups = (taps + JT - 1) / JT;
    const int job = blockIdx.y * NW + wave;
    const bool active = job < ncb * nib * tapgroups;
    const int tg = job % tapgroups, pair = job / tapgroups;
    const int cb = pair / nib, ib = pair % nib;
    const int tap0 = tg * JT;                                   // multiple of KW by construction (JT % KW == 0)
    const int Co8 = a.Co / 8, Ci8 = a.Ci / 8;
    const int n_g8 = kBwTM * Co8, n_a8 = rowtaps * n_pa * Ci8;

    // Staging slots, the same for every chunk: slot i moves 16 bytes (8 channels of one pixel) from pixel
    // q0 + dq[i], channel col[i], to LDS offset lds[i].  Unused slots have lds < 0.
    int g_dq[PG], g_off[PG], g_lds[PG];
    int a_px[PA], a_off[PA], a_lds[PA];
    unsigned a_rt[PA];
#pragma unroll
    for (int i = 0; i < PG; ++i) {
        const int v = tid + i * NT;
        const int p = v / Co8, c8 = v % Co8;
        g_dq[i] = p;
        g_off[i] = p * a.Co + 8 * c8;   // element offset from the chunk's first pixel
        g_lds[i] = v < n_g8 ? p * CoP + 8 * c8 : -1;
    }
#pragma unroll
    for (int i = 0; i < PA; ++i) {
        const int v = tid + i * NT;
        const int rt = v / (n_pa * Ci8), r = v % (n_pa * Ci8);
        const int p = r / Ci8, c8 = r % Ci8;
        a_px[i] = p - KW / 2;
        a_off[i] = v < n_a8 ? ((int)rowtap_offset(rt, d) - KW / 2 + p) * a.Ci + 8 * c8 : 0;   // may be negative
        a_rt[i] = v < n_a8 ? 1u << rt : 0u;
        a_lds[i] = v < n_a8 ? (rt * kBwSlab + p) * CiP + 8 * c8 : -1;
    }

    uint4 rg[PG], ra[PA];
    float bsum[PG][8];
#pragma unroll
    for (int i = 0; i < PG; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) bsum[i][e] = 0.f;

    // prefetch loads are unconditional (clamped address); validity is applied when they are stashed
    unsigned g_ok = 0u, a_ok = 0u;
    // (segment, row, slice, frame) of the chunk to fetch, advanced chunk by chunk without divisions
    const int segs = (d.W + kBwTM - 1) / kBwTM;
    PixDims cd = d;
    cd.W = segs;
    PixCoord cc{0, 0, 0, 0}, cstep{0, 0, 0, 0};
    long long crow = 0, rstep = 0;
    auto fetch = [&]() {
        const int w0 = cc.w * kBwTM;
        unsigned rows_ok = 0u;
        {
            int rt = 0;
            for (int it = 0; it < d.kt; ++it)
                for (int id = 0; id < d.kd; ++id)
                    for (int ih = 0; ih < d.kh; ++ih, ++rt) {
                        const bool v = (unsigned)(cc.t + it - d.kt / 2) < (unsigned)d.T && (unsigned)(cc.dd + id - d.kd / 2) < (unsigned)d.D &&
                                       (unsigned)(cc.h + ih - d.kh / 2) < (unsigned)d.H;
                        rows_ok |= (v ? 1u : 0u) << rt;
                    }
        }
        const long long q0 = crow * d.W + w0;
        const unsigned short* gbase = a.g + q0 * a.Co;   // uniform; per-slot offsets are 32-bit constants
        const unsigned short* abase = a.a + q0 * a.Ci;
        crow += rstep + (cc.w + cstep.w >= segs ? 1 : 0);
        pix_advance(cc, cstep, cd);
        g_ok = 0u;
        a_ok = 0u;
#pragma unroll
        for (int i = 0; i < PG; ++i) {
            const bool ok = g_lds[i] >= 0 && w0 + g_dq[i] < d.W;
            rg[i] = *reinterpret_cast<const uint4*>(ok ? gbase + g_off[i] : a.g);
            g_ok |= (ok ? 1u : 0u) << i;
        }
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const bool ok = (rows_ok & a_rt[i]) != 0u && (unsigned)(w0 + a_px[i]) < (unsigned)d.W;
            ra[i] = *reinterpret_cast<const uint4*>(ok ? abase + a_off[i] : a.a);
            a_ok |= (ok ? 1u : 0u) << i;
        }
    };
    auto stash = [&](int buf) {
        unsigned short* gsT = smem16 + buf * buf_elems;
        unsigned short* asT = gsT + as_off;
#pragma unroll
        for (int i = 0; i < PG; ++i) {
            if (g_lds[i] >= 0) {
                const unsigned mk = ((g_ok >> i) & 1u) ? 0xffffffffu : 0u;
                const unsigned w4[4] = {rg[i].x & mk, rg[i].y & mk, rg[i].z & mk, rg[i].w & mk};
                *reinterpret_cast<uint4*>(gsT + g_lds[i]) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
                if (a.bias_partial != nullptr) {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        bsum[i][e] += (e & 1) ? __uint_as_float(w4[e >> 1] & 0xffff0000u) : __uint_as_float(w4[e >> 1] << 16);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            if (a_lds[i] >= 0) {
                const unsigned mk = ((a_ok >> i) & 1u) ? 0xffffffffu : 0u;
                unsigned w4[4] = {ra[i].x & mk, ra[i].y & mk, ra[i].z & mk, ra[i].w & mk};
                if (a.relu_in) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) w4[e] = relu_bf16x2(w4[e]);
                }
                *reinterpret_cast<uint4*>(asT + a_lds[i]) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
            }
        }
    };

    floatx16 acc[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    const int ci = ib * 32 + m;
    const int rt0 = tap0 / KW;
    // per-lane offsets of the transposing reads: row s/4 and columns 16*(group%2) + 4*(s%4) inside the
    // wave's 32-channel block, pixels 8h.. of the K-block (group = lane/16, s = lane%16, h = group/2)
    const int tr_row = 8 * h + ((lane & 15) >> 2), tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const int g_rd = tr_row * CoP + cb * 32 + tr_col;
    const int a_rd = as_off + tr_row * CiP + ib * 32 + tr_col;

    // Pipeline over this workgroup's chunks c0, c1, ...: while the MFMAs of chunk i read LDS buffer i%2,
    // chunk i+1 (fetched one step earlier) is written to the other buffer and chunk i+2 is requested from
    // HBM; one barrier per chunk.  Layers whose two buffers do not fit LDS use one buffer and two barriers.
    const long long n_chunks = (d.Q / d.W) * segs;
    const XcdRange xr = xcd_range(n_chunks);
    long long chunk = xr.first;
    if (chunk < xr.end) {
        cc = pix_coord(chunk, cd);
        cstep = pix_coord(xr.stride, cd);
        crow = chunk / segs;
        rstep = xr.stride / segs;
    }
    auto compute = [&](int buf) {
        if (active) {
            const unsigned short* base = smem16 + buf * buf_elems;
#pragma unroll
            for (int kb = 0; kb < kBwTM / 16; ++kb) {
                const uint2 g0 = lds_read_tr16(base + g_rd + (16 * kb) * CoP), g1 = lds_read_tr16(base + g_rd + (16 * kb + 4) * CoP);
                const bf16x8 gv = __builtin_bit_cast(bf16x8, make_uint4(g0.x, g0.y, g1.x, g1.y));
#pragma unroll
                for (int jr = 0; jr < JT / KW; ++jr) {
                    const int rt = rt0 + jr < rowtaps ? rt0 + jr : rowtaps - 1;
                    // window of slab pixels px .. px+11 of this lane's input channel as six 32-bit words
                    const unsigned short* row = base + a_rd + (rt * kBwSlab + 16 * kb) * CiP;
                    const uint2 w0 = lds_read_tr16(row), w1 = lds_read_tr16(row + 4 * CiP);
                    uint2 w2 = make_uint2(0u, 0u);
                    if (KW > 1) w2 = lds_read_tr16(row + 8 * CiP);
                    const unsigned dws[6] = {w0.x, w0.y, w1.x, w1.y, w2.x, w2.y};
#pragma unroll
                    for (int dw = 0; dw < KW; ++dw) {
                        const int j = jr * KW + dw;
                        uint4 b;
                        if (dw % 2 == 0) {
                            b = make_uint4(dws[dw / 2], dws[dw / 2 + 1], dws[dw / 2 + 2], dws[dw / 2 + 3]);
                        } else {
                            b.x = __builtin_amdgcn_alignbit(dws[dw / 2 + 1], dws[dw / 2], 16);
                            b.y = __builtin_amdgcn_alignbit(dws[dw / 2 + 2], dws[dw / 2 + 1], 16);
                            b.z = __builtin_amdgcn_alignbit(dws[dw / 2 + 3], dws[dw / 2 + 2], 16);
                            b.w = __builtin_amdgcn_alignbit(dws[dw / 2 + 4], dws[dw / 2 + 3], 16);
                        }
                        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gv, __builtin_bit_cast(bf16x8, b), acc[j], 0, 0, 0);
                    }
                }
            }
        }
    };
    if (a.two_buf) {
        if (chunk < xr.end) {
            fetch();
            stash(0);
            if (chunk + xr.stride < xr.end) fetch();
        }
        __syncthreads();
        int buf = 0;
        for (; chunk < xr.end; chunk += xr.stride) {
            const long long next = chunk + xr.stride, next2 = next + xr.stride;
            if (next < xr.end) stash(buf ^ 1);
            if (next2 < xr.end) fetch();
            compute(buf);
            __syncthreads();
            buf ^= 1;
        }
    } else {   // one buffer (large layers): write the next chunk between two barriers
        if (chunk < xr.end) {
            fetch();
            stash(0);
        }
        __syncthreads();
        for (; chunk < xr.end; chunk += xr.stride) {
            const long long next = chunk + xr.stride;
            if (next < xr.end) fetch();
            compute(0);
            __syncthreads();
            if (next < xr.end) stash(0);
            __syncthreads();
        }
    }
    if (active) {
        float* dst = a.partial + (size_t)blockIdx.x * a.Co * taps * a.Ci;
#pragma unroll
        for (int j = 0; j < JT; ++j) {
            const int tap = tap0 + j;
            if (tap >= taps || ci >= a.Ci) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int cc = cb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (cc < a.Co) dst[((size_t)cc * taps + tap) * a.Ci + ci] = acc[j][r];
            }
        }
    }
    if (a.bias_partial != nullptr && blockIdx.y == 0) {
        __syncthreads();
        float* red = reinterpret_cast<float*>(smem16);   // [PG*NT][8] floats; fits: checked by the launcher
#pragma unroll
        for (int i = 0; i < PG; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) red[(tid + i * NT) * 8 + e] = (tid + i * NT) < n_g8 ? bsum[i][e] : 0.f;
        __syncthreads();
        if (tid < a.Co) {
            const int c8 = tid / 8, e = tid % 8;
            float t = 0.f;
            for (int v = c8; v < PG * NT; v += Co8) t += red[v * 8 + e];
            a.bias_partial[(size_t)blockIdx.x * a.Co + tid] = t;
        }
    }
}

template <int JT, int KW, int NW, int PG, int PA>
static void launch_wgrad_bf16_k(const WgradBf16Args& a, dim3 grid, size_t lds, hipStream_t st) {
    static bool once = false;
    if (!once) {
        (void)hipFuncSetAttribute((const void*)wgrad_bf16_kernel<JT, KW, NW, PG, PA>, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        once = true;
    }
    hipLaunchKernelGGL((wgrad_bf16_kernel<JT, KW, NW, PG, PA>), grid, dim3(NW * 64), lds, st, a);
}

// Supported: Co, Ci multiples of 8 (16-byte rows), kw in {1, 3}; the caller checks and falls back otherwise.
hipError_t launch_wgrad_bf16(const WgradBf16Args& a_in, int n_split, hipStream_t stream) {
    WgradBf16Args a = a_in;
    const PixDims& d = a_in.d;
    const int rowtaps = d.kt * d.kd * d.kh, taps = rowtaps * d.kw;
    char name[56];
    snprintf(name, sizeof(name), "conv_bf16_wgrad_%dto%d_t%d", a.Ci, a.Co, taps);
    KernelScope ks(name, 2.0 * (double)d.Q * a.Ci * a.Co * taps, 2.0 * (double)d.Q * (a.Ci + a.Co), stream);
    constexpr int NW = 8, NT = NW * 64;
    size_t lds = wgrad_bf16_lds_bytes(a.Co, a.Ci, d.kt, d.kd, d.kh, d.kw);
    {
        const size_t one = ((size_t)kBwTM * bw_row(a.Co) + (size_t)(d.kt * d.kd * d.kh) * kBwSlab * bw_row(a.Ci) + 7) / 8 * 8 *
                           sizeof(unsigned short);
        a.two_buf = 2 * one <= kBwLdsMax ? 1 : 0;
    }
    const size_t red = (size_t)2 * NT * 8 * sizeof(float);
    if (lds < red) lds = red;
    const int ncb = (a.Co + 31) / 32, nib = (a.Ci + 31) / 32;
    const int n_pa = kBwTM + d.kw - 1;
    // staging slots per thread must fit the compile-time bounds (2 for g, 8 for a)
    if (kBwTM * (a.Co / 8) > 2 * NT || rowtaps * n_pa * (a.Ci / 8) > 8 * NT || lds > 150 * 1024) return hipErrorInvalidValue;
    // few staging slots (channel counts up to 128 with 3 row taps) keep the kernel free of register spills
    const bool small = kBwTM * (a.Co / 8) <= NT && rowtaps * n_pa * (a.Ci / 8) <= 4 * NT;
    if (d.kw == 3) {
        const int jt = 9, tapgroups = (taps + jt - 1) / jt;
        dim3 grid(n_split, (ncb * nib * tapgroups + NW - 1) / NW);
        if (small) launch_wgrad_bf16_k<9, 3, NW, 1, 4>(a, grid, lds, stream);
        else launch_wgrad_bf16_k<9, 3, NW, 2, 8>(a, grid, lds, stream);
    } else if (d.kw == 1) {
        const int jt = 3, tapgroups = (taps + jt - 1) / jt;
        dim3 grid(n_split, (ncb * nib * tapgroups + NW - 1) / NW);
        if (small) launch_wgrad_bf16_k<3, 1, NW, 1, 4>(a, grid, lds, stream);
        else launch_wgrad_bf16_k<3, 1, NW, 2, 8>(a, grid, lds, stream);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace gleam
