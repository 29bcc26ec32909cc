// Two-channel-OUTPUT convolution (last layer of the prox, Eq. 4-5) on the matrix cores.
//
// out[p][n] = b[n] + sum_{tap,k} W[n][tap][k] * in[p + off(tap)][k] is split into a dense product and a shifted
// sum: first c[p][tap][n] = sum_k W[n][tap][k] * in[p][k] for every pixel of a tile and its halo (a
// [2*taps x K] . [K x pixels] product, the rows padded to one 32-row MFMA block), then
// out[p][n] = b[n] + sum_tap c[p + off(tap)][tap][n] from LDS.  The kernel reads its input once (plus the halo,
// served by L2) and is bound by that read; the lane-per-pixel kernel it replaces spent its time on scalar
// weight loads and LDS traffic.
//
// Kernel shapes: KP x KP taps in the image plane (KP = 3 is what is launched), times KO taps (1 or 3) along one
// outer axis (the depth of a 3x3x3 layer).  The outer taps are a loop: per outer tap the plane it points at is
// multiplied with that tap's 2*KP*KP weight rows and summed into the same outputs.
//
// A workgroup of four waves owns 8 x 32 output pixels of one plane; the (8 + KP - 1) x (32 + KP - 1) input
// region is padded to 32-pixel blocks (eleven for KP = 3, eight for KP = 1) that are dealt to the waves.  Lane
// (m, h) of a wave loads the channels of ITS pixel slot straight from memory into the B operand (float32:
// channels K/2*h .. K/2*h + K/2 - 1, one per v_mfma_f32_32x32x2_f32; bfloat16: eight channels 16*i + 8*h .. per
// v_mfma_f32_32x32x16_bf16), so the input never passes through LDS; the weights sit in registers as the A
// operand for the life of the workgroup.
#include <type_traits>

#include "prox_common.h"

namespace gleam {

struct ThinOutMfmaArgs {
    const void* in;       // [NI][H][W][K] float32 or bfloat16, NI = all planes (batch, time, depth)
    const float* wts;     // [2][KO*KP*KP][K]
    const float* bias;    // [2] or null
    const float* add;     // [NI][H][W][2] or null
    float* out;           // [NI][H][W][2]
    int relu_in, relu_out, H, W, bx_n, by_n;
    int o_n, o_stride;    // outer axis: extent, and its stride in planes (plane index = (.. * o_n + pos) * o_stride + ..)
    long long n_blocks;
};

constexpr int kTOStride = 20;   // floats per pixel slot in LDS: up to 18 tap contributions + 2

template <int K, bool BF, int KP, int KO>
__global__ __launch_bounds__(256) void conv_thin_out_mfma_kernel(ThinOutMfmaArgs a) {
    constexpr int NM = BF ? K / 16 : K / 2;   // MFMAs per 32-pixel block
    constexpr int RW = 32 + KP - 1, RPX = (8 + KP - 1) * RW, NBLK = (RPX + 31) / 32, PT = KP * KP;
    static_assert(NBLK > 4 && NBLK <= 12, "two or three blocks per wave");
    __shared__ __attribute__((aligned(16))) float c[NBLK * 32 * kTOStride];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, h = lane >> 5;
    const int H = a.H, W = a.W;

    // A operand: row j = 2*(tap in the plane) + n of the 32-row block, rows 2*PT..31 are zero; one set per outer tap
    float wf[BF ? 1 : KO][BF ? 1 : NM];
    bf16x8 wb[BF ? KO : 1][BF ? NM : 1];
    {
        const bool row_ok = m < 2 * PT;
#pragma unroll
        for (int ko = 0; ko < KO; ++ko) {
            const float* wrow = a.wts + (size_t)((m & 1) * (KO * PT) + ko * PT + (row_ok ? (m >> 1) : 0)) * K;
            if constexpr (BF) {
#pragma unroll
                for (int i = 0; i < NM; ++i) {
                    const float* wp = wrow + 16 * i + 8 * h;
                    uint4 u;
                    u.x = pack_bf16x2(wp[0], wp[1]); u.y = pack_bf16x2(wp[2], wp[3]);
                    u.z = pack_bf16x2(wp[4], wp[5]); u.w = pack_bf16x2(wp[6], wp[7]);
                    if (!row_ok) u = make_uint4(0u, 0u, 0u, 0u);
                    wb[ko][i] = __builtin_bit_cast(bf16x8, u);
                }
            } else {
#pragma unroll
                for (int i = 0; i < NM; ++i) wf[ko][i] = row_ok ? wrow[NM * h + i] : 0.f;
            }
        }
    }
    const float bias0 = a.bias ? a.bias[0] : 0.f, bias1 = a.bias ? a.bias[1] : 0.f;

    const XcdRange xr = xcd_range(a.n_blocks);
    for (long long item = xr.first; item < xr.end; item += xr.stride) {
        const int bx = (int)(item % a.bx_n);
        const long long rest = item / a.bx_n;
        const int by = (int)(rest % a.by_n);
        const long long img = rest / a.by_n;
        const int x0 = bx * 32, y0 = by * 8;
        int opos = 0;
        if constexpr (KO > 1) opos = (int)((img / a.o_stride) % a.o_n);
        float o0 = bias0, o1 = bias1;
#pragma unroll
        for (int ko = 0; ko < KO; ++ko) {
            long long src = img;
            if constexpr (KO > 1) {
                const int z = opos + ko - KO / 2;
                if (z < 0 || z >= a.o_n) continue;   // uniform: the plane of this outer tap lies outside the grid
                src = img + (long long)(ko - KO / 2) * a.o_stride;
            }
            // the wave's blocks are wave, wave + 4 and (where there are that many) wave + 8; the loads of a block
            // are issued before the MFMAs of the block ahead of it
            using Vec = typename std::conditional<BF, uint4, float4>::type;
            constexpr int NV = BF ? NM : NM / 4;
            auto slot_ok = [&](int b) {
                const int s = 32 * b + m;
                const int ry = s / RW, rx = s - ry * RW;
                const int y = y0 - KP / 2 + ry, x = x0 - KP / 2 + rx;
                return s < RPX && y >= 0 && y < H && x >= 0 && x < W;
            };
            auto load = [&](int b, Vec* v) {
                const int s = 32 * b + m;
                const int ry = s / RW, rx = s - ry * RW;
                const long long pix = slot_ok(b) ? (src * H + (y0 - KP / 2 + ry)) * W + (x0 - KP / 2 + rx) : 0;   // clamped: the loads are unconditional
                if constexpr (BF) {
                    const unsigned short* p = reinterpret_cast<const unsigned short*>(a.in) + pix * K + 8 * h;
#pragma unroll
                    for (int i = 0; i < NV; ++i) v[i] = *reinterpret_cast<const uint4*>(p + 16 * i);
                } else {
                    const float* p = reinterpret_cast<const float*>(a.in) + pix * K + NM * h;
#pragma unroll
                    for (int q = 0; q < NV; ++q) v[q] = *reinterpret_cast<const float4*>(p + 4 * q);
                }
            };
            auto compute = [&](int b, const Vec* v) {
                const bool ok = slot_ok(b);
                floatx16 acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0.f;
                if constexpr (BF) {
#pragma unroll
                    for (int i = 0; i < NV; ++i) {
                        uint4 u = v[i];
                        if (a.relu_in) { u.x = relu_bf16x2(u.x); u.y = relu_bf16x2(u.y); u.z = relu_bf16x2(u.z); u.w = relu_bf16x2(u.w); }
                        if (!ok) u = make_uint4(0u, 0u, 0u, 0u);
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[ko][i], __builtin_bit_cast(bf16x8, u), acc, 0, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < NV; ++q) {
                        const float e[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            float xv = a.relu_in ? fmaxf(e[t], 0.f) : e[t];
                            xv = ok ? xv : 0.f;
                            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[ko][4 * q + t], xv, acc, 0, 0, 0);
                        }
                    }
                }
                // accumulator r holds row 8*(r/4) + 4*h + r%4 of this lane's pixel: rows 0..19 are kept
                float* cs = c + (32 * b + m) * kTOStride;
                *reinterpret_cast<float4*>(cs + 4 * h) = make_float4(acc[0], acc[1], acc[2], acc[3]);
                if (PT > 4) {
                    *reinterpret_cast<float4*>(cs + 8 + 4 * h) = make_float4(acc[4], acc[5], acc[6], acc[7]);
                    if (h == 0) *reinterpret_cast<float4*>(cs + 16) = make_float4(acc[8], acc[9], acc[10], acc[11]);
                }
            };
            {
                const bool third = wave + 8 < NBLK;   // uniform per wave
                Vec va[NV], vb[NV];
                load(wave, va);
                load(wave + 4, vb);
                __builtin_amdgcn_sched_barrier(0);   // all loads of both blocks are in flight before the first MFMA
                compute(wave, va);
                __builtin_amdgcn_sched_barrier(0);
                if (third) load(wave + 8, va);
                __builtin_amdgcn_sched_barrier(0);
                compute(wave + 4, vb);
                if (third) compute(wave + 8, va);
            }
            __syncthreads();
            {
                const int oy = tid >> 5, ox = tid & 31;
#pragma unroll
                for (int dy = 0; dy < KP; ++dy)
#pragma unroll
                    for (int dx = 0; dx < KP; ++dx) {
                        const float2 v = *reinterpret_cast<const float2*>(c + ((oy + dy) * RW + ox + dx) * kTOStride + (dy * KP + dx) * 2);
                        o0 += v.x;
                        o1 += v.y;
                    }
            }
            __syncthreads();   // the next pass overwrites c
        }
        {
            const int y = y0 + (tid >> 5), x = x0 + (tid & 31);
            if (y < H && x < W) {
                const long long q = (img * H + y) * W + x;
                if (a.relu_out) { o0 = fmaxf(o0, 0.f); o1 = fmaxf(o1, 0.f); }
                if (a.add) {
                    const float2 av = *reinterpret_cast<const float2*>(a.add + 2 * q);
                    o0 += av.x;
                    o1 += av.y;
                }
                *reinterpret_cast<float2*>(a.out + 2 * q) = make_float2(o0, o1);
            }
        }
    }
}

// 3x1x1 layers (three taps along time, none in the plane): a tile is 32 neighbouring positions of one volume times
// ALL frames, so the shifted sum out[t] = b + sum_dt c[t + dt - 1][dt] never leaves the tile and every input value is
// read exactly once.  Frame t of the tile is one 32-pixel block (dealt to wave t % 4); rows 2*dt + n of the product.
constexpr int kTOTimeMaxT = 32;

struct ThinOutTimeArgs {
    const float* in;      // [B][T][S][K], S = D*H*W positions per frame
    const float* wts;     // [2][3][K]
    const float* bias;    // [2] or null
    const float* add;     // [B][T][S][2] or null
    float* out;           // [B][T][S][2]
    int relu_in, relu_out, T, segs;
    long long S, n_blocks;   // n_blocks = B * segs, segs = ceil(S / 32)
};

template <int K>
__global__ __launch_bounds__(256) void conv_thin_out_time_mfma_kernel(ThinOutTimeArgs a) {
    constexpr int NM = K / 2, NV = NM / 4;
    __shared__ __attribute__((aligned(16))) float c[kTOTimeMaxT * 32 * 8];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, h = lane >> 5;
    const int T = a.T;
    float wf[NM];   // A operand: row j = 2*dt + n, rows 6..31 are zero
#pragma unroll
    for (int i = 0; i < NM; ++i) wf[i] = m < 6 ? a.wts[(size_t)((m & 1) * 3 + (m >> 1)) * K + NM * h + i] : 0.f;
    const float bias0 = a.bias ? a.bias[0] : 0.f, bias1 = a.bias ? a.bias[1] : 0.f;
    const XcdRange xr = xcd_range(a.n_blocks);
    for (long long item = xr.first; item < xr.end; item += xr.stride) {
        const long long b = item / a.segs;
        const long long s0 = (item - b * a.segs) * 32;
        const bool px_ok = s0 + m < a.S;
        auto load = [&](int t, float4* v) {
            const long long pix = px_ok ? (b * T + t) * a.S + s0 + m : 0;   // clamped: the loads are unconditional
            const float* p = a.in + pix * K + NM * h;
#pragma unroll
            for (int q = 0; q < NV; ++q) v[q] = *reinterpret_cast<const float4*>(p + 4 * q);
        };
        auto compute = [&](int t, const float4* v) {
            floatx16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const float e[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    float xv = a.relu_in ? fmaxf(e[u], 0.f) : e[u];
                    xv = px_ok ? xv : 0.f;
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[4 * q + u], xv, acc, 0, 0, 0);
                }
            }
            // accumulator r holds row 4*h + r (r < 4) of this lane's pixel: rows 0..7 are kept
            *reinterpret_cast<float4*>(c + (t * 32 + m) * 8 + 4 * h) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        };
        // frames wave, wave + 4, ...: the loads of a frame are issued before the MFMAs of the frame ahead of it
        {
            float4 va[NV], vb[NV];
            if (wave < T) load(wave, va);
            for (int t = wave; t < T; t += 8) {
                if (t + 4 < T) load(t + 4, vb);
                __builtin_amdgcn_sched_barrier(0);
                compute(t, va);
                __builtin_amdgcn_sched_barrier(0);
                if (t + 8 < T) load(t + 8, va);
                __builtin_amdgcn_sched_barrier(0);
                if (t + 4 < T) compute(t + 4, vb);
            }
        }
        __syncthreads();
        for (int t = tid >> 5; t < T; t += 8) {
            const int px = tid & 31;
            float o0 = bias0, o1 = bias1;
#pragma unroll
            for (int dt = 0; dt < 3; ++dt) {
                const int tt = t + dt - 1;
                if (tt >= 0 && tt < T) {
                    const float2 v = *reinterpret_cast<const float2*>(c + (tt * 32 + px) * 8 + 2 * dt);
                    o0 += v.x;
                    o1 += v.y;
                }
            }
            if (s0 + px < a.S) {
                const long long q = (b * T + t) * a.S + s0 + px;
                if (a.relu_out) { o0 = fmaxf(o0, 0.f); o1 = fmaxf(o1, 0.f); }
                if (a.add) {
                    const float2 av = *reinterpret_cast<const float2*>(a.add + 2 * q);
                    o0 += av.x;
                    o1 += av.y;
                }
                *reinterpret_cast<float2*>(a.out + 2 * q) = make_float2(o0, o1);
            }
        }
        __syncthreads();   // the next tile overwrites c
    }
}

// 3x3x3 layers with 32 input channels: a walk along the depth.  conv_thin_out_mfma_kernel<K, BF, 3, 3> visits every
// input slice three times (once per output slice it contributes to) and was bound by those re-reads (2.7 times the
// input left the L2 on the 3D volume).  Here a workgroup owns an 8 x 32-pixel column of the volume and walks a run of
// slices: input slice z is read once, multiplied with the weight rows of all three depth taps (54 rows = 27 taps x 2
// outputs, packed into two 32-row MFMA blocks instead of three) and its shifted sums go to the outputs of slices
// z + 1, z and z - 1, which a thread keeps in registers for its pixel until slice z + 1 has added the last of them.
// The next slice's pixels are requested before the MFMAs of the current one.
struct ThinOutWalkArgs {
    const float* in;      // [volumes][D][H][W][K]
    const float* wts;     // [2][27][K]
    const float* bias;    // [2] or null
    const float* add;     // [volumes][D][H][W][2] or null
    float* out;
    int relu_in, relu_out, D, H, W, bx_n, by_n;
    int seg_len, segs_per_col;   // output slices per run, runs per column
    long long n_items;
};

constexpr int kTWStride = 56;   // floats per pixel slot in LDS: 54 tap contributions + 2

template <int K>
__global__ __launch_bounds__(256, 2) void conv_thin_out_walk_kernel(ThinOutWalkArgs a) {
    constexpr int NM = K / 2, NV = NM / 4;   // MFMAs per 32-pixel block and row set; float4 loads per lane and block
    constexpr int RW = 34, RPX = 10 * RW, NBLK = (RPX + 31) / 32;   // 340 region pixels in 11 blocks: three per wave, the last wave two
    __shared__ __attribute__((aligned(16))) float c[NBLK * 32 * kTWStride];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, h = lane >> 5;
    const int H = a.H, W = a.W, D = a.D;

    // A operands: row m of set s is (tap 16*s + m/2, output m & 1); taps past the 27th are zero rows
    float wf[2][NM];
#pragma unroll
    for (int s_ = 0; s_ < 2; ++s_) {
        const int tap = 16 * s_ + (m >> 1);
        const float* wrow = a.wts + (size_t)((m & 1) * 27 + (tap < 27 ? tap : 0)) * K + NM * h;
#pragma unroll
        for (int i = 0; i < NM; ++i) wf[s_][i] = tap < 27 ? wrow[i] : 0.f;
    }
    const float bias0 = a.bias ? a.bias[0] : 0.f, bias1 = a.bias ? a.bias[1] : 0.f;
    const int oy = tid >> 5, ox = tid & 31;

    const XcdRange xr = xcd_range(a.n_items);
    for (long long item = xr.first; item < xr.end; item += xr.stride) {
        const int by = (int)(item % a.by_n);
        long long rest = item / a.by_n;
        const int bx = (int)(rest % a.bx_n);
        rest /= a.bx_n;
        const int seg = (int)(rest % a.segs_per_col);
        const long long vol = rest / a.segs_per_col;
        const int x0 = bx * 32, y0 = by * 8;
        const int z0 = seg * a.seg_len, z1 = z0 + a.seg_len < D ? z0 + a.seg_len : D;

        // this lane's pixel slots (blocks wave, wave + 4, wave + 8): offset inside a slice, or -1 outside the image
        int pix_off[3];
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const int s_ = 32 * (wave + 4 * j) + m;
            const int ry = s_ / RW, rx = s_ - ry * RW;
            const int y = y0 - 1 + ry, x = x0 - 1 + rx;
            pix_off[j] = (wave + 4 * j < NBLK && s_ < RPX && y >= 0 && y < H && x >= 0 && x < W) ? y * W + x : -1;
        }
        const bool third = wave + 8 < NBLK;   // uniform per wave
        auto load = [&](int z, float4 (*v)[NV]) {
            const float* plane = a.in + ((vol * D + z) * H) * (long long)W * K + NM * h;
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                if (j == 2 && !third) continue;
                const float* p = plane + (long long)(pix_off[j] >= 0 ? pix_off[j] : 0) * K;   // clamped: the loads are unconditional
#pragma unroll
                for (int q = 0; q < NV; ++q) v[j][q] = *reinterpret_cast<const float4*>(p + 4 * q);
            }
        };
        auto compute = [&](int j, const float4* v) {
            const bool ok = pix_off[j] >= 0;
            float* cs = c + (32 * (wave + 4 * j) + m) * kTWStride;
#pragma unroll
            for (int s_ = 0; s_ < 2; ++s_) {
                floatx16 acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    const float e[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        float xv = a.relu_in ? fmaxf(e[t], 0.f) : e[t];
                        xv = ok ? xv : 0.f;
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[s_][4 * q + t], xv, acc, 0, 0, 0);
                    }
                }
                // accumulator r holds row 8*(r/4) + 4*h + r%4 of this lane's pixel; set 1 keeps rows 0..21
#pragma unroll
                for (int rg = 0; rg < (s_ == 0 ? 4 : 3); ++rg)
                    *reinterpret_cast<float4*>(cs + 32 * s_ + 8 * rg + 4 * h) =
                        make_float4(acc[4 * rg], acc[4 * rg + 1], acc[4 * rg + 2], acc[4 * rg + 3]);
            }
        };

        // o[k]: sums of this thread's pixel in slices zi - 1, zi, zi + 1 while input slice zi is worked on
        float o[3][2] = {{bias0, bias1}, {bias0, bias1}, {bias0, bias1}};
        float4 cur[3][NV], nxt[3][NV];
        const int zi_first = z0 - 1 >= 0 ? z0 - 1 : 0, zi_last = z1 < D ? z1 : D - 1;
        load(zi_first, cur);
        for (int zi = zi_first; zi <= zi_last; ++zi) {
            if (zi + 1 <= zi_last) load(zi + 1, nxt);
            __builtin_amdgcn_sched_barrier(0);   // the next slice's loads are in flight before the first MFMA
            compute(0, cur[0]);
            compute(1, cur[1]);
            if (third) compute(2, cur[2]);
            __syncthreads();
#pragma unroll
            for (int ko = 0; ko < 3; ++ko)
#pragma unroll
                for (int dy = 0; dy < 3; ++dy)
#pragma unroll
                    for (int dx = 0; dx < 3; ++dx) {
                        const float2 v = *reinterpret_cast<const float2*>(c + ((oy + dy) * RW + ox + dx) * kTWStride + 2 * (ko * 9 + dy * 3 + dx));
                        o[2 - ko][0] += v.x;
                        o[2 - ko][1] += v.y;
                    }
            // slice zi - 1 has received its last contribution (slice zi - 1 = z0 - 1 or earlier is not this run's)
            {
                const int zo = zi - 1, y = y0 + oy, x = x0 + ox;
                if (zo >= z0 && zo < z1 && y < H && x < W) {
                    const long long q = ((vol * D + zo) * H + y) * W + x;
                    float r0 = o[0][0], r1 = o[0][1];
                    if (a.relu_out) { r0 = fmaxf(r0, 0.f); r1 = fmaxf(r1, 0.f); }
                    if (a.add) {
                        const float2 av = *reinterpret_cast<const float2*>(a.add + 2 * q);
                        r0 += av.x;
                        r1 += av.y;
                    }
                    *reinterpret_cast<float2*>(a.out + 2 * q) = make_float2(r0, r1);
                }
            }
            o[0][0] = o[1][0]; o[0][1] = o[1][1];
            o[1][0] = o[2][0]; o[1][1] = o[2][1];
            o[2][0] = bias0; o[2][1] = bias1;
#pragma unroll
            for (int j = 0; j < 3; ++j)
#pragma unroll
                for (int q = 0; q < NV; ++q) cur[j][q] = nxt[j][q];
            __syncthreads();   // the next slice overwrites c
        }
        // the last slices of the run: when the volume ends at z1 no input slice z1 exists to push them out
        for (int zo = zi_last; zo < z1; ++zo) {
            const int y = y0 + oy, x = x0 + ox;
            if (zo >= z0 && y < H && x < W) {
                const long long q = ((vol * D + zo) * H + y) * W + x;
                float r0 = o[0][0], r1 = o[0][1];
                if (a.relu_out) { r0 = fmaxf(r0, 0.f); r1 = fmaxf(r1, 0.f); }
                if (a.add) {
                    const float2 av = *reinterpret_cast<const float2*>(a.add + 2 * q);
                    r0 += av.x;
                    r1 += av.y;
                }
                *reinterpret_cast<float2*>(a.out + 2 * q) = make_float2(r0, r1);
            }
            o[0][0] = o[1][0]; o[0][1] = o[1][1];
        }
    }
}

// 0: not covered; 1: 3x3 in the plane; 2: 3x3x3 (outer axis = depth); 3: 3x1x1 on tiles that span all frames (as a
// loop over three planes of an 8 x 32 tile it re-read every input three times and was slower than the lane-per-pixel
// kernel, 125 against 97 us).
static int thin_out_mfma_shape(const PixDims& d, int K, bool bf) {
    const bool on = !(kernel_policy() & GLEAM_POLICY_NO_THIN_MFMA);   // else the lane-per-pixel kernel
    if (!on) return 0;
    if (d.kt == 1 && d.kd == 1 && d.kh == 3 && d.kw == 3) return (bf ? (K == 64 || K == 128) : (K == 32 || K == 64 || K == 128)) ? 1 : 0;
    if (d.kt == 1 && d.kd == 3 && d.kh == 3 && d.kw == 3) return (!bf && (K == 32 || K == 64)) ? 2 : 0;
    if (d.kt == 3 && d.kd == 1 && d.kh == 1 && d.kw == 1) return (!bf && (K == 32 || K == 64) && d.T <= kTOTimeMaxT) ? 3 : 0;
    return 0;
}

bool conv_thin_out_mfma_applies(const PixDims& d, int K, bool bf) { return thin_out_mfma_shape(d, K, bf) != 0; }

template <int K, bool BF, int KP, int KO>
static void launch_thin_out_mfma_t(const ThinOutMfmaArgs& a, hipStream_t st) {
    // persistent workgroups: three per CU (four measured slower on the 64-channel float32 layer), two where the
    // instantiation's registers (weights of all outer taps + two blocks of input) leave room for no more
    constexpr int per_cu = (!BF && K * KO >= 128) ? 2 : 3;
    const long long cap = 256LL * per_cu;
    const long long gx = ((a.n_blocks < cap ? a.n_blocks : cap) + 7) / 8 * 8;
    hipLaunchKernelGGL((conv_thin_out_mfma_kernel<K, BF, KP, KO>), dim3((unsigned)gx), dim3(256), 0, st, a);
}

// wts: [2][taps][K] float32 (theta's own layout of a K -> 2 layer); in is bfloat16 when bf.
hipError_t launch_conv_thin_out_mfma(const void* in, const float* wts, const float* bias, const float* add, float* out, int K,
                                     int relu_in, int relu_out, const PixDims& d, bool bf, hipStream_t st) {
    const int shape = thin_out_mfma_shape(d, K, bf);
    if (shape == 0) return hipErrorInvalidValue;
    if (shape == 3) {
        ThinOutTimeArgs t{};
        t.in = reinterpret_cast<const float*>(in); t.wts = wts; t.bias = bias; t.add = add; t.out = out;
        t.relu_in = relu_in; t.relu_out = relu_out; t.T = d.T;
        t.S = (long long)d.D * d.H * d.W;
        t.segs = (int)((t.S + 31) / 32);
        t.n_blocks = d.Q / ((long long)d.T * t.S) * t.segs;
        const long long cap = 256LL * 3;
        const long long gx = ((t.n_blocks < cap ? t.n_blocks : cap) + 7) / 8 * 8;
        if (K == 32) hipLaunchKernelGGL((conv_thin_out_time_mfma_kernel<32>), dim3((unsigned)gx), dim3(256), 0, st, t);
        else hipLaunchKernelGGL((conv_thin_out_time_mfma_kernel<64>), dim3((unsigned)gx), dim3(256), 0, st, t);
        return hipGetLastError();
    }
    ThinOutMfmaArgs a{};
    a.in = in; a.wts = wts; a.bias = bias; a.add = add; a.out = out;
    a.relu_in = relu_in; a.relu_out = relu_out; a.H = d.H; a.W = d.W;
    a.bx_n = (d.W + 31) / 32;
    a.by_n = (d.H + 7) / 8;
    a.n_blocks = d.Q / ((long long)d.H * d.W) * a.bx_n * a.by_n;
    a.o_n = 1; a.o_stride = 1;
    if (shape == 2) { a.o_n = d.D; a.o_stride = 1; }        // planes are ordered (batch, time, depth)
    if (shape == 1) {
        if (bf) {
            if (K == 64) launch_thin_out_mfma_t<64, true, 3, 1>(a, st);
            else launch_thin_out_mfma_t<128, true, 3, 1>(a, st);
        } else {
            if (K == 32) launch_thin_out_mfma_t<32, false, 3, 1>(a, st);
            else if (K == 64) launch_thin_out_mfma_t<64, false, 3, 1>(a, st);
            else launch_thin_out_mfma_t<128, false, 3, 1>(a, st);
        }
    } else if (K == 32) {   // walk along the depth: every input slice read once
        ThinOutWalkArgs w{};
        w.in = reinterpret_cast<const float*>(in); w.wts = wts; w.bias = bias; w.add = add; w.out = out;
        w.relu_in = relu_in; w.relu_out = relu_out; w.D = d.D; w.H = d.H; w.W = d.W;
        w.bx_n = a.bx_n; w.by_n = a.by_n;
        const long long cols = d.Q / ((long long)d.D * d.H * d.W) * a.bx_n * a.by_n;
        const long long cap = 512;   // two workgroups per CU
        // runs per column: the split that minimises (runs per workgroup) x (run length + the two extra slices a run reads)
        double best = 1e300;
        w.seg_len = d.D; w.segs_per_col = 1;
        for (int n = 1; n <= 64 && n <= d.D; ++n) {
            const int len = (d.D + n - 1) / n, nseg = (d.D + len - 1) / len;
            const long long items = cols * nseg, wgs = items < cap ? items : cap;
            const double cost = (double)((items + wgs - 1) / wgs) * (len + 2.0);
            if (cost < best) { best = cost; w.seg_len = len; w.segs_per_col = nseg; }
        }
        w.n_items = cols * w.segs_per_col;
        const long long gx = ((w.n_items < cap ? w.n_items : cap) + 7) / 8 * 8;
        hipLaunchKernelGGL((conv_thin_out_walk_kernel<32>), dim3((unsigned)gx), dim3(256), 0, st, w);
    } else {
        launch_thin_out_mfma_t<64, false, 3, 3>(a, st);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------------
// Two-channel-INPUT 3x3 (KD = 1) or 3x3x3 (KD = 3) convolution (first layer of the prox; data gradient of the last
// layer) on the matrix cores.
//
// out[p][n] = b[n] + sum_{tap,e} W[n][tap][e] * in[p + off(tap)][e] with e = 0, 1: one v_mfma_f32_32x32x2_f32 per
// tap and block of 32 output channels, its depth of two being exactly the two input channels.  Lane (m, h) of a
// wave supplies W[32*nb + m][tap][h] (registers, for the life of the wave) and in[p_m + off(tap)][h] (4-byte loads,
// 256 contiguous bytes per wave, zero outside the grid), and ends up with 16 output channels of its pixel in groups
// of four, which go through the usual fused epilogue (bias, ReLU, ReLU mask, add) into 16-byte (float32) or 8-byte
// (bfloat16) stores after a turn through the wave's own LDS rows.  No barriers in the loop: every wave walks down
// 32-pixel column segments on its own.  The kernel it replaces for these shapes computes on the vector ALUs,
// 2*taps multiply-adds per output.

template <int KD, int NB, int NH, bool BF, bool EPI>   // EPI: the call has a ReLU mask source or an add operand
__global__ __launch_bounds__(256) void conv_thin_in_mfma_kernel(ThinInMfmaArgs a, int runs, int run_len) {
    // NH passes of NB blocks of 32 output channels each: Nn = 32 * NB * NH
    static_assert(KD == 1 || KD == 3, "the walk keeps KD slices of three rows");
    constexpr int TAPS = 9 * KD, NP = 32 * NB, NN = NP * NH, SS = NP + 4;   // SS: floats per pixel row of the wave's LDS rows
    __shared__ __attribute__((aligned(16))) float stage_all[4 * 32 * SS];
    const PixDims d = a.d;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int m = lane & 31, h = lane >> 5;
    float* stage = stage_all + wave * 32 * SS;
    float wreg[NH][NB][TAPS];
#pragma unroll
    for (int hb = 0; hb < NH; ++hb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int t = 0; t < TAPS; ++t)
                wreg[hb][nb][t] = a.w[(NP * hb + 32 * nb + m) * a.sn + (a.flip ? TAPS - 1 - t : t) * a.st + h * a.sk];
    // A wave walks down the rows of one 32-pixel column segment of one slice: of the 9 KD input values a row needs (KD
    // slices x three rows x three columns) those of the two upper rows are the previous row's, so a row costs 3 KD loads,
    // and all of its addresses are a wave-uniform row pointer plus a lane constant.  Item = (slice of an image, segment,
    // run of run_len rows).
    const int segs = (d.W + 31) / 32;
    const long long planes = d.Q / ((long long)d.H * d.W);   // images x slices
    const long long n_items = planes * segs * runs;
    const long long first = (long long)blockIdx.x * 4 + wave, step = (long long)gridDim.x * 4;
    // epilogue pieces: pass u of a 32-pixel x NP-channel block covers pixel (64 u + lane) / (NP / 4), channels 4 ((64 u + lane) % (NP / 4)) ..
    constexpr int PASSES = NB * 4;
    // loads and stores go through buffer resources: a wave-uniform row offset in a scalar register plus a 32-bit lane
    // offset, so that no lane forms a 64-bit address (the launcher checks that both tensors are below 4 GB)
    const __amdgpu_buffer_rsrc_t r_in = __builtin_amdgcn_make_buffer_rsrc((void*)a.in, 0, (unsigned)(d.Q * 8), 0x00020000);
    constexpr unsigned ES = BF ? 2u : 4u;   // bytes per output element
    const unsigned out_bytes = (unsigned)(d.Q * NN * ES);
    const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, out_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t r_ref =
        __builtin_amdgcn_make_buffer_rsrc((void*)(a.mask_ref ? a.mask_ref : (const void*)a.out), 0, a.mask_ref ? out_bytes : 0u, 0x00020000);
    const __amdgpu_buffer_rsrc_t r_add =
        __builtin_amdgcn_make_buffer_rsrc((void*)(a.add ? a.add : (const void*)a.out), 0, a.add ? out_bytes : 0u, 0x00020000);
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    // the mask source and the add operand of a pass over the channels are requested before its MFMAs where the registers
    // allow (32 channels per pass, or bfloat16 pieces of 8 bytes); else they are loaded in the epilogue
    constexpr bool PRE = NB == 1 || BF;
    // four output-sized values (16 bytes of float32, 8 of bfloat16) at lane offset off of the row at byte offset row
    auto load_piece = [&](__amdgpu_buffer_rsrc_t r, unsigned off, unsigned row) -> u32x4 {
        if constexpr (BF) {
            const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(r, off, row, 0);
            return u32x4{w[0], w[1], 0u, 0u};
        } else {
            return __builtin_amdgcn_raw_buffer_load_b128(r, off, row, 0);
        }
    };
    auto piece_values = [&](u32x4 w) -> float4 {
        if constexpr (BF)
            return make_float4(bf16_to_f32((unsigned short)w[0]), bf16_to_f32((unsigned short)(w[0] >> 16)),
                               bf16_to_f32((unsigned short)w[1]), bf16_to_f32((unsigned short)(w[1] >> 16)));
        else
            return make_float4(__uint_as_float(w[0]), __uint_as_float(w[1]), __uint_as_float(w[2]), __uint_as_float(w[3]));
    };
    const int in_floor_i = a.relu_in ? 0 : (int)0x80000000;
    const float out_floor = a.relu_out ? 0.f : -__builtin_huge_valf();
    __shared__ __attribute__((aligned(16))) float bias_s[NN];
    if ((int)threadIdx.x < NN) bias_s[threadIdx.x] = a.bias ? a.bias[threadIdx.x] : 0.f;
    __syncthreads();
    for (long long item = first; item < n_items; item += step) {
        // segments fastest: the four waves of a workgroup walk down neighbouring segments of the same rows
        const int seg = (int)(item % segs);
        const int rn = (int)((item / segs) % runs);
        const long long plane = item / ((long long)runs * segs);
        const int z = (int)(plane % d.D);
        const int x_seg = 32 * seg, x = x_seg + m;
        const int y0 = rn * run_len, y1 = y0 + run_len < d.H ? y0 + run_len : d.H;
        // byte offset of this lane's value for column tap ix inside a row, clamped into the row (the value is dropped when
        // the column is outside), and whether it counts
        unsigned col_off[3], col_ok[3];   // (col_ok: all ones or zero)
#pragma unroll
        for (int ix = 0; ix < 3; ++ix) {
            const int xc = x + ix - 1;
            col_ok[ix] = (x < d.W && xc >= 0 && xc < d.W) ? 0xffffffffu : 0u;
            const int xcl = xc < 0 ? 0 : (xc >= d.W ? d.W - 1 : xc);
            col_off[ix] = (unsigned)(2 * xcl + h) * 4u;
        }
        const bool z_ok[3] = {KD == 1 || z >= 1, true, KD == 1 || z + 1 < d.D};   // (KD = 1: only [0] is used)
        // epilogue piece u of this lane: inside the row?  byte offset from the segment's first piece (0 if not: the loads
        // are unconditional)
        bool okk_item[PASSES];
        unsigned oo_item[PASSES];
#pragma unroll
        for (int u = 0; u < PASSES; ++u) {
            const int j = u * 64 + lane;
            const int px = j / (NP / 4), cq = j - px * (NP / 4);
            okk_item[u] = x_seg + px < d.W;
            oo_item[u] = okk_item[u] ? (unsigned)(px * NN + 4 * cq) * ES : 0u;
        }
        float v[KD][3][3];   // [slice tap][row slot][column tap]; row y + iy - 1 sits in slot (y + iy - 1 - (y0 - 1)) % 3
        auto load_row = [&](int yy, int slot) __attribute__((always_inline)) {
            const bool y_ok = yy >= 0 && yy < d.H;
#pragma unroll
            for (int iz = 0; iz < KD; ++iz) {
                // a row outside the image is read at row 0 of the tensor and masked away: the nine loads of a row are
                // unconditional, so that they are all in flight together (a uniform branch around each made them wait
                // for one another)
                const bool ok = y_ok && z_ok[iz];   // uniform
                const unsigned row = ok ? (unsigned)((((plane + iz - KD / 2) * d.H + yy) * d.W) * 8) : 0u;   // byte offset of the row
                const unsigned row_mask = ok ? 0xffffffffu : 0u;
#pragma unroll
                for (int ix = 0; ix < 3; ++ix) {
                    const unsigned f = __builtin_amdgcn_raw_buffer_load_b32(r_in, col_off[ix], row, 0);
                    // (ReLU as a signed-integer maximum: negative floats are negative integers)
                    const int fi = (int)(f & (row_mask & col_ok[ix]));
                    v[iz][slot][ix] = __int_as_float(fi > in_floor_i ? fi : in_floor_i);
                }
            }
        };
        load_row(y0 - 1, 0);
        load_row(y0, 1);
        int y = y0;
        // ROT: slot of row y - 1
        auto row_step = [&](auto rot_c) __attribute__((always_inline)) {
            constexpr int ROT = decltype(rot_c)::value;
            load_row(y + 1, (ROT + 2) % 3);
            const long long q0 = (plane * d.H + y) * d.W + x_seg;   // first pixel of the segment
#pragma unroll
            for (int hb = 0; hb < NH; ++hb) {
                floatx16 acc[NB];
                u32x4 refq[PRE ? PASSES : 1], addq[PRE ? PASSES : 1];
                if constexpr (EPI && PRE) {
                    const unsigned rb = (unsigned)((q0 * NN + NP * hb) * ES);
#pragma unroll
                    for (int u = 0; u < PASSES; ++u) {
                        refq[u] = load_piece(r_ref, oo_item[u], rb);
                        addq[u] = load_piece(r_add, oo_item[u], rb);
                    }
                }
                // row taps in the order upper, middle, lower: the lower row's values are the ones just requested
#pragma unroll
                for (int k = 0; k < TAPS; ++k) {
                    const int iy = k / (3 * KD), iz = (k / 3) % KD, ix = k % 3, t = 9 * iz + 3 * iy + ix;
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        floatx16 c;
                        if (k == 0) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) c[r] = 0.f;
                        } else {
                            c = acc[nb];
                        }
                        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(wreg[hb][nb][t], v[iz][(ROT + iy) % 3][ix], c, 0, 0, 0);
                    }
                }
                // accumulator r of block nb: output channel NP*hb + 32*nb + 8*(r/4) + 4*h + r%4 of this lane's pixel.  The
                // wave turns its 32 pixels x NP channels around in its own LDS rows, so that the epilogue's loads and stores
                // cover whole runs of NP channels per pixel; LDS accesses of one wave complete in order, no barrier.
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        *reinterpret_cast<float4*>(stage + m * SS + 32 * nb + 8 * g + 4 * h) =
                            make_float4(acc[nb][4 * g], acc[nb][4 * g + 1], acc[nb][4 * g + 2], acc[nb][4 * g + 3]);
                __builtin_amdgcn_wave_barrier();
                constexpr int UN = 4;   // 64 pieces of four channels per pass
                const unsigned row_byte = (unsigned)((q0 * NN + NP * hb) * ES);   // uniform: byte offset of the segment's first piece
#pragma unroll
                for (int p0 = 0; p0 < PASSES; p0 += UN) {
                    float4 accv[UN], refv[UN], addv[UN];
                    unsigned oo[UN];
                    bool okk[UN];
#pragma unroll
                    for (int u = 0; u < UN; ++u) {
                        const int j = (p0 + u) * 64 + lane;
                        const int px = j / (NP / 4), cq = j - px * (NP / 4);
                        okk[u] = okk_item[p0 + u];
                        oo[u] = oo_item[p0 + u];
                        accv[u] = *reinterpret_cast<const float4*>(stage + px * SS + 4 * cq);
                        refv[u] = make_float4(1.f, 1.f, 1.f, 1.f);
                        addv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                        if constexpr (EPI) {   // (an absent operand reads zeros through its empty resource and is not used)
                            const u32x4 w2 = PRE ? refq[PRE ? p0 + u : 0] : load_piece(r_ref, oo[u], row_byte);
                            const u32x4 w3 = PRE ? addq[PRE ? p0 + u : 0] : load_piece(r_add, oo[u], row_byte);
                            if (a.mask_ref) refv[u] = piece_values(w2);
                            addv[u] = piece_values(w3);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < UN; ++u) {
                        const int j = (p0 + u) * 64 + lane;
                        const int co = NP * hb + 4 * (j % (NP / 4));
                        const float4 bv = *reinterpret_cast<const float4*>(bias_s + co);
                        float xv[4] = {accv[u].x + bv.x, accv[u].y + bv.y, accv[u].z + bv.z, accv[u].w + bv.w};
                        const float rr[4] = {refv[u].x, refv[u].y, refv[u].z, refv[u].w};
                        const float aa[4] = {addv[u].x, addv[u].y, addv[u].z, addv[u].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            xv[e] = fmaxf(xv[e], out_floor);
                            if constexpr (EPI) {
                                if (a.mask_acc) xv[e] = rr[e] > 0.f ? xv[e] : 0.f;
                                xv[e] += (a.mask_add && !(rr[e] > 0.f)) ? 0.f : aa[e];
                            }
                        }
                        if (okk[u]) {
                            if constexpr (BF) {
                                const u32x2 pk = {pack_bf16x2(xv[0], xv[1]), pack_bf16x2(xv[2], xv[3])};
                                __builtin_amdgcn_raw_buffer_store_b64(pk, r_out, oo[u], row_byte, 0);
                            } else {
                                typedef float f32x4 __attribute__((ext_vector_type(4)));
                                const f32x4 pk = {xv[0], xv[1], xv[2], xv[3]};
                                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((ext_vector_type(4))) unsigned, pk), r_out, oo[u], row_byte, 0);
                            }
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
            ++y;
        };
        while (true) {
            row_step(std::integral_constant<int, 0>{});
            if (y >= y1) break;
            row_step(std::integral_constant<int, 1>{});
            if (y >= y1) break;
            row_step(std::integral_constant<int, 2>{});
            if (y >= y1) break;
        }
    }
}

template <int KD, int NB, int NH, bool BF, bool EPI>
static void launch_thin_in_mfma_e(const ThinInMfmaArgs& a, hipStream_t st) {
    static const int per_cu = [] {   // persistent waves: what the instantiation's registers allow, at most four workgroups
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, conv_thin_in_mfma_kernel<KD, NB, NH, BF, EPI>, 256, 0) != hipSuccess) n = 1;
        return n < 1 ? 1 : (n > 4 ? 4 : n);
    }();
    // runs of rows per (slice, segment) column: the split that minimises (columns per wave) x (run length + the two rows a
    // run loads before its first)
    const long long cols = a.d.Q / ((long long)a.d.H * a.d.W) * ((a.d.W + 31) / 32), waves = 4LL * 256 * per_cu;
    int runs = 1, run_len = a.d.H;
    double best = 1e300;
    for (int n = 1; n <= a.d.H; ++n) {
        const int len = (a.d.H + n - 1) / n;
        if ((a.d.H + len - 1) / len != n) continue;
        const long long items = cols * n;
        const double cost = (double)((items + waves - 1) / waves) * (len + 2.0);
        if (cost < best) { best = cost; runs = n; run_len = len; }
    }
    const long long n_items = cols * runs;
    const long long want = (n_items + 3) / 4, cap = 256LL * per_cu;
    hipLaunchKernelGGL((conv_thin_in_mfma_kernel<KD, NB, NH, BF, EPI>), dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0, st, a, runs, run_len);
}

template <int KD, int NB, int NH, bool BF>
static void launch_thin_in_mfma_t(const ThinInMfmaArgs& a, hipStream_t st) {
    if (a.mask_ref || a.add) launch_thin_in_mfma_e<KD, NB, NH, BF, true>(a, st);
    else launch_thin_in_mfma_e<KD, NB, NH, BF, false>(a, st);
}

template <int KD, bool BF>
static void launch_thin_in_mfma_n(const ThinInMfmaArgs& a, hipStream_t st) {
    switch (a.Nn / 32) {
        case 1: launch_thin_in_mfma_t<KD, 1, 1, BF>(a, st); break;
        case 2: launch_thin_in_mfma_t<KD, 2, 1, BF>(a, st); break;
        default: launch_thin_in_mfma_t<KD, 2, 2, BF>(a, st); break;
    }
}

bool conv_thin_in_mfma_applies(const PixDims& d, int Nn) {
    const bool on = !(kernel_policy() & GLEAM_POLICY_NO_THIN_MFMA);   // else the vector-ALU kernel
    if (!on || !(d.kt == 1 && (d.kd == 3 || d.kd == 1) && d.kh == 3 && d.kw == 3)) return false;
    // byte offsets into the input and the output are 32 bits in the kernel
    if ((double)d.Q * 8.0 >= 4.0e9 || (double)d.Q * Nn * 4.0 >= 4.0e9) return false;
    return Nn == 32 || Nn == 64 || Nn == 128;
}

hipError_t launch_conv_thin_in_mfma(const ThinInMfmaArgs& a, bool bf, hipStream_t st) {
    if (!conv_thin_in_mfma_applies(a.d, a.Nn)) return hipErrorInvalidValue;
    if (a.d.kd == 3) {
        if (bf) launch_thin_in_mfma_n<3, true>(a, st);
        else launch_thin_in_mfma_n<3, false>(a, st);
    } else {
        if (bf) launch_thin_in_mfma_n<1, true>(a, st);
        else launch_thin_in_mfma_n<1, false>(a, st);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------------
// Weight gradient of a layer with the 2-channel image on one side, 3x3 (KD = 1) or 3x3x3 (KD = 3) taps, on the matrix
// cores:
//   THIN_IN  (first layer):  dw[c][tap][e] = sum_q wide[q][c] * thin[q + off(tap)][e]      wide = output gradient
//   !THIN_IN (last layer):   dw[e][tap][c] = sum_q wide[q][c] * thin[q - off(tap)][e]      wide = input activation
// One v_mfma_f32_32x32x2_f32 takes two pixels as its depth: A = the wide tensor (rows = 32 channels, lane (m, h) loads
// channel m of pixel h: 256 contiguous bytes per wave), B = the thin tensor seen through the taps (columns = (tap, e)
// pairs, 18 or 54 of them in one or two blocks of 32; lane (n, h) loads the value its pair needs for pixel h).  A wave
// walks down the rows of a 32-pixel column segment and keeps the thin rows around the current row in its own LDS rows
// (one new row per slice tap and image row, fetched a row ahead), from where the B operands are 4-byte LDS reads at
// lane-constant offsets (read straight from memory, a wave-wide load gathered from up to 27 rows and took as long as
// the MFMAs).  All global loads go through buffer resources that span one image row: pixels outside the row arrive
// as zeros and a row outside the volume gets a resource of size 0, so nothing is masked.  The vector-ALU kernel this
// replaces for these shapes spends 2 * taps multiply-adds per wide value and is bound by them.
struct WgradThinWalkKArgs {
    WgradThinWalkArgs a;
    int runs, run_len;
};

template <int KD, int NCB, bool THIN_IN, bool BF>
__global__ __launch_bounds__(256) void wgrad_thin_walk_kernel(WgradThinWalkKArgs ka) {
    constexpr int TAPS = 9 * KD, NCOL = 2 * TAPS, NBLK = (NCOL + 31) / 32, WC = 32 * NCB;
    constexpr int ES = BF ? 2 : 4;
    constexpr unsigned kOutside = 0x80000000u;
    __shared__ float red[2][NCB * NBLK * 16 * 64];
    // bfloat16 wide tensors with 64 channels or more are loaded as channel pairs (4 bytes per lane): row i of block c is
    // channel 64 (c / 2) + 2 i + c % 2 then, else channel 32 c + i
    constexpr bool PAIRS = BF && NCB >= 2;
    auto chan = [](int c, int i) { return PAIRS ? 64 * (c / 2) + 2 * i + (c & 1) : 32 * c + i; };
    // the thin rows around the current row, per wave: [slice tap][ring of 4 rows][36 pixels][2]; pixel pp = image column
    // x_seg - 1 + pp.  Rows and columns outside the volume hold zeros (they are loaded through a resource that spans one
    // image row, of size 0 for a row outside), so the B operand reads need no masks.
    constexpr int kSlabPx = 36;
    __shared__ __attribute__((aligned(8))) float slab_all[4][KD * 4 * kSlabPx * 2];
    const WgradThinWalkArgs& a = ka.a;
    const PixDims d = a.d;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int m = lane & 31, h = lane >> 5;
    float* const slab = slab_all[wave];
    constexpr int sgn = THIN_IN ? 1 : -1;
    // this lane's (tap, e) pair per column block
    int dz[NBLK], dy[NBLK], dx[NBLK], ee[NBLK];
    bool col_used[NBLK];
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
        const int n = 32 * b + m, tap = n >> 1;
        col_used[b] = n < NCOL;
        ee[b] = n & 1;
        dz[b] = KD == 1 ? 0 : sgn * (tap / 9 - 1);
        dy[b] = sgn * ((tap / 3) % 3 - 1);
        dx[b] = sgn * (tap % 3 - 1);
    }
    floatx16 acc[NCB][NBLK];
#pragma unroll
    for (int c = 0; c < NCB; ++c)
#pragma unroll
        for (int b = 0; b < NBLK; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[c][b][r] = 0.f;
    float bs[THIN_IN ? NCB : 1];
#pragma unroll
    for (int c = 0; c < (THIN_IN ? NCB : 1); ++c) bs[c] = 0.f;

    const int segs = (d.W + 31) / 32;
    const long long planes = d.Q / ((long long)d.H * d.W);
    const long long n_items = planes * segs * ka.runs;
    const unsigned wide_row_bytes = (unsigned)d.W * WC * ES;
    const int relu_floor = a.relu_in ? 0 : (int)0x80000000;   // ReLU as a signed-integer maximum on the bit pattern

    for (long long item = (long long)blockIdx.x * 4 + wave; item < n_items; item += (long long)gridDim.x * 4) {
        // segments fastest: the four waves of a workgroup walk down neighbouring segments of the same rows
        const int seg = (int)(item % segs);
        const int rn = (int)((item / segs) % ka.runs);
        const long long plane = item / ((long long)ka.runs * segs);
        const int z = (int)(plane % d.D);
        const int x_seg = 32 * seg;
        const int y0 = rn * ka.run_len, y1 = y0 + ka.run_len < d.H ? y0 + ka.run_len : d.H;
        // thin side: lanes 0 .. 35 fetch pixel pp = lane of a row segment (8 bytes); float offset of this lane's B value
        // inside a slab row
        const unsigned thin_lane = lane < kSlabPx ? (unsigned)((x_seg - 1 + lane) * 8) : kOutside;
        int b_in_row[NBLK];
#pragma unroll
        for (int b = 0; b < NBLK; ++b) b_in_row[b] = ((KD == 1 ? 0 : dz[b] + 1) * 4 * kSlabPx + h + dx[b] + 1) * 2 + ee[b];
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        u32x2 tq[KD];
        auto fetch_thin = [&](int ys) __attribute__((always_inline)) {   // row ys of the KD slices
#pragma unroll
            for (int iz = 0; iz < KD; ++iz) {
                const int zz = z + iz - KD / 2;
                const bool ok = ys >= 0 && ys < d.H && (KD == 1 || (zz >= 0 && zz < d.D));   // uniform
                const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
                    (void*)(a.thin + (ok ? ((plane + iz - KD / 2) * d.H + ys) * d.W * 2 : 0)), 0, ok ? (unsigned)d.W * 8u : 0u, 0x00020000);
                tq[iz] = __builtin_amdgcn_raw_buffer_load_b64(r, thin_lane, 0, 0);
            }
        };
        auto store_thin = [&](int ys) __attribute__((always_inline)) {
            const int slot = (ys - y0 + 1) & 3;
            if (lane < kSlabPx) {
#pragma unroll
                for (int iz = 0; iz < KD; ++iz) {
                    int v0 = (int)tq[iz][0], v1 = (int)tq[iz][1];
                    if (THIN_IN) { v0 = v0 > relu_floor ? v0 : relu_floor; v1 = v1 > relu_floor ? v1 : relu_floor; }
                    *reinterpret_cast<float2*>(slab + ((iz * 4 + slot) * kSlabPx + lane) * 2) = make_float2(__int_as_float(v0), __int_as_float(v1));
                }
            }
        };
        // (LDS operations of one wave execute in order: no barrier between this wave's stores and its reads)
        fetch_thin(y0 - 1); store_thin(y0 - 1);
        fetch_thin(y0); store_thin(y0);
        fetch_thin(y0 + 1); store_thin(y0 + 1);
        const unsigned wide_lane = (unsigned)((h * WC + (PAIRS ? 2 * m : m)) * ES);
        for (int y = y0; y < y1; ++y) {
            fetch_thin(y + 2);   // stored after this row's reads, into the slot of row y - 2
            const __amdgpu_buffer_rsrc_t r_wide = __builtin_amdgcn_make_buffer_rsrc(
                (void*)((const char*)a.wide + ((plane * d.H + y) * d.W) * (long long)(WC * ES)), 0, wide_row_bytes, 0x00020000);
            const float* brow[NBLK];
#pragma unroll
            for (int b = 0; b < NBLK; ++b) brow[b] = slab + b_in_row[b] + ((y + dy[b] - y0 + 1) & 3) * (kSlabPx * 2);
            float av[NCB][16], bv[NBLK][16];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
#pragma unroll
                for (int c = 0; c < NCB; c += PAIRS ? 2 : 1) {
                    const unsigned off = wide_lane + (unsigned)(((x_seg + 2 * j) * WC + 32 * c) * ES);
                    if constexpr (PAIRS) {
                        const unsigned w2 = __builtin_amdgcn_raw_buffer_load_b32(r_wide, off, 0, 0);
                        int lo = (int)(w2 << 16), hi = (int)(w2 & 0xffff0000u);
                        if (!THIN_IN) { lo = lo > relu_floor ? lo : relu_floor; hi = hi > relu_floor ? hi : relu_floor; }
                        av[c][j] = __int_as_float(lo);
                        av[c + 1][j] = __int_as_float(hi);
                    } else {
                        int bits;
                        if constexpr (BF) bits = (int)((unsigned)(unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r_wide, off, 0, 0) << 16);
                        else bits = (int)__builtin_amdgcn_raw_buffer_load_b32(r_wide, off, 0, 0);
                        if (!THIN_IN) bits = bits > relu_floor ? bits : relu_floor;
                        av[c][j] = __int_as_float(bits);
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < 16; ++j)
#pragma unroll
                for (int b = 0; b < NBLK; ++b) bv[b][j] = brow[b][4 * j];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
#pragma unroll
                for (int c = 0; c < NCB; ++c)
#pragma unroll
                    for (int b = 0; b < NBLK; ++b) acc[c][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[c][j], bv[b][j], acc[c][b], 0, 0, 0);
                // bias gradient: column sums of the output gradient, which is the wide tensor (THIN_IN) or the thin one
                // (there the centre tap's columns hold the pixel itself)
                if (THIN_IN) {
#pragma unroll
                    for (int c = 0; c < NCB; ++c) bs[c] += av[c][j];
                } else {
                    bs[0] += bv[0][j];
                }
            }
            store_thin(y + 2);
        }
    }

    // fold the four waves of the workgroup (waves 2, 3 into 0, 1, then 1 into 0), then wave 0 writes the partial block in
    // dw layout
    const int Co = THIN_IN ? WC : 2, Ci = THIN_IN ? 2 : WC;
    float* dst = a.partial + (size_t)blockIdx.x * Co * TAPS * Ci;
    float bsum[THIN_IN ? NCB : 1];
#pragma unroll
    for (int c = 0; c < (THIN_IN ? NCB : 1); ++c) bsum[c] = bs[c] + __shfl_xor(bs[c], 32);
    auto put = [&](int slot) {
#pragma unroll
        for (int c = 0; c < NCB; ++c)
#pragma unroll
            for (int b = 0; b < NBLK; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) red[slot][((c * NBLK + b) * 16 + r) * 64 + lane] = acc[c][b][r];
    };
    auto take = [&](int slot) {
#pragma unroll
        for (int c = 0; c < NCB; ++c)
#pragma unroll
            for (int b = 0; b < NBLK; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[c][b][r] += red[slot][((c * NBLK + b) * 16 + r) * 64 + lane];
    };
    __shared__ float bred[4][THIN_IN ? 32 * NCB : 64];
#pragma unroll
    for (int c = 0; c < (THIN_IN ? NCB : 1); ++c)
        if (h == 0) bred[wave][32 * c + m] = bsum[c];
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) take(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave == 0) {
        take(0);
#pragma unroll
        for (int c = 0; c < NCB; ++c)
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int n = 32 * b + m;
                if (n < NCOL) {
                    const int tap = n >> 1, e = n & 1;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int ch = chan(c, 8 * (r >> 2) + 4 * h + (r & 3));
                        dst[THIN_IN ? ((size_t)ch * TAPS + tap) * 2 + e : ((size_t)e * TAPS + tap) * WC + ch] = acc[c][b][r];
                    }
                }
            }
    }
    if (a.bias_partial != nullptr) {
        if (THIN_IN) {
            if ((int)threadIdx.x < WC) {
                const int c = threadIdx.x >> 5, i = threadIdx.x & 31;
                a.bias_partial[(size_t)blockIdx.x * Co + chan(c, i)] =
                    (bred[0][threadIdx.x] + bred[1][threadIdx.x]) + (bred[2][threadIdx.x] + bred[3][threadIdx.x]);
            }
        } else if (threadIdx.x < 2) {
            const int col = 2 * (TAPS / 2) + threadIdx.x;   // centre tap
            a.bias_partial[(size_t)blockIdx.x * Co + threadIdx.x] = (bred[0][col] + bred[1][col]) + (bred[2][col] + bred[3][col]);
        }
    }
}

bool wgrad_thin_walk_applies(const PixDims& d, int WC, bool bf) {
    if (kernel_policy() & GLEAM_POLICY_NO_THIN_MFMA) return false;
    if (!(d.kt == 1 && (d.kd == 1 || d.kd == 3) && d.kh == 3 && d.kw == 3)) return false;
    // byte offsets into the thin tensor and into an image row of the wide one are 32 bits in the kernel
    if ((double)d.Q * 8.0 >= 2.0e9 || (double)d.W * WC * 4.0 >= 2.0e9) return false;
    (void)bf;
    return WC == 32 || WC == 64 || WC == 128;
}

template <int KD, int NCB, bool THIN_IN, bool BF>
static hipError_t launch_wgrad_thin_walk_t(const WgradThinWalkArgs& a, size_t partial_floats, int* used_split, hipStream_t st) {
    static const int per_cu = [] {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, wgrad_thin_walk_kernel<KD, NCB, THIN_IN, BF>, 256, 0) != hipSuccess) n = 1;
        return n < 1 ? 1 : (n > 4 ? 4 : n);
    }();
    const PixDims& d = a.d;
    const long long cols = d.Q / ((long long)d.H * d.W) * ((d.W + 31) / 32);
    const size_t block = (size_t)(32 * NCB) * 9 * KD * 2;
    long long wgs = 256LL * per_cu;
    const long long fit = (long long)(partial_floats / block);
    if (wgs > fit) wgs = fit;
    if (wgs > kThinWalkSplit) wgs = kThinWalkSplit;
    if (wgs < 1) return hipErrorInvalidValue;
    WgradThinWalkKArgs ka{a, 1, d.H};
    double best = 1e300;
    for (int n = 1; n <= d.H; ++n) {
        const int len = (d.H + n - 1) / n;
        if ((d.H + len - 1) / len != n) continue;
        const long long items = cols * n;
        const double cost = (double)((items + 4 * wgs - 1) / (4 * wgs)) * (len + 0.5);
        if (cost < best) { best = cost; ka.runs = n; ka.run_len = len; }
    }
    const long long want = (cols * ka.runs + 3) / 4;
    const long long gx = want < wgs ? want : wgs;
    hipLaunchKernelGGL((wgrad_thin_walk_kernel<KD, NCB, THIN_IN, BF>), dim3((unsigned)gx), dim3(256), 0, st, ka);
    *used_split = (int)gx;
    return hipGetLastError();
}

template <int KD, bool THIN_IN, bool BF>
static hipError_t launch_wgrad_thin_walk_c(const WgradThinWalkArgs& a, size_t partial_floats, int* used_split, hipStream_t st) {
    switch (a.WC / 32) {
        case 1: return launch_wgrad_thin_walk_t<KD, 1, THIN_IN, BF>(a, partial_floats, used_split, st);
        case 2: return launch_wgrad_thin_walk_t<KD, 2, THIN_IN, BF>(a, partial_floats, used_split, st);
        default: return launch_wgrad_thin_walk_t<KD, 4, THIN_IN, BF>(a, partial_floats, used_split, st);
    }
}

hipError_t launch_wgrad_thin_walk(const WgradThinWalkArgs& a, size_t partial_floats, int* used_split, hipStream_t st) {
    if (!wgrad_thin_walk_applies(a.d, a.WC, a.bf != 0)) return hipErrorInvalidValue;
#define GLEAM_TW(KD_)                                                                                       \
    if (a.thin_in) {                                                                                        \
        if (a.bf) return launch_wgrad_thin_walk_c<KD_, true, true>(a, partial_floats, used_split, st);     \
        return launch_wgrad_thin_walk_c<KD_, true, false>(a, partial_floats, used_split, st);              \
    } else {                                                                                                \
        if (a.bf) return launch_wgrad_thin_walk_c<KD_, false, true>(a, partial_floats, used_split, st);    \
        return launch_wgrad_thin_walk_c<KD_, false, false>(a, partial_floats, used_split, st);             \
    }
    if (a.d.kd == 3) { GLEAM_TW(3) } else { GLEAM_TW(1) }
#undef GLEAM_TW
}

}  // namespace gleam
