// Weight gradient of a 3x3 layer with 128 input channels, bfloat16 operands, float32 sums:
//     dW[co][ky][kx][ci] = sum over images and pixels (y, x) of g[y][x][co] * a[y + ky - 1][x + kx - 1][ci]
// The three row taps pair gradient row y with input rows y - 1, y, y + 1, so a workgroup walks down a strip of 64
// columns and every input row segment is brought into LDS once (a kernel that stages the three rows per gradient
// row reads each input three times and pays the staging instructions three times).  Nothing is staged through
// registers: row segments go from memory to LDS by direct loads, one image row ahead of the matrix cores; pixels
// outside the image are loaded from a 16-byte block of zeros, so the loop has no masks and no LDS stores.
// A workgroup of 8 waves (two per SIMD) owns 64 output channels x 128 input channels: wave (wi, wc) holds the nine taps
// of input channels 32 wi .. + 31 against output channels 32 wc .. + 31 (9 accumulators; 18 per wave would be 288
// registers, more than the 256 accumulation registers an MFMA can address, and the compiler then moves accumulators
// to and fro all the time).  Per 16 pixels it reads its input window (3 transposing LDS reads per input row, the kx
// shifts are register shifts of that window) and its gradient operand, 11 LDS reads for 9 MFMAs.  v_mfma_f32_32x32x16_bf16: contraction index = pixel; A = gradient (rows = output channels),
// B = input window (columns = input channels), so a lane's accumulators are one input channel and lanes are
// contiguous in the [Co][tap][Ci] partial block every workgroup writes once.
// The four input buffers and the two gradient buffers are separate LDS objects and the walk is written out over
// its four rotations: the compiler then knows which buffer a read touches and does not make operand reads wait for
// the direct loads in flight.
#include "prox_common.h"

namespace gleam {

namespace {

constexpr int kWW = 64;                  // columns of a strip
constexpr int kWXRow = 128 + 16;         // elements per pixel of an input segment: 128 channels + 32 bytes (bank spread)
constexpr int kWGRow = 64 + 16;          // elements per pixel of a gradient segment
constexpr int kWXPix = kWW + 2;          // pixels of an input segment that are loaded (one halo column each side)
constexpr int kWXQuads = 20 * 64;        // 16-byte slots of an input buffer: 68 pixels (the windows of the last lanes
                                         // reach two pixels past the loaded ones; what they read there is not used)
constexpr int kWXLoads = 19;             // wave-wide direct loads that cover the 66 loaded pixels (18 slots each)
constexpr int kWGQuads = 10 * 64;        // 64 pixels x 10 slots
constexpr int kWGLoads = 10;

__device__ __attribute__((aligned(16))) unsigned w_zero_quad[4];   // zero-initialised: the source of every out-of-image pixel

__device__ __forceinline__ void w_dma16(const unsigned short* g, unsigned short* l) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)l, 16, 0, 0);
}

typedef short w_short4 __attribute__((ext_vector_type(4)));
// ds_read_b64_tr_b16: within each group of 16 lanes, lane s passes the address of 4 consecutive 16-bit values of
// row s/4, columns 4*(s%4)..+3 of a 4 x 16 block; lane j gets column j of the block, rows 0..3
__device__ __forceinline__ uint2 w_read_tr16(const unsigned short* p) {
    const w_short4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((w_short4 __attribute__((address_space(3)))*)(p));
    return __builtin_bit_cast(uint2, v);
}

}  // namespace

struct WalkWgradBf16Args {
    const unsigned short* g;   // [Q][Co]
    const unsigned short* a;   // [Q][128]
    float* partial;            // [gridDim.x][Co][9][128]
    float* bias_partial;       // [gridDim.x][Co] or null
    int Co, H, W;
    int strips, runs, run_len; // strips of 64 columns per image row, runs of run_len rows per strip
    long long n_items;         // images x strips x runs
};

template <bool RELU>
__global__ __launch_bounds__(512) void wgrad_bf16_walk_kernel(WalkWgradBf16Args a) {
    __shared__ __attribute__((aligned(16))) unsigned short X0[kWXQuads * 8];
    __shared__ __attribute__((aligned(16))) unsigned short X1[kWXQuads * 8];
    __shared__ __attribute__((aligned(16))) unsigned short X2[kWXQuads * 8];
    __shared__ __attribute__((aligned(16))) unsigned short X3[kWXQuads * 8];
    __shared__ __attribute__((aligned(16))) unsigned short G0[kWGQuads * 8];
    __shared__ __attribute__((aligned(16))) unsigned short G1[kWGQuads * 8];
    __shared__ float bred[4][64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 1, wc = wave & 1;
    const int m = lane & 31, h = lane >> 5;
    const int co0 = 64 * (int)blockIdx.y;
    constexpr int Ci = 128;

    // Direct loads.  Input buffer: slot s = 64 (wave + 8 i) + lane holds channel quad s % 18 (16, 17: padding) of segment
    // pixel s / 18 = image column x0 - 1 + s / 18.  Gradient buffer: slot s holds quad s % 10 (8, 9: padding) of pixel
    // s / 10 = column x0 + s / 10.  Padding slots and pixels that are not loaded fetch the zeros as well.
    int x_off[3], x_col[3], g_off[2], g_col[2];   // element offset from (row, x0), column offset; column 1 << 20: never valid
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int s = 64 * (wave + 8 * i) + lane, pp = s / 18, c8 = s % 18;
        const bool data = c8 < 16 && pp < kWXPix;
        x_col[i] = data ? pp - 1 : (1 << 20);
        x_off[i] = data ? (pp - 1) * Ci + 8 * c8 : 0;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int s = 64 * (wave + 8 * i) + lane, p = s / 10, c8 = s % 10;
        const bool data = c8 < 8;
        g_col[i] = data ? p : (1 << 20);
        g_off[i] = data ? p * a.Co + 8 * c8 : 0;
    }
    const unsigned short* const zero = reinterpret_cast<const unsigned short*>(w_zero_quad);

    // per-lane element offsets of the transposing reads: pixel 8h + (lane % 16) / 4 of the 16-pixel block, channels
    // 16 ((lane / 16) % 2) + 4 (lane % 4) .. + 3 of the wave's 32-channel block
    const int tr_row = 8 * h + ((lane & 15) >> 2), tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const int g_rd = tr_row * kWGRow + wc * 32 + tr_col;
    const int x_rd = tr_row * kWXRow + wi * 32 + tr_col;

    floatx16 acc[9];
#pragma unroll
    for (int j = 0; j < 9; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    float bsum = 0.f;

    // one image row of the strip: input rows y - 1, y, y + 1 in xm, xz, xp, gradient row y in gc
    auto run = [&](const unsigned short* xm, const unsigned short* xz, const unsigned short* xp, const unsigned short* gc)
                   __attribute__((always_inline)) {
#pragma unroll
        for (int kb = 0; kb < kWW / 16; ++kb) {
            const unsigned short* gp = gc + g_rd + 16 * kb * kWGRow;
            const uint2 g0 = w_read_tr16(gp), g1 = w_read_tr16(gp + 4 * kWGRow);
            const bf16x8 gv = __builtin_bit_cast(bf16x8, make_uint4(g0.x, g0.y, g1.x, g1.y));
            if (kb == wi) {   // bias gradient: of the four waves with these output channels, each sums one of the four pixel blocks
                const unsigned w4[4] = {g0.x, g0.y, g1.x, g1.y};
#pragma unroll
                for (int e = 0; e < 4; ++e) bsum += __uint_as_float(w4[e] << 16) + __uint_as_float(w4[e] & 0xffff0000u);
            }
#pragma unroll
            for (int rt = 0; rt < 3; ++rt) {
                // window of segment pixels 16 kb + 8 h .. + 11 of this lane's input channel, six 32-bit words
                const unsigned short* row = (rt == 0 ? xm : rt == 1 ? xz : xp) + x_rd + 16 * kb * kWXRow;
                const uint2 w0 = w_read_tr16(row), w1 = w_read_tr16(row + 4 * kWXRow), w2 = w_read_tr16(row + 8 * kWXRow);
                unsigned dws[5] = {w0.x, w0.y, w1.x, w1.y, w2.x};
                if (RELU) {
#pragma unroll
                    for (int e = 0; e < 5; ++e) dws[e] = relu_bf16x2(dws[e]);
                }
#pragma unroll
                for (int dw = 0; dw < 3; ++dw) {
                    uint4 b;
                    if (dw == 1) {
                        b.x = __builtin_amdgcn_alignbit(dws[1], dws[0], 16);
                        b.y = __builtin_amdgcn_alignbit(dws[2], dws[1], 16);
                        b.z = __builtin_amdgcn_alignbit(dws[3], dws[2], 16);
                        b.w = __builtin_amdgcn_alignbit(dws[4], dws[3], 16);
                    } else {
                        b = make_uint4(dws[dw / 2], dws[dw / 2 + 1], dws[dw / 2 + 2], dws[dw / 2 + 3]);
                    }
                    acc[3 * rt + dw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gv, __builtin_bit_cast(bf16x8, b), acc[3 * rt + dw], 0, 0, 0);
                }
            }
        }
    };

    for (long long item = blockIdx.x; item < a.n_items; item += gridDim.x) {
        const int rn = (int)(item % a.runs);
        const int strip = (int)((item / a.runs) % a.strips);
        const long long img = item / ((long long)a.runs * a.strips);
        const int x0 = strip * kWW;
        const int y0 = rn * a.run_len, y1 = y0 + a.run_len < a.H ? y0 + a.run_len : a.H;
        // which of this thread's slots hold pixels inside the image row
        bool x_in[3], g_in[2];
#pragma unroll
        for (int i = 0; i < 3; ++i) x_in[i] = (unsigned)(x0 + x_col[i]) < (unsigned)a.W;
#pragma unroll
        for (int i = 0; i < 2; ++i) g_in[i] = (unsigned)(x0 + g_col[i]) < (unsigned)a.W;
        const unsigned short* const xa = a.a + ((img * a.H) * a.W + x0) * Ci;          // (row 0, x0) of the image
        const unsigned short* const ga = a.g + ((img * a.H) * a.W + x0) * a.Co + co0;
        auto load_x = [&](int y, unsigned short* dst) __attribute__((always_inline)) {
            const bool row_ok = y >= 0 && y < a.H;
            const unsigned short* const base = xa + (long long)(row_ok ? y : 0) * a.W * Ci;
#pragma unroll
            for (int i = 0; i < 3; ++i)
                if (wave + 8 * i < kWXLoads) w_dma16(row_ok && x_in[i] ? base + x_off[i] : zero, dst + (wave + 8 * i) * 512);
        };
        auto load_g = [&](int y, unsigned short* dst) __attribute__((always_inline)) {
            const unsigned short* const base = ga + (long long)y * a.W * a.Co;   // rows y0 .. y1 - 1 only
#pragma unroll
            for (int i = 0; i < 2; ++i)
                if (wave + 8 * i < kWGLoads) w_dma16(g_in[i] ? base + g_off[i] : zero, dst + (wave + 8 * i) * 512);
        };
        // the previous item ended with a barrier: all buffers are free
        load_x(y0 - 1, X0);
        load_x(y0, X1);
        load_x(y0 + 1, X2);
        load_g(y0, G0);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        int y = y0;
        // row y: the input row y + 2 goes to the buffer that held row y - 2, the next gradient row to the other buffer
        auto step = [&](const unsigned short* xm, const unsigned short* xz, const unsigned short* xp, unsigned short* xn,
                        const unsigned short* gc, unsigned short* gn) __attribute__((always_inline)) {
            if (y + 1 < y1) {
                load_x(y + 2, xn);
                load_g(y + 1, gn);
            }
            __builtin_amdgcn_sched_barrier(0);
            run(xm, xz, xp, gc);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            ++y;
        };
        while (true) {
            step(X0, X1, X2, X3, G0, G1);
            if (y >= y1) break;
            step(X1, X2, X3, X0, G1, G0);
            if (y >= y1) break;
            step(X2, X3, X0, X1, G0, G1);
            if (y >= y1) break;
            step(X3, X0, X1, X2, G1, G0);
            if (y >= y1) break;
        }
    }

    float* const pout = a.partial + (size_t)blockIdx.x * a.Co * 9 * Ci;
#pragma unroll
    for (int j = 0; j < 9; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int co = co0 + 32 * wc + 8 * (r >> 2) + 4 * h + (r & 3), ci = 32 * wi + m;
            pout[((size_t)co * 9 + j) * Ci + ci] = acc[j][r];
        }
    if (a.bias_partial) {
        const float tot = bsum + __shfl_xor(bsum, 32);
        if (h == 0) bred[wi][32 * wc + m] = tot;
        __syncthreads();
        if (tid < 64) a.bias_partial[(size_t)blockIdx.x * a.Co + co0 + tid] = (bred[0][tid] + bred[1][tid]) + (bred[2][tid] + bred[3][tid]);
    }
}

bool wgrad_bf16_walk_applies(const PixDims& d, int Ci, int Co) {
    // element offsets inside a row of strips are 32 bits in the kernel
    return d.kt == 1 && d.kd == 1 && d.kh == 3 && d.kw == 3 && Ci == 128 && Co % 64 == 0 && Co >= 64 &&
           d.W < (1 << 20) && (double)(d.W + 2 * kWW) * (Ci > Co ? Ci : Co) < 2.0e9;
}

// Runs per strip.  In units of the time of one image row of a strip: a run of n rows costs n + 3 (its first rows), the
// chip holds 256 workgroups at a time, and every partial block (64 x 9 x 128 sums, written once and read once by the
// reduction) costs about 0.15.
static void wgrad_bf16_walk_split(const PixDims& d, int Co, int* runs, int* run_len, long long* n_items, int* splits) {
    const long long n_img = d.Q / ((long long)d.H * d.W), strips = (d.W + kWW - 1) / kWW, ny = Co / 64;
    const long long per_y = 256 / ny > 0 ? 256 / ny : 1;   // workgroups of one channel block that run together
    long long best_r = 1;
    double best = 1e300;
    for (long long r = 1; r <= d.H; ++r) {
        const long long len = (d.H + r - 1) / r;
        if ((d.H + len - 1) / len != r) continue;   // same run length as a smaller count
        const long long items = n_img * strips * r;
        const long long rounds = (items + per_y - 1) / per_y;
        const double cost = (double)rounds * (double)(len + 3) + 0.15 * (double)((items < per_y ? items : per_y) * ny);
        if (cost < best) { best = cost; best_r = r; }
    }
    *runs = (int)best_r;
    *run_len = (int)((d.H + best_r - 1) / best_r);
    *n_items = n_img * strips * best_r;
    *splits = (int)(*n_items < per_y ? *n_items : per_y);
}

int wgrad_bf16_walk_splits(const PixDims& d, int Co) {
    int runs, run_len, splits;
    long long n_items;
    wgrad_bf16_walk_split(d, Co, &runs, &run_len, &n_items, &splits);
    return splits;
}

size_t wgrad_bf16_walk_partial_floats(const PixDims& d, int Ci, int Co) { return (size_t)wgrad_bf16_walk_splits(d, Co) * 9 * Ci * Co; }

hipError_t launch_wgrad_bf16_walk(const WgradBf16Args& w, hipStream_t st) {
    const PixDims& d = w.d;
    WalkWgradBf16Args a{};
    a.g = w.g; a.a = w.a; a.partial = w.partial; a.bias_partial = w.bias_partial;
    a.Co = w.Co; a.H = d.H; a.W = d.W;
    a.strips = (d.W + kWW - 1) / kWW;
    int splits;
    wgrad_bf16_walk_split(d, w.Co, &a.runs, &a.run_len, &a.n_items, &splits);
    char name[56];
    snprintf(name, sizeof(name), "conv_bf16_wgrad_%dto%d_t9", w.Ci, w.Co);
    KernelScope ks(name, 2.0 * (double)d.Q * w.Ci * w.Co * 9, 2.0 * (double)d.Q * (w.Ci + w.Co), st);
    dim3 grid((unsigned)splits, (unsigned)(w.Co / 64));
    if (w.relu_in) hipLaunchKernelGGL((wgrad_bf16_walk_kernel<true>), grid, dim3(512), 0, st, a);
    else hipLaunchKernelGGL((wgrad_bf16_walk_kernel<false>), grid, dim3(512), 0, st, a);
    return hipGetLastError();
}

}  // namespace gleam
