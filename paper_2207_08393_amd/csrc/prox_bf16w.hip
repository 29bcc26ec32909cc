// Weight gradient of a 3x3 layer with 128 input channels, bfloat16 operands, float32 sums:
//     dW[co][ky][kx][ci] = sum over images and pixels (y, x) of g[y][x][co] * a[y + ky - 1][x + kx - 1][ci]
// The three row taps pair gradient row y with input rows y - 1, y, y + 1, so a workgroup walks down a strip of 64
// columns and every input row segment is brought into LDS once (a kernel that stages the three rows per gradient
// row reads each input three times and pays the staging instructions three times).  Nothing is staged through
// registers: row segments go from memory to LDS by direct loads, one image row ahead of the matrix cores; pixels
// outside the image fall outside the buffer resource of their image row and arrive as zeros, so the loop has no
// masks, no selects and no LDS stores.
// A workgroup of 8 waves (two per SIMD) owns 64 output channels x 128 input channels: wave (wi, wc) holds the nine taps
// of input channels 32 wi .. + 31 against output channels 32 wc .. + 31 (9 accumulators; 18 per wave would be 288
// registers, more than the 256 accumulation registers an MFMA can address, and the compiler then moves accumulators
// to and fro all the time).  Per 16 pixels and input row it reads its input window with 4 transposing LDS reads (the
// taps kx = 0 and kx = 2 as they lie, kx = 1 by register shifts of the two) and per 16 pixels its gradient operand with 2;
// the bias sums are packed dot products with ones.  v_mfma_f32_32x32x16_bf16: contraction index = pixel; A = gradient
// (rows = output channels), B = input window (columns = input channels), so a lane's accumulators are one input
// channel and lanes are contiguous in the [Co][tap][Ci] partial block every workgroup writes once.
// The four input buffers and the two gradient buffers are separate LDS objects and the walk is written out over
// its four rotations: the compiler then knows which buffer a read touches and does not make operand reads wait for
// the direct loads in flight.
#include "prox_common.h"

namespace gleam {

namespace {

constexpr int kWW = 64;                  // columns of a strip
// LDS layout of a segment: pixel p, channel c at element p * row + 16 * ((p / 8) % 2) + c, with rows of 320 bytes
// (input, 128 channels) and 192 bytes (gradient, 64 channels).  A transposing read touches, per group of 16 lanes,
// 32 bytes of each of 4 consecutive pixels, the lane halves of a wave are 8 pixels apart and the two groups of a
// half 32 bytes: with row = 64 (mod 256) bytes the four pixels of a half fill the 64 banks exactly, and the extra 32
// bytes of every other block of 8 pixels keep the halves apart whichever lanes the hardware serves together.
// (With 288-byte rows the counters showed two conflict cycles per cycle of LDS work.)
constexpr int kWXRow = 160;              // elements per pixel of an input segment
constexpr int kWGRow = 96;               // elements per pixel of a gradient segment
constexpr int kWXPix = kWW + 2;          // pixels of an input segment that are loaded (one halo column each side)
constexpr int kWXQuads = 21 * 64;        // 16-byte slots of an input buffer: 66 pixels of 20 slots and the shift
constexpr int kWXLoads = 21;             // wave-wide direct loads that cover the 66 loaded pixels
constexpr int kWGQuads = 12 * 64;        // 64 pixels x 12 slots
constexpr int kWGLoads = 12;

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
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 1, wc = wave & 1;
    const int m = lane & 31, h = lane >> 5;
    const int co0 = 64 * (int)blockIdx.y;
    constexpr int Ci = 128;

    // Direct loads through a buffer resource that spans one image row: a slot whose byte offset falls outside the row
    // (columns left of 0 come out as huge unsigned offsets, columns right of W - 1 exceed the size) is filled with zeros
    // by the hardware, a row outside the image gets a resource of size 0, and padding slots an offset that is always
    // outside; no selects, no LDS stores.  Input buffer: slot s = 64 (wave + 8 i) + lane belongs to segment pixel
    // pp = s / 20 = image column x0 - 1 + pp and holds its channel quad s % 20 - 2 ((pp / 8) % 2) if that is one of
    // 0 .. 15.  Gradient buffer: pixel p = s / 12 = column x0 + p, quad s % 12 - 2 ((p / 8) % 2) of 0 .. 7.
    constexpr unsigned kOutside = 0x80000000u;   // (row sizes are below 2^31 bytes: checked by the launcher)
    unsigned x_slot[3], g_slot[2];               // byte offset from column x0 of the row
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int s = 64 * (wave + 8 * i) + lane, pp = s / 20, c8 = s % 20 - 2 * ((pp >> 3) & 1);
        x_slot[i] = (c8 >= 0 && c8 < 16 && pp < kWXPix) ? (unsigned)((pp - 1) * Ci * 2 + 16 * c8) : kOutside;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int s = 64 * (wave + 8 * i) + lane, p = s / 12, c8 = s % 12 - 2 * ((p >> 3) & 1);
        g_slot[i] = (c8 >= 0 && c8 < 8) ? (unsigned)(p * a.Co * 2 + 2 * co0 + 16 * c8) : kOutside;
    }
    const unsigned x_row_bytes = (unsigned)a.W * Ci * 2, g_row_bytes = (unsigned)a.W * (unsigned)a.Co * 2;

    // per-lane element offsets of the transposing reads: pixel 8h + (lane % 16) / 4 (+ 2, 4, 6) of the 16-pixel block,
    // channels 16 ((lane / 16) % 2) + 4 (lane % 4) .. + 3 of the wave's 32-channel block
    const int tr_row = 8 * h + ((lane & 15) >> 2), tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    auto px_off = [](int p, int row) { return p * row + 16 * ((p >> 3) & 1); };
    const int g_rd = px_off(tr_row, kWGRow) + wc * 32 + tr_col;        // (+ 4 pixels: the same block of 8)
    const int x_rd = px_off(tr_row, kWXRow) + wi * 32 + tr_col;        // (+ 2, + 4 pixels: the same block of 8)
    const int x_rd6 = px_off(tr_row + 6, kWXRow) + wi * 32 + tr_col;

    floatx16 acc[9];
#pragma unroll
    for (int j = 0; j < 9; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    float bsum = 0.f;
    const bf16x2v ones = {(__bf16)1.0f, (__bf16)1.0f};

    // one image row of the strip: input rows y - 1, y, y + 1 in xm, xz, xp, gradient row y in gc
    auto run = [&](const unsigned short* xm, const unsigned short* xz, const unsigned short* xp, const unsigned short* gc)
                   __attribute__((always_inline)) {
        // 12 operand groups (16-pixel block kb, input row rt): 4 window reads (+ 2 gradient reads when rt = 0) and 3 MFMAs
        // each; the reads of a group are issued two groups ahead of its MFMAs.  Of this lane's input channel a group
        // reads segment pixels 16 kb + 8 h + 0 .. 7 (tap kx = 0) and + 2 .. 9 (kx = 2) as they are (four registers that
        // start at an odd one are no MFMA operand, and the copies would cost more than the second pair of reads);
        // kx = 1 is shifted out of the two.
        uint2 wq[3][4], gq[2][2];
        auto read_group = [&](int g) __attribute__((always_inline)) {
            const int kb = g / 3, rt = g - 3 * kb;
            if (rt == 0) {
                const unsigned short* gp = gc + g_rd + 16 * kb * kWGRow;
                gq[kb & 1][0] = w_read_tr16(gp);
                gq[kb & 1][1] = w_read_tr16(gp + 4 * kWGRow);
            }
            const unsigned short* row = (rt == 0 ? xm : rt == 1 ? xz : xp) + 16 * kb * kWXRow;
            wq[g % 3][0] = w_read_tr16(row + x_rd);
            wq[g % 3][1] = w_read_tr16(row + x_rd + 4 * kWXRow);
            wq[g % 3][2] = w_read_tr16(row + x_rd + 2 * kWXRow);
            wq[g % 3][3] = w_read_tr16(row + x_rd6);
        };
        read_group(0);
        read_group(1);
#pragma unroll
        for (int g = 0; g < 12; ++g) {
            const int kb = g / 3, rt = g - 3 * kb;
            if (g + 2 < 12) read_group(g + 2);
            __builtin_amdgcn_sched_barrier(0);
            const uint2 g0 = gq[kb & 1][0], g1 = gq[kb & 1][1];
            const bf16x8 gv = __builtin_bit_cast(bf16x8, make_uint4(g0.x, g0.y, g1.x, g1.y));
            if (rt == 0) {   // bias gradient (the four waves with these output channels all form it; one of them writes it)
                const unsigned w4[4] = {g0.x, g0.y, g1.x, g1.y};
#pragma unroll
                for (int e = 0; e < 4; ++e) bsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2v, w4[e]), ones, bsum, false);
            }
            uint2* w = wq[g % 3];
            if (RELU) {
#pragma unroll
                for (int e = 0; e < 4; ++e) { w[e].x = relu_bf16x2(w[e].x); w[e].y = relu_bf16x2(w[e].y); }
            }
            uint4 b1;   // pixels 1 .. 8 of the window
            b1.x = __builtin_amdgcn_alignbit(w[0].y, w[0].x, 16);
            b1.y = __builtin_amdgcn_alignbit(w[1].x, w[0].y, 16);
            b1.z = __builtin_amdgcn_alignbit(w[1].y, w[1].x, 16);
            b1.w = __builtin_amdgcn_alignbit(w[3].y, w[1].y, 16);
            const uint4 b0 = make_uint4(w[0].x, w[0].y, w[1].x, w[1].y), b2 = make_uint4(w[2].x, w[2].y, w[3].x, w[3].y);
            acc[3 * rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gv, __builtin_bit_cast(bf16x8, b0), acc[3 * rt], 0, 0, 0);
            acc[3 * rt + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gv, __builtin_bit_cast(bf16x8, b1), acc[3 * rt + 1], 0, 0, 0);
            acc[3 * rt + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gv, __builtin_bit_cast(bf16x8, b2), acc[3 * rt + 2], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    for (long long item = blockIdx.x; item < a.n_items; item += gridDim.x) {
        const int rn = (int)(item % a.runs);
        const int strip = (int)((item / a.runs) % a.strips);
        const long long img = item / ((long long)a.runs * a.strips);
        const int x0 = strip * kWW;
        const int y0 = rn * a.run_len, y1 = y0 + a.run_len < a.H ? y0 + a.run_len : a.H;
        unsigned x_at[3], g_at[2];   // byte offsets of this thread's slots inside an image row
#pragma unroll
        for (int i = 0; i < 3; ++i) x_at[i] = x_slot[i] + (unsigned)(x0 * Ci * 2);
#pragma unroll
        for (int i = 0; i < 2; ++i) g_at[i] = g_slot[i] + (unsigned)(x0 * a.Co * 2);
        const unsigned short* const xa = a.a + (img * a.H) * a.W * Ci;     // row 0 of the image
        const unsigned short* const ga = a.g + (img * a.H) * a.W * a.Co;
        auto load_x = [&](int y, unsigned short* dst) __attribute__((always_inline)) {
            const bool row_ok = y >= 0 && y < a.H;
            const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(xa + (long long)(row_ok ? y : 0) * a.W * Ci), 0, row_ok ? x_row_bytes : 0u, 0x00020000);
#pragma unroll
            for (int i = 0; i < 3; ++i)
                if (wave + 8 * i < kWXLoads)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)(dst + (wave + 8 * i) * 512), 16,
                                                             x_at[i], 0, 0, 0);
        };
        auto load_g = [&](int y, unsigned short* dst) __attribute__((always_inline)) {   // rows y0 .. y1 - 1 only
            const __amdgpu_buffer_rsrc_t r =
                __builtin_amdgcn_make_buffer_rsrc((void*)(ga + (long long)y * a.W * a.Co), 0, g_row_bytes, 0x00020000);
#pragma unroll
            for (int i = 0; i < 2; ++i)
                if (wave + 8 * i < kWGLoads)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)(dst + (wave + 8 * i) * 512), 16,
                                                             g_at[i], 0, 0, 0);
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
    if (a.bias_partial && wi == 0) {
        const float tot = bsum + __shfl_xor(bsum, 32);
        if (h == 0) a.bias_partial[(size_t)blockIdx.x * a.Co + co0 + 32 * wc + m] = tot;
    }
}

bool wgrad_bf16_walk_applies(const PixDims& d, int Ci, int Co) {
    // element offsets inside a row of strips are 32 bits in the kernel
    return d.kt == 1 && d.kd == 1 && d.kh == 3 && d.kw == 3 && Ci == 128 && Co % 64 == 0 && Co >= 64 &&
           (double)(d.W + 2 * kWW) * 2.0 * (Ci > Co ? Ci : Co) < 2.0e9;   // byte offsets inside an image row: 31 bits
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
