// Weight gradient of a temporal 3x1x1 layer (the time half of a (2+1)D convolution), float32:
//     dW[co][kt][ci] = sum over samples, frames t and pixels p of g[t][p][co] * x[t + kt - 1][p][ci]
// The three taps pair one input frame tau with the gradients of frames tau + 1, tau and tau - 1, so a workgroup
// walks the frames of a 32-pixel segment in order and every input and every gradient segment is read from memory
// once (a kernel that treats the taps as independent reads each input three times).  A workgroup of 4 waves owns
// a 64 x 64 channel block; wave (jo, ji) holds the three taps of one 32 x 32 sub-block (3 MFMA accumulators) and
// needs four operand reads per three MFMAs: its input channels once, its output channels of three frames.
// The input segments alternate between two LDS buffers and the gradient segments rotate through four, filled by
// direct global -> LDS loads one frame ahead.  The six buffers are separate LDS objects and the loop is written
// out over the four rotations, so that the compiler knows which buffer every read touches and does not make
// operand reads wait for the loads in flight.  Contraction index of v_mfma_f32_32x32x2_f32 = pixel pair; a lane
// holds one channel and one pixel of the pair.  Every workgroup writes its partial sums [Co][3][Ci] once; the
// fixed-order reduction of the other weight-gradient kernels follows.
#include "prox_common.h"

namespace gleam {

namespace {

constexpr int kTPix = 32;                    // pixels per segment
constexpr int kTSlots = kTPix * 16;          // 16-byte quads of a segment of 64 channels
constexpr int kTLoads = kTSlots / 64;        // wave-wide direct loads per segment

__device__ __forceinline__ void dma16(const float* g, float* l) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)l, 16, 0, 0);
}

}  // namespace

template <bool RELU>
__global__ __launch_bounds__(256, 3) void wgrad_time_kernel(TimeWgradArgs a) {
    // element (pixel p, channel c) of a segment sits at p*64 + (c ^ 32*(p & 1)): the two lane halves of an operand
    // read (neighbouring pixels) then use different banks
    __shared__ __attribute__((aligned(16))) float X0[kTSlots * 4];
    __shared__ __attribute__((aligned(16))) float X1[kTSlots * 4];
    __shared__ __attribute__((aligned(16))) float G0[kTSlots * 4];
    __shared__ __attribute__((aligned(16))) float G1[kTSlots * 4];
    __shared__ __attribute__((aligned(16))) float G2[kTSlots * 4];
    __shared__ __attribute__((aligned(16))) float G3[kTSlots * 4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jo = wave >> 1, ji = wave & 1;
    const int m = lane & 31, h = lane >> 5;
    const int nci = a.Ci / 64;
    const int co0 = 64 * ((int)blockIdx.y / nci), ci0 = 64 * ((int)blockIdx.y % nci);
    float* const pout = a.partial + (size_t)blockIdx.x * a.Co * 3 * a.Ci;
    const XcdRange xr = xcd_range(a.n_items);
    if (xr.first >= xr.end) {   // nothing to do: the partial of this workgroup is zero
        for (int i = tid; i < 64 * 3 * 64; i += 256) {
            const int co = i / 192, kt = (i / 64) % 3, ci = i & 63;
            pout[((size_t)(co0 + co) * 3 + kt) * a.Ci + ci0 + ci] = 0.f;
        }
        if (a.bias_partial && ci0 == 0 && tid < 64) a.bias_partial[(size_t)blockIdx.x * a.Co + co0 + tid] = 0.f;
        return;
    }

    // Direct loads: slot s = tid + 256*i (16 bytes at float offset 4*s) holds channel quad (s & 15) ^ 8*(p & 1) of
    // pixel p = s >> 4.  They go through a buffer resource that spans one frame of the tensor: pixels past the end of
    // the frame arrive as zeros with the data, and a frame that does not exist gets a resource of size 0 (no bounds
    // checks, no LDS stores of zeros, which would have to wait for the direct loads in flight into the buffer).
    unsigned s_slot[2];   // pixel and channel quad of the slot
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int s = tid + 256 * i;
        s_slot[i] = (unsigned)(((s >> 4) << 4) | ((s & 15) ^ (8 * ((s >> 4) & 1))));
    }
    // frame: first element of the frame's channel block (or null), C channels per pixel, p0 first pixel of the segment
    auto fill = [&](const float* frame, long long p0, int C, float* dst) {
        const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)(frame ? frame : a.a), 0,
                                                                           frame ? (unsigned)(a.P * C * 4) : 0u, 0x00020000);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const unsigned voff = (((unsigned)p0 + (s_slot[i] >> 4)) * (unsigned)C + 4u * (s_slot[i] & 15u)) * 4u;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)(dst + (wave + 4 * i) * 256), 16, voff, 0, 0, 0);
        }
    };

    // LDS float offsets of this lane's operands at contraction step k (pixels 2k, 2k + 1): + 128*k
    const int offx = h * 64 + 32 * (ji ^ h) + m;   // input channel 32*ji + m
    const int offg = h * 64 + 32 * (jo ^ h) + m;   // output channel 32*jo + m

    floatx16 acc[3];
#pragma unroll
    for (int kt = 0; kt < 3; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[kt][r] = 0.f;
    float bsum = 0.f;

    // gp / gz / gm: gradient segments of frames tau + 1, tau, tau - 1 (taps 0, 1, 2)
    auto run = [&](const float* x, const float* gp, const float* gz, const float* gm) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kTPix / 2; ++k) {
            float xv = x[offx + 128 * k];
            if (RELU) xv = __int_as_float(__float_as_int(xv) > 0 ? __float_as_int(xv) : 0);
            const float g0 = gp[offg + 128 * k], g1 = gz[offg + 128 * k], g2 = gm[offg + 128 * k];
            bsum += g1;
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(g0, xv, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(g1, xv, acc[1], 0, 0, 0);
            acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(g2, xv, acc[2], 0, 0, 0);
        }
    };

    for (long long item = xr.first; item < xr.end; item += xr.stride) {
        const long long seg = item % a.segs, vol = item / a.segs;   // segment of the frame, sample
        const long long p0 = seg * kTPix;
        // frame 0 of this sample, at the workgroup's channel block
        const float* const ox = a.a + ((vol * a.T) * a.P) * a.Ci + ci0;
        const float* const og = a.g + ((vol * a.T) * a.P) * a.Co + co0;
        auto load_x = [&](int tau, float* dst) { fill(tau >= 0 && tau < a.T ? ox + (long long)tau * a.P * a.Ci : nullptr, p0, a.Ci, dst); };
        auto load_g = [&](int tau, float* dst) { fill(tau >= 0 && tau < a.T ? og + (long long)tau * a.P * a.Co : nullptr, p0, a.Co, dst); };
        // the previous chunk ended with a barrier: all buffers are free
        load_x(0, X0);
        load_g(1, G0);
        load_g(0, G1);
        load_g(-1, G2);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        int tau = 0;
        // chunk tau: input in xc, gradients of frames tau + 1, tau, tau - 1 in gp, gz, gm; the next chunk's input goes to
        // xn and the gradient frame tau + 2 to gn (the buffer that held frame tau - 2)
        auto chunk = [&](const float* xc, float* xn, const float* gp, const float* gz, const float* gm, float* gn)
                         __attribute__((always_inline)) {
            if (tau + 1 < a.T) {
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
            if (tau >= a.T) break;
            chunk(X1, X0, G3, G0, G1, G2);
            if (tau >= a.T) break;
            chunk(X0, X1, G2, G3, G0, G1);
            if (tau >= a.T) break;
            chunk(X1, X0, G1, G2, G3, G0);
            if (tau >= a.T) break;
        }
    }

#pragma unroll
    for (int kt = 0; kt < 3; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int co = co0 + 32 * jo + 8 * (r >> 2) + 4 * h + (r & 3), ci = ci0 + 32 * ji + m;
            pout[((size_t)co * 3 + kt) * a.Ci + ci] = acc[kt][r];
        }
    if (a.bias_partial && ci0 == 0 && ji == 0) {
        const float tot = bsum + __shfl_xor(bsum, 32);
        if (h == 0) a.bias_partial[(size_t)blockIdx.x * a.Co + co0 + 32 * jo + m] = tot;
    }
}

bool wgrad_time_applies(const PixDims& d, int Ci, int Co) {
    const double P = (double)d.D * d.H * d.W;
    // byte offsets inside a frame are 32 bits in the kernel
    return d.kt == 3 && d.kd == 1 && d.kh == 1 && d.kw == 1 && Ci % 64 == 0 && Co % 64 == 0 && (P + kTPix) * (Ci > Co ? Ci : Co) * 4.0 < 4.0e9;
}

int wgrad_time_splits(const PixDims& d) {
    const long long P = (long long)d.D * d.H * d.W;
    const long long items = d.Q / ((long long)d.T * P) * ((P + kTPix - 1) / kTPix);
    const long long cap = 768;   // three workgroups per CU
    return (int)(((items < cap ? items : cap) + 7) / 8 * 8);
}

size_t wgrad_time_partial_floats(const PixDims& d, int Ci, int Co) { return (size_t)wgrad_time_splits(d) * 3 * Ci * Co; }

hipError_t launch_wgrad_time(TimeWgradArgs a, const PixDims& d, int relu_in, hipStream_t st) {
    a.T = d.T;
    a.P = (long long)d.D * d.H * d.W;
    a.segs = (a.P + kTPix - 1) / kTPix;
    a.n_items = d.Q / ((long long)d.T * a.P) * a.segs;
    dim3 grid((unsigned)wgrad_time_splits(d), (unsigned)((a.Co / 64) * (a.Ci / 64)));
    if (relu_in) hipLaunchKernelGGL((wgrad_time_kernel<true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((wgrad_time_kernel<false>), grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------------
// Forward / data gradient of a temporal 3x1x1 layer with 64 input channels, float32:
//     out[t][p][n] = b[n] + sum over kt and k of W[n][kt][k] * in[t + kt - 1][p][k]
// Output frame t needs input frames t - 1, t, t + 1, so a workgroup walks the frames of a 64-pixel segment in order
// and every input segment is read from memory once (as three independent taps of a flattened-pixel kernel each is
// staged three times).  The weights stay in registers: wave (cb, pb) of 4 owns 32 output channels x 32 pixels and
// keeps W[32 cb + m][kt][32 h + i] for the whole kernel (96 registers: the A operands).  Contraction step i of
// v_mfma_f32_32x32x2_f32 pairs input channels i and 32 + i (any pairing is a sum over all 64), so that a lane's B
// operands of a tap are 32 consecutive floats of its pixel: eight 16-byte LDS reads.  Input segments go from memory
// to LDS by direct loads through a buffer resource that spans one frame (pixels past the frame's end arrive as
// zeros, a frame outside 0 .. T - 1 gets a resource of size 0), one frame ahead, into a ring of four buffers that are
// separate LDS objects; the walk is written out over the four rotations.  The epilogue is branch-free through buffer
// resources (a pixel past the frame's end has its stores dropped) and its mask source / add operand are requested
// before the MFMAs of the frame.
namespace {
constexpr int kCPix = 64;                 // pixels per segment
constexpr int kCRow = 68;                 // floats per pixel in LDS: 64 channels + 16 bytes (bank spread of the 16-byte reads)
constexpr int kCLoads = 17;               // wave-wide direct loads per segment: 64 pixels x 17 slots of 16 bytes
}  // namespace

template <bool RELU, bool EPI>
__global__ __launch_bounds__(256, 2) void conv_time_kernel(TimeConvArgs a) {
    __shared__ __attribute__((aligned(16))) float F0[kCLoads * 256];
    __shared__ __attribute__((aligned(16))) float F1[kCLoads * 256];
    __shared__ __attribute__((aligned(16))) float F2[kCLoads * 256];
    __shared__ __attribute__((aligned(16))) float F3[kCLoads * 256];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cb = wave & 1, pb = wave >> 1;
    const int m = lane & 31, h = lane >> 5;
    const int co0 = 64 * (int)blockIdx.y + 32 * cb;
    constexpr unsigned kOutside = 0x80000000u;
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

    float wreg[3][32];
#pragma unroll
    for (int kt = 0; kt < 3; ++kt)
#pragma unroll
        for (int i = 0; i < 32; ++i) wreg[kt][i] = a.w[(co0 + m) * a.sn + (a.flip ? 2 - kt : kt) * a.st + (32 * h + i) * a.sk];

    // direct loads: slot s = 64 (wave + 4 i) + lane holds channel quad s % 17 (16: padding) of segment pixel s / 17
    unsigned slot_off[5];
#pragma unroll
    for (int i = 0; i < 5; ++i) {
        const int s = 64 * (wave + 4 * i) + lane, px = s / 17, q = s % 17;
        slot_off[i] = q < 16 ? (unsigned)((px * 64 + 4 * q) * 4) : kOutside;
    }
    const unsigned in_frame_bytes = (unsigned)(a.P * 256);
    const unsigned out_frame_bytes = (unsigned)(a.P * a.Nn * 4);
    const int b_rd = (32 * pb + m) * kCRow + 32 * h;   // this lane's pixel and channel half
    // epilogue: accumulators 4 g .. 4 g + 3 are output channels co0 + 8 g + 4 h .. + 3 of pixel 32 pb + m
    const unsigned out_lane = (unsigned)(((32 * pb + m) * a.Nn + co0 + 4 * h) * 4);
    __shared__ __attribute__((aligned(16))) float bias_s[64];   // of the workgroup's 64 output channels
    if (tid < 64) bias_s[tid] = a.bias ? a.bias[64 * (int)blockIdx.y + tid] : 0.f;
    __syncthreads();
    const float out_floor = a.relu_out ? 0.f : -__builtin_huge_valf();

    for (long long item = blockIdx.x; item < a.n_items; item += gridDim.x) {
        const long long seg = item % a.segs, vol = item / a.segs;
        const unsigned p_off_in = (unsigned)(seg * kCPix * 256), p_off_out = (unsigned)(seg * kCPix * a.Nn * 4);
        auto load = [&](int tau, float* dst) __attribute__((always_inline)) {
            const bool ok = tau >= 0 && tau < a.T;
            const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(a.in + ((vol * a.T + (ok ? tau : 0)) * a.P) * 64), 0, ok ? in_frame_bytes : 0u, 0x00020000);
#pragma unroll
            for (int i = 0; i < 5; ++i)
                if (wave + 4 * i < kCLoads)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)(dst + (wave + 4 * i) * 256), 16,
                                                             slot_off[i] + p_off_in, 0, 0, 0);
        };
        // the previous item ended with a barrier: all buffers are free
        load(-1, F0);
        load(0, F1);
        load(1, F2);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        int t = 0;
        auto step = [&](const float* fm, const float* fz, const float* fp, float* fn) __attribute__((always_inline)) {
            if (t + 1 < a.T) load(t + 2, fn);
            const long long frame = vol * a.T + t;
            const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc((void*)(a.out + frame * a.P * a.Nn), 0, out_frame_bytes, 0x00020000);
            u32x4 refq[4], addq[4];
            if constexpr (EPI) {
                const __amdgpu_buffer_rsrc_t r_ref = __builtin_amdgcn_make_buffer_rsrc(
                    (void*)(a.mask_ref ? a.mask_ref + frame * a.P * a.Nn : a.out), 0, a.mask_ref ? out_frame_bytes : 0u, 0x00020000);
                const __amdgpu_buffer_rsrc_t r_add = __builtin_amdgcn_make_buffer_rsrc(
                    (void*)(a.add ? a.add + frame * a.P * a.Nn : a.out), 0, a.add ? out_frame_bytes : 0u, 0x00020000);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    refq[g] = __builtin_amdgcn_raw_buffer_load_b128(r_ref, out_lane + p_off_out + 32u * g, 0, 0);
                    addq[g] = __builtin_amdgcn_raw_buffer_load_b128(r_add, out_lane + p_off_out + 32u * g, 0, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            // the 32 B operands of a tap are read while the MFMAs of the tap before it run
            floatx16 acc;
            float4 vq[2][8];
            auto read_tap = [&](int kt) __attribute__((always_inline)) {
                const float* fb = (kt == 0 ? fm : kt == 1 ? fz : fp) + b_rd;
#pragma unroll
                for (int q = 0; q < 8; ++q) vq[kt & 1][q] = *reinterpret_cast<const float4*>(fb + 4 * q);
            };
            read_tap(0);
#pragma unroll
            for (int kt = 0; kt < 3; ++kt) {
                if (kt + 1 < 3) read_tap(kt + 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const float4 v4 = vq[kt & 1][q];
                    float v[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (RELU) v[e] = __int_as_float(__float_as_int(v[e]) > 0 ? __float_as_int(v[e]) : 0);
                        floatx16 c;
                        if (kt == 0 && q == 0 && e == 0) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) c[r] = 0.f;
                        } else {
                            c = acc;
                        }
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wreg[kt][4 * q + e], v[e], c, 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 b4 = *reinterpret_cast<const float4*>(bias_s + 32 * cb + 8 * g + 4 * h);
                const float bb[4] = {b4.x, b4.y, b4.z, b4.w};
                u32x4 pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float x = fmaxf(acc[4 * g + e] + bb[e], out_floor);
                    if constexpr (EPI) {
                        const bool pos = a.mask_ref ? __uint_as_float(refq[g][e]) > 0.f : true;
                        if (a.mask_acc) x = pos ? x : 0.f;
                        x += (a.mask_add && !pos) ? 0.f : __uint_as_float(addq[g][e]);
                    }
                    pk[e] = __float_as_uint(x);
                }
                __builtin_amdgcn_raw_buffer_store_b128(pk, r_out, out_lane + p_off_out + 32u * g, 0, 0);
            }
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            ++t;
        };
        while (true) {
            step(F0, F1, F2, F3);
            if (t >= a.T) break;
            step(F1, F2, F3, F0);
            if (t >= a.T) break;
            step(F2, F3, F0, F1);
            if (t >= a.T) break;
            step(F3, F0, F1, F2);
            if (t >= a.T) break;
        }
    }
}

bool conv_time_applies(const PixDims& d, int K, int Nn) {
    const long long P = (long long)d.D * d.H * d.W;
    // byte offsets inside a frame are 32 bits in the kernel (and below the offset that marks padding slots)
    return d.kt == 3 && d.kd == 1 && d.kh == 1 && d.kw == 1 && K == 64 && Nn % 64 == 0 && Nn >= 64 &&
           (double)(P + kCPix) * (Nn > 64 ? Nn : 64) * 4.0 < 2.0e9;
}

hipError_t launch_conv_time(TimeConvArgs a, const PixDims& d, hipStream_t st) {
    a.T = d.T;
    a.P = (long long)d.D * d.H * d.W;
    a.segs = (a.P + kCPix - 1) / kCPix;
    a.n_items = d.Q / ((long long)d.T * a.P) * a.segs;
    const long long cap = 512 / (a.Nn / 64) > 8 ? 512 / (a.Nn / 64) : 8;   // two workgroups per CU in total
    dim3 grid((unsigned)(a.n_items < cap ? a.n_items : cap), (unsigned)(a.Nn / 64));
    const bool epi = a.mask_ref || a.add;
    if (a.relu_in) {
        if (epi) hipLaunchKernelGGL((conv_time_kernel<true, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((conv_time_kernel<true, false>), grid, dim3(256), 0, st, a);
    } else {
        if (epi) hipLaunchKernelGGL((conv_time_kernel<false, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((conv_time_kernel<false, false>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace gleam
