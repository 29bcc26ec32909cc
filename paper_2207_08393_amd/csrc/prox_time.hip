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
    // pixel p = s >> 4.  Lanes past the end of the frame, and every lane when the frame does not exist, store zeros
    // themselves (a direct load writes lane l's 16 bytes at the wave's base + 16*l; masked-off lanes write nothing);
    // the zero stores come before the loads, because a store into a buffer waits for loads in flight into it.
    int s_px[2];
    unsigned s_qd[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int s = tid + 256 * i;
        s_px[i] = s >> 4;
        s_qd[i] = (unsigned)((s & 15) ^ (8 * ((s >> 4) & 1)));
    }
    auto fill = [&](const float* origin, bool frame_ok, int n_px, int C, float* dst) {
        bool ok[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            ok[i] = frame_ok && s_px[i] < n_px;
            if (!ok[i]) *reinterpret_cast<float4*>(dst + (wave + 4 * i) * 256 + lane * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
            if (ok[i]) dma16(origin + (size_t)s_px[i] * C + 4 * s_qd[i], dst + (wave + 4 * i) * 256);
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
        const int n_px = a.P - p0 < kTPix ? (int)(a.P - p0) : kTPix;
        // origins of the segment in frame 0 of this sample; only ever dereferenced for frames 0 .. T-1
        const float* const ox = a.a + ((vol * a.T) * a.P + p0) * a.Ci + ci0;
        const float* const og = a.g + ((vol * a.T) * a.P + p0) * a.Co + co0;
        auto load_x = [&](int tau, float* dst) { fill(ox + (long long)tau * a.P * a.Ci, tau >= 0 && tau < a.T, n_px, a.Ci, dst); };
        auto load_g = [&](int tau, float* dst) { fill(og + (long long)tau * a.P * a.Co, tau >= 0 && tau < a.T, n_px, a.Co, dst); };
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
    return d.kt == 3 && d.kd == 1 && d.kh == 1 && d.kw == 1 && Ci % 64 == 0 && Co % 64 == 0;
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

}  // namespace gleam
