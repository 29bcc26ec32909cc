// Declarations shared by the float32 (prox.hip) and bfloat16 (prox_bf16.hip) prox kernels.
#pragma once
#include <hip/hip_runtime.h>

#include "internal.h"
#include "xcd.h"

namespace gleam {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kConvThreads = 256;
constexpr int kConvTM = 256;  // pixels per workgroup tile of the forward / data-gradient kernel

struct PixDims {
    int T, D, H, W;
    int kt, kd, kh, kw;
    long long Q;
};

// Bit `tap` is set when pixel q + off(tap) lies inside the grid (same sample, frame, slice, row).
__device__ __forceinline__ unsigned tap_validity(long long q, const PixDims& d) {
    if (q >= d.Q) return 0u;
    const int w = (int)(q % d.W);
    long long r = q / d.W;
    const int h = (int)(r % d.H);
    r /= d.H;
    const int dd = (int)(r % d.D);
    r /= d.D;
    const int t = (int)(r % d.T);
    unsigned bits = 0u;
    int tap = 0;
    for (int it = 0; it < d.kt; ++it)
        for (int id = 0; id < d.kd; ++id)
            for (int ih = 0; ih < d.kh; ++ih)
                for (int iw = 0; iw < d.kw; ++iw, ++tap) {
                    const int tt = t + it - d.kt / 2, d2 = dd + id - d.kd / 2;
                    const int hh = h + ih - d.kh / 2, ww = w + iw - d.kw / 2;
                    const bool ok = tt >= 0 && tt < d.T && d2 >= 0 && d2 < d.D && hh >= 0 && hh < d.H && ww >= 0 && ww < d.W;
                    bits |= (ok ? 1u : 0u) << tap;
                }
    return bits;
}

// The same bits for a pixel tracked by its coordinates, for kernels that walk the pixel index in equal
// steps and cannot afford the divisions of tap_validity per step.
struct PixCoord {
    int w, h, dd, t;
};
__device__ __forceinline__ PixCoord pix_coord(long long q, const PixDims& d) {
    PixCoord c;
    c.w = (int)(q % d.W);
    long long r = q / d.W;
    c.h = (int)(r % d.H);
    r /= d.H;
    c.dd = (int)(r % d.D);
    r /= d.D;
    c.t = (int)(r % d.T);
    return c;
}
// c += step, where step holds the coordinates of the step length (pix_coord(step_pixels)).
__device__ __forceinline__ void pix_advance(PixCoord& c, const PixCoord& step, const PixDims& d) {
    c.w += step.w;
    int carry = c.w >= d.W ? 1 : 0;
    c.w -= carry ? d.W : 0;
    c.h += step.h + carry;
    carry = c.h >= d.H ? 1 : 0;
    c.h -= carry ? d.H : 0;
    c.dd += step.dd + carry;
    carry = c.dd >= d.D ? 1 : 0;
    c.dd -= carry ? d.D : 0;
    c.t += step.t + carry;
    c.t -= c.t >= d.T ? d.T : 0;
}
__device__ __forceinline__ unsigned tap_validity_at(const PixCoord& c, const PixDims& d) {
    unsigned bits = 0u;
    int tap = 0;
    for (int it = 0; it < d.kt; ++it)
        for (int id = 0; id < d.kd; ++id)
            for (int ih = 0; ih < d.kh; ++ih)
                for (int iw = 0; iw < d.kw; ++iw, ++tap) {
                    const int tt = c.t + it - d.kt / 2, d2 = c.dd + id - d.kd / 2;
                    const int hh = c.h + ih - d.kh / 2, ww = c.w + iw - d.kw / 2;
                    const bool ok = (unsigned)tt < (unsigned)d.T && (unsigned)d2 < (unsigned)d.D && (unsigned)hh < (unsigned)d.H &&
                                    (unsigned)ww < (unsigned)d.W;
                    bits |= (ok ? 1u : 0u) << tap;
                }
    return bits;
}

// Flattened pixel offset of row-tap rt = (it, id, ih), before the kw taps along W.
__device__ __forceinline__ long long rowtap_offset(int rt, const PixDims& d) {
    const int ih = rt % d.kh, id = (rt / d.kh) % d.kd, it = rt / (d.kh * d.kd);
    return (((long long)(it - d.kt / 2) * d.D + (id - d.kd / 2)) * d.H + (ih - d.kh / 2)) * d.W;
}


// ------------------------------------------------------------------ bfloat16 helpers
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ unsigned short f32_to_bf16(float f) {   // round to nearest even
    unsigned u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(unsigned short h) { return __uint_as_float((unsigned)h << 16); }
// two values at once: gfx950's packed conversion (v_cvt_pk_bf16_f32, round to nearest even like f32_to_bf16)
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    const float2v f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2v));
}
// max(x, 0) on two packed bf16 values: a negative bf16 has the sign bit of its 16-bit pattern set, so a
// packed signed 16-bit max with 0 is ReLU (one instruction)
typedef short short2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned relu_bf16x2(unsigned x) {
    const short2v zero = {0, 0};
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(short2v, x), zero));
}

// Walks the chunks of one pixel tile in order (row tap major, input-channel chunk minor) and keeps the
// flattened pixel offset of the row tap, without divisions.
struct ChunkIter {
    int c, rt, kc, ih, id, it;
    long long off;   // rowtap_offset(rt)
};
__device__ __forceinline__ ChunkIter chunk_first(const PixDims& d) {
    ChunkIter x;
    x.c = x.rt = x.kc = x.ih = x.id = x.it = 0;
    x.off = (((long long)(0 - d.kt / 2) * d.D + (0 - d.kd / 2)) * d.H + (0 - d.kh / 2)) * d.W;
    return x;
}
__device__ __forceinline__ ChunkIter chunk_next(ChunkIter x, int n_kc, int nck, const PixDims& d) {
    if (x.c + 1 == nck) return chunk_first(d);
    ++x.c;
    if (++x.kc == n_kc) {
        x.kc = 0;
        ++x.rt;
        x.off += d.W;                                        // next row
        if (++x.ih == d.kh) {
            x.ih = 0;
            x.off += (long long)(d.H - d.kh) * d.W;           // next slice, first row tap
            if (++x.id == d.kd) {
                x.id = 0;
                x.off += (long long)(d.D - d.kd) * d.H * d.W;   // next frame, first slice tap
                ++x.it;
            }
        }
    }
    return x;
}

// Launch arguments of the bf16 MFMA convolution (forward and data gradient): in/out/mask_ref/add are
// bfloat16 [Q][channels] unless out_f32 (then out and add are float32).  wt: bf16 LDS images.
// Winograd F(2x2, 3x3) convolution, float32 (prox_wino.hip).  Same fused epilogue as the direct kernels.
struct WinoArgs {
    const float* in;        // [NI][H][W][K]
    float* out;             // [NI][H][W][Nn]
    const float* u;         // transformed weights (set by the launcher)
    const float* zero;      // one quad of zeros in global memory (set by the launcher)
    const float* bias;      // [Nn] or null
    const float* mask_ref;  // [Q][Nn] or null: ReLU mask source (value > 0 passes)
    const float* add;       // [Q][Nn] or null
    const unsigned* bits_in;   // or null: sign words of the mask source written by an earlier launch (replace mask_ref)
    unsigned* bits_out;        // or null: sign words of this launch's output, conv_wino_sign_words() of them
    int K, Nn, relu_out, mask_acc, mask_add;
    long long NI;           // images (B*T*D)
    int H, W, bx_n, by_n;
    long long n_blocks;
    int D;                  // slices per volume (3x3x3 kernel only)
};
bool conv_wino_applies(const PixDims& d, int K, int Nn);
size_t conv_wino_weight_floats(int K, int Nn);
// 32-bit words of the sign-bit image of a [pixels][Nn] tensor as the Winograd kernel's threads write and read it
size_t conv_wino_sign_words(const PixDims& d, int Nn);
// u_ready: transformed weights made earlier by wino_weights_batch (then w and the strides are not used);
// otherwise they are made now, into u_scratch.
hipError_t launch_conv_wino(WinoArgs a, const float* w, long long sn, long long st, long long sk, int flip, int relu_in,
                            float* u_scratch, const float* u_ready, const char* name, hipStream_t stream);
// 3x3x3 layers: Winograd inside every slice, plain sum over the three depth taps (prox_wino3.hip).  The transformed
// weights (conv_wino3_weight_floats(K, Nn) floats) are made at launch into u_scratch.
bool conv_wino3_applies(const PixDims& d, int K, int Nn);
size_t conv_wino3_weight_floats(int K, int Nn);
hipError_t launch_conv_wino3(WinoArgs a, const float* w, long long sn, long long st, long long sk, int flip, int relu_in,
                             float* u_scratch, const char* name, hipStream_t stream);
// Weight gradient of a 3x3x3 layer by the same scheme (prox_wino3.hip): partial sums of the 3 x 16 transformed products
// per workgroup, then reduce_partials_kernel and wgrad_wino3_finish.
struct Wino3WgradArgs {
    const float* g;         // [volumes][D][H][W][Co]  gradient at the conv output (already ReLU-masked)
    const float* a;         // [volumes][D][H][W][Ci]  conv input before its optional ReLU
    float* partial;         // [gridDim.x][3][16][Co][Ci], followed by [3][16][Co][Ci] for the reduced sums
    float* bias_partial;    // [gridDim.x][Co] or null
    int Co, Ci;
    int D, H, W, bx_n, by_n;            // set by the launcher
    int seg_len, segs_per_col;          // slices per run, runs per column
    long long n_items;                  // runs in total
};
bool wgrad_wino3_applies(const PixDims& d, int Ci, int Co);
int wgrad_wino3_splits(const PixDims& d);                                  // workgroups along x = partial sums written
size_t wgrad_wino3_partial_floats(const PixDims& d, int Ci, int Co);      // partials and reduced sums
hipError_t launch_wgrad_wino3(Wino3WgradArgs a, const PixDims& d, int relu_in, hipStream_t stream);
hipError_t wgrad_wino3_finish(const float* psum, int Co, int Ci, float* grad_w, hipStream_t stream);
// Weight gradient of a temporal 3x1x1 layer by a walk along the frames (prox_time.hip): partial sums
// [gridDim.x][Co][3][Ci] for reduce_partials_kernel.
struct TimeWgradArgs {
    const float* g;         // [samples][T][P][Co]  gradient at the conv output (already ReLU-masked)
    const float* a;         // [samples][T][P][Ci]  conv input before its optional ReLU
    float* partial;
    float* bias_partial;    // [gridDim.x][Co] or null
    int Co, Ci;
    int T;                  // set by the launcher: frames, pixels per frame, segments per frame, segments in total
    long long P, segs, n_items;
};
bool wgrad_time_applies(const PixDims& d, int Ci, int Co);
int wgrad_time_splits(const PixDims& d);
size_t wgrad_time_partial_floats(const PixDims& d, int Ci, int Co);
hipError_t launch_wgrad_time(TimeWgradArgs a, const PixDims& d, int relu_in, hipStream_t stream);
// Forward / data gradient of a temporal 3x1x1 layer with 64 input channels by a walk along the frames (prox_time.hip).
struct TimeConvArgs {
    const float* in;        // [samples][T][P][64]
    float* out;             // [samples][T][P][Nn]
    const float* bias;      // [Nn] or null
    const float* mask_ref;  // [..][Nn] or null: ReLU mask source (value > 0 passes)
    const float* add;       // [..][Nn] or null
    const float* w;         // element (output n, tap t, input k) at w[n*sn + t*st + k*sk]; flip: taps mirrored
    long long sn, st, sk;
    int flip, Nn, relu_in, relu_out, mask_acc, mask_add;
    int T;                  // set by the launcher: frames, pixels per frame, 64-pixel segments per frame, segments in total
    long long P, segs, n_items;
};
bool conv_time_applies(const PixDims& d, int K, int Nn);
hipError_t launch_conv_time(TimeConvArgs a, const PixDims& d, hipStream_t stream);
// Transformed weights of several layers in one launch (a launch costs more than the transform of one layer).
struct WinoWeightJob {
    const float* w;
    long long sn, st, sk;
    int flip, K, Nn;
    float* u;          // conv_wino_weight_floats(K, Nn) floats
};
struct WinoWeightBatch {
    int n;
    WinoWeightJob job[kMaxLayers];
};
hipError_t wino_weights_batch(const WinoWeightBatch& b, hipStream_t stream);

// Winograd weight gradient of a 3x3 layer, float32 (prox_wino.hip): partial sums of the 16 transformed
// products per workgroup, then a fixed-order reduction and the back-transform to the nine taps.
struct WinoWgradArgs {
    const float* g;         // [NI][H][W][Co]  gradient at the conv output (already ReLU-masked)
    const float* a;         // [NI][H][W][Ci]  conv input before its optional ReLU
    float* partial;         // [gridDim.x][16][Co][Ci], followed by [16][Co][Ci] for the reduced sums
    float* bias_partial;    // [gridDim.x][Co] or null
    int Co, Ci;
    long long NI;
    int H, W, bx_n, by_n;
    long long n_chunks;
};
bool wgrad_wino_applies(const PixDims& d, int Ci, int Co);
size_t wgrad_wino_partial_floats(int Ci, int Co, int n_split);   // partials and reduced sums
// Runs the kernel with n_split workgroups; the partials then need wgrad_wino_finish.
hipError_t launch_wgrad_wino(WinoWgradArgs a, int relu_in, int n_split, hipStream_t stream);
// grad_w[co][tap][ci] = G^T (sum of partials) G  (call after the partials have been reduced into
// partial + n_split*16*Co*Ci by reduce_partials_kernel)
hipError_t wgrad_wino_finish(const float* psum, int Co, int Ci, float* grad_w, hipStream_t stream);

// Two-channel-output 3x3 layer on the matrix cores (prox_thin.hip); wts is [2][9][K] float32, in is bfloat16 when bf.
bool conv_thin_out_mfma_applies(const PixDims& d, int K, bool bf);
hipError_t launch_conv_thin_out_mfma(const void* in, const float* wts, const float* bias, const float* add, float* out, int K,
                                     int relu_in, int relu_out, const PixDims& d, bool bf, hipStream_t stream);

// Two-channel-input 3x3x3 layer on the matrix cores (prox_thin.hip).  out, mask_ref and add are bfloat16 when
// the launch says so; the 2-channel input and the weights are float32; weight (n, tap, e) at w[n*sn + tapidx*st + e*sk],
// taps mirrored when flip.
struct ThinInMfmaArgs {
    const float* in;        // [Q][2]
    void* out;              // [Q][Nn]
    const float* bias;      // [Nn] or null
    const void* mask_ref;   // [Q][Nn] or null: ReLU mask source (value > 0 passes)
    const void* add;        // [Q][Nn] or null
    const float* w;
    long long sn, st, sk;
    int Nn, flip, relu_in, relu_out, mask_acc, mask_add;
    PixDims d;
};
bool conv_thin_in_mfma_applies(const PixDims& d, int Nn);

// Weight gradient of a layer with the 2-channel image on one side, 3x3 or 3x3x3 taps, on the matrix cores (prox_thin.hip)
struct WgradThinWalkArgs {
    const void* wide;      // [Q][WC] float32 or bfloat16 (bf)
    const float* thin;     // [Q][2]
    float* partial;        // [workgroups][Co][taps][Ci]
    float* bias_partial;   // [workgroups][Co] or null
    int WC, relu_in, thin_in, bf;   // thin_in: the layer's input is the thin side (wide = output gradient)
    PixDims d;
};
constexpr int kThinWalkSplit = 1024;   // most partial blocks the kernel writes
bool wgrad_thin_walk_applies(const PixDims& d, int WC, bool bf);
hipError_t launch_wgrad_thin_walk(const WgradThinWalkArgs& a, size_t partial_floats, int* used_split, hipStream_t stream);
hipError_t launch_conv_thin_in_mfma(const ThinInMfmaArgs& a, bool bf, hipStream_t stream);

struct ConvBf16Args {
    const unsigned short* in;
    void* out;
    const unsigned short* wt;
    const float* bias;
    const unsigned short* mask_ref;
    const void* add;
    const unsigned* bits_in;   // or null: sign words of the mask source written by an earlier launch (replace mask_ref)
    unsigned* bits_out;        // or null: sign words of this launch's output, conv_bf16_sign_words() of them
    int K, Nn;
    int out_f32;
    int relu_in, relu_out, mask_acc, mask_add;
    PixDims d;
};
// Whether a (K -> Nn) layer with bfloat16 output runs on the two-dimensional-tile kernel, whose launches can leave
// and take ReLU masks as sign words, and how many 32-bit words those are for a [pixels][Nn] tensor.
// 0: neither; 1: the two-dimensional-tile kernel; 2: the kernel with register-resident weights.
int conv_bf16_takes_sign_words(const PixDims& d, int K, int Nn);
size_t conv_bf16_sign_words(const PixDims& d, int Nn, int variant);
hipError_t launch_conv_bf16(const ConvBf16Args& a, const float* w, long long sn, long long st, long long sk, int flip,
                            unsigned short* wt_scratch, hipStream_t stream);
size_t conv_bf16_wimg_elems(int K, int Nn, int taps);

// Weight gradient with bf16 operands: g [Q][Co], a [Q][Ci] bfloat16; partial sums float32.
struct WgradBf16Args {
    const unsigned short* g;
    const unsigned short* a;
    float* partial;        // [gridDim.x][Co][taps][Ci]
    float* bias_partial;   // [gridDim.x][Co] or null
    int Co, Ci, relu_in;
    int two_buf;           // set by the launcher: LDS holds two staging buffers
    PixDims d;
};
hipError_t launch_wgrad_bf16(const WgradBf16Args& a, int n_split, hipStream_t stream);
size_t wgrad_bf16_lds_bytes(int Co, int Ci, int kt, int kd, int kh, int kw);
// 3x3 layers with 128 input channels: walk down strips of 64 columns (prox_bf16w.hip); writes
// wgrad_bf16_walk_splits partial blocks (two_buf is not used)
bool wgrad_bf16_walk_applies(const PixDims& d, int Ci, int Co);
int wgrad_bf16_walk_splits(const PixDims& d, int Co);
size_t wgrad_bf16_walk_partial_floats(const PixDims& d, int Ci, int Co);
hipError_t launch_wgrad_bf16_walk(const WgradBf16Args& a, hipStream_t stream);

}  // namespace gleam
