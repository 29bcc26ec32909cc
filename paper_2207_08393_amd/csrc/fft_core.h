// In-LDS mixed-radix Stockham FFT building blocks for gfx950 (wave64).
//
// A transform of length N is a product of radices chosen at compile time (see next_radix: e.g. 368 = 23 * 4 * 4,
// 320 = 20 * 4 * 4, 640 = 20 * 4 * 4 * 2, 46 = 2 * 23).  Each stage reads R points at stride
// N/R from the LDS buffer, applies the stage twiddles and an R-point DFT held in registers, and
// writes them back autosorted (in place, with a barrier between the reads and the writes), so the
// result comes out in natural order with no bit-reversal pass.  Transforms are unnormalised here; callers scale at their global store.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

namespace gleam {

// ------------------------------------------------------------------ compile-time trigonometry
constexpr double kPi = 3.14159265358979323846264338327950288;

constexpr double ct_sin_small(double x) {  // |x| <= pi
    double term = x, sum = x, x2 = x * x;
    for (int n = 1; n < 16; ++n) {
        term *= -x2 / ((2 * n) * (2 * n + 1));
        sum += term;
    }
    return sum;
}
constexpr double ct_cos_small(double x) {
    double term = 1.0, sum = 1.0, x2 = x * x;
    for (int n = 1; n < 16; ++n) {
        term *= -x2 / ((2 * n - 1) * (2 * n));
        sum += term;
    }
    return sum;
}
// cos / sin of 2*pi*m/R for integers, reduced to [-pi, pi] first.
constexpr double ct_cos_frac(int m, int R) {
    m %= R;
    if (2 * m > R) m -= R;
    return ct_cos_small(2.0 * kPi * m / R);
}
constexpr double ct_sin_frac(int m, int R) {
    m %= R;
    if (2 * m > R) m -= R;
    return ct_sin_small(2.0 * kPi * m / R);
}

template <int I> using ic = std::integral_constant<int, I>;
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(ic<Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// ------------------------------------------------------------------ complex helpers
__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float2 cmul_conj(float2 a, float2 b) {  // a * conj(b)
    return make_float2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}
// multiply by -i (forward) or +i (inverse)
template <bool INV> __device__ __forceinline__ float2 mul_mi(float2 a) {
    return INV ? make_float2(-a.y, a.x) : make_float2(a.y, -a.x);
}

// ------------------------------------------------------------------ small DFTs in registers
template <bool INV> __device__ __forceinline__ void dft2(float2& a, float2& b) {
    float2 t = csub(a, b);
    a = cadd(a, b);
    b = t;
}

template <bool INV> __device__ __forceinline__ void dft4(float2& b0, float2& b1, float2& b2, float2& b3) {
    float2 s02 = cadd(b0, b2), d02 = csub(b0, b2);
    float2 s13 = cadd(b1, b3), d13 = mul_mi<INV>(csub(b1, b3));
    b0 = cadd(s02, s13);
    b2 = csub(s02, s13);
    b1 = cadd(d02, d13);
    b3 = csub(d02, d13);
}

template <bool INV> __device__ __forceinline__ void dft8(float2 (&u)[8]) {
    constexpr float h = 0.70710678118654752440f;
    float2 a0 = cadd(u[0], u[4]), a4 = csub(u[0], u[4]);
    float2 a1 = cadd(u[1], u[5]), a5 = csub(u[1], u[5]);
    float2 a2 = cadd(u[2], u[6]), a6 = csub(u[2], u[6]);
    float2 a3 = cadd(u[3], u[7]), a7 = csub(u[3], u[7]);
    // a5 *= w8, a6 *= w8^2, a7 *= w8^3 with w8 = exp(-+ i pi/4)
    a5 = INV ? make_float2(h * (a5.x - a5.y), h * (a5.x + a5.y)) : make_float2(h * (a5.x + a5.y), h * (a5.y - a5.x));
    a6 = mul_mi<INV>(a6);
    a7 = INV ? make_float2(-h * (a7.x + a7.y), h * (a7.x - a7.y)) : make_float2(h * (a7.y - a7.x), -h * (a7.x + a7.y));
    dft4<INV>(a0, a1, a2, a3);
    dft4<INV>(a4, a5, a6, a7);
    u[0] = a0; u[2] = a1; u[4] = a2; u[6] = a3;
    u[1] = a4; u[3] = a5; u[5] = a6; u[7] = a7;
}

// Odd prime length R by conjugate-pair folding: with a_r = u_r + u_{R-r}, b_r = u_r - u_{R-r},
//   X_q     = u_0 + sum_r cos(2 pi q r / R) a_r  -+ i sum_r sin(2 pi q r / R) b_r
//   X_{R-q} = the same with the opposite sign of the second sum,
// which halves the multiplications of the direct R x R product; all constants are literals.
template <int R, bool INV> __device__ __forceinline__ void dft_odd(float2 (&u)[R]) {
    constexpr int Hn = (R - 1) / 2;
    float2 a[Hn], b[Hn];
#pragma unroll
    for (int r = 1; r <= Hn; ++r) {
        a[r - 1] = cadd(u[r], u[R - r]);
        b[r - 1] = csub(u[r], u[R - r]);
    }
    const float2 u0 = u[0];
    float2 s = u0;
#pragma unroll
    for (int r = 0; r < Hn; ++r) s = cadd(s, a[r]);
    u[0] = s;
    static_for<Hn>([&](auto qi) {
        constexpr int q = decltype(qi)::value + 1;
        float2 A = u0, Bv = make_float2(0.f, 0.f);
        static_for<Hn>([&](auto ri) {
            constexpr int r = decltype(ri)::value + 1;
            constexpr float c = (float)ct_cos_frac(q * r, R);
            constexpr float sn = (float)ct_sin_frac(q * r, R);
            A.x = fmaf(c, a[r - 1].x, A.x);
            A.y = fmaf(c, a[r - 1].y, A.y);
            Bv.x = fmaf(sn, b[r - 1].x, Bv.x);
            Bv.y = fmaf(sn, b[r - 1].y, Bv.y);
        });
        // forward: X_q = A - i Bv ; inverse: X_q = A + i Bv
        const float2 lo = make_float2(A.x + Bv.y, A.y - Bv.x), hi = make_float2(A.x - Bv.y, A.y + Bv.x);
        u[q] = INV ? hi : lo;
        u[R - q] = INV ? lo : hi;
    });
}

// First factor of an in-register DFT of length R: R itself for the base cases (2, 4, 8, odd primes).
constexpr int first_factor(int R) {
    if (R == 2 || R == 4 || R == 8) return R;
    if (R % 8 == 0) return 8;
    if (R % 4 == 0) return 4;
    if (R % 2 == 0) return 2;
    for (int p = 3; p * p <= R; p += 2)
        if (R % p == 0) return p;
    return R;
}

// DFT of any small length held in registers.  Composite R = R1*R2 is one Cooley-Tukey step with
// literal twiddles: X[q1 + R1*q2] = sum_r2 w_R2^(r2 q2) * w_R^(r2 q1) * (sum_r1 w_R1^(r1 q1) u[r1*R2 + r2]).
template <int R, bool INV> __device__ __forceinline__ void dft_r(float2 (&u)[R]) {
    constexpr int R1 = first_factor(R);
    if constexpr (R == 1) {
    } else if constexpr (R1 == R) {
        if constexpr (R == 2) dft2<INV>(u[0], u[1]);
        else if constexpr (R == 4) dft4<INV>(u[0], u[1], u[2], u[3]);
        else if constexpr (R == 8) dft8<INV>(u);
        else dft_odd<R, INV>(u);
    } else {
        constexpr int R2 = R / R1;
        float2 y[R];
        static_for<R2>([&](auto r2c) {
            constexpr int r2 = decltype(r2c)::value;
            float2 v[R1];
            static_for<R1>([&](auto r1c) { v[decltype(r1c)::value] = u[decltype(r1c)::value * R2 + r2]; });
            dft_r<R1, INV>(v);
            static_for<R1>([&](auto q1c) {
                constexpr int q1 = decltype(q1c)::value;
                if constexpr (q1 * r2 == 0) {
                    y[q1 * R2 + r2] = v[q1];
                } else {
                    constexpr float c = (float)ct_cos_frac(q1 * r2, R);
                    constexpr float sn = (float)ct_sin_frac(q1 * r2, R);   // forward twiddle = c - i sn
                    const float2 w = make_float2(c, INV ? sn : -sn);
                    y[q1 * R2 + r2] = cmul(v[q1], w);
                }
            });
        });
        static_for<R1>([&](auto q1c) {
            constexpr int q1 = decltype(q1c)::value;
            float2 v[R2];
            static_for<R2>([&](auto r2c) { v[decltype(r2c)::value] = y[q1 * R2 + decltype(r2c)::value]; });
            dft_r<R2, INV>(v);
            static_for<R2>([&](auto q2c) { u[q1 + R1 * decltype(q2c)::value] = v[decltype(q2c)::value]; });
        });
    }
}

// ------------------------------------------------------------------ radix plan
// Radix of the stage that follows a partial product P (P divides N), for one of two plans.
// PLAN 0: whatever is left once it fits in registers (<= 24 points), otherwise the largest power of two up to 16,
//         otherwise a small prime (368 = 16.23, 320 = 16.20, 640 = 16.8.5, 160 = 16.10): few stages, few barriers.
// PLAN 1: one large in-register DFT first - it needs no stage twiddles - then radix-4 stages (640 = 20.4.4.2,
//         368 = 23.4.4, 320 = 20.4.4, 192 = 12.4.4, 160 = 10.4.4), which with the right number of lines per tile gives
//         every stage a whole multiple of 256 butterflies, so that the four waves of a 256-thread workgroup carry the
//         same load in every stage; lengths without such a split fall back to plan 0.
// Which plan a sweep uses is part of its tile configuration (sense.hip), chosen by measurement.
constexpr int plan1_first_radix(int N) {
    switch (N) {
        case 640: return 20;
        case 368: return 23;
        case 320: return 20;
        case 192: return 12;
        case 160: return 10;
        default: return 0;
    }
}
constexpr int next_radix(int N, int P, int PLAN = 0) {
    int m = N / P;
    if (PLAN == 1 && plan1_first_radix(N) != 0) {
        if (P == 1) return plan1_first_radix(N);
        return m % 4 == 0 ? 4 : m;
    }
    if (m <= 24) return m;
    if (m % 16 == 0) return 16;
    if (m % 8 == 0) return 8;
    if (m % 4 == 0) return 4;
    if (m % 2 == 0) return 2;
    for (int r = 3; r <= m; r += 2)
        if (m % r == 0) return r;
    return 1;
}

// LDS layout of a tile of L lines: position-major, element p of line l at p*(L + PAD) + l, and threads
// walk l fastest.  With L a multiple of 16 every butterfly access of a wave covers whole 128-byte rows,
// so the stages are bank-conflict free.  PAD = 1 lets a kernel whose GLOBAL rows run along p (threads
// walking p fastest while loading and storing) transpose into this layout without conflicts either.
template <int N, int L, int PAD> struct Layout {
    static constexpr int kStride = L + PAD;
    static constexpr int kElems = N * kStride;
    __device__ static __forceinline__ int at(int line, int p) { return p * kStride + line; }
};

// One Stockham stage over L lines held in one LDS buffer, in place: every thread first pulls the
// inputs of all its butterflies into registers, the workgroup synchronises, then results are written
// back autosorted.  Ends with a barrier, so the buffer is ready for the next stage or for readers.
template <int N, int L, int PAD, bool INV, int P, int NT, int PLAN>
__device__ __forceinline__ void fft_stage(float2* __restrict__ buf, const float2* __restrict__ tw) {
    constexpr int R = next_radix(N, P, PLAN);
    constexpr int T = N / R;
    constexpr int PER = (L * T + NT - 1) / NT;
    using Lay = Layout<N, L, PAD>;
    float2 u[PER][R];
#pragma unroll
    for (int m = 0; m < PER; ++m) {
        const int idx = threadIdx.x + m * NT;
        if (PER * NT == L * T || idx < L * T) {
            const int line = idx % L, i = idx / L;
#pragma unroll
            for (int r = 0; r < R; ++r) u[m][r] = buf[Lay::at(line, i + r * T)];
        }
    }
    __syncthreads();
#pragma unroll
    for (int m = 0; m < PER; ++m) {
        const int idx = threadIdx.x + m * NT;
        if (PER * NT == L * T || idx < L * T) {
            const int line = idx % L, i = idx / L;
            const int k = i % P;
            if constexpr (P > 1) {
                constexpr int step = N / (P * R);
#pragma unroll
                for (int r = 1; r < R; ++r) {
                    const float2 w = tw[r * k * step];
                    u[m][r] = INV ? cmul_conj(u[m][r], w) : cmul(u[m][r], w);
                }
            }
            dft_r<R, INV>(u[m]);
            const int j = (i - k) * R + k;
#pragma unroll
            for (int r = 0; r < R; ++r) buf[Lay::at(line, j + r * P)] = u[m][r];
        }
    }
    __syncthreads();
}

// All stages, in place.  The caller synchronises after filling `buf`; the result is visible to the
// whole workgroup on return.
template <int N, int L, int PAD, bool INV, int NT, int PLAN = 0, int P = 1>
__device__ __forceinline__ void fft_lines(float2* buf, const float2* tw) {
    if constexpr (P < N) {
        fft_stage<N, L, PAD, INV, P, NT, PLAN>(buf, tw);
        fft_lines<N, L, PAD, INV, NT, PLAN, P * next_radix(N, P, PLAN)>(buf, tw);
    }
}

// Forward twiddles w[k] = exp(-2 pi i k / N), k < N, evaluated in double.
template <int N, int NT> __device__ __forceinline__ void fill_twiddles(float2* tw) {
    for (int k = threadIdx.x; k < N; k += NT) {
        double s, c;
        sincospi(-2.0 * (double)k / (double)N, &s, &c);
        tw[k] = make_float2((float)c, (float)s);
    }
}

}  // namespace gleam
