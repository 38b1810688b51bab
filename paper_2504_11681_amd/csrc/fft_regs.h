// Register-resident small transforms for the fused kernels: every index and every twiddle is a
// compile-time constant, so a transform is a straight line of VALU instructions on VGPRs.
//
//  RegFFT<L, DIR>        full L-point DFT, L in {1,2,4,8,16,32}, natural order in and out
//  dft_prune_out<T,Q>    first Q outputs of a T-point DFT     (output pruning: the forward transform only
//                        feeds retained modes, Sec. 3.3 "FFT pruning")
//  dft_prune_in<T,Q>     T-point DFT of an input whose bins Q..T-1 are zero (input pruning: the inverse
//                        transform of a zero-padded spectrum, Sec. 3.3)
// DIR = -1: exp(-2 pi i k n / L) (forward);  DIR = +1: inverse, unscaled.
#pragma once
#include "common.h"
#include <type_traits>

namespace tfno {

template <int I, int E, class F>
TFNO_HD void static_for(F &&f)
{
    if constexpr (I < E) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, E>(f);
    }
}

// cos(2 pi m / 32), built from the first quadrant so that the symmetries are exact.
__host__ __device__ constexpr float cos32(int m)
{
    constexpr float q[9] = {1.0f, 9.807852804e-01f, 9.238795325e-01f, 8.314696123e-01f, 7.071067812e-01f,
                            5.555702330e-01f, 3.826834324e-01f, 1.950903220e-01f, 0.0f};
    m &= 31;
    return m <= 8 ? q[m] : m <= 16 ? -q[16 - m] : m <= 24 ? -q[m - 16] : q[32 - m];
}
__host__ __device__ constexpr float sin32(int m) { return cos32(m + 24); }

// a * exp(DIR * 2 pi i * M / L), with L | 32; trivial factors cost no multiply.
template <int L, int DIR, int M>
TFNO_HD c64 mul_tw(c64 a)
{
    constexpr int m = (((M % L) + L) % L) * (32 / L);   // index into the 32nd roots
    if constexpr (m == 0) return a;
    else if constexpr (m == 16) return make_float2(-a.x, -a.y);
    else if constexpr (m == 8) return DIR > 0 ? make_float2(-a.y, a.x) : make_float2(a.y, -a.x);
    else if constexpr (m == 24) return DIR > 0 ? make_float2(a.y, -a.x) : make_float2(-a.y, a.x);
    else {
        constexpr float c = cos32(m), s = DIR * sin32(m);
        return make_float2(fmaf(a.x, c, -(a.y * s)), fmaf(a.x, s, a.y * c));
    }
}

// acc + a * exp(DIR * 2 pi i * M / L)
template <int L, int DIR, int M>
TFNO_HD c64 mac_tw(c64 acc, c64 a)
{
    constexpr int m = (((M % L) + L) % L) * (32 / L);
    if constexpr (m == 0 || m == 8 || m == 16 || m == 24) return cadd(acc, mul_tw<L, DIR, M>(a));
    else {
        constexpr float c = cos32(m), s = DIR * sin32(m);
        float re = fmaf(a.x, c, acc.x);
        re = fmaf(-a.y, s, re);
        float im = fmaf(a.x, s, acc.y);
        im = fmaf(a.y, c, im);
        return make_float2(re, im);
    }
}

// lo = e + w o, hi = e - w o with w = exp(DIR * 2 pi i * M / L).  For a general twiddle the product is folded into
// the sum (4 FMAs) and hi = 2 e - lo (2 FMAs): 6 instructions instead of 8.
template <int L, int DIR, int M>
TFNO_HD void butterfly_tw(c64 e, c64 o, c64 &lo, c64 &hi)
{
    constexpr int m = (((M % L) + L) % L) * (32 / L);
    if constexpr (m % 8 == 0) {
        const c64 t = mul_tw<L, DIR, M>(o);
        lo = cadd(e, t);
        hi = csub(e, t);
    } else {
        constexpr float c = cos32(m), s = DIR * sin32(m);
        lo.x = fmaf(-o.y, s, fmaf(o.x, c, e.x));
        lo.y = fmaf(o.x, s, fmaf(o.y, c, e.y));
        hi.x = fmaf(2.f, e.x, -lo.x);
        hi.y = fmaf(2.f, e.y, -lo.y);
    }
}

// Recursive radix-2 decimation in time on registers.  in[i * STRIDE], i < L  ->  out[k], k < L.
template <int L, int DIR, int STRIDE = 1>
struct RegFFT {
    TFNO_HD static void run(const c64 *in, c64 *out)
    {
        c64 e[L / 2], o[L / 2];
        RegFFT<L / 2, DIR, 2 * STRIDE>::run(in, e);
        RegFFT<L / 2, DIR, 2 * STRIDE>::run(in + STRIDE, o);
        static_for<0, L / 2>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            butterfly_tw<L, DIR, k>(e[k], o[k], out[k], out[k + L / 2]);
        });
    }
};
template <int DIR, int STRIDE>
struct RegFFT<1, DIR, STRIDE> {
    TFNO_HD static void run(const c64 *in, c64 *out) { out[0] = in[0]; }
};

// First (decimation-in-frequency) level of an L-point transform: after it the input registers are dead, so a
// caller can refill them from memory while the two half-size transforms run.
//   even outputs  X[2k]   = DFT_{L/2}(a)[k],  a[i] = v[i] + v[i + L/2]
//   odd outputs   X[2k+1] = DFT_{L/2}(b)[k],  b[i] = (v[i] - v[i + L/2]) exp(DIR 2 pi i i / L)
template <int L, int DIR>
TFNO_HD void dif_first_level(const c64 *v, c64 *a, c64 *b)
{
    static_for<0, L / 2>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        a[i] = cadd(v[i], v[i + L / 2]);
        b[i] = mul_tw<L, DIR, i>(csub(v[i], v[i + L / 2]));
    });
}

// out[q] = sum_{t<T} in(t) exp(DIR 2 pi i t q / T),  q < Q,  Q | T.     in: callable int -> c64
// t = t1 + S t2 (S = T/Q):  S full Q-point transforms of the decimated input, then a twiddled S-term sum.
// The input is consumed Q values at a time, so a caller that reads it from LDS keeps only one group live.
// One group of the network: g = inputs t1, t1 + S, ..., t1 + (Q-1) S (destroyed); adds its share to out.
template <int T, int Q, int DIR, int T1>
TFNO_HD void dft_prune_out_group(c64 *g, c64 *out)
{
    c64 F[Q];
    RegFFT<Q, DIR, 1>::run(g, F);
    static_for<0, Q>([&](auto qc) {
        constexpr int q = decltype(qc)::value;
        if constexpr (T1 == 0) out[q] = F[q];
        else out[q] = mac_tw<T, DIR, T1 * q>(out[q], F[q]);
    });
}

template <int T, int Q, int DIR, class In>
TFNO_HD void dft_prune_out(In &&in, c64 *out)
{
    constexpr int S = T / Q;
    static_for<0, S>([&](auto t1c) {
        constexpr int t1 = decltype(t1c)::value;
        c64 g[Q];
        static_for<0, Q>([&](auto t2c) {
            constexpr int t2 = decltype(t2c)::value;
            g[t2] = in(std::integral_constant<int, t1 + S * t2>{});
        });
        dft_prune_out_group<T, Q, DIR, t1>(g, out);
    });
}

// emit(t, sum_{q<Q} in[q] exp(DIR 2 pi i t q / T)),  t < T.   (the transpose of the network above)
// emit: callable (integral_constant t, c64); outputs are produced Q at a time.
template <int T, int Q, int DIR, class Emit>
TFNO_HD void dft_prune_in(const c64 *in, Emit &&emit)
{
    constexpr int S = T / Q;
    static_for<0, S>([&](auto t1c) {
        constexpr int t1 = decltype(t1c)::value;
        c64 g[Q], G[Q];
        static_for<0, Q>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            g[q] = mul_tw<T, DIR, t1 * q>(in[q]);
        });
        RegFFT<Q, DIR, 1>::run(g, G);
        static_for<0, Q>([&](auto t2c) {
            constexpr int t2 = decltype(t2c)::value;
            emit(std::integral_constant<int, t1 + S * t2>{}, G[t2]);
        });
    });
}

}  // namespace tfno
