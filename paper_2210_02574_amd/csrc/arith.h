// Device arithmetic on residues of primes below 2^60 (gfx950).
//
// Two forms are used.  Integer: 64-bit values built from 32-bit multiplies -- Shoup products for
// multiplications by table constants (w, floor(w 2^64 / q)), 128-bit accumulation with one final
// reduction for sums of products of two variable residues.  Floating point, for primes below
// 2^50: a residue is a double holding an exact integer and a modular product is the error-free
// sequence h = y*w, l = fma(y,w,-h), c = rint(h/q), r = fma(-c,q,h) + l; on this GPU FP64 FMA
// issues at the rate of 32-bit integer ops, so this is a quarter of the instructions of the
// integer form.  Both give exact results; only canonical residues are ever stored to buffers
// that leave the library.
#pragma once
#include <hip/hip_runtime.h>

#include "he_internal.h"

__device__ __forceinline__ u64 mulhi64(u64 a, u64 b) { return __umul64hi(a, b); }
__device__ __forceinline__ u64 csub(u64 x, u64 q) { return x >= q ? x - q : x; }
// w*x mod q up to one extra q, for any 64-bit x; w < q with wp = floor(w 2^64 / q)
__device__ __forceinline__ u64 mul_shoup_lazy(u64 x, ShoupConst w, u64 q) { return x * w.w - mulhi64(x, w.wp) * q; }
__device__ __forceinline__ u64 mul_shoup(u64 x, ShoupConst w, u64 q) { return csub(mul_shoup_lazy(x, w, q), q); }
// The same product with a cheaper quotient: of the four 32-bit partial products of x * wp only the high one and
// the high halves of the two middle ones are kept, so the estimate is at most three below floor(x wp / 2^64)
// and the result lies in [0, 4q) for any 64-bit x (exact arithmetic modulo 2^64, since 4q < 2^64).
__device__ __forceinline__ u64 mul_shoup_sloppy(u64 x, ShoupConst w, u64 q)
{
    const unsigned xl = (unsigned)x, xh = (unsigned)(x >> 32);
    const unsigned pl = (unsigned)w.wp, ph = (unsigned)(w.wp >> 32);
    u64 quo = (u64)xh * ph;
    quo += __umulhi(xh, pl);
    quo += __umulhi(xl, ph);
    return x * w.w - quo * q;
}

struct U128 {
    u64 lo, hi;
};
__device__ __forceinline__ void mac128(U128 &acc, u64 a, u64 b)
{
    const u64 lo = a * b;
    const u64 hi = mulhi64(a, b);
    acc.lo += lo;
    acc.hi += hi + (acc.lo < lo ? 1 : 0);
}
// (hi 2^64 + lo) mod q for any 128-bit value
__device__ __forceinline__ u64 reduce128(U128 v, const ModConst &m)
{
    const u64 a = mul_shoup_lazy(v.hi, m.r, m.q);      // hi * (2^64 mod q)   in [0, 2q)
    const u64 b = v.lo - mulhi64(v.lo, m.one_p) * m.q; // lo mod q            in [0, 2q)
    return csub(csub(a + b, 2 * m.q), m.q);
}
__device__ __forceinline__ u64 reduce64(u64 v, const ModConst &m) { return csub(v - mulhi64(v, m.one_p) * m.q, m.q); }
__device__ __forceinline__ u64 mul_mod(u64 a, u64 b, const ModConst &m)
{
    U128 p{a * b, mulhi64(a, b)};
    return reduce128(p, m);
}

// exact conversions between integers below 2^52 and doubles (mantissa tricks, two instructions)
__device__ __forceinline__ double u2d(u64 v) { return __longlong_as_double(v | 0x4330000000000000ull) - 4503599627370496.0; }
__device__ __forceinline__ u64 d2u(double v)
{
    return (u64)__double_as_longlong(v + 4503599627370496.0) & 0x000FFFFFFFFFFFFFull;
}

// error-free modular product of two exact-integer doubles, |y w / q| < 2^52: the result lies
// within about (1/2 + 3|y|/(16 q)) q of zero
__device__ __forceinline__ double fp_mulmod(double y, double w, double q, double qinv)
{
    const double h = y * w;
    const double l = __builtin_fma(y, w, -h);
    const double c = __builtin_rint(h * qinv);
    return __builtin_fma(-c, q, h) + l;
}
// v - rint(v/q) q: |result| <= q/2 (+1)
__device__ __forceinline__ double fp_reduce(double v, double q, double qinv)
{
    return __builtin_fma(-__builtin_rint(v * qinv), q, v);
}
// canonical residue of a double with |v| < 2^52 q-multiples away
__device__ __forceinline__ u64 fp_canon(double v, double q, double qinv)
{
    const double r = fp_reduce(v, q, qinv);
    return d2u(r < 0.0 ? r + q : r);
}

// ---- arithmetic policies for the NTT kernels ---------------------------------------------------------
//
// V is the in-register form.  load/store_final convert from/to canonical residues; load_mid and
// store_mid are the form kept in LDS and between the two kernels of one transform.  fwd16 runs four
// forward stages s_base..s_base+3 on the 16 elements of a thread (G = index of the thread's group
// at stage s_base; twiddle index 2^s + (G << (s - s_base)) + group within the 16); inv16 runs the
// same stages backwards, and with LAST also folds the factors n0 = 1/N (times an optional extra
// constant) and n1 = n0 * twiddle into stage 0.
//
// ArithFp ranges: values are signed; a forward phase entered with |v| <= 1q (canonical input) or
// after reduce_first (|v| <= q/2) ends below 4.7q; an inverse phase reduces the sum path at its
// second and fourth stage and never exceeds 7.4q.  Everything stays below 8q < 2^53.

struct ArithFp {
    typedef double V;
    static constexpr bool IS_FP = true;
    double q, qinv, n0, n1;
    const double *twf, *twi;
    __device__ __forceinline__ V reduce(V v) const { return fp_reduce(v, q, qinv); }
    __device__ __forceinline__ V mulmod(V y, V w) const { return fp_mulmod(y, w, q, qinv); }
    __device__ __forceinline__ V load(u64 m) const { return u2d(m); }
    __device__ __forceinline__ V load_mid(u64 m) const { return __longlong_as_double(m); }
    __device__ __forceinline__ u64 store_mid(V v) const { return (u64)__double_as_longlong(v); }
    __device__ __forceinline__ u64 store_final(V v) const { return fp_canon(v, q, qinv); }
    // tw(c): twiddle c of the 15 this step uses, stage sp's at c = 2^sp - 1 .. 2^(sp+1) - 2
    template <class F> __device__ __forceinline__ void fwd16_with(V (&a)[16], bool reduce_first, F tw) const
    {
        if (reduce_first) {
#pragma unroll
            for (int k = 0; k < 16; k++) a[k] = reduce(a[k]);
        }
#pragma unroll
        for (int sp = 0; sp < 4; sp++) {
            const int dist = 8 >> sp;
#pragma unroll
            for (int g = 0; g < (1 << sp); g++) {
                const double w = tw((1 << sp) - 1 + g);
#pragma unroll
                for (int e = 0; e < dist; e++) {
                    const int k0 = g * 2 * dist + e, k1 = k0 + dist;
                    const double t = mulmod(a[k1], w), x = a[k0];
                    a[k0] = x + t;
                    a[k1] = x - t;
                }
            }
        }
    }
    // Three forward stages on 8 elements (pairs 4, 2, 1 apart); tw(sp, g): twiddle of stage sp, group g < 2^sp.
    // Entered with |v| <= q/2 (reduce_first) it ends below 2.7q.
    template <class F> __device__ __forceinline__ void fwd8_with(V (&a)[8], bool reduce_first, F tw) const
    {
        if (reduce_first) {
#pragma unroll
            for (int k = 0; k < 8; k++) a[k] = reduce(a[k]);
        }
#pragma unroll
        for (int sp = 0; sp < 3; sp++) {
            const int dist = 4 >> sp;
#pragma unroll
            for (int g = 0; g < (1 << sp); g++) {
                const double w = tw(sp, g);
#pragma unroll
                for (int e = 0; e < dist; e++) {
                    const int k0 = g * 2 * dist + e, k1 = k0 + dist;
                    const double t = mulmod(a[k1], w), x = a[k0];
                    a[k0] = x + t;
                    a[k1] = x - t;
                }
            }
        }
    }
    // Two forward stages on each of the two groups a[0..3], a[4..7] (pairs 2, 1 apart); tw(h, sp, g): twiddle
    // of group h, stage sp, pair group g < 2^sp.
    template <class F> __device__ __forceinline__ void fwd4x2_with(V (&a)[8], bool reduce_first, F tw) const
    {
        if (reduce_first) {
#pragma unroll
            for (int k = 0; k < 8; k++) a[k] = reduce(a[k]);
        }
#pragma unroll
        for (int h = 0; h < 2; h++) {
#pragma unroll
            for (int sp = 0; sp < 2; sp++) {
                const int dist = 2 >> sp;
#pragma unroll
                for (int g = 0; g < (1 << sp); g++) {
                    const double w = tw(h, sp, g);
#pragma unroll
                    for (int e = 0; e < dist; e++) {
                        const int k0 = 4 * h + g * 2 * dist + e, k1 = k0 + dist;
                        const double t = mulmod(a[k1], w), x = a[k0];
                        a[k0] = x + t;
                        a[k1] = x - t;
                    }
                }
            }
        }
    }
    // index in twf of twiddle c (as above) of the step that starts at stage s_base in group G
    static __device__ __forceinline__ unsigned fwd16_twiddle(unsigned s_base, unsigned G, unsigned c)
    {
        const unsigned sp = 31u - (unsigned)__clz((int)(c + 1));
        return (1u << (s_base + sp)) + (G << sp) + (c + 1 - (1u << sp));
    }
    __device__ __forceinline__ void fwd16(V (&a)[16], unsigned s_base, unsigned G, bool reduce_first) const
    {
        fwd16_with(a, reduce_first, [&](int c) { return twf[fwd16_twiddle(s_base, G, (unsigned)c)]; });
    }
    template <bool LAST> __device__ __forceinline__ void inv16(V (&a)[16], unsigned s_base, unsigned G) const
    {
#pragma unroll
        for (int sp = 3; sp >= 0; sp--) {
            const int dist = 8 >> sp;
            const unsigned idx0 = (1u << (s_base + sp)) + (G << sp);
#pragma unroll
            for (int g = 0; g < (1 << sp); g++) {
                const bool fin = LAST && sp == 0;
                const double w = fin ? n1 : twi[idx0 + g];
#pragma unroll
                for (int e = 0; e < dist; e++) {
                    const int k0 = g * 2 * dist + e, k1 = k0 + dist;
                    const double u = a[k0], v = a[k1];
                    double s = u + v;
                    if (fin)
                        s = mulmod(s, n0);
                    else if (sp == 2 || sp == 0)
                        s = reduce(s);
                    a[k0] = s;
                    a[k1] = mulmod(u - v, w);
                }
            }
        }
    }
    // Stage 0 of a 32-element column step (N = 2^17): pairs (lo[k], hi[k]) are N/2 apart, twiddle index 1.
    // Forward: inputs within 1q of zero (reduced or canonical).  Inverse: last stage, with the 1/N factors.
    __device__ __forceinline__ void fwd_stage0(V (&lo)[16], V (&hi)[16], bool reduce_first) const
    {
        const double w = twf[1];
        if (reduce_first) {
#pragma unroll
            for (int k = 0; k < 16; k++) lo[k] = reduce(lo[k]), hi[k] = reduce(hi[k]);
        }
#pragma unroll
        for (int k = 0; k < 16; k++) {
            const double t = mulmod(hi[k], w), x = lo[k];
            lo[k] = x + t;
            hi[k] = x - t;
        }
    }
    __device__ __forceinline__ void inv_stage0_last(V (&lo)[16], V (&hi)[16]) const
    {
#pragma unroll
        for (int k = 0; k < 16; k++) {
            const double u = lo[k], v = hi[k];
            lo[k] = mulmod(u + v, n0);
            hi[k] = mulmod(u - v, n1);
        }
    }
};

// ArithInt ranges (q < 2^60, so 8q < 2^63): values stay in [0, 8q) between forward stages and in [0, 4q) between
// inverse stages; every product with a table constant uses the cheaper quotient and lands in [0, 4q).
struct ArithInt {
    typedef u64 V;
    static constexpr bool IS_FP = false;
    u64 q, q2, q4;
    ShoupConst n0, n1, post; // post: optional extra constant applied by store_final (post.w == 0: none)
    const ShoupConst *twf, *twi;
    __device__ __forceinline__ V load(u64 m) const { return m; }
    __device__ __forceinline__ V load_mid(u64 m) const { return m; }
    __device__ __forceinline__ u64 store_mid(V v) const { return v; }
    __device__ __forceinline__ u64 store_final(V v) const
    {
        const u64 r = csub(csub(csub(v, q4), q2), q);
        return post.w ? mul_shoup(r, post, q) : r;
    }
    __device__ __forceinline__ void fwd_bfly(V &lo, V &hi, ShoupConst w) const
    {
        const u64 u = csub(lo, q4);
        const u64 v = mul_shoup_sloppy(hi, w, q);
        lo = u + v;
        hi = u - v + q4;
    }
    __device__ __forceinline__ void fwd16(V (&a)[16], unsigned s_base, unsigned G, bool) const
    {
#pragma unroll
        for (int sp = 0; sp < 4; sp++) {
            const int dist = 8 >> sp;
            const unsigned idx0 = (1u << (s_base + sp)) + (G << sp);
#pragma unroll
            for (int g = 0; g < (1 << sp); g++) {
                const ShoupConst w = twf[idx0 + g];
#pragma unroll
                for (int e = 0; e < dist; e++) fwd_bfly(a[g * 2 * dist + e], a[g * 2 * dist + e + dist], w);
            }
        }
    }
    template <bool LAST> __device__ __forceinline__ void inv16(V (&a)[16], unsigned s_base, unsigned G) const
    {
#pragma unroll
        for (int sp = 3; sp >= 0; sp--) {
            const int dist = 8 >> sp;
            const unsigned idx0 = (1u << (s_base + sp)) + (G << sp);
#pragma unroll
            for (int g = 0; g < (1 << sp); g++) {
                const bool fin = LAST && sp == 0;
                const ShoupConst w = fin ? n1 : twi[idx0 + g];
#pragma unroll
                for (int e = 0; e < dist; e++) {
                    const int k0 = g * 2 * dist + e, k1 = k0 + dist;
                    const u64 u = a[k0], v = a[k1];
                    a[k0] = fin ? mul_shoup_sloppy(u + v, n0, q) : csub(u + v, q4);
                    a[k1] = mul_shoup_sloppy(u - v + q4, w, q);
                }
            }
        }
    }
    __device__ __forceinline__ void fwd_stage0(V (&lo)[16], V (&hi)[16], bool) const
    {
        const ShoupConst w = twf[1];
#pragma unroll
        for (int k = 0; k < 16; k++) fwd_bfly(lo[k], hi[k], w);
    }
    __device__ __forceinline__ void inv_stage0_last(V (&lo)[16], V (&hi)[16]) const
    {
#pragma unroll
        for (int k = 0; k < 16; k++) {
            const u64 u = lo[k], v = hi[k];
            lo[k] = mul_shoup_sloppy(u + v, n0, q);
            hi[k] = mul_shoup_sloppy(u - v + q4, n1, q);
        }
    }
};

// extra_d / extra: optional constant folded into the final 1/N scaling of an inverse transform
__device__ __forceinline__ ArithFp make_fp(const DevTables &T, unsigned mi, int logN, double extra_d = 0.0)
{
    ArithFp A;
    A.q = T.mod[mi].qd;
    A.qinv = T.mod[mi].qinvd;
    A.twf = T.twd_fwd + ((size_t)mi << logN);
    A.twi = T.twd_inv + ((size_t)mi << logN);
    A.n0 = T.ninvd[2 * mi];
    A.n1 = T.ninvd[2 * mi + 1];
    if (extra_d != 0.0) {
        A.n0 = A.reduce(A.mulmod(A.n0, extra_d));
        A.n1 = A.reduce(A.mulmod(A.n1, extra_d));
    }
    return A;
}
__device__ __forceinline__ ArithInt make_int(const DevTables &T, unsigned mi, int logN, ShoupConst extra = ShoupConst{0, 0})
{
    ArithInt A;
    A.q = T.mod[mi].q;
    A.q2 = 2 * A.q;
    A.q4 = 4 * A.q;
    A.twf = T.tw_fwd + ((size_t)mi << logN);
    A.twi = T.tw_inv + ((size_t)mi << logN);
    A.n0 = T.ninv[2 * mi];
    A.n1 = T.ninv[2 * mi + 1];
    A.post = extra;
    return A;
}
