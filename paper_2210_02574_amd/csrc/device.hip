// HIP kernels (gfx950) and device-side entry points of the RNS-CKKS library.
//
// All arithmetic is on 64-bit residues of primes below 2^62, built from 32-bit integer
// multiplies: Shoup products for multiplications by table constants, and 128-bit
// accumulation with one final reduction for sums of products of two variable residues.
// Every buffer leaving a public entry point holds canonical residues in [0, q).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <functional>
#include <vector>

#include "he_internal.h"

// ------------------------------------------------------------------------------- modular helpers

__device__ __forceinline__ u64 mulhi64(u64 a, u64 b) { return __umul64hi(a, b); }
__device__ __forceinline__ u64 csub(u64 x, u64 q) { return x >= q ? x - q : x; }
// w*x mod q up to one extra q, for any 64-bit x; w < q with wp = floor(w 2^64 / q)
__device__ __forceinline__ u64 mul_shoup_lazy(u64 x, ShoupConst w, u64 q) { return x * w.w - mulhi64(x, w.wp) * q; }
__device__ __forceinline__ u64 mul_shoup(u64 x, ShoupConst w, u64 q) { return csub(mul_shoup_lazy(x, w, q), q); }

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
    const u64 a = mul_shoup_lazy(v.hi, m.r, m.q);       // hi * (2^64 mod q)   in [0, 2q)
    const u64 b = v.lo - mulhi64(v.lo, m.one_p) * m.q;  // lo mod q            in [0, 2q)
    return csub(csub(a + b, 2 * m.q), m.q);
}
__device__ __forceinline__ u64 reduce64(u64 v, const ModConst &m) { return csub(v - mulhi64(v, m.one_p) * m.q, m.q); }
__device__ __forceinline__ u64 mul_mod(u64 a, u64 b, const ModConst &m)
{
    U128 p{a * b, mulhi64(a, b)};
    return reduce128(p, m);
}

// ------------------------------------------------------------------------------------ limb lists

#define HE_MAXB 512
// A launch works on up to HE_MAXB limbs: limb b lives at base + slot[b]*N and uses modulus mod[b].
struct LimbBatch {
    uint16_t slot[HE_MAXB];
    uint8_t mod[HE_MAXB];
};

// ------------------------------------------------------------------------------------------ NTT
//
// Forward transform = decimation in time with the powers of psi in bit-reversed order; stage s
// (s = 0 .. logN-1) pairs elements N/2^(s+1) apart and uses twiddle index 2^s + (j >> (logN-s)).
// Each thread keeps 16 elements in registers and runs four stages on them (a radix-16 step);
// between steps the work-group exchanges data through LDS.  A limb of N = 2^16 takes two
// kernels: stages 0-7 on 16 columns x 256 rows (row stride 256 elements, 128-byte segments),
// then stages 8-15 on 16 contiguous blocks of 256.
//
// Two arithmetic policies share the kernel bodies:
//  * ArithFp, for primes below 2^50: residues are carried as doubles (exact integers below 2^53)
//    and a modular product is an error-free FMA sequence -- h = y*w, l = fma(y,w,-h),
//    c = rint(h/q), r = fma(-c,q,h) + l -- eight full-rate FP64 instructions per butterfly
//    against about thirty-five for the 64-bit integer form.  Values are signed and grow by a
//    bounded amount per stage; a reduction v - rint(v/q)*q every four forward stages (every second
//    inverse stage on the sum path) keeps every magnitude below 8q < 2^53, so every operation
//    is exact.
//  * ArithInt, for any prime below 2^62 (the ~60-bit special primes): Shoup products on 32-bit
//    integer multiplies with values in [0, 4q) between forward stages ([0, 2q) inverse).
// Only the last step writes canonical residues; between the two kernels of a transform the
// buffer holds the policy's internal form.

__device__ __forceinline__ double u2d(u64 v) { return __longlong_as_double(v | 0x4330000000000000ull) - 4503599627370496.0; }
__device__ __forceinline__ u64 d2u(double v)
{
    return (u64)__double_as_longlong(v + 4503599627370496.0) & 0x000FFFFFFFFFFFFFull;
}

// error-free modular product of two exact-integer doubles, |y w / q| < 2^52: result within about
// (1/2 + 3|y|/(16 q)) q of zero
__device__ __forceinline__ double fp_mulmod(double y, double w, double q, double qinv)
{
    const double h = y * w;
    const double l = __builtin_fma(y, w, -h);
    const double c = __builtin_rint(h * qinv);
    return __builtin_fma(-c, q, h) + l;
}
__device__ __forceinline__ double fp_reduce(double v, double q, double qinv)
{
    return __builtin_fma(-__builtin_rint(v * qinv), q, v);
}

struct ArithFp {
    typedef double V;
    double q, qinv;
    const double *twf, *twi, *nv;
    __device__ __forceinline__ V reduce(V v) const { return __builtin_fma(-__builtin_rint(v * qinv), q, v); }
    __device__ __forceinline__ V mulmod(V y, V w) const
    {
        const double h = y * w;
        const double l = __builtin_fma(y, w, -h);
        const double c = __builtin_rint(h * qinv);
        return __builtin_fma(-c, q, h) + l;
    }
    __device__ __forceinline__ V load(u64 m) const { return u2d(m); }
    __device__ __forceinline__ V load_mid(u64 m) const { return __longlong_as_double(m); }
    __device__ __forceinline__ u64 store_mid(V v) const { return (u64)__double_as_longlong(v); }
    __device__ __forceinline__ u64 store_final(V v) const
    {
        const double r = reduce(v);
        return d2u(r < 0.0 ? r + q : r);
    }
    __device__ __forceinline__ void fwd16(V (&a)[16], unsigned s_base, unsigned G, bool reduce_first) const
    {
        if (reduce_first) {
#pragma unroll
            for (int k = 0; k < 16; k++) a[k] = reduce(a[k]);
        }
#pragma unroll
        for (int sp = 0; sp < 4; sp++) {
            const int dist = 8 >> sp;
            const unsigned idx0 = (1u << (s_base + sp)) + (G << sp);
#pragma unroll
            for (int g = 0; g < (1 << sp); g++) {
                const double w = twf[idx0 + g];
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
    template <bool LAST> __device__ __forceinline__ void inv16(V (&a)[16], unsigned s_base, unsigned G) const
    {
#pragma unroll
        for (int sp = 3; sp >= 0; sp--) {
            const int dist = 8 >> sp;
            const unsigned idx0 = (1u << (s_base + sp)) + (G << sp);
#pragma unroll
            for (int g = 0; g < (1 << sp); g++) {
                const bool fin = LAST && sp == 0;
                const double w = fin ? nv[1] : twi[idx0 + g];
#pragma unroll
                for (int e = 0; e < dist; e++) {
                    const int k0 = g * 2 * dist + e, k1 = k0 + dist;
                    const double u = a[k0], v = a[k1];
                    double s = u + v;
                    if (fin)
                        s = mulmod(s, nv[0]);
                    else if (sp == 2 || sp == 0)
                        s = reduce(s);
                    a[k0] = s;
                    a[k1] = mulmod(u - v, w);
                }
            }
        }
    }
};

struct ArithInt {
    typedef u64 V;
    u64 q, q2;
    const ShoupConst *twf, *twi, *nv;
    __device__ __forceinline__ V load(u64 m) const { return m; }
    __device__ __forceinline__ V load_mid(u64 m) const { return m; }
    __device__ __forceinline__ u64 store_mid(V v) const { return v; }
    __device__ __forceinline__ u64 store_final(V v) const { return csub(csub(v, q2), q); }
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
                for (int e = 0; e < dist; e++) {
                    const int k0 = g * 2 * dist + e, k1 = k0 + dist;
                    const u64 u = csub(a[k0], q2);
                    const u64 v = mul_shoup_lazy(a[k1], w, q);
                    a[k0] = u + v;
                    a[k1] = u - v + q2;
                }
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
                const ShoupConst w = fin ? nv[1] : twi[idx0 + g];
#pragma unroll
                for (int e = 0; e < dist; e++) {
                    const int k0 = g * 2 * dist + e, k1 = k0 + dist;
                    const u64 u = a[k0], v = a[k1];
                    a[k0] = fin ? mul_shoup_lazy(u + v, nv[0], q) : csub(u + v, q2);
                    a[k1] = mul_shoup_lazy(u - v + q2, w, q);
                }
            }
        }
    }
};

__device__ __forceinline__ ArithFp make_fp(const DevTables &T, unsigned mi, int logN)
{
    ArithFp A;
    A.q = T.mod[mi].qd;
    A.qinv = T.mod[mi].qinvd;
    A.twf = T.twd_fwd + ((size_t)mi << logN);
    A.twi = T.twd_inv + ((size_t)mi << logN);
    A.nv = T.ninvd + 2 * mi;
    return A;
}
__device__ __forceinline__ ArithInt make_int(const DevTables &T, unsigned mi, int logN)
{
    ArithInt A;
    A.q = T.mod[mi].q;
    A.q2 = 2 * A.q;
    A.twf = T.tw_fwd + ((size_t)mi << logN);
    A.twi = T.tw_inv + ((size_t)mi << logN);
    A.nv = T.ninv + 2 * mi;
    return A;
}

// LDS tile of 16 groups x 256 elements; one pad word per 16 elements and 16 pad words per group
// keep both the "stride-16" and the "16 consecutive" access patterns free of bank conflicts.
#define TILE_GROUP 272
#define TILE_WORDS (16 * TILE_GROUP)
__device__ __forceinline__ unsigned tile_at(unsigned grp, unsigned i) { return grp * TILE_GROUP + i + (i >> 4); }
// column pass: row r (0..255) of column c (0..15); 16 pad words after every 16 rows
__device__ __forceinline__ unsigned col_at(unsigned r, unsigned c) { return (r >> 4) * TILE_GROUP + (r & 15) * 16 + c; }

// ---- "block" pass: the last eight forward stages (first eight inverse stages) on 16 contiguous
// blocks of 256 elements per work-group.
template <int LOGN, class A>
__device__ __forceinline__ void fwd_blocks_body(u64 *__restrict__ limb, const A &ar, u64 *lds, unsigned tile)
{
    const unsigned blk = threadIdx.x >> 4, il = threadIdx.x & 15;
    const unsigned bg = tile * 16 + blk; // block index within the limb
    typename A::V a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) {
        const u64 m = limb[bg * 256 + il + 16 * k];
        a[k] = LOGN > 8 ? ar.load_mid(m) : ar.load(m);
    }
    ar.fwd16(a, LOGN - 8, bg, true);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, il + 16 * k)] = ar.store_mid(a[k]);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load_mid(lds[tile_at(blk, 16 * il + k)]);
    ar.fwd16(a, LOGN - 4, bg * 16 + il, true);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, 16 * il + k)] = ar.store_final(a[k]);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) limb[bg * 256 + il + 16 * k] = lds[tile_at(blk, il + 16 * k)];
}

template <int LOGN, class A>
__device__ __forceinline__ void inv_blocks_body(u64 *__restrict__ limb, const A &ar, u64 *lds, unsigned tile)
{
    const unsigned blk = threadIdx.x >> 4, il = threadIdx.x & 15;
    const unsigned bg = tile * 16 + blk;
    typename A::V a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, il + 16 * k)] = limb[bg * 256 + il + 16 * k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load(lds[tile_at(blk, 16 * il + k)]);
    ar.template inv16<false>(a, LOGN - 4, bg * 16 + il);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, 16 * il + k)] = ar.store_mid(a[k]);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load_mid(lds[tile_at(blk, il + 16 * k)]);
    ar.template inv16<false>(a, LOGN - 8, bg);
#pragma unroll
    for (int k = 0; k < 16; k++) limb[bg * 256 + il + 16 * k] = ar.store_mid(a[k]); // the column pass finishes
}

// grid.x = (N/4096) * batch
template <int LOGN>
__global__ __launch_bounds__(256) void k_ntt_fwd_blocks(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    __shared__ u64 lds[TILE_WORDS];
    constexpr unsigned TILES = (1u << LOGN) / 4096;
    const unsigned tile = blockIdx.x % TILES, b = blockIdx.x / TILES;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << LOGN);
    if (T.mod[mi].qd != 0.0)
        fwd_blocks_body<LOGN>(limb, make_fp(T, mi, LOGN), lds, tile);
    else
        fwd_blocks_body<LOGN>(limb, make_int(T, mi, LOGN), lds, tile);
}

template <int LOGN>
__global__ __launch_bounds__(256) void k_ntt_inv_blocks(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    __shared__ u64 lds[TILE_WORDS];
    constexpr unsigned TILES = (1u << LOGN) / 4096;
    const unsigned tile = blockIdx.x % TILES, b = blockIdx.x / TILES;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << LOGN);
    if (T.mod[mi].qd != 0.0)
        inv_blocks_body<LOGN>(limb, make_fp(T, mi, LOGN), lds, tile);
    else
        inv_blocks_body<LOGN>(limb, make_int(T, mi, LOGN), lds, tile);
}

// ---- "column" pass for N = 2^16: stages 0-7 on 256 rows x 16 columns per work-group (element
// (r, c) at r*256 + c).
template <class A> __device__ __forceinline__ void fwd_cols16_body(u64 *__restrict__ limb, const A &ar, u64 *lds)
{
    const unsigned rl = threadIdx.x >> 4, c = threadIdx.x & 15;
    typename A::V a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load(limb[(rl + 16 * k) * 256 + c]);
    ar.fwd16(a, 0, 0, false);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[col_at(rl + 16 * k, c)] = ar.store_mid(a[k]);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load_mid(lds[col_at(16 * rl + k, c)]);
    ar.fwd16(a, 4, rl, true);
#pragma unroll
    for (int k = 0; k < 16; k++) limb[(16 * rl + k) * 256 + c] = ar.store_mid(a[k]); // the block pass finishes
}

template <class A> __device__ __forceinline__ void inv_cols16_body(u64 *__restrict__ limb, const A &ar, u64 *lds)
{
    const unsigned rl = threadIdx.x >> 4, c = threadIdx.x & 15;
    typename A::V a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load_mid(limb[(16 * rl + k) * 256 + c]);
    ar.template inv16<false>(a, 4, rl);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[col_at(16 * rl + k, c)] = ar.store_mid(a[k]);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load_mid(lds[col_at(rl + 16 * k, c)]);
    ar.template inv16<true>(a, 0, 0);
#pragma unroll
    for (int k = 0; k < 16; k++) limb[(rl + 16 * k) * 256 + c] = ar.store_final(a[k]);
}

// grid.x = 16 * batch
__global__ __launch_bounds__(256) void k_ntt_fwd_cols16(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    __shared__ u64 lds[TILE_WORDS];
    const unsigned tile = blockIdx.x & 15, b = blockIdx.x >> 4;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << 16) + tile * 16;
    if (T.mod[mi].qd != 0.0)
        fwd_cols16_body(limb, make_fp(T, mi, 16), lds);
    else
        fwd_cols16_body(limb, make_int(T, mi, 16), lds);
}

__global__ __launch_bounds__(256) void k_ntt_inv_cols16(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    __shared__ u64 lds[TILE_WORDS];
    const unsigned tile = blockIdx.x & 15, b = blockIdx.x >> 4;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << 16) + tile * 16;
    if (T.mod[mi].qd != 0.0)
        inv_cols16_body(limb, make_fp(T, mi, 16), lds);
    else
        inv_cols16_body(limb, make_int(T, mi, 16), lds);
}

// ---- "column" pass for N = 2^12: stages 0-3 on 16 rows x 256 columns, one thread per column.
template <class A> __device__ __forceinline__ void fwd_cols12_body(u64 *__restrict__ limb, const A &ar)
{
    const unsigned c = threadIdx.x;
    typename A::V a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load(limb[k * 256 + c]);
    ar.fwd16(a, 0, 0, false);
#pragma unroll
    for (int k = 0; k < 16; k++) limb[k * 256 + c] = ar.store_mid(a[k]);
}
template <class A> __device__ __forceinline__ void inv_cols12_body(u64 *__restrict__ limb, const A &ar)
{
    const unsigned c = threadIdx.x;
    typename A::V a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load_mid(limb[k * 256 + c]);
    ar.template inv16<true>(a, 0, 0);
#pragma unroll
    for (int k = 0; k < 16; k++) limb[k * 256 + c] = ar.store_final(a[k]);
}

__global__ __launch_bounds__(256) void k_ntt_fwd_cols12(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    const unsigned mi = lb.mod[blockIdx.x];
    u64 *limb = data + ((size_t)lb.slot[blockIdx.x] << 12);
    if (T.mod[mi].qd != 0.0)
        fwd_cols12_body(limb, make_fp(T, mi, 12));
    else
        fwd_cols12_body(limb, make_int(T, mi, 12));
}

__global__ __launch_bounds__(256) void k_ntt_inv_cols12(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    const unsigned mi = lb.mod[blockIdx.x];
    u64 *limb = data + ((size_t)lb.slot[blockIdx.x] << 12);
    if (T.mod[mi].qd != 0.0)
        inv_cols12_body(limb, make_fp(T, mi, 12));
    else
        inv_cols12_body(limb, make_int(T, mi, 12));
}

// ---------------------------------------------------------------------------------- elementwise

// op 0 add, 1 sub, 2 mul.  Limb l of the flat [limbs][N] buffers uses modulus l % level;
// b_limbs = number of limbs of b before it repeats (pmult: the plaintext has `level` limbs).
__global__ __launch_bounds__(256) void k_limbwise(const u64 *__restrict__ a, const u64 *__restrict__ b,
                                                  u64 *__restrict__ out, DevTables T, int op, int level, int b_limbs,
                                                  int logN)
{
    const unsigned l = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const ModConst m = T.mod[l % level];
    const u64 x = a[((size_t)l << logN) + n], y = b[((size_t)(l % b_limbs) << logN) + n];
    u64 r;
    if (op == 0)
        r = csub(x + y, m.q);
    else if (op == 1)
        r = csub(x + m.q - y, m.q);
    else
        r = mul_mod(x, y, m);
    out[((size_t)l << logN) + n] = r;
}

struct ScalarArgs {
    ShoupConst s[64];
};
__global__ __launch_bounds__(256) void k_cmult(const u64 *__restrict__ a, u64 *__restrict__ out, DevTables T,
                                               ScalarArgs sc, int level, int logN)
{
    const unsigned l = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const unsigned i = l % level;
    out[((size_t)l << logN) + n] = mul_shoup(a[((size_t)l << logN) + n], sc.s[i], T.mod[i].q);
}

// Tensor product: d0 = a0 b0, d1 = a0 b1 + a1 b0 -> out (may alias A or B); d2 = a1 b1 -> d2 and d2copy.
__global__ __launch_bounds__(256) void k_tensor(const u64 *A, const u64 *B, u64 *out, u64 *__restrict__ d2,
                                                u64 *__restrict__ d2copy, DevTables T, int level, int logN)
{
    const unsigned i = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const ModConst m = T.mod[i];
    const size_t o0 = ((size_t)i << logN) + n, o1 = ((size_t)(level + i) << logN) + n;
    const u64 a0 = A[o0], a1 = A[o1], b0 = B[o0], b1 = B[o1];
    U128 acc{0, 0};
    mac128(acc, a0, b1);
    mac128(acc, a1, b0);
    const u64 r0 = mul_mod(a0, b0, m), r1 = reduce128(acc, m), r2 = mul_mod(a1, b1, m);
    out[o0] = r0;
    out[o1] = r1;
    d2[o0] = r2;
    d2copy[o0] = r2;
}

// ----------------------------------------------------------------------------------- key switch

__device__ __forceinline__ int active_mod(int a, int level, int L) { return a < level ? a : L + (a - level); }

// NTT-domain index of the automorphism sigma_g: out[k] = in[k'] with
// 2 brv(k') + 1 = (2 brv(k) + 1) g mod 2N.
__device__ __forceinline__ unsigned galois_index(unsigned k, unsigned g, int logN)
{
    const unsigned b = __brev(k) >> (32 - logN);
    const unsigned e = ((2 * b + 1) * g) & ((2u << logN) - 1);
    return __brev((e - 1) >> 1) >> (32 - logN);
}

// Digit decomposition + ModUp.  x: coefficient-domain limbs [level][N]; d: the same polynomial in
// the NTT domain.  For digit j = blockIdx.y: y_i = x_i (D/q_i)^-1 mod q_i, and for every active
// modulus t outside the digit raised[j][a] = sum_i y_i (D/q_i mod t) mod t (coefficient domain,
// no correction of the overshoot); inside the digit raised[j][a] = d[a] (already transformed).
// blockIdx.z selects a contiguous share of the target limbs.  When all ciphertext primes are
// below 2^50 (fp != 0) the products for targets below 2^50 are FP64 error-free products.
template <int AMAX>
__global__ __launch_bounds__(256) void k_modup(const u64 *__restrict__ x, const u64 *__restrict__ d,
                                               u64 *__restrict__ raised, DevTables T, int level, int L, int K,
                                               int alpha, int logN, int fp)
{
    const int j = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int M = L + K, Ma = level + K;
    const int lo = j * alpha, hi = min(lo + alpha, level), na = hi - lo;
    const size_t slot = (size_t)j * alpha + (na - 1);
    const int per = (Ma + gridDim.z - 1) / gridDim.z;
    const int a_lo = blockIdx.z * per, a_hi = min(a_lo + per, Ma);
    u64 yi[AMAX];
    double yd[AMAX];
#pragma unroll
    for (int ii = 0; ii < AMAX; ii++) {
        yi[ii] = 0;
        yd[ii] = 0.0;
        if (ii < na) {
            const u64 v = x[((size_t)(lo + ii) << logN) + n];
            const ModConst m = T.mod[lo + ii];
            if (fp) {
                const double r = fp_reduce(fp_mulmod(u2d(v), T.up_inv_d[slot * alpha + ii], m.qd, m.qinvd), m.qd, m.qinvd);
                yd[ii] = r < 0.0 ? r + m.qd : r;
                yi[ii] = d2u(yd[ii]);
            } else
                yi[ii] = mul_shoup(v, T.up_inv[slot * alpha + ii], m.q);
            if (blockIdx.z == 0) raised[(((size_t)j * Ma + lo + ii) << logN) + n] = d[((size_t)(lo + ii) << logN) + n];
        }
    }
    for (int a = a_lo; a < a_hi; a++) {
        if (a >= lo && a < hi) continue;
        const int mi = active_mod(a, level, L);
        const ModConst m = T.mod[mi];
        u64 out;
        if (fp && m.qd != 0.0) {
            double acc = 0.0;
#pragma unroll
            for (int ii = 0; ii < AMAX; ii++)
                if (ii < na) acc += fp_mulmod(yd[ii], T.up_hat_d[(slot * alpha + ii) * M + mi], m.qd, m.qinvd);
            const double r = fp_reduce(acc, m.qd, m.qinvd);
            out = d2u(r < 0.0 ? r + m.qd : r);
        } else {
            U128 acc{0, 0};
#pragma unroll
            for (int ii = 0; ii < AMAX; ii++)
                if (ii < na) mac128(acc, yi[ii], T.up_hat[(slot * alpha + ii) * M + mi]);
            out = reduce128(acc, m);
        }
        raised[(((size_t)j * Ma + a) << logN) + n] = out;
    }
}

// Inner product with the evaluation key on active limb a = blockIdx.y:
// u[c][a][n] = sum_j raised[j][a][pi_g(n)] * evk[j][c][mod(a)][n].
__global__ __launch_bounds__(256) void k_inner(const u64 *__restrict__ raised, const u64 *__restrict__ evk,
                                               u64 *__restrict__ u, DevTables T, int level, int L, int K, int beta,
                                               unsigned g, int logN)
{
    const int a = blockIdx.y;
    const unsigned n = blockIdx.x * 256 + threadIdx.x;
    const int M = L + K, Ma = level + K;
    const int mi = active_mod(a, level, L);
    const unsigned src = g == 1 ? n : galois_index(n, g, logN);
    U128 acc0{0, 0}, acc1{0, 0};
    for (int j = 0; j < beta; j++) {
        const u64 dv = raised[(((size_t)j * Ma + a) << logN) + src];
        const u64 kb = evk[((((size_t)j * 2 + 0) * M + mi) << logN) + n];
        const u64 ka = evk[((((size_t)j * 2 + 1) * M + mi) << logN) + n];
        mac128(acc0, dv, kb);
        mac128(acc1, dv, ka);
    }
    const ModConst m = T.mod[mi];
    u[(((size_t)0 * Ma + a) << logN) + n] = reduce128(acc0, m);
    u[(((size_t)1 * Ma + a) << logN) + n] = reduce128(acc1, m);
}

// ModDown, conversion step.  u: [2][level+K][N] whose special limbs are in the coefficient
// domain.  y_k = w_k (P/p_k)^-1 mod p_k; r[c][i] = sum_k y_k (P/p_k mod q_i) mod q_i.
__global__ __launch_bounds__(256) void k_moddown_conv(const u64 *__restrict__ u, u64 *__restrict__ r, DevTables T,
                                                      int level, int L, int K, int logN)
{
    const int c = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int Ma = level + K;
    const int per = (level + gridDim.z - 1) / gridDim.z;
    const int i_lo = blockIdx.z * per, i_hi = min(i_lo + per, level);
    u64 y[16];
#pragma unroll
    for (int k = 0; k < 16; k++)
        y[k] = k < K ? mul_shoup(u[(((size_t)c * Ma + level + k) << logN) + n], T.dn_inv[k], T.mod[L + k].q) : 0;
    for (int i = i_lo; i < i_hi; i++) {
        U128 acc{0, 0};
#pragma unroll
        for (int k = 0; k < 16; k++)
            if (k < K) mac128(acc, y[k], T.dn_hat[(size_t)k * L + i]);
        r[(((size_t)c * level + i) << logN) + n] = reduce128(acc, T.mod[i]);
    }
}

// ModDown, final step: out[c][i] = (u[c][i] - r[c][i]) P^-1 + addend, all in the NTT domain.
// addend: mode 0 none; 1 out itself (hmult: d0, d1 already there); 2 rotation: component 0 gets
// c0 read through pi_g, component 1 nothing.
__global__ __launch_bounds__(256) void k_moddown_fin(const u64 *__restrict__ u, const u64 *__restrict__ r,
                                                     u64 *out, const u64 *__restrict__ c0, DevTables T, int level,
                                                     int K, int mode, unsigned g, int logN)
{
    const int ci = blockIdx.y; // c * level + i
    const int c = ci / level, i = ci % level;
    const unsigned n = blockIdx.x * 256 + threadIdx.x;
    const int Ma = level + K;
    const u64 q = T.mod[i].q;
    const u64 uv = u[(((size_t)c * Ma + i) << logN) + n];
    const u64 rv = r[((size_t)ci << logN) + n];
    u64 v = mul_shoup(uv + q - rv, T.dn_pinv[i], q);
    if (mode == 1)
        v = csub(v + out[((size_t)ci << logN) + n], q);
    else if (mode == 2 && c == 0)
        v = csub(v + c0[((size_t)i << logN) + galois_index(n, g, logN)], q);
    out[((size_t)ci << logN) + n] = v;
}

// Rescale, conversion: t[c] = last limb in the coefficient domain; r[c][i] = centred(t) mod q_i.
__global__ __launch_bounds__(256) void k_rescale_conv(const u64 *__restrict__ t, u64 *__restrict__ r, DevTables T,
                                                      int level, int logN)
{
    const int c = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const u64 ql = T.mod[level - 1].q;
    const u64 v = t[((size_t)c << logN) + n];
    const bool neg = v > (ql - 1) / 2;
    const u64 mag = neg ? ql - v : v;
    for (int i = 0; i < level - 1; i++) {
        const ModConst m = T.mod[i];
        const u64 w = reduce64(mag, m);
        r[(((size_t)c * (level - 1) + i) << logN) + n] = neg ? (w ? m.q - w : 0) : w;
    }
}

// Rescale, final: out[c][i] = (ct[c][i] - r[c][i]) q_last^-1.
__global__ __launch_bounds__(256) void k_rescale_fin(const u64 *__restrict__ ct, const u64 *__restrict__ r,
                                                     u64 *__restrict__ out, DevTables T, int level, int L, int logN)
{
    const int ci = blockIdx.y; // c * (level-1) + i
    const int c = ci / (level - 1), i = ci % (level - 1);
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const u64 q = T.mod[i].q;
    const u64 cv = ct[(((size_t)c * level + i) << logN) + n];
    const u64 rv = r[((size_t)ci << logN) + n];
    out[((size_t)ci << logN) + n] = mul_shoup(cv + q - rv, T.rs_inv[(size_t)(level - 1) * L + i], q);
}

// ===================================================================================== host side

#define HIP_TRY(ctx, expr)                                                                                           \
    do {                                                                                                             \
        hipError_t e_ = (expr);                                                                                      \
        if (e_ != hipSuccess) {                                                                                      \
            (ctx)->hip_err = std::string(#expr) + ": " + hipGetErrorString(e_);                                      \
            return HE_EHIP;                                                                                          \
        }                                                                                                            \
    } while (0)

template <class Tv> static int32_t upload(he_ctx *c, const std::vector<Tv> &v, const Tv **out)
{
    void *p = nullptr;
    const size_t bytes = std::max<size_t>(v.size() * sizeof(Tv), 16);
    HIP_TRY(c, hipMalloc(&p, bytes));
    c->dev_allocs.push_back(p);
    if (!v.empty()) HIP_TRY(c, hipMemcpy(p, v.data(), v.size() * sizeof(Tv), hipMemcpyHostToDevice));
    *out = (const Tv *)p;
    return HE_OK;
}

int32_t dev_upload_tables(he_ctx *c)
{
    if (c->logN != 12 && c->logN != 16) return HE_EINVAL;
    if (c->alpha > 16 || c->K > 16 || c->M > 64) return HE_EINVAL;
    HIP_TRY(c, hipSetDevice(c->device));
    int32_t rc;
#define UP(field)                                                                                                    \
    if ((rc = upload(c, c->field, &c->dev.field)) != HE_OK) return rc;
    if ((rc = upload(c, c->modc, &c->dev.mod)) != HE_OK) return rc;
    UP(tw_fwd) UP(tw_inv) UP(ninv) UP(twd_fwd) UP(twd_inv) UP(ninvd) UP(up_inv) UP(up_inv_d) UP(up_hat_d) UP(up_hat) UP(dn_inv) UP(dn_hat) UP(dn_pinv) UP(rs_inv)
#undef UP
    return HE_OK;
}

void dev_free_tables(he_ctx *c)
{
    for (void *p : c->dev_allocs) (void)hipFree(p);
    c->dev_allocs.clear();
}

int32_t dev_upload_evk(he_evk *k)
{
    he_ctx *c = const_cast<he_ctx *>(k->ctx);
    HIP_TRY(c, hipSetDevice(c->device));
    HIP_TRY(c, hipMalloc((void **)&k->dev, k->host.size() * sizeof(u64)));
    HIP_TRY(c, hipMemcpy(k->dev, k->host.data(), k->host.size() * sizeof(u64), hipMemcpyHostToDevice));
    return HE_OK;
}

void dev_free_evk(he_evk *k)
{
    if (k->dev) (void)hipFree(k->dev);
    k->dev = nullptr;
}

extern "C" int32_t he_evk_to_host(const he_evk *evk, uint64_t *h_out)
{
    if (!evk || !h_out) return HE_EINVAL;
    const he_ctx *c = evk->ctx;
    const size_t words = (size_t)c->dnum * 2 * c->M * c->N;
    if (evk->dev) {
        he_ctx *cm = const_cast<he_ctx *>(c);
        HIP_TRY(cm, hipMemcpy(h_out, evk->dev, words * sizeof(u64), hipMemcpyDeviceToHost));
    } else
        memcpy(h_out, evk->host.data(), words * sizeof(u64));
    return HE_OK;
}

// ---- optional per-kernel timing with HIP events on the launch stream (he_profile_start/stop)
enum KernelId {
    KID_NTT_FWD_COLS, KID_NTT_FWD_BLOCKS, KID_NTT_INV_BLOCKS, KID_NTT_INV_COLS, KID_LIMBWISE, KID_CMULT, KID_TENSOR,
    KID_MODUP, KID_INNER, KID_MODDOWN_CONV, KID_MODDOWN_FIN, KID_RESCALE_CONV, KID_RESCALE_FIN, KID_COPY, KID_COUNT
};
static const char *const kKernelNames[KID_COUNT] = {
    "k_ntt_fwd_cols", "k_ntt_fwd_blocks", "k_ntt_inv_blocks", "k_ntt_inv_cols", "k_limbwise", "k_cmult", "k_tensor",
    "k_modup", "k_inner", "k_moddown_conv", "k_moddown_fin", "k_rescale_conv", "k_rescale_fin", "copy"};

static void prof_begin(he_ctx *c, hipStream_t st, int kid, double bytes)
{
    ProfRecord r;
    r.kid = kid;
    r.bytes = bytes;
    r.a = r.b = nullptr;
    if (hipEventCreate((hipEvent_t *)&r.a) != hipSuccess || hipEventCreate((hipEvent_t *)&r.b) != hipSuccess) return;
    (void)hipEventRecord((hipEvent_t)r.a, st);
    c->prof.push_back(r);
}
static void prof_end(he_ctx *c, hipStream_t st)
{
    if (!c->prof.empty()) (void)hipEventRecord((hipEvent_t)c->prof.back().b, st);
}
// Launch wrapper: `bytes` = bytes the launch has to move by the definition of its step
#define KLAUNCH(c, st, kid, bytes, ...)                                                                              \
    do {                                                                                                             \
        if ((c)->prof_on) prof_begin((c), (st), (kid), (double)(bytes));                                             \
        __VA_ARGS__;                                                                                                 \
        if ((c)->prof_on) prof_end((c), (st));                                                                       \
    } while (0)

extern "C" int32_t he_profile_start(he_ctx *ctx)
{
    if (!ctx) return HE_EINVAL;
    if (ctx->device < 0) return HE_ENODEV;
    ctx->prof_on = true;
    return HE_OK;
}

extern "C" int32_t he_profile_stop(he_ctx *ctx, he_kernel_stat *out, int32_t max_out, int32_t *n_out)
{
    if (!ctx || !out || !n_out || max_out < 0) return HE_EINVAL;
    ctx->prof_on = false;
    double ms[KID_COUNT] = {0}, bytes[KID_COUNT] = {0};
    int64_t cnt[KID_COUNT] = {0};
    int32_t rc = HE_OK;
    for (ProfRecord &r : ctx->prof) {
        float t = 0.f;
        if (r.a && r.b && hipEventSynchronize((hipEvent_t)r.b) == hipSuccess &&
            hipEventElapsedTime(&t, (hipEvent_t)r.a, (hipEvent_t)r.b) == hipSuccess) {
            ms[r.kid] += t;
            bytes[r.kid] += r.bytes;
            cnt[r.kid]++;
        } else
            rc = HE_EHIP;
        if (r.a) (void)hipEventDestroy((hipEvent_t)r.a);
        if (r.b) (void)hipEventDestroy((hipEvent_t)r.b);
    }
    ctx->prof.clear();
    int32_t n = 0;
    for (int k = 0; k < KID_COUNT && n < max_out; k++) {
        if (!cnt[k]) continue;
        memset(&out[n], 0, sizeof(out[n]));
        strncpy(out[n].name, kKernelNames[k], sizeof(out[n].name) - 1);
        out[n].launches = cnt[k];
        out[n].total_ms = ms[k];
        out[n].bytes = bytes[k];
        n++;
    }
    *n_out = n;
    return rc;
}

static inline int32_t launch_ok(he_ctx *c)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        c->hip_err = std::string("kernel launch: ") + hipGetErrorString(e);
        return HE_EHIP;
    }
    return HE_OK;
}

// NTT of the limbs listed in (slots, mods), all relative to `base`
static int32_t run_ntt(he_ctx *c, u64 *base, const std::vector<int> &slots, const std::vector<int> &mods, bool inverse,
                       hipStream_t st)
{
    const int total = (int)slots.size();
    // limbs on the integer path take about three times longer: schedule them first
    std::vector<int> order(total);
    for (int b = 0; b < total; b++) order[b] = b;
    std::stable_partition(order.begin(), order.end(), [&](int b) { return c->modc[mods[b]].qd == 0.0; });
    for (int off = 0; off < total; off += HE_MAXB) {
        const int nb = std::min(HE_MAXB, total - off);
        LimbBatch lb;
        for (int b = 0; b < nb; b++) {
            lb.slot[b] = (uint16_t)slots[order[off + b]];
            lb.mod[b] = (uint8_t)mods[order[off + b]];
        }
        // each pass reads and writes every limb of the batch once
        const double bytes = (double)nb * (double)c->N * 16.0;
        if (c->logN == 16) {
            if (!inverse) {
                KLAUNCH(c, st, KID_NTT_FWD_COLS, bytes, k_ntt_fwd_cols16<<<16 * nb, 256, 0, st>>>(base, c->dev, lb));
                KLAUNCH(c, st, KID_NTT_FWD_BLOCKS, bytes,
                        k_ntt_fwd_blocks<16><<<16 * nb, 256, 0, st>>>(base, c->dev, lb));
            } else {
                KLAUNCH(c, st, KID_NTT_INV_BLOCKS, bytes,
                        k_ntt_inv_blocks<16><<<16 * nb, 256, 0, st>>>(base, c->dev, lb));
                KLAUNCH(c, st, KID_NTT_INV_COLS, bytes, k_ntt_inv_cols16<<<16 * nb, 256, 0, st>>>(base, c->dev, lb));
            }
        } else {
            if (!inverse) {
                KLAUNCH(c, st, KID_NTT_FWD_COLS, bytes, k_ntt_fwd_cols12<<<nb, 256, 0, st>>>(base, c->dev, lb));
                KLAUNCH(c, st, KID_NTT_FWD_BLOCKS, bytes, k_ntt_fwd_blocks<12><<<nb, 256, 0, st>>>(base, c->dev, lb));
            } else {
                KLAUNCH(c, st, KID_NTT_INV_BLOCKS, bytes, k_ntt_inv_blocks<12><<<nb, 256, 0, st>>>(base, c->dev, lb));
                KLAUNCH(c, st, KID_NTT_INV_COLS, bytes, k_ntt_inv_cols12<<<nb, 256, 0, st>>>(base, c->dev, lb));
            }
        }
        int32_t rc = launch_ok(c);
        if (rc != HE_OK) return rc;
    }
    return HE_OK;
}

static int32_t dev_guard(he_ctx *c)
{
    if (!c) return HE_EINVAL;
    if (c->device < 0) return HE_ENODEV;
    return HE_OK;
}

static int32_t ntt_api(he_ctx *ctx, uint64_t *d_limbs, const int32_t *h_mod_idx, int32_t batch, void *stream, bool inv)
{
    int32_t rc = dev_guard(ctx);
    if (rc != HE_OK) return rc;
    if (!d_limbs || !h_mod_idx || batch < 0) return HE_EINVAL;
    for (int b = 0; b < batch; b++)
        if (h_mod_idx[b] < 0 || h_mod_idx[b] >= ctx->M) return HE_EINVAL;
    // slots are 16-bit: walk the buffer in windows
    const int WIN = 32768;
    for (int off = 0; off < batch; off += WIN) {
        const int nb = std::min(WIN, batch - off);
        std::vector<int> slots(nb), mods(nb);
        for (int b = 0; b < nb; b++) {
            slots[b] = b;
            mods[b] = h_mod_idx[off + b];
        }
        rc = run_ntt(ctx, d_limbs + (size_t)off * ctx->N, slots, mods, inv, (hipStream_t)stream);
        if (rc != HE_OK) return rc;
    }
    return HE_OK;
}

extern "C" int32_t he_ntt(he_ctx *ctx, uint64_t *d_limbs, const int32_t *h_mod_idx, int32_t batch, void *stream)
{
    return ntt_api(ctx, d_limbs, h_mod_idx, batch, stream, false);
}
extern "C" int32_t he_intt(he_ctx *ctx, uint64_t *d_limbs, const int32_t *h_mod_idx, int32_t batch, void *stream)
{
    return ntt_api(ctx, d_limbs, h_mod_idx, batch, stream, true);
}

static int32_t level_guard(he_ctx *c, int level)
{
    int32_t rc = dev_guard(c);
    if (rc != HE_OK) return rc;
    if (level < 1 || level > c->L) return HE_ELEVEL;
    return HE_OK;
}

static int32_t limbwise(he_ctx *c, const u64 *a, const u64 *b, u64 *out, int level, int op, int limbs, int b_limbs,
                        void *stream)
{
    int32_t rc = level_guard(c, level);
    if (rc != HE_OK) return rc;
    if (!a || !b || !out) return HE_EINVAL;
    dim3 grid((unsigned)(c->N / 256), (unsigned)limbs);
    KLAUNCH(c, (hipStream_t)stream, KID_LIMBWISE, (double)(2 * limbs + b_limbs) * c->N * 8.0,
            k_limbwise<<<grid, 256, 0, (hipStream_t)stream>>>(a, b, out, c->dev, op, level, b_limbs, c->logN));
    return launch_ok(c);
}

extern "C" int32_t he_add(he_ctx *ctx, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out, int32_t level,
                          void *stream)
{
    return limbwise(ctx, d_a, d_b, d_out, level, 0, 2 * level, 2 * level, stream);
}
extern "C" int32_t he_sub(he_ctx *ctx, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out, int32_t level,
                          void *stream)
{
    return limbwise(ctx, d_a, d_b, d_out, level, 1, 2 * level, 2 * level, stream);
}
extern "C" int32_t he_pmult(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *d_pt, uint64_t *d_out, int32_t level,
                            void *stream)
{
    return limbwise(ctx, d_ct, d_pt, d_out, level, 2, 2 * level, level, stream);
}

extern "C" int32_t he_cmult(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *h_scalar, uint64_t *d_out, int32_t level,
                            void *stream)
{
    int32_t rc = level_guard(ctx, level);
    if (rc != HE_OK) return rc;
    if (!d_ct || !h_scalar || !d_out) return HE_EINVAL;
    ScalarArgs sc;
    memset(&sc, 0, sizeof(sc));
    for (int i = 0; i < level; i++) {
        if (h_scalar[i] >= ctx->mod[i]) return HE_EINVAL;
        sc.s[i] = hostmath::shoup(h_scalar[i], ctx->mod[i]);
    }
    dim3 grid((unsigned)(ctx->N / 256), (unsigned)(2 * level));
    KLAUNCH(ctx, (hipStream_t)stream, KID_CMULT, 4.0 * level * ctx->N * 8.0,
            k_cmult<<<grid, 256, 0, (hipStream_t)stream>>>(d_ct, d_out, ctx->dev, sc, level, ctx->logN));
    return launch_ok(ctx);
}

// ---- workspace layout (in limbs of N words)
struct WsLayout {
    size_t x, d, raised, u, r, tmp, total;
};
static WsLayout ws_layout(const he_ctx *c, int level)
{
    const size_t Ma = level + c->K, beta = (level + c->alpha - 1) / c->alpha;
    WsLayout w;
    size_t o = 0;
    w.x = o, o += level;
    w.d = o, o += level;
    w.raised = o, o += beta * Ma;
    w.u = o, o += 2 * Ma;
    w.r = o, o += 2 * level;
    w.tmp = o, o += 2 * level;
    w.total = o;
    return w;
}

extern "C" int32_t he_workspace_bytes(const he_ctx *ctx, int32_t level, int32_t max_hoist, size_t *out)
{
    if (!ctx || !out || max_hoist < 1) return HE_EINVAL;
    if (level < 1 || level > ctx->L) return HE_ELEVEL;
    *out = ws_layout(ctx, level).total * ctx->N * sizeof(u64);
    return HE_OK;
}

// Steps 1-2 of the key switch: x (a copy of d at ws.x, NTT domain) -> iNTT -> ModUp -> NTT of the
// limbs outside each digit.  d_ntt: the polynomial in the NTT domain.
static int32_t ks_raise(he_ctx *c, const u64 *d_ntt, u64 *ws, const WsLayout &w, int level, hipStream_t st)
{
    const size_t N = c->N;
    const int K = c->K, Ma = level + K, beta = (level + c->alpha - 1) / c->alpha;
    std::vector<int> slots, mods;
    for (int i = 0; i < level; i++) slots.push_back(i), mods.push_back(i);
    int32_t rc = run_ntt(c, ws + w.x * N, slots, mods, true, st);
    if (rc != HE_OK) return rc;
    dim3 grid((unsigned)(N / 256), (unsigned)beta);
    // reads the level coefficient-domain limbs (and the NTT-domain copies), writes beta*(level+K) limbs
    grid.z = 4;
#define MODUP_LAUNCH(AMAX)                                                                                           \
    KLAUNCH(c, st, KID_MODUP, (double)(2 * level + beta * Ma) * N * 8.0,                                             \
            k_modup<AMAX><<<grid, 256, 0, st>>>(ws + w.x * N, d_ntt, ws + w.raised * N, c->dev, level, c->L, K,      \
                                                c->alpha, c->logN, c->conv_fp ? 1 : 0))
    if (c->alpha <= 1)
        MODUP_LAUNCH(1);
    else if (c->alpha <= 2)
        MODUP_LAUNCH(2);
    else if (c->alpha <= 4)
        MODUP_LAUNCH(4);
    else if (c->alpha <= 8)
        MODUP_LAUNCH(8);
    else
        MODUP_LAUNCH(16);
#undef MODUP_LAUNCH
    if ((rc = launch_ok(c)) != HE_OK) return rc;
    slots.clear(), mods.clear();
    for (int j = 0; j < beta; j++) {
        const int lo = j * c->alpha, hi = std::min(lo + c->alpha, level);
        for (int a = 0; a < Ma; a++) {
            if (a >= lo && a < hi) continue;
            slots.push_back(j * Ma + a);
            mods.push_back(a < level ? a : c->L + (a - level));
        }
    }
    return run_ntt(c, ws + w.raised * N, slots, mods, false, st);
}

// Steps 3-5: inner product through pi_g, ModDown of both components into `out` with the addend
// selected by mode (see k_moddown_fin).
static int32_t ks_apply(he_ctx *c, const he_evk *evk, u64 *ws, const WsLayout &w, int level, u64 *out, const u64 *c0,
                        int mode, hipStream_t st)
{
    const size_t N = c->N;
    const int K = c->K, Ma = level + K, beta = (level + c->alpha - 1) / c->alpha;
    const unsigned g = (unsigned)evk->galois;
    dim3 grid((unsigned)(N / 256), (unsigned)Ma);
    // reads beta raised limbs and 2*beta key limbs per active modulus, writes 2 limbs per active modulus
    KLAUNCH(c, st, KID_INNER, (double)(3 * beta + 2) * Ma * N * 8.0,
            k_inner<<<grid, 256, 0, st>>>(ws + w.raised * N, evk->dev, ws + w.u * N, c->dev, level, c->L, K, beta, g,
                                          c->logN));
    int32_t rc = launch_ok(c);
    if (rc != HE_OK) return rc;
    std::vector<int> slots, mods;
    for (int cc = 0; cc < 2; cc++)
        for (int k = 0; k < K; k++) slots.push_back(cc * Ma + level + k), mods.push_back(c->L + k);
    if ((rc = run_ntt(c, ws + w.u * N, slots, mods, true, st)) != HE_OK) return rc;
    dim3 grid2((unsigned)(N / 256), 2, (unsigned)std::min(level, 6));
    KLAUNCH(c, st, KID_MODDOWN_CONV, (double)(2 * K + 2 * level) * N * 8.0,
            k_moddown_conv<<<grid2, 256, 0, st>>>(ws + w.u * N, ws + w.r * N, c->dev, level, c->L, K, c->logN));
    if ((rc = launch_ok(c)) != HE_OK) return rc;
    slots.clear(), mods.clear();
    for (int cc = 0; cc < 2; cc++)
        for (int i = 0; i < level; i++) slots.push_back(cc * level + i), mods.push_back(i);
    if ((rc = run_ntt(c, ws + w.r * N, slots, mods, false, st)) != HE_OK) return rc;
    dim3 grid3((unsigned)(N / 256), (unsigned)(2 * level));
    KLAUNCH(c, st, KID_MODDOWN_FIN, (double)(6 * level + (mode == 1 ? 2 * level : mode == 2 ? level : 0)) * N * 8.0,
            k_moddown_fin<<<grid3, 256, 0, st>>>(ws + w.u * N, ws + w.r * N, out, c0, c->dev, level, K, mode, g,
                                                 c->logN));
    return launch_ok(c);
}

static int32_t ks_guard(he_ctx *c, const he_evk *evk, int level, void *ws, size_t ws_bytes)
{
    int32_t rc = level_guard(c, level);
    if (rc != HE_OK) return rc;
    if (!evk || evk->ctx != c || !evk->dev) return HE_ENOKEY;
    if (!ws) return HE_EINVAL;
    if (ws_bytes < ws_layout(c, level).total * c->N * sizeof(u64)) return HE_EWORKSPACE;
    return HE_OK;
}

extern "C" int32_t he_hmult_relin(he_ctx *ctx, const he_evk *relin, const uint64_t *d_a, const uint64_t *d_b,
                                  uint64_t *d_out, int32_t level, void *d_ws, size_t ws_bytes, void *stream)
{
    int32_t rc = ks_guard(ctx, relin, level, d_ws, ws_bytes);
    if (rc != HE_OK) return rc;
    if (relin->galois != 1) return HE_ENOKEY;
    if (!d_a || !d_b || !d_out) return HE_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    u64 *ws = (u64 *)d_ws;
    const WsLayout w = ws_layout(ctx, level);
    const size_t N = ctx->N;
    dim3 grid((unsigned)(N / 256), (unsigned)level);
    KLAUNCH(ctx, st, KID_TENSOR, 8.0 * level * N * 8.0,
            k_tensor<<<grid, 256, 0, st>>>(d_a, d_b, d_out, ws + w.d * N, ws + w.x * N, ctx->dev, level, ctx->logN));
    if ((rc = launch_ok(ctx)) != HE_OK) return rc;
    if ((rc = ks_raise(ctx, ws + w.d * N, ws, w, level, st)) != HE_OK) return rc;
    return ks_apply(ctx, relin, ws, w, level, d_out, nullptr, 1, st);
}

extern "C" int32_t he_hrot_many(he_ctx *ctx, const he_evk *const *rots, int32_t count, const uint64_t *d_ct,
                                uint64_t *const *h_d_outs, int32_t level, void *d_ws, size_t ws_bytes, void *stream)
{
    if (!rots || count < 1 || !h_d_outs) return HE_EINVAL;
    int32_t rc;
    for (int r = 0; r < count; r++) {
        if ((rc = ks_guard(ctx, rots[r], level, d_ws, ws_bytes)) != HE_OK) return rc;
        if (rots[r]->galois == 1) return HE_ENOKEY;
        if (!h_d_outs[r] || h_d_outs[r] == d_ct) return HE_EINVAL;
    }
    if (!d_ct) return HE_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    u64 *ws = (u64 *)d_ws;
    const WsLayout w = ws_layout(ctx, level);
    const size_t N = ctx->N;
    const u64 *c1 = d_ct + (size_t)level * N;
    hipError_t e = hipMemcpyAsync(ws + w.x * N, c1, (size_t)level * N * sizeof(u64), hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) {
        ctx->hip_err = std::string("hipMemcpyAsync: ") + hipGetErrorString(e);
        return HE_EHIP;
    }
    if ((rc = ks_raise(ctx, c1, ws, w, level, st)) != HE_OK) return rc;
    for (int r = 0; r < count; r++)
        if ((rc = ks_apply(ctx, rots[r], ws, w, level, h_d_outs[r], d_ct, 2, st)) != HE_OK) return rc;
    return HE_OK;
}

extern "C" int32_t he_hrot(he_ctx *ctx, const he_evk *rot, const uint64_t *d_ct, uint64_t *d_out, int32_t level,
                           void *d_ws, size_t ws_bytes, void *stream)
{
    uint64_t *outs[1] = {d_out};
    const he_evk *keys[1] = {rot};
    return he_hrot_many(ctx, keys, 1, d_ct, outs, level, d_ws, ws_bytes, stream);
}

extern "C" int32_t he_rotate_sum(he_ctx *ctx, const he_evk *const *rots, int32_t count, uint64_t *d_ct, int32_t level,
                                 void *d_ws, size_t ws_bytes, void *stream)
{
    if (!rots || count < 0) return HE_EINVAL;
    int32_t rc = level_guard(ctx, level);
    if (rc != HE_OK) return rc;
    if (!d_ws || !d_ct) return HE_EINVAL;
    const WsLayout w = ws_layout(ctx, level);
    if (ws_bytes < w.total * ctx->N * sizeof(u64)) return HE_EWORKSPACE;
    u64 *tmp = (u64 *)d_ws + w.tmp * ctx->N;
    for (int k = 0; k < count; k++) {
        if ((rc = he_hrot(ctx, rots[k], d_ct, tmp, level, d_ws, ws_bytes, stream)) != HE_OK) return rc;
        if ((rc = he_add(ctx, d_ct, tmp, d_ct, level, stream)) != HE_OK) return rc;
    }
    return HE_OK;
}

extern "C" int32_t he_rescale(he_ctx *ctx, const uint64_t *d_ct, uint64_t *d_out, int32_t level, void *d_ws,
                              size_t ws_bytes, void *stream)
{
    int32_t rc = level_guard(ctx, level);
    if (rc != HE_OK) return rc;
    if (level < 2) return HE_ELEVEL;
    if (!d_ct || !d_out || !d_ws || d_ct == d_out) return HE_EINVAL;
    const WsLayout w = ws_layout(ctx, level);
    if (ws_bytes < w.total * ctx->N * sizeof(u64)) return HE_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    u64 *ws = (u64 *)d_ws;
    const size_t N = ctx->N;
    u64 *t = ws + w.x * N; // two limbs: the last limb of each component
    u64 *r = ws + w.r * N; // [2][level-1][N]
    for (int c = 0; c < 2; c++) {
        hipError_t e = hipMemcpyAsync(t + c * N, d_ct + ((size_t)c * level + level - 1) * N, N * sizeof(u64),
                                      hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) {
            ctx->hip_err = std::string("hipMemcpyAsync: ") + hipGetErrorString(e);
            return HE_EHIP;
        }
    }
    std::vector<int> slots{0, 1}, mods{level - 1, level - 1};
    if ((rc = run_ntt(ctx, t, slots, mods, true, st)) != HE_OK) return rc;
    dim3 grid((unsigned)(N / 256), 2);
    KLAUNCH(ctx, st, KID_RESCALE_CONV, (double)(2 + 2 * (level - 1)) * N * 8.0,
            k_rescale_conv<<<grid, 256, 0, st>>>(t, r, ctx->dev, level, ctx->logN));
    if ((rc = launch_ok(ctx)) != HE_OK) return rc;
    slots.clear(), mods.clear();
    for (int c = 0; c < 2; c++)
        for (int i = 0; i < level - 1; i++) slots.push_back(c * (level - 1) + i), mods.push_back(i);
    if ((rc = run_ntt(ctx, r, slots, mods, false, st)) != HE_OK) return rc;
    dim3 grid2((unsigned)(N / 256), (unsigned)(2 * (level - 1)));
    KLAUNCH(ctx, st, KID_RESCALE_FIN, 6.0 * (level - 1) * N * 8.0,
            k_rescale_fin<<<grid2, 256, 0, st>>>(d_ct, r, d_out, ctx->dev, level, ctx->L, ctx->logN));
    return launch_ok(ctx);
}
