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
// then stages 8-15 on 16 contiguous blocks of 256.  Values stay in [0, 4q) between stages
// (inverse: [0, 2q)); only the last step writes canonical residues.

__device__ __forceinline__ void bfly_fwd(u64 &x, u64 &y, ShoupConst w, u64 q, u64 q2)
{
    const u64 u = csub(x, q2);
    const u64 v = mul_shoup_lazy(y, w, q);
    x = u + v;
    y = u - v + q2;
}

__device__ __forceinline__ void bfly_inv(u64 &x, u64 &y, ShoupConst w, u64 q, u64 q2)
{
    const u64 u = x, v = y;
    x = csub(u + v, q2);
    y = mul_shoup_lazy(u - v + q2, w, q);
}

// four forward stages s_base .. s_base+3 on the 16 elements of one thread; G = index of the
// thread's group at stage s_base
__device__ __forceinline__ void fwd16(u64 (&a)[16], const ShoupConst *__restrict__ tw, unsigned s_base, unsigned G,
                                      u64 q)
{
    const u64 q2 = 2 * q;
#pragma unroll
    for (int sp = 0; sp < 4; sp++) {
        const int dist = 8 >> sp;
        const unsigned idx0 = (1u << (s_base + sp)) + (G << sp);
#pragma unroll
        for (int g = 0; g < (1 << sp); g++) {
            const ShoupConst w = tw[idx0 + g];
#pragma unroll
            for (int e = 0; e < dist; e++) bfly_fwd(a[g * 2 * dist + e], a[g * 2 * dist + e + dist], w, q, q2);
        }
    }
}

// the inverse of fwd16: stages s_base+3 down to s_base.  When `last` is set, stage 0 also
// multiplies by N^-1 (ninv[0] = N^-1, ninv[1] = N^-1 * twiddle).
template <bool LAST>
__device__ __forceinline__ void inv16(u64 (&a)[16], const ShoupConst *__restrict__ tw, unsigned s_base, unsigned G,
                                      u64 q, const ShoupConst *__restrict__ ninv)
{
    const u64 q2 = 2 * q;
#pragma unroll
    for (int sp = 3; sp >= 0; sp--) {
        const int dist = 8 >> sp;
        const unsigned idx0 = (1u << (s_base + sp)) + (G << sp);
#pragma unroll
        for (int g = 0; g < (1 << sp); g++) {
            if (LAST && sp == 0) {
                const ShoupConst n0 = ninv[0], n1 = ninv[1];
#pragma unroll
                for (int e = 0; e < dist; e++) {
                    const u64 u = a[e], v = a[e + dist];
                    a[e] = mul_shoup_lazy(u + v, n0, q);
                    a[e + dist] = mul_shoup_lazy(u - v + q2, n1, q);
                }
            } else {
                const ShoupConst w = tw[idx0 + g];
#pragma unroll
                for (int e = 0; e < dist; e++) bfly_inv(a[g * 2 * dist + e], a[g * 2 * dist + e + dist], w, q, q2);
            }
        }
    }
}

// LDS tile of 16 groups x 256 elements; one pad word per 16 elements and 16 pad words per group
// keep both the "stride-16" and the "16 consecutive" access patterns free of bank conflicts.
#define TILE_GROUP 272
#define TILE_WORDS (16 * TILE_GROUP)
__device__ __forceinline__ unsigned tile_at(unsigned grp, unsigned i) { return grp * TILE_GROUP + i + (i >> 4); }

// ---- "block" pass: the last eight forward stages (first eight inverse stages) on 16 contiguous
// blocks of 256 elements per work-group.  grid.x = (N/4096) * batch.
template <int LOGN>
__global__ __launch_bounds__(256) void k_ntt_fwd_blocks(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    __shared__ u64 lds[TILE_WORDS];
    constexpr unsigned TILES = (1u << LOGN) / 4096;
    const unsigned tile = blockIdx.x % TILES, b = blockIdx.x / TILES;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << LOGN);
    const u64 q = T.mod[mi].q;
    const ShoupConst *tw = T.tw_fwd + ((size_t)mi << LOGN);
    const unsigned blk = threadIdx.x >> 4, il = threadIdx.x & 15;
    const unsigned bg = tile * 16 + blk; // block index within the limb
    u64 a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = limb[bg * 256 + il + 16 * k];
    fwd16(a, tw, LOGN - 8, bg, q);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, il + 16 * k)] = a[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = lds[tile_at(blk, 16 * il + k)];
    fwd16(a, tw, LOGN - 4, bg * 16 + il, q);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, 16 * il + k)] = csub(csub(a[k], 2 * q), q);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) limb[bg * 256 + il + 16 * k] = lds[tile_at(blk, il + 16 * k)];
}

template <int LOGN>
__global__ __launch_bounds__(256) void k_ntt_inv_blocks(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    __shared__ u64 lds[TILE_WORDS];
    constexpr unsigned TILES = (1u << LOGN) / 4096;
    const unsigned tile = blockIdx.x % TILES, b = blockIdx.x / TILES;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << LOGN);
    const u64 q = T.mod[mi].q;
    const ShoupConst *tw = T.tw_inv + ((size_t)mi << LOGN);
    const ShoupConst *ninv = T.ninv + 2 * mi;
    const unsigned blk = threadIdx.x >> 4, il = threadIdx.x & 15;
    const unsigned bg = tile * 16 + blk;
    u64 a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, il + 16 * k)] = limb[bg * 256 + il + 16 * k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = lds[tile_at(blk, 16 * il + k)];
    inv16<false>(a, tw, LOGN - 4, bg * 16 + il, q, ninv);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, 16 * il + k)] = a[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = lds[tile_at(blk, il + 16 * k)];
    inv16<false>(a, tw, LOGN - 8, bg, q, ninv);
#pragma unroll
    for (int k = 0; k < 16; k++) limb[bg * 256 + il + 16 * k] = a[k]; // in [0, 2q): the column pass finishes
}

// ---- "column" pass for N = 2^16: stages 0-7 on 256 rows x 16 columns per work-group (element
// (r, c) at r*256 + c).  grid.x = 16 * batch.
__global__ __launch_bounds__(256) void k_ntt_fwd_cols16(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    __shared__ u64 lds[TILE_WORDS];
    const unsigned tile = blockIdx.x & 15, b = blockIdx.x >> 4;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << 16) + tile * 16;
    const u64 q = T.mod[mi].q;
    const ShoupConst *tw = T.tw_fwd + ((size_t)mi << 16);
    const unsigned rl = threadIdx.x >> 4, c = threadIdx.x & 15;
    u64 a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = limb[(rl + 16 * k) * 256 + c];
    fwd16(a, tw, 0, 0, q);
    // LDS index: row r of column c at (r>>4)*272 + (r&15)*17... reuse the tile helper with the
    // roles (group = r>>4, element = (r&15)*16 + c)
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(k, rl * 16 + c)] = a[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = lds[tile_at(rl, k * 16 + c)];
    fwd16(a, tw, 4, rl, q);
#pragma unroll
    for (int k = 0; k < 16; k++) limb[(16 * rl + k) * 256 + c] = a[k]; // in [0, 4q): the block pass finishes
}

__global__ __launch_bounds__(256) void k_ntt_inv_cols16(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    __shared__ u64 lds[TILE_WORDS];
    const unsigned tile = blockIdx.x & 15, b = blockIdx.x >> 4;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << 16) + tile * 16;
    const u64 q = T.mod[mi].q;
    const ShoupConst *tw = T.tw_inv + ((size_t)mi << 16);
    const ShoupConst *ninv = T.ninv + 2 * mi;
    const unsigned rl = threadIdx.x >> 4, c = threadIdx.x & 15;
    u64 a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = limb[(16 * rl + k) * 256 + c];
    inv16<false>(a, tw, 4, rl, q, ninv);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(rl, k * 16 + c)] = a[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = lds[tile_at(k, rl * 16 + c)];
    inv16<true>(a, tw, 0, 0, q, ninv);
#pragma unroll
    for (int k = 0; k < 16; k++) limb[(rl + 16 * k) * 256 + c] = csub(a[k], q);
}

// ---- "column" pass for N = 2^12: stages 0-3 on 16 rows x 256 columns, one thread per column.
__global__ __launch_bounds__(256) void k_ntt_fwd_cols12(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    const unsigned b = blockIdx.x;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << 12);
    const u64 q = T.mod[mi].q;
    const ShoupConst *tw = T.tw_fwd + ((size_t)mi << 12);
    const unsigned c = threadIdx.x;
    u64 a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = limb[k * 256 + c];
    fwd16(a, tw, 0, 0, q);
#pragma unroll
    for (int k = 0; k < 16; k++) limb[k * 256 + c] = a[k];
}

__global__ __launch_bounds__(256) void k_ntt_inv_cols12(u64 *__restrict__ data, DevTables T, LimbBatch lb)
{
    const unsigned b = blockIdx.x;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << 12);
    const u64 q = T.mod[mi].q;
    const ShoupConst *tw = T.tw_inv + ((size_t)mi << 12);
    const ShoupConst *ninv = T.ninv + 2 * mi;
    const unsigned c = threadIdx.x;
    u64 a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = limb[k * 256 + c];
    inv16<true>(a, tw, 0, 0, q, ninv);
#pragma unroll
    for (int k = 0; k < 16; k++) limb[k * 256 + c] = csub(a[k], q);
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
__global__ __launch_bounds__(256) void k_modup(const u64 *__restrict__ x, const u64 *__restrict__ d,
                                               u64 *__restrict__ raised, DevTables T, int level, int L, int K,
                                               int alpha, int logN)
{
    const int j = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int M = L + K, Ma = level + K;
    const int lo = j * alpha, hi = min(lo + alpha, level), na = hi - lo;
    const size_t slot = (size_t)j * alpha + (na - 1);
    u64 y[16];
#pragma unroll 4
    for (int ii = 0; ii < na; ii++) {
        const u64 v = x[((size_t)(lo + ii) << logN) + n];
        y[ii] = mul_shoup(v, T.up_inv[slot * alpha + ii], T.mod[lo + ii].q);
        raised[(((size_t)j * Ma + lo + ii) << logN) + n] = d[((size_t)(lo + ii) << logN) + n];
    }
    for (int a = 0; a < Ma; a++) {
        if (a >= lo && a < hi) continue;
        const int mi = active_mod(a, level, L);
        U128 acc{0, 0};
        for (int ii = 0; ii < na; ii++) mac128(acc, y[ii], T.up_hat[(slot * alpha + ii) * M + mi]);
        raised[(((size_t)j * Ma + a) << logN) + n] = reduce128(acc, T.mod[mi]);
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
    u64 y[16];
    for (int k = 0; k < K; k++)
        y[k] = mul_shoup(u[(((size_t)c * Ma + level + k) << logN) + n], T.dn_inv[k], T.mod[L + k].q);
    for (int i = 0; i < level; i++) {
        U128 acc{0, 0};
        for (int k = 0; k < K; k++) mac128(acc, y[k], T.dn_hat[(size_t)k * L + i]);
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
    UP(tw_fwd) UP(tw_inv) UP(ninv) UP(up_inv) UP(up_hat) UP(dn_inv) UP(dn_hat) UP(dn_pinv) UP(rs_inv)
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
    for (int off = 0; off < total; off += HE_MAXB) {
        const int nb = std::min(HE_MAXB, total - off);
        LimbBatch lb;
        for (int b = 0; b < nb; b++) {
            lb.slot[b] = (uint16_t)slots[off + b];
            lb.mod[b] = (uint8_t)mods[off + b];
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
    KLAUNCH(c, st, KID_MODUP, (double)(2 * level + beta * Ma) * N * 8.0,
            k_modup<<<grid, 256, 0, st>>>(ws + w.x * N, d_ntt, ws + w.raised * N, c->dev, level, c->L, K, c->alpha,
                                          c->logN));
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
    dim3 grid2((unsigned)(N / 256), 2);
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
