// Streaming kernels of the ciphertext operations: limb-wise arithmetic, the tensor product of
// Mult, and the inner product of key switching with the evaluation key.
#pragma once
#include "kernels_ntt.h"

// op 0 add, 1 sub, 2 mul.  Limb l of the flat [limbs][N] buffers uses modulus l % level;
// b_limbs = number of limbs of b before it repeats (pmult: the plaintext has `level` limbs).
// blockIdx.z = operation of a strided batch: the three buffers advance by sa, sb, so limbs.
__global__ __launch_bounds__(256) void k_limbwise(const u64 *__restrict__ a, const u64 *__restrict__ b,
                                                  u64 *__restrict__ out, DevTables T, int op, int level, int b_limbs,
                                                  int logN, int sa, int sb, int so)
{
    const unsigned l = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    a += ((size_t)blockIdx.z * sa) << logN;
    b += ((size_t)blockIdx.z * sb) << logN;
    out += ((size_t)blockIdx.z * so) << logN;
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

// c0 += constant (one residue per limb), c1 copied
__global__ __launch_bounds__(256) void k_addconst(const u64 *__restrict__ a, u64 *__restrict__ out, DevTables T,
                                                  ScalarArgs sc, int level, int logN)
{
    const unsigned l = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const u64 v = a[((size_t)l << logN) + n];
    const unsigned ll = l % (2 * level); // stacked ciphertexts: c0 limbs first, then c1
    out[((size_t)l << logN) + n] = ll < (unsigned)level ? csub(v + sc.s[ll].w, T.mod[ll].q) : v;
}

// Tensor product: d0 = a0 b0, d1 = a0 b1 + a1 b0 -> out (may alias A or B); d2 = a1 b1 -> d2.
// blockIdx.z = operation of a batch: ciphertexts 2*level limbs apart, d2 buffers d2_stride limbs apart.
__global__ __launch_bounds__(256) void k_tensor(const u64 *A, const u64 *B, u64 *out, u64 *__restrict__ d2,
                                                DevTables T, int level, int logN, int d2_stride)
{
    const unsigned i = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const ModConst m = T.mod[i];
    const size_t ct_off = ((size_t)blockIdx.z * 2 * level) << logN;
    A += ct_off, B += ct_off, out += ct_off;
    d2 += ((size_t)blockIdx.z * d2_stride) << logN;
    const size_t o0 = ((size_t)i << logN) + n, o1 = ((size_t)(level + i) << logN) + n;
    const u64 a0 = A[o0], a1 = A[o1], b0 = B[o0], b1 = B[o1];
    u64 r0, r1, r2;
    if (m.qd != 0.0) {
        const double x0 = u2d(a0), x1 = u2d(a1), y0 = u2d(b0), y1 = u2d(b1);
        r0 = fp_canon(fp_mulmod(x0, y0, m.qd, m.qinvd), m.qd, m.qinvd);
        r1 = fp_canon(fp_mulmod(x0, y1, m.qd, m.qinvd) + fp_mulmod(x1, y0, m.qd, m.qinvd), m.qd, m.qinvd);
        r2 = fp_canon(fp_mulmod(x1, y1, m.qd, m.qinvd), m.qd, m.qinvd);
    } else {
        U128 acc{0, 0};
        mac128(acc, a0, b1);
        mac128(acc, a1, b0);
        r0 = mul_mod(a0, b0, m), r1 = reduce128(acc, m), r2 = mul_mod(a1, b1, m);
    }
    out[o0] = r0;
    out[o1] = r1;
    d2[o0] = r2;
}

// Inner product with the evaluation key on active limb a = blockIdx.y:
// u[c][a][n] = sum_j D_j[a][pi_g(n)] * evk[j][c][mod(a)][n], where D_j[a] is the raised digit
// (raised[j][a]) outside digit j and the NTT-domain input d[a] inside it.
// blockIdx.z = operation of a batch (same key for all): raised / u buffers ws_stride limbs apart, d
// buffers d_stride limbs apart.
__global__ __launch_bounds__(256) void k_inner(const u64 *__restrict__ raised, const u64 *__restrict__ d,
                                               const u64 *__restrict__ evk, u64 *__restrict__ u, DevTables T,
                                               int level, int L, int K, int alpha, int beta, unsigned g, int logN,
                                               int ws_stride, int d_stride)
{
    const int a = blockIdx.y;
    raised += ((size_t)blockIdx.z * ws_stride) << logN;
    u += ((size_t)blockIdx.z * ws_stride) << logN;
    d += ((size_t)blockIdx.z * d_stride) << logN;
    const unsigned n = blockIdx.x * 256 + threadIdx.x;
    const int M = L + K, Ma = level + K;
    const int mi = active_mod(a, level, L);
    const unsigned src = g == 1 ? n : galois_index(n, g, logN);
    const int own = a < level ? a / alpha : -1;
    const ModConst m = T.mod[mi];
    u64 r0, r1;
    if (m.qd != 0.0) {
        double acc0 = 0.0, acc1 = 0.0;
        for (int j = 0; j < beta; j++) {
            const u64 *dj = j == own ? d + ((size_t)a << logN) : raised + (((size_t)j * Ma + a) << logN);
            const double dv = u2d(dj[src]);
            acc0 += fp_mulmod(dv, u2d(evk[((((size_t)j * 2 + 0) * M + mi) << logN) + n]), m.qd, m.qinvd);
            acc1 += fp_mulmod(dv, u2d(evk[((((size_t)j * 2 + 1) * M + mi) << logN) + n]), m.qd, m.qinvd);
            if ((j & 3) == 3) {
                acc0 = fp_reduce(acc0, m.qd, m.qinvd);
                acc1 = fp_reduce(acc1, m.qd, m.qinvd);
            }
        }
        r0 = fp_canon(acc0, m.qd, m.qinvd);
        r1 = fp_canon(acc1, m.qd, m.qinvd);
    } else {
        U128 acc0{0, 0}, acc1{0, 0};
        for (int j = 0; j < beta; j++) {
            const u64 *dj = j == own ? d + ((size_t)a << logN) : raised + (((size_t)j * Ma + a) << logN);
            const u64 dv = dj[src];
            mac128(acc0, dv, evk[((((size_t)j * 2 + 0) * M + mi) << logN) + n]);
            mac128(acc1, dv, evk[((((size_t)j * 2 + 1) * M + mi) << logN) + n]);
        }
        r0 = reduce128(acc0, m);
        r1 = reduce128(acc1, m);
    }
    u[(((size_t)0 * Ma + a) << logN) + n] = r0;
    u[(((size_t)1 * Ma + a) << logN) + n] = r1;
}
