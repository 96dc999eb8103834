// Streaming kernels of the ciphertext operations: limb-wise arithmetic and the tensor product of Mult.
// Not templates: included by device.hip alone.
#pragma once
#include "arith.h"

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

// out = sum_k ct_k * pt_k: `count` ciphertexts [2][level][N], each times its own plaintext [level][N]
// (the inner sums of a baby-step/giant-step matrix product, one pass instead of count products and sums).
#define PMULT_SUM_MAX 64
struct PmultSumArgs {
    const u64 *ct[PMULT_SUM_MAX];
    const u64 *pt[PMULT_SUM_MAX];
    int count;
};
__global__ __launch_bounds__(256) void k_pmult_sum(PmultSumArgs a, u64 *__restrict__ out, DevTables T, int level, int logN)
{
    const unsigned l = blockIdx.y, i = l % level;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t oc = ((size_t)l << logN) + n, op = ((size_t)i << logN) + n;
    const ModConst m = T.mod[i];
    u64 r;
    if (m.qd != 0.0) {
        double acc = 0.0;
        for (int k = 0; k < a.count; k++) {
            acc += fp_mulmod(u2d(a.ct[k][oc]), u2d(a.pt[k][op]), m.qd, m.qinvd);
            if ((k & 3) == 3) acc = fp_reduce(acc, m.qd, m.qinvd);
        }
        r = fp_canon(acc, m.qd, m.qinvd);
    } else {
        U128 acc{0, 0};
        u64 part = 0;
        for (int k = 0; k < a.count; k++) {
            mac128(acc, a.ct[k][oc], a.pt[k][op]);
            if ((k & 7) == 7) { // eight products of two residues below 2^62 fit 128 bits
                part = csub(part + reduce128(acc, m), m.q);
                acc = U128{0, 0};
            }
        }
        r = csub(part + reduce128(acc, m), m.q);
    }
    out[oc] = r;
}

// Tensor product: d0 = a0 b0, d1 = a0 b1 + a1 b0 -> out (may alias A or B); d2 = a1 b1 -> d2.
// blockIdx.z = operation of a batch: input ciphertexts 2*level limbs apart, out buffers out_stride and d2
// buffers d2_stride limbs apart.
__global__ __launch_bounds__(256) void k_tensor(const u64 *A, const u64 *B, u64 *out, u64 *__restrict__ d2,
                                                DevTables T, int level, int logN, int d2_stride, int out_stride)
{
    const unsigned i = blockIdx.y;
    const size_t n = (size_t)blockIdx.x * 256 + threadIdx.x;
    const ModConst m = T.mod[i];
    const size_t ct_off = ((size_t)blockIdx.z * 2 * level) << logN;
    A += ct_off, B += ct_off;
    out += ((size_t)blockIdx.z * out_stride) << logN;
    d2 += ((size_t)blockIdx.z * d2_stride) << logN;
    const size_t o0 = ((size_t)i << logN) + n, o1 = ((size_t)(level + i) << logN) + n;
    // every operand is read once and every result is for a later launch: streamed past the caches
    const u64 a0 = __builtin_nontemporal_load(A + o0), a1 = __builtin_nontemporal_load(A + o1);
    const u64 b0 = __builtin_nontemporal_load(B + o0), b1 = __builtin_nontemporal_load(B + o1);
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
    __builtin_nontemporal_store(r0, out + o0);
    __builtin_nontemporal_store(r1, out + o1);
    __builtin_nontemporal_store(r2, d2 + o0);
}
