// Negacyclic NTT kernels with fused base-conversion prologues and ModDown/rescale epilogues.
//
// Forward transform = decimation in time with the powers of psi in bit-reversed order; stage s
// (s = 0 .. logN-1) pairs elements N/2^(s+1) apart and uses twiddle index 2^s + (j >> (logN-s)).
// Each thread keeps 16 elements in registers and runs four stages on them (a radix-16 step);
// between steps the 256-thread work-group exchanges data through LDS.  A limb of N = 2^16 takes
// two kernels: the column pass (stages 0-7 on 16 columns x 256 rows, row stride 256 elements,
// 128-byte global segments) and the block pass (stages 8-15 on 16 contiguous blocks of 256).
// N = 2^17 keeps the two kernels: its column pass runs nine stages on 512 rows (32 elements per thread).
// N = 2^12 uses a four-stage column pass (one thread per column) and the same block pass.
// The inverse runs the block pass first and the column pass last.
//
// Fusions, all bit-identical to the unfused steps:
//  * the forward column pass can build its input on the fly: ModUp (sum over the digit's limbs of
//    y_i * (D/q_i mod t)), ModDown (sum over the special limbs of y_k * (P/p_k mod q_i)) or the
//    centred residue of a dropped limb (rescale);
//  * the inverse column pass can fold (D/q_i)^-1 or (P/p_k)^-1 into its 1/N scaling, so it emits
//    the y values those sums need;
//  * the forward block pass can finish ModDown / rescale: out = (u - ntt) * const + addend;
//  * ModDown followed by rescale takes one transform per limb instead of two: with t the centred dropped
//    limb of the ModDown result, NTT(r) P^-1 + NTT(t) = NTT(r + P t) P^-1, so the column pass transforms
//    r + P t and the block pass finishes out = (u - ntt) (P q_l)^-1 + d q_l^-1.
#pragma once
#include "arith.h"

// limbs per launch: the table below travels as a kernel argument (10 KiB); large launches matter, halving this
// costs the conversion passes 11-14 %
#ifndef HE_MAXB
#define HE_MAXB 2048
#endif
// operations per launch that can carry a key, a Galois element, a level and pointers of their own
#ifndef HE_OPS_MAX
#define HE_OPS_MAX 32
#endif
// A launch works on up to HE_MAXB limbs: limb b is written at dst + slot[b]*N, read (inverse block
// pass only) at src + src[b]*N, and uses modulus index mod[b].
struct LimbBatch {
    uint16_t slot[HE_MAXB];
    uint16_t src[HE_MAXB];
    uint8_t mod[HE_MAXB];
};

enum { PRO_LOAD = 0, PRO_MODUP = 1, PRO_MODDOWN = 2, PRO_RESCALE = 3, PRO_MODDOWN_RS = 4 };
__host__ __device__ constexpr bool pro_is_moddown(int pro) { return pro == PRO_MODDOWN || pro == PRO_MODDOWN_RS; }
enum { SCALE_NONE = 0, SCALE_MODUP = 1, SCALE_MODDOWN = 2 };
enum { EPI_STORE = 0, EPI_FIN = 1 };

// Batches: `count` independent ciphertexts are laid out with fixed strides (in limbs); a limb's slot
// is op * stride + local index, so op = slot / stride and the local index keeps its single-op meaning.
struct ConvArgs {
    const u64 *src; // ModUp: y limbs [level][N]; ModDown: u [2][level+K][N]; rescale: t [2][N]
    int level, L, K, alpha;
    int dst_stride; // limbs between two operations in the buffer being transformed
    int src_stride; // limbs between two operations in src
    // ModDown + rescale: the dropped limb of component c (coefficient domain) at src2 + (c*level + level-1) limbs
    const u64 *src2;
    int src2_stride;
    // centred-limb prologue (rescale, ModRaise): modulus index of the source limb, limbs per component in dst
    int rs_mod, rs_nl;
    // Corrected conversions selected: ModUp takes out floor(sum_i y_i / q_i) D, ModDown rint(sum_k y'_k / p_k) P,
    // the sums in double precision, one rounding per operation, sources in order.
    int exact;
    // Operations of one launch at different levels (mixed-level rotations): op_level[o] != 0 is the level of
    // operation o, while `level` stays the level the buffers are laid out for (the largest of the launch).
    uint8_t op_level[HE_OPS_MAX];
};
// level of the operation that owns destination slot `slot`
__device__ __forceinline__ int conv_op_level(const ConvArgs &cv, unsigned slot)
{
    const unsigned op = slot / (unsigned)cv.dst_stride;
    const int l = op < HE_OPS_MAX ? cv.op_level[op] : 0;
    return l ? l : cv.level;
}

// A limb's slot within its operation decodes as component c = slot / nl, limb i = slot % nl.
struct FinArgs {
    const u64 *u;   // minuend limbs, component stride u_cstride limbs
    u64 *out;       // component stride out_cstride limbs
    const u64 *add; // mode 2: c0 limbs [nl][N], read through the automorphism index map; mode 3: component
                    // stride add_cstride limbs
    const u64 *self; // mode 4: [2][nl][N] per operation, self_stride limbs apart
    const ShoupConst *cst, *cst2;
    const double *cst_d, *cst2_d;
    // mode 0: no addend; 1: add what `out` holds; 2: add sigma_g(c0) to component 0; 3: add the limb of `add`
    // times cst2 (cst2 == nullptr: as it is); 4: as 2, plus the limb of `self` (rotate-and-add)
    int u_cstride, out_cstride, add_cstride, self_stride, nl, mode;
    unsigned g;
    int hoisted; // operation o writes to out[o] and uses Galois element g[o] of the HoistOuts argument
    int dst_stride, u_stride, out_stride, add_stride; // limbs between two operations in each buffer
};

__device__ __forceinline__ int active_mod(int a, int level, int L) { return a < level ? a : L + (a - level); }

// NTT-domain index of the automorphism sigma_g: out[k] = in[k'] with
// 2 brv(k') + 1 = (2 brv(k) + 1) g mod 2N.
__device__ __forceinline__ unsigned galois_index(unsigned k, unsigned g, int logN)
{
    const unsigned b = __brev(k) >> (32 - logN);
    const unsigned e = ((2 * b + 1) * g) & ((2u << logN) - 1);
    return __brev((e - 1) >> 1) >> (32 - logN);
}

// ---- prologues: element `pos` of the limb the column pass is about to transform ----------------------

template <int NSMAX> struct ConvSetup {
    const u64 *sp[NSMAX];         // source limbs; entries past the real count repeat entry 0 with zero constants
    double cd[NSMAX], cdh[NSMAX]; // constants as balanced doubles (cdh: constant * 2^31)
    u64 ci[NSMAX], cp[NSMAX];     // constants as residues and their companions floor(c 2^64 / t) (integer targets)
    // ModDown: source digit s counts as y - p_s when y > hs[s]; each such digit subtracts P mod q_i
    u64 hs[NSMAX];
    u64 pm_i;
    double pm_d;
    double r50;  // ModDown, SPLIT 2: 2^50 mod q
    // rescale
    u64 ql, half;
    double qld;
    const u64 *tp; // ModDown + rescale: the dropped limb of this component
    // corrected conversions: 1.0 / (double)modulus of source s (0 past the real count), D mod t (ModUp)
    double rq[NSMAX];
    u64 dm_i;
    double dm_d;
};

// slot = position of the limb in the destination buffer; mi = its modulus index
template <int PRO, int NSMAX, int LOGN>
__device__ __forceinline__ ConvSetup<NSMAX> conv_setup(const ConvArgs &cv, const DevTables &T, unsigned slot, unsigned mi)
{
    ConvSetup<NSMAX> S;
    S.ql = S.half = 0;
    S.qld = 0.0;
    S.pm_i = 0;
    S.pm_d = 0.0;
    S.r50 = 0.0;
    S.tp = nullptr;
    S.dm_i = 0;
    S.dm_d = 0.0;
    const int M = cv.L + cv.K, Ma = cv.level + cv.K;
    const int op_level = conv_op_level(cv, slot);
    const unsigned op = slot / (unsigned)cv.dst_stride;
    slot -= op * (unsigned)cv.dst_stride;
    const u64 *src = cv.src + (((size_t)op * cv.src_stride) << LOGN);
#pragma unroll
    for (int s = 0; s < NSMAX; s++) {
        S.sp[s] = src;
        S.ci[s] = S.cp[s] = 0;
        S.cd[s] = S.cdh[s] = 0.0;
        S.hs[s] = ~(u64)0;
        S.rq[s] = 0.0;
    }
    if (PRO == PRO_MODUP) {
        const int j = slot / Ma;
        const int lo = j * cv.alpha, hi = min(lo + cv.alpha, op_level);
        const int ns = hi - lo;
        const size_t cs = ((size_t)j * cv.alpha + (ns - 1)) * cv.alpha;
#pragma unroll
        for (int s = 0; s < NSMAX; s++) {
            const bool on = s < ns;
            const size_t ci = (cs + (on ? s : 0)) * M + mi;
            S.sp[s] = src + ((size_t)(lo + (on ? s : 0)) << LOGN);
            S.ci[s] = on ? T.up_hat[ci] : 0;
            S.cp[s] = on ? T.up_hat_p[ci] : 0;
            S.cd[s] = on ? T.up_hat_d[ci] : 0.0;
            S.cdh[s] = on ? T.up_hat_dh[ci] : 0.0;
            S.rq[s] = on ? T.rq[lo + s] : 0.0;
        }
        S.dm_i = T.up_dmod[((size_t)j * cv.alpha + (ns - 1)) * M + mi];
        S.dm_d = T.up_dmod_d[((size_t)j * cv.alpha + (ns - 1)) * M + mi];
    } else if (pro_is_moddown(PRO)) {
        const int c = slot / cv.level, i = slot % cv.level;
#pragma unroll
        for (int s = 0; s < NSMAX; s++) {
            const bool on = s < cv.K;
            const size_t ci = (size_t)(on ? s : 0) * cv.L + i;
            S.sp[s] = src + (((size_t)c * Ma + cv.level + (on ? s : 0)) << LOGN);
            S.ci[s] = on ? T.dn_hat[ci] : 0;
            S.cd[s] = on ? T.dn_hat_d[ci] : 0.0;
            S.cdh[s] = on ? T.dn_hat_dh[ci] : 0.0;
            S.hs[s] = on ? (T.mod[cv.L + s].q - 1) / 2 : ~(u64)0;
            S.rq[s] = on ? T.rq[cv.L + s] : 0.0;
        }
        S.pm_i = T.dn_pmod[i];
        S.pm_d = T.dn_pmod_d[i];
        S.r50 = T.dn_r50_d[i];
        if (PRO == PRO_MODDOWN_RS) {
            S.tp = cv.src2 + (((size_t)op * cv.src2_stride + (size_t)c * cv.level + cv.level - 1) << LOGN);
            S.ql = T.mod[cv.level - 1].q;
            S.half = (S.ql - 1) / 2;
            S.qld = T.mod[cv.level - 1].qd;
        }
    } else if (PRO == PRO_RESCALE) {
        const int c = slot / cv.rs_nl;
        S.sp[0] = src + ((size_t)c << LOGN);
        S.ql = T.mod[cv.rs_mod].q;
        S.half = (S.ql - 1) / 2;
        S.qld = T.mod[cv.rs_mod].qd;
    }
    return S;
}

// SPLIT 1: the sources may be 2^50 or larger, so an FP64 target splits each at bit 31; SPLIT 2 (ModDown): it folds
// each at bit 50 instead, y = yh 2^50 + yl = yh r50 + yl modulo q with r50 = 2^50 mod q small (one product, not two).  TINT (ModDown + rescale):
// the dropped limb is 2^50 or larger and is reduced with integers first; a template parameter rather than a
// run-time branch, because the integer code would cost every launch 100 registers.
template <int PRO, int SPLIT, bool TINT, bool EX, int NSMAX>
__device__ __forceinline__ double conv_get(const ConvSetup<NSMAX> &S, const ArithFp &ar, const ModConst &m, unsigned pos)
{
    if (PRO == PRO_RESCALE) {
        const u64 tv = S.sp[0][pos];
        if (S.qld != 0.0) return u2d(tv) - (tv > S.half ? S.qld : 0.0); // centred value, |v| < q_last / 2
        const bool neg = tv > S.half; // q_last >= 2^50: reduce the magnitude with integers first
        const double w = u2d(reduce64(neg ? S.ql - tv : tv, m));
        return neg ? -w : w;
    }
    double acc = 0.0, sv = 0.0;
    int neg = 0; // ModDown: number of digits that stand for y - p
#pragma unroll
    for (int s = 0; s < NSMAX; s++) {
        const u64 y = S.sp[s][pos];
        const bool ng = pro_is_moddown(PRO) && y > S.hs[s];
        if (pro_is_moddown(PRO)) neg += ng ? 1 : 0;
        if (EX) { // the source as a fraction of its modulus (ModDown: of the centred digit)
            const double yd = !pro_is_moddown(PRO) ? (SPLIT ? (double)y : u2d(y))
                              : ng               ? -(double)(2 * S.hs[s] + 1 - y)
                                                 : (double)y;
            sv = sv + yd * S.rq[s];
        }
        if (!SPLIT)
            acc += ar.mulmod(u2d(y), S.cd[s]);
        else if (SPLIT == 2) {
            // y = yh 2^50 + yl = yh r50 + yl modulo q: below 2^50 + 2^10 2^40, exact, and one product instead of two
            const double yh = (double)(unsigned)(y >> 50), yl = u2d(y & 0x3FFFFFFFFFFFFull);
            acc += ar.mulmod(__builtin_fma(yh, S.r50, yl), S.cd[s]);
        } else {
            const double yh = (double)(unsigned)(y >> 31), yl = (double)(unsigned)(y & 0x7FFFFFFFu);
            acc += ar.mulmod(yh, S.cdh[s]) + ar.mulmod(yl, S.cd[s]);
        }
        if ((s & 3) == 3 && s + 1 < NSMAX) acc = ar.reduce(acc);
    }
    if (PRO == PRO_MODUP && EX) acc -= __builtin_floor(sv) * S.dm_d; // at most (sources - 1) D
    if (pro_is_moddown(PRO)) {
        if (NSMAX > 4) acc = ar.reduce(acc);
        // p_s * (P/p_s) = P for every centred digit; corrected: plus rint(sv) P, together between 0 and K times P
        acc -= ((double)neg + (EX ? __builtin_rint(sv) : 0.0)) * S.pm_d;
    }
    if (PRO == PRO_MODDOWN_RS) { // + P t with t the centred dropped limb
        const u64 tv = S.tp[pos];
        double tc;
        if (!TINT)
            tc = u2d(tv) - (tv > S.half ? S.qld : 0.0);
        else {
            const bool tneg = tv > S.half;
            const double w = u2d(reduce64(tneg ? S.ql - tv : tv, m));
            tc = tneg ? -w : w;
        }
        acc += ar.mulmod(tc, S.pm_d);
    }
    return acc;
}

template <int PRO, int SPLIT, bool TINT, bool EX, int NSMAX>
__device__ __forceinline__ u64 conv_get(const ConvSetup<NSMAX> &S, const ArithInt &, const ModConst &m, unsigned pos)
{
    if (PRO == PRO_RESCALE) {
        const u64 tv = S.sp[0][pos];
        const bool neg = tv > S.half;
        const u64 w = reduce64(neg ? S.ql - tv : tv, m);
        return neg ? (w ? m.q - w : 0) : w;
    }
    if (PRO == PRO_MODUP && NSMAX <= 4) {
        // up to four products in [0, 4q) each, summed without reduction: below 16q < 2^64
        u64 lazy = 0;
        double sv = 0.0;
#pragma unroll
        for (int s = 0; s < NSMAX; s++) {
            const u64 y = S.sp[s][pos];
            lazy += mul_shoup_sloppy(y, ShoupConst{S.ci[s], S.cp[s]}, m.q);
            if (EX) sv = sv + (double)y * S.rq[s];
        }
        lazy = csub(lazy, 8 * m.q); // the range the transform takes
        if (EX) {
            const u64 r = csub(csub(csub(lazy, 4 * m.q), 2 * m.q), m.q);
            return csub(r + m.q - mul_mod((u64)__builtin_floor(sv), S.dm_i, m), m.q);
        }
        return lazy;
    }
    U128 acc{0, 0};
    double sv = 0.0;
    u64 corr = 0; // ModDown: every digit that stands for y - p takes out one P
#pragma unroll
    for (int s = 0; s < NSMAX; s++) {
        const u64 y = S.sp[s][pos];
        mac128(acc, y, S.ci[s]);
        const bool ng = pro_is_moddown(PRO) && y > S.hs[s];
        if (pro_is_moddown(PRO)) corr = csub(corr + (ng ? S.pm_i : 0), m.q);
        if (EX) {
            const double yd = ng ? -(double)(2 * S.hs[s] + 1 - y) : (double)y;
            sv = sv + yd * S.rq[s];
        }
    }
    u64 r = reduce128(acc, m);
    if (PRO == PRO_MODUP && EX) r = csub(r + m.q - mul_mod((u64)__builtin_floor(sv), S.dm_i, m), m.q);
    if (pro_is_moddown(PRO)) {
        if (EX) { // the correction rint(sv), at most NSMAX / 2 in size, times P
            const int v = (int)__builtin_rint(sv);
#pragma unroll
            for (int t = 0; t < NSMAX / 2; t++) {
                if (t < v) corr = csub(corr + S.pm_i, m.q);
                if (t < -v) corr = csub(corr + m.q - S.pm_i, m.q);
            }
        }
        r = csub(r + m.q - corr, m.q);
    }
    if (PRO == PRO_MODDOWN_RS) {
        const u64 tv = S.tp[pos];
        const bool tneg = tv > S.half;
        const u64 pw = mul_mod(reduce64(tneg ? S.ql - tv : tv, m), S.pm_i, m);
        r = tneg ? csub(r + m.q - pw, m.q) : csub(r + pw, m.q);
    }
    return r;
}

// ---- epilogue: what the forward block pass does with a finished (canonical) NTT value ---------------------

#define HOIST_OUT_MAX HE_OPS_MAX
struct HoistOuts {
    u64 *out[HOIST_OUT_MAX];
    unsigned g[HOIST_OUT_MAX];
    // mixed-level rotations: the operation's input c0 limbs (mode 2 addend) and the limbs per component of its
    // output; null / 0: the launch-wide values of FinArgs
    const u64 *add[HOIST_OUT_MAX];
    uint8_t cstride[HOIST_OUT_MAX];
};

// Operands of the epilogue for one output: issued before the transform so that the loads overlap it.
struct FinOperands {
    u64 uv, av;
};
template <int LOGN>
__device__ __forceinline__ FinOperands fin_load(const FinArgs &fa, const HoistOuts &ho, const DevTables &T, unsigned slot,
                                                unsigned pos)
{
    const unsigned op = slot / (unsigned)fa.dst_stride;
    slot -= op * (unsigned)fa.dst_stride;
    const unsigned c = slot / fa.nl, i = slot % fa.nl;
    FinOperands o;
    o.uv = __builtin_nontemporal_load(fa.u + ((((size_t)op * fa.u_stride + (size_t)c * fa.u_cstride + i) << LOGN) + pos));
    o.av = 0;
    if (fa.mode == 1)
        o.av = fa.out[(((size_t)op * fa.out_stride + (size_t)c * fa.out_cstride + i) << LOGN) + pos];
    else if (fa.mode == 2 && c == 0) {
        const u64 *add = fa.hoisted && ho.add[op] ? ho.add[op] : fa.add + (((size_t)op * fa.add_stride) << LOGN);
        o.av = add[((size_t)i << LOGN) + galois_index(pos, fa.hoisted ? ho.g[op] : fa.g, LOGN)];
    }
    else if (fa.mode == 3)
        o.av = fa.add[(((size_t)op * fa.add_stride + (size_t)c * fa.add_cstride + i) << LOGN) + pos];
    else if (fa.mode == 4) {
        const u64 sv = fa.self[(((size_t)op * fa.self_stride + (size_t)c * fa.nl + i) << LOGN) + pos];
        const u64 rv = c == 0 ? fa.add[(((size_t)op * fa.add_stride + i) << LOGN) + galois_index(pos, fa.g, LOGN)] : 0;
        o.av = csub(sv + rv, T.mod[i].q);
    }
    return o;
}

// FP: the limb's modulus is on the floating-point path (known from the transform's arithmetic at compile time)
template <int LOGN, bool FP>
__device__ __forceinline__ void fin_store(const FinArgs &fa, const HoistOuts &ho, const DevTables &T, unsigned slot,
                                          unsigned pos, u64 rv, const FinOperands &fo)
{
    const unsigned op = slot / (unsigned)fa.dst_stride;
    slot -= op * (unsigned)fa.dst_stride;
    const unsigned c = slot / fa.nl, i = slot % fa.nl;
    const ModConst m = T.mod[i];
    const unsigned out_cstride = fa.hoisted && ho.cstride[op] ? ho.cstride[op] : (unsigned)fa.out_cstride;
    const size_t o = (((size_t)op * fa.out_stride + (size_t)c * out_cstride + i) << LOGN) + pos;
    const bool scaled = fa.mode == 3 && fa.cst2 != nullptr;
    u64 res;
    if (FP) {
        const double av = scaled ? fp_mulmod(u2d(fo.av), fa.cst2_d[i], m.qd, m.qinvd) : u2d(fo.av);
        res = fp_canon(fp_mulmod(u2d(fo.uv) - u2d(rv), fa.cst_d[i], m.qd, m.qinvd) + av, m.qd, m.qinvd);
    } else {
        const u64 av = scaled ? mul_shoup(fo.av, fa.cst2[i], m.q) : fo.av;
        res = csub(mul_shoup(fo.uv + m.q - rv, fa.cst[i], m.q) + av, m.q);
    }
    __builtin_nontemporal_store(res, (fa.hoisted ? ho.out[op] : fa.out) + o); // a result: nothing in this launch reads it
}

// LDS tile of the block pass: 16 groups x 256 elements; one pad word per 16 elements and 16 pad words per
// group keep both the "stride-16" and the "16 consecutive" access patterns free of bank conflicts.
#define TILE_GROUP 272
// threads per work-group of the block pass: 16 threads per 256-element block
#ifndef BLK_THREADS
#define BLK_THREADS 256
#endif
#define BLK_PER_WG (BLK_THREADS / 16)
__device__ __forceinline__ unsigned tile_at(unsigned grp, unsigned i) { return grp * TILE_GROUP + i + (i >> 4); }
// Exchange through LDS among the 16 lanes that own one 256-element block.  They belong to one wave, and a wave's
// LDS operations execute in order, so no work-group barrier is needed: only the compiler has to be kept from
// moving LDS accesses across this point.
__device__ __forceinline__ void block_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
static_assert(BLK_THREADS % 64 == 0, "a block's 16 lanes must not straddle two waves");
// column pass: row r of column c (0..15).  The 16 lanes of a column group always touch 16 consecutive words,
// so this tile needs no padding: 32 KiB at N = 2^16, five work-groups per compute unit.
#define COL_GROUP 256
__device__ __forceinline__ unsigned col_at(unsigned r, unsigned c) { return (r >> 4) * COL_GROUP + (r & 15) * 16 + c; }

// ---- block pass ---------------------------------------------------------------------------------------------

template <int LOGN, int EPI, class A>
__device__ __forceinline__ void fwd_blocks_body(u64 *__restrict__ limb, const A &ar, u64 *lds, unsigned tile,
                                                const FinArgs &fa, const HoistOuts &ho, const DevTables &T, unsigned slot)
{
    const unsigned blk = threadIdx.x >> 4, il = threadIdx.x & 15;
    const unsigned bg = tile * BLK_PER_WG + blk; // block index within the limb
    typename A::V a[16];
    FinOperands fo[EPI == EPI_FIN ? 16 : 1];
#pragma unroll
    for (int k = 0; k < 16; k++)
        a[k] = ar.load_mid(__builtin_nontemporal_load(limb + bg * 256 + il + 16 * k)); // read once: the column pass wrote it
    if (EPI == EPI_FIN) {
#pragma unroll
        for (int k = 0; k < 16; k++) fo[k] = fin_load<LOGN>(fa, ho, T, slot, bg * 256 + il + 16 * k);
    }
    ar.fwd16(a, LOGN - 8, bg, true);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, il + 16 * k)] = ar.store_mid(a[k]);
    block_sync();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load_mid(lds[tile_at(blk, 16 * il + k)]);
    ar.fwd16(a, LOGN - 4, bg * 16 + il, true);
    block_sync();
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, 16 * il + k)] = ar.store_final(a[k]);
    block_sync();
#pragma unroll
    for (int k = 0; k < 16; k++) {
        const unsigned pos = bg * 256 + il + 16 * k;
        const u64 v = lds[tile_at(blk, il + 16 * k)];
        if (EPI == EPI_FIN)
            fin_store<LOGN, A::IS_FP>(fa, ho, T, slot, pos, v, fo[k]);
        else
            __builtin_nontemporal_store(v, limb + pos);
    }
}

template <int LOGN, class A>
__device__ __forceinline__ void inv_blocks_body(const u64 *in, u64 *limb, const A &ar,
                                                u64 *lds, unsigned tile)
{
    // out of place: part of a conversion, whose batch is far larger than the caches; in place (a plain inverse
    // transform) the column pass that follows finds the stores in the last-level cache
    const bool stream = in != limb;
    const unsigned blk = threadIdx.x >> 4, il = threadIdx.x & 15;
    const unsigned bg = tile * BLK_PER_WG + blk;
    typename A::V a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) {
        const u64 *src = in + bg * 256 + il + 16 * k;
        lds[tile_at(blk, il + 16 * k)] = __builtin_nontemporal_load(src); // read once
    }
    block_sync();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load(lds[tile_at(blk, 16 * il + k)]);
    ar.template inv16<false>(a, LOGN - 4, bg * 16 + il);
    block_sync();
#pragma unroll
    for (int k = 0; k < 16; k++) lds[tile_at(blk, 16 * il + k)] = ar.store_mid(a[k]);
    block_sync();
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load_mid(lds[tile_at(blk, il + 16 * k)]);
    ar.template inv16<false>(a, LOGN - 8, bg);
#pragma unroll
    for (int k = 0; k < 16; k++) { // the column pass finishes
        u64 *dst = limb + bg * 256 + il + 16 * k;
        if (stream)
            __builtin_nontemporal_store(ar.store_mid(a[k]), dst);
        else
            *dst = ar.store_mid(a[k]);
    }
}

// grid.x = (N/4096) * batch
template <int LOGN, int EPI>
__global__ __launch_bounds__(BLK_THREADS, EPI == EPI_FIN ? 4 : 1) void k_ntt_fwd_blocks(u64 *__restrict__ data, DevTables T, LimbBatch lb, FinArgs fa,
                                                                HoistOuts ho)
{
    __shared__ u64 lds[BLK_PER_WG * TILE_GROUP];
    constexpr unsigned TILES = (1u << LOGN) / (256 * BLK_PER_WG);
    const unsigned tile = blockIdx.x % TILES, b = blockIdx.x / TILES;
    const unsigned mi = lb.mod[b], slot = lb.slot[b];
    u64 *limb = data + ((size_t)slot << LOGN);
    if (T.mod[mi].qd != 0.0)
        fwd_blocks_body<LOGN, EPI>(limb, make_fp(T, mi, LOGN), lds, tile, fa, ho, T, slot);
    else
        fwd_blocks_body<LOGN, EPI>(limb, make_int(T, mi, LOGN), lds, tile, fa, ho, T, slot);
}

template <int LOGN>
__global__ __launch_bounds__(BLK_THREADS) void k_ntt_inv_blocks(const u64 *src, u64 *dst,
                                                        DevTables T, LimbBatch lb)
{
    __shared__ u64 lds[BLK_PER_WG * TILE_GROUP];
    constexpr unsigned TILES = (1u << LOGN) / (256 * BLK_PER_WG);
    const unsigned tile = blockIdx.x % TILES, b = blockIdx.x / TILES;
    const unsigned mi = lb.mod[b];
    const u64 *in = src + ((size_t)lb.src[b] << LOGN);
    u64 *limb = dst + ((size_t)lb.slot[b] << LOGN);
    if (T.mod[mi].qd != 0.0)
        inv_blocks_body<LOGN>(in, limb, make_fp(T, mi, LOGN), lds, tile);
    else
        inv_blocks_body<LOGN>(in, limb, make_int(T, mi, LOGN), lds, tile);
}

// ---- column pass, N = 2^16 and 2^17: all rows x 16 columns per work-group (element (r, c) at r*256 + c) ---------
//
// N = 2^16: 256 rows, 16 elements per thread, stages 0-3 then 4-7.  N = 2^17: 512 rows, 32 elements per thread:
// stage 0 pairs the two halves of the rows, each half then takes stages 1-4 as a 16-element step, and after
// the exchange every thread runs stages 5-8 on two groups of 16 consecutive rows.

template <int LOGN> struct ColsGeom {
    static constexpr int ROWS = 1 << (LOGN - 8);
    static constexpr int HALVES = ROWS / 256;          // 16-element register steps per thread and phase
    static constexpr int LDS_WORDS = 16 * COL_GROUP;   // one half of the rows at a time: 32 KiB at either size
};

// the 16 inputs of one thread in rows rl + 16 k + 256 h (plain load or base conversion)
template <int PRO, int SPLIT, bool TINT, bool EX, int NSMAX, class A>
__device__ __forceinline__ void cols_inputs(typename A::V (&a)[16], const u64 *__restrict__ limb, unsigned col0, int h,
                                            const A &ar, const ConvSetup<NSMAX> &S, const ModConst &m)
{
    const unsigned rl = threadIdx.x >> 4, c = threadIdx.x & 15;
#pragma unroll
    for (int k = 0; k < 16; k++) {
        const unsigned pos = (rl + 16 * k + 256 * h) * 256 + col0 + c;
        a[k] = PRO == PRO_LOAD ? ar.load(__builtin_nontemporal_load(limb + pos)) : conv_get<PRO, SPLIT, TINT, EX>(S, ar, m, pos);
    }
}
// second phase of the forward column pass for rows 16 g .. 16 g + 15, held in LDS as group gl.  STREAM: the
// output is a new buffer that a later kernel reads, so it is stored past the sources that stay in L2
template <int S_BASE, bool STREAM, class A>
__device__ __forceinline__ void cols_finish_group(typename A::V (&a)[16], u64 *__restrict__ limb, unsigned col0, unsigned g,
                                                  unsigned gl, const A &ar, const u64 *lds)
{
    const unsigned c = threadIdx.x & 15;
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = ar.load_mid(lds[col_at(16 * gl + k, c)]);
    ar.fwd16(a, S_BASE, g, true);
#pragma unroll
    for (int k = 0; k < 16; k++) { // the block pass finishes
        u64 *dst = limb + (16 * g + k) * 256 + col0 + c;
        if (STREAM)
            __builtin_nontemporal_store(ar.store_mid(a[k]), dst);
        else
            *dst = ar.store_mid(a[k]);
    }
}

template <int LOGN, int PRO, int SPLIT, bool TINT, bool EX, int NSMAX, class A>
__device__ __forceinline__ void fwd_cols_body(u64 *__restrict__ limb, unsigned col0, const A &ar, u64 *lds,
                                              const ConvSetup<NSMAX> &S, const ModConst &m)
{
    constexpr int H = ColsGeom<LOGN>::HALVES;
    const unsigned rl = threadIdx.x >> 4, c = threadIdx.x & 15;
    typename A::V a0[16];
    cols_inputs<PRO, SPLIT, TINT, EX>(a0, limb, col0, 0, ar, S, m);
    if (H == 1) {
        ar.fwd16(a0, 0, 0, PRO != PRO_LOAD);
#pragma unroll
        for (int k = 0; k < 16; k++) lds[col_at(rl + 16 * k, c)] = ar.store_mid(a0[k]);
        __syncthreads();
        cols_finish_group<4, PRO != PRO_LOAD>(a0, limb, col0, rl, rl, ar, lds);
    } else {
        typename A::V a1[16];
        // one half's source loads at a time: 32 outputs x up to 8 sources in flight would not fit the registers
        if (PRO != PRO_LOAD) __builtin_amdgcn_sched_barrier(0);
        cols_inputs<PRO, SPLIT, TINT, EX>(a1, limb, col0, 1, ar, S, m);
        ar.fwd_stage0(a0, a1, PRO != PRO_LOAD);
        ar.fwd16(a0, 1, 0, true);
        ar.fwd16(a1, 1, 1, true);
        // after stage 0 the two halves of the rows are independent: they go through the same 32 KiB of LDS in turn
#pragma unroll
        for (int k = 0; k < 16; k++) lds[col_at(rl + 16 * k, c)] = ar.store_mid(a0[k]);
        __syncthreads();
        cols_finish_group<5, PRO != PRO_LOAD>(a0, limb, col0, rl, rl, ar, lds);
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; k++) lds[col_at(rl + 16 * k, c)] = ar.store_mid(a1[k]);
        __syncthreads();
        cols_finish_group<5, PRO != PRO_LOAD>(a1, limb, col0, rl + 16, rl, ar, lds);
    }
}

// STREAM: the input is the first half of a conversion's inverse transform, read this once only
template <int LOGN, bool STREAM, class A>
__device__ __forceinline__ void inv_cols_body(u64 *__restrict__ limb, unsigned col0, const A &ar, u64 *lds)
{
    constexpr int H = ColsGeom<LOGN>::HALVES;
    const unsigned rl = threadIdx.x >> 4, c = threadIdx.x & 15;
    typename A::V a[H][16];
    // each half of the rows: stages logN-9 .. logN-12 on 16 consecutive rows, exchange through the same 32 KiB of
    // LDS, then stages 3 .. 0 (N = 2^16) or 4 .. 1 (N = 2^17: stage 0 pairs the halves afterwards)
#pragma unroll
    for (int h = 0; h < H; h++) {
        const unsigned g = rl + 16 * h;
#pragma unroll
        for (int k = 0; k < 16; k++) {
            const u64 *src = limb + (16 * g + k) * 256 + col0 + c;
            a[h][k] = ar.load_mid(STREAM ? __builtin_nontemporal_load(src) : *src);
        }
        ar.template inv16<false>(a[h], H + 3, g);
        if (h > 0) __syncthreads(); // the previous half has been read back by every thread
#pragma unroll
        for (int k = 0; k < 16; k++) lds[col_at(16 * rl + k, c)] = ar.store_mid(a[h][k]);
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; k++) a[h][k] = ar.load_mid(lds[col_at(rl + 16 * k, c)]);
        if (H == 1)
            ar.template inv16<true>(a[h], 0, 0);
        else
            ar.template inv16<false>(a[h], 1, h);
    }
    if (H == 2) ar.inv_stage0_last(a[0], a[H - 1]);
#pragma unroll
    for (int h = 0; h < H; h++)
#pragma unroll
        for (int k = 0; k < 16; k++) limb[(rl + 16 * k + 256 * h) * 256 + col0 + c] = ar.store_final(a[h][k]);
}

// column pass of limb b of the launch (the arithmetic path and the prologue's variant follow from its modulus)
template <int LOGN, int PRO, int NSMAX, bool EX>
__device__ __forceinline__ void fwd_cols_limb(u64 *__restrict__ data, const DevTables &T, const LimbBatch &lb,
                                              const ConvArgs &cv, unsigned tile, unsigned b, u64 *lds)
{
    const unsigned mi = lb.mod[b], slot = lb.slot[b];
    u64 *limb = data + ((size_t)slot << LOGN);
    const ModConst m = T.mod[mi];
    const ConvSetup<NSMAX> S = conv_setup<PRO, NSMAX, LOGN>(cv, T, slot, mi);
    const bool split = PRO == PRO_MODUP ? T.up_split != 0 : pro_is_moddown(PRO) ? T.dn_split != 0 : false;
    const bool fold = pro_is_moddown(PRO) && !EX && NSMAX <= 4 && T.dn_fold != 0; // the common case only: each variant costs code
    const bool tint = PRO == PRO_MODDOWN_RS && S.qld == 0.0; // dropped limb on the integer path
    if (m.qd == 0.0)
        fwd_cols_body<LOGN, PRO, 0, false, EX>(limb, tile * 16, make_int(T, mi, LOGN), lds, S, m);
    else if (PRO == PRO_MODDOWN_RS && tint) {
        if (split)
            fwd_cols_body<LOGN, PRO, 1, PRO == PRO_MODDOWN_RS, EX>(limb, tile * 16, make_fp(T, mi, LOGN), lds, S, m);
        else
            fwd_cols_body<LOGN, PRO, 0, PRO == PRO_MODDOWN_RS, EX>(limb, tile * 16, make_fp(T, mi, LOGN), lds, S, m);
    } else if (fold)
        fwd_cols_body<LOGN, PRO, pro_is_moddown(PRO) && !EX && NSMAX <= 4 ? 2 : 0, false, EX>(limb, tile * 16, make_fp(T, mi, LOGN), lds, S, m);
    else if (split)
        fwd_cols_body<LOGN, PRO, 1, false, EX>(limb, tile * 16, make_fp(T, mi, LOGN), lds, S, m);
    else
        fwd_cols_body<LOGN, PRO, 0, false, EX>(limb, tile * 16, make_fp(T, mi, LOGN), lds, S, m);
}
template <int LOGN, int PRO, int NSMAX, bool EX>
__device__ __forceinline__ void fwd_cols_kernel(u64 *__restrict__ data, const DevTables &T, const LimbBatch &lb,
                                                const ConvArgs &cv)
{
    __shared__ u64 lds[ColsGeom<LOGN>::LDS_WORDS];
    fwd_cols_limb<LOGN, PRO, NSMAX, EX>(data, T, lb, cv, blockIdx.x & 15, blockIdx.x >> 4, lds);
}

// ModUp column pass for two limbs per work-group (N = 2^16; grid.x = 16 * ceil(batch / 2)): limbs 2i and 2i+1 of
// the launch.  When both are floating-point targets of the same digit of the same operation (the usual case:
// the targets of a digit follow each other in a launch), the digit's source limbs are read and converted to
// doubles once and both base conversions are formed from them, term by term as in conv_get; every target
// otherwise re-reads the same source tile through L2.  Any other pair is processed one limb after the other.
template <int NSMAX, bool EX>
__global__ __launch_bounds__(256) void k_ntt_fwd_cols16_modup2(u64 *__restrict__ data, DevTables T, LimbBatch lb,
                                                                ConvArgs cv, int nb)
{
    __shared__ u64 lds[ColsGeom<16>::LDS_WORDS];
    const unsigned tile = blockIdx.x & 15, b0 = (blockIdx.x >> 4) * 2, b1 = b0 + 1;
    if (b1 >= (unsigned)nb) {
        fwd_cols_limb<16, PRO_MODUP, NSMAX, EX>(data, T, lb, cv, tile, b0, lds);
        return;
    }
    const unsigned mi0 = lb.mod[b0], mi1 = lb.mod[b1], slot0 = lb.slot[b0], slot1 = lb.slot[b1];
    const ConvSetup<NSMAX> S0 = conv_setup<PRO_MODUP, NSMAX, 16>(cv, T, slot0, mi0);
    const ConvSetup<NSMAX> S1 = conv_setup<PRO_MODUP, NSMAX, 16>(cv, T, slot1, mi1);
    bool same = T.up_split == 0 && T.mod[mi0].qd != 0.0 && T.mod[mi1].qd != 0.0;
#pragma unroll
    for (int s = 0; s < NSMAX; s++) same = same && S0.sp[s] == S1.sp[s];
    if (!same) {
        fwd_cols_limb<16, PRO_MODUP, NSMAX, EX>(data, T, lb, cv, tile, b0, lds);
        __syncthreads(); // the first limb's second phase has read the tile
        fwd_cols_limb<16, PRO_MODUP, NSMAX, EX>(data, T, lb, cv, tile, b1, lds);
        return;
    }
    const ArithFp ar0 = make_fp(T, mi0, 16), ar1 = make_fp(T, mi1, 16);
    const unsigned rl = threadIdx.x >> 4, c = threadIdx.x & 15, col0 = tile * 16;
    double a0[16], a1[16];
#pragma unroll
    for (int k = 0; k < 16; k++) {
        const unsigned pos = (rl + 16 * k) * 256 + col0 + c;
        double acc0 = 0.0, acc1 = 0.0, sv = 0.0;
#pragma unroll
        for (int s = 0; s < NSMAX; s++) {
            const double y = u2d(S0.sp[s][pos]);
            if (EX) sv = sv + y * S0.rq[s];
            acc0 += ar0.mulmod(y, S0.cd[s]);
            acc1 += ar1.mulmod(y, S1.cd[s]);
            if ((s & 3) == 3 && s + 1 < NSMAX) acc0 = ar0.reduce(acc0), acc1 = ar1.reduce(acc1);
        }
        if (EX) { // one estimate of the multiple of D for both targets
            const double v = __builtin_floor(sv);
            acc0 -= v * S0.dm_d, acc1 -= v * S1.dm_d;
        }
        a0[k] = acc0, a1[k] = acc1;
    }
    u64 *limb0 = data + ((size_t)slot0 << 16), *limb1 = data + ((size_t)slot1 << 16);
    ar0.fwd16(a0, 0, 0, true);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[col_at(rl + 16 * k, c)] = ar0.store_mid(a0[k]);
    __syncthreads();
    cols_finish_group<4, true>(a0, limb0, col0, rl, rl, ar0, lds);
    __syncthreads();
    ar1.fwd16(a1, 0, 0, true);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[col_at(rl + 16 * k, c)] = ar1.store_mid(a1[k]);
    __syncthreads();
    cols_finish_group<4, true>(a1, limb1, col0, rl, rl, ar1, lds);
}
// grid.x = 16 * batch
// EX: the corrected conversions (a kernel of its own: their extra registers would cost the default form waves)
template <int PRO, int NSMAX, bool EX>
__global__ __launch_bounds__(256) void k_ntt_fwd_cols16(u64 *__restrict__ data, DevTables T, LimbBatch lb, ConvArgs cv)
{
    fwd_cols_kernel<16, PRO, NSMAX, EX>(data, T, lb, cv);
}
template <int PRO, int NSMAX, bool EX>
__global__ __launch_bounds__(256) void k_ntt_fwd_cols17(u64 *__restrict__ data, DevTables T, LimbBatch lb, ConvArgs cv)
{
    fwd_cols_kernel<17, PRO, NSMAX, EX>(data, T, lb, cv);
}

// extra constant of the inverse column pass for modulus index mi
__device__ __forceinline__ void scale_consts(int scale, const ConvArgs &cv, const DevTables &T, unsigned mi, unsigned slot,
                                             ShoupConst &ci, double &cd)
{
    ci = ShoupConst{0, 0};
    cd = 0.0;
    if (scale == SCALE_MODUP) {
        const int j = mi / cv.alpha, ii = mi - j * cv.alpha;
        const int na = min(cv.alpha, conv_op_level(cv, slot) - j * cv.alpha);
        const size_t idx = ((size_t)j * cv.alpha + (na - 1)) * cv.alpha + ii;
        ci = T.up_inv[idx];
        cd = T.up_inv_d[idx];
    } else if (scale == SCALE_MODDOWN) {
        ci = T.dn_inv[mi - cv.L];
        cd = T.dn_inv_d[mi - cv.L];
    }
}

template <int LOGN, int SCALE>
__device__ __forceinline__ void inv_cols_kernel(u64 *__restrict__ data, const DevTables &T, const LimbBatch &lb,
                                                const ConvArgs &cv)
{
    __shared__ u64 lds[ColsGeom<LOGN>::LDS_WORDS];
    const unsigned tile = blockIdx.x & 15, b = blockIdx.x >> 4;
    const unsigned mi = lb.mod[b];
    u64 *limb = data + ((size_t)lb.slot[b] << LOGN);
    ShoupConst ci;
    double cd;
    scale_consts(SCALE, cv, T, mi, lb.slot[b], ci, cd);
    if (T.mod[mi].qd != 0.0)
        inv_cols_body<LOGN, true>(limb, tile * 16, make_fp(T, mi, LOGN, cd), lds);
    else
        inv_cols_body<LOGN, true>(limb, tile * 16, make_int(T, mi, LOGN, ci), lds);
}
template <int SCALE>
__global__ __launch_bounds__(256) void k_ntt_inv_cols16(u64 *__restrict__ data, DevTables T, LimbBatch lb, ConvArgs cv)
{
    inv_cols_kernel<16, SCALE>(data, T, lb, cv);
}
template <int SCALE>
__global__ __launch_bounds__(256, 3) void k_ntt_inv_cols17(u64 *__restrict__ data, DevTables T, LimbBatch lb, ConvArgs cv)
{
    inv_cols_kernel<17, SCALE>(data, T, lb, cv);
}

// ---- column pass, N = 2^12: 16 rows x 256 columns, one thread per column --------------------------------------

template <int PRO, int SPLIT, bool TINT, bool EX, int NSMAX, class A>
__device__ __forceinline__ void fwd_cols12_body(u64 *__restrict__ limb, const A &ar, const ConvSetup<NSMAX> &S,
                                                const ModConst &m)
{
    const unsigned c = threadIdx.x;
    typename A::V a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) a[k] = PRO == PRO_LOAD ? ar.load(limb[k * 256 + c]) : conv_get<PRO, SPLIT, TINT, EX>(S, ar, m, k * 256 + c);
    ar.fwd16(a, 0, 0, PRO != PRO_LOAD);
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

template <int PRO, int NSMAX, bool EX>
__global__ __launch_bounds__(256) void k_ntt_fwd_cols12(u64 *__restrict__ data, DevTables T, LimbBatch lb, ConvArgs cv)
{
    const unsigned mi = lb.mod[blockIdx.x], slot = lb.slot[blockIdx.x];
    u64 *limb = data + ((size_t)slot << 12);
    const ModConst m = T.mod[mi];
    const ConvSetup<NSMAX> S = conv_setup<PRO, NSMAX, 12>(cv, T, slot, mi);
    const bool split = PRO == PRO_MODUP ? T.up_split != 0 : pro_is_moddown(PRO) ? T.dn_split != 0 : false;
    const bool tint = PRO == PRO_MODDOWN_RS && S.qld == 0.0; // dropped limb on the integer path
    const bool fold = pro_is_moddown(PRO) && !EX && NSMAX <= 4 && T.dn_fold != 0; // the common case only: each variant costs code
    if (m.qd == 0.0)
        fwd_cols12_body<PRO, 0, false, EX>(limb, make_int(T, mi, 12), S, m);
    else if (PRO == PRO_MODDOWN_RS && tint) {
        if (split)
            fwd_cols12_body<PRO, 1, PRO == PRO_MODDOWN_RS, EX>(limb, make_fp(T, mi, 12), S, m);
        else
            fwd_cols12_body<PRO, 0, PRO == PRO_MODDOWN_RS, EX>(limb, make_fp(T, mi, 12), S, m);
    } else if (fold)
        fwd_cols12_body<PRO, pro_is_moddown(PRO) && !EX && NSMAX <= 4 ? 2 : 0, false, EX>(limb, make_fp(T, mi, 12), S, m);
    else if (split)
        fwd_cols12_body<PRO, 1, false, EX>(limb, make_fp(T, mi, 12), S, m);
    else
        fwd_cols12_body<PRO, 0, false, EX>(limb, make_fp(T, mi, 12), S, m);
}

template <int SCALE>
__global__ __launch_bounds__(256) void k_ntt_inv_cols12(u64 *__restrict__ data, DevTables T, LimbBatch lb, ConvArgs cv)
{
    const unsigned mi = lb.mod[blockIdx.x];
    u64 *limb = data + ((size_t)lb.slot[blockIdx.x] << 12);
    ShoupConst ci;
    double cd;
    scale_consts(SCALE, cv, T, mi, lb.slot[blockIdx.x], ci, cd);
    if (T.mod[mi].qd != 0.0)
        inv_cols12_body(limb, make_fp(T, mi, 12, cd));
    else
        inv_cols12_body(limb, make_int(T, mi, 12, ci));
}
