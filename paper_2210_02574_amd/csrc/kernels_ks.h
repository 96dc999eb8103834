// The inner product of key switching with the evaluation key.
#pragma once
#include "kernels_ntt.h"

// ---- inner product with the evaluation key, block pass of the raised digits' forward NTT fused in -----------
//
// u[c][a][n] = sum_j D_j[a][pi_g(n)] * evk[j][c][mod(a)][n] on every active limb a, where D_j[a] is the
// raised digit outside digit j and the NTT-domain input d[a] inside it.
// One work-group produces INNER_TILE consecutive outputs (a few blocks of 256) of one active limb.  The index map of
// sigma_g sends aligned groups of 2^m consecutive NTT-domain indices to aligned groups (the low bits of
// (2 brv(k) + 1) g depend only on the low bits of brv(k), i.e. on the high bits of k), so the sources of
// these outputs are the indices of one input tile of that size.  For a limb on the floating-point path the raised
// digits arrive as the column pass left them; each is finished here (stages logN-8 .. logN-1) into LDS
// and read back through the index map, so the transformed digits never travel to memory.  Limbs on
// the integer path read digits that the block-pass kernel has finished.  With inv_special the special
// limbs of u leave this kernel with the block pass of their inverse transform already applied.

typedef u64 u64x2 __attribute__((ext_vector_type(2)));
typedef double f64x2 __attribute__((ext_vector_type(2)));

struct InnerArgs {
    const u64 *raised, *d, *evk;
    u64 *u;
    int level, L, K, alpha, beta;
    unsigned g;
    int raised_stride, u_stride, d_stride; // limbs between two operations of a batch in each buffer
    int inv_special;
    int hoisted; // operation z uses key and Galois element z of the HoistKeys argument (one raised input for all)
    int count;   // operations in this launch
};
#define HOIST_MAX HE_OPS_MAX
struct HoistKeys {
    const u64 *evk[HOIST_MAX];
    unsigned g[HOIST_MAX];
    // mixed-level rotations: the operation's level (0: InnerArgs.level, which always gives the buffer layout)
    // and its NTT-domain input polynomial (null: InnerArgs.d + operation * d_stride)
    const u64 *d[HOIST_MAX];
    uint8_t level[HOIST_MAX];
};

// One-dimensional grid of inner_grid() work-groups; every buffer is 16-byte aligned.  Work-groups go to the
// eight XCDs round-robin by index, and each XCD has its own L2: index 8 s + x runs on XCD x, and the `count`
// operations of one (tile, limb) take consecutive s there, so the key slice they share is fetched from
// memory once per XCD visit instead of once per operation.
#define XCDS 8u
__host__ __device__ inline unsigned inner_grid(unsigned tiles, unsigned limbs, unsigned count)
{
    return (tiles * limbs + XCDS - 1) / XCDS * XCDS * count;
}

// Eight elements per thread and 128 threads per work-group: measured at 512, 256, 128 and 64 threads, work-groups of
// 128 win by 3 to 8 % because the barriers between the phases of a digit then stall two waves instead of eight while
// the other work-groups of the compute unit run.  25 KiB of LDS (exchange tile, twiddles, the next digit) allow six
// work-groups per compute unit, three waves per SIMD, at up to 170 registers.  A 256-element
// block belongs to 32 lanes (half a wave) and its block pass runs as three register steps, stages 0-2, 3-5 and
// 6-7 of the block, with two exchanges through LDS among those lanes:
//   step 1: lane t holds e = t + 32 k;   step 2: lane (g = t & 7, r = t >> 3) holds e = 32 g + r + 4 k;
//   step 3: lane t holds e = 4 t + k' and 128 + 4 t + k' (k' < 4).
// With one pad word per 16 elements every 16 consecutive lanes of each pattern hit 16 different 8-byte banks.
// All 255 twiddles of a block's eight stages sit in LDS, the one of local stage m and group i at 2^m - 1 + i.
// In the product phase thread t owns the pairs (INNER_TILE tile + 2 INNER_THREADS i + 2 t, + 1), i < 4.

#ifndef INNER_THREADS
#define INNER_THREADS 128
#endif
#define INNER_TILE (INNER_THREADS * 8)      // outputs per work-group
#define INNER_BLOCKS (INNER_THREADS / 32)   // 256-element blocks per work-group
#define INNER_TLOG (INNER_THREADS == 512 ? 12 : INNER_THREADS == 256 ? 11 : INNER_THREADS == 128 ? 10 : 9)
static_assert(INNER_THREADS == 512 || INNER_THREADS == 256 || INNER_THREADS == 128 || INNER_THREADS == 64, "tile of 4096, 2048, 1024 or 512 outputs");
__device__ __forceinline__ unsigned pair8_at(unsigned i) { return 2u * INNER_THREADS * i + 2u * threadIdx.x; }

// Inverse block pass of the special limbs from the pairs of the product phase: the results go through LDS to the
// first half of the threads, which run the 16-element form; the other threads only take part in the barriers.
template <int LOGN, class A>
__device__ __forceinline__ void inv_blocks_from_pairs8(const u64 (&r)[8], u64 *limb, const A &ar, u64 *lds, unsigned tile)
{
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const unsigned p = pair8_at(i);
        lds[tile_at(p >> 8, p & 255u)] = r[2 * i];
        lds[tile_at(p >> 8, (p & 255u) + 1)] = r[2 * i + 1];
    }
    __syncthreads();
    if (threadIdx.x < INNER_THREADS / 2) {
        const unsigned blk = threadIdx.x >> 4, il = threadIdx.x & 15, bg = tile * INNER_BLOCKS + blk;
        typename A::V a[16];
#pragma unroll
        for (int k = 0; k < 16; k++) a[k] = ar.load(lds[tile_at(blk, 16 * il + k)]);
        ar.template inv16<false>(a, LOGN - 4, bg * 16 + il);
#pragma unroll
        for (int k = 0; k < 16; k++) lds[tile_at(blk, 16 * il + k)] = ar.store_mid(a[k]);
        block_sync();
#pragma unroll
        for (int k = 0; k < 16; k++) a[k] = ar.load_mid(lds[tile_at(blk, il + 16 * k)]);
        ar.template inv16<false>(a, LOGN - 8, bg);
#pragma unroll
        for (int k = 0; k < 16; k++) limb[bg * 256 + il + 16 * k] = ar.store_mid(a[k]);
    }
    __syncthreads();
}

// Addresses are formed as a wave-uniform base plus a 32-bit lane offset so that they stay in scalar registers;
// the three LDS patterns of the block pass are one base each plus compile-time offsets (with the pad word per
// 16 elements: t + 32 k sits at t + (t >> 4) + 34 k, 32 g + r + 4 k at 34 g + r + 4 k + (k >> 2), and
// 128 h + 4 t + k' at 4 t + (t >> 2) + 136 h + k').
template <class Tv> __device__ __forceinline__ Tv ld_at(const void *base, unsigned byte_off)
{
    return *(const Tv *)((const char *)base + byte_off);
}

template <int LOGN> __global__ __launch_bounds__(INNER_THREADS, 4) void k_inner_blocks8(InnerArgs ia, DevTables T, HoistKeys hk)
{
    __shared__ u64 lds[INNER_BLOCKS * TILE_GROUP];
    __shared__ double tws[INNER_BLOCKS * 256];
    __shared__ u64 pre[INNER_BLOCKS * 256]; // the next raised digit of this tile, as it lies in memory
    const int level = ia.level, M = ia.L + ia.K, Ma = level + ia.K;
    const unsigned ntile = 1u << (LOGN - INNER_TLOG);
    const unsigned slot = blockIdx.x / XCDS, op = slot % (unsigned)ia.count;
    const unsigned tl = slot / (unsigned)ia.count * XCDS + blockIdx.x % XCDS;
    if (tl >= ntile * (unsigned)Ma) return; // padding of the last group of eight (whole work-group)
    const int a = Ma - 1 - (int)(tl / ntile); // special limbs (the slowest) first
    const unsigned tile = tl % ntile;
    const unsigned g = ia.hoisted ? hk.g[op] : ia.g;
    // an operation below the layout's level has no limbs a in [its level, level) and fewer digits
    const int op_level = ia.hoisted && hk.level[op] ? hk.level[op] : level;
    if (a < level && a >= op_level) return;
    const int beta = (op_level + ia.alpha - 1) / ia.alpha;
    const int mi = active_mod(a, level, ia.L);
    const int own = a < level ? a / ia.alpha : -1;
    const ModConst m = T.mod[mi];
    const unsigned blk = threadIdx.x >> 5, t = threadIdx.x & 31;
    const unsigned tile_in = g == 1 ? tile : galois_index(tile << INNER_TLOG, g, LOGN) >> INNER_TLOG;
    // wave-uniform bases (bytes): raised digit 0 and key component 0 of digit 0 for this limb and tile; digit j is
    // raised_step / key_step further on, key component 1 comp_step after component 0
    const char *raised0 = (const char *)(ia.raised + ((((size_t)op * ia.raised_stride + a) << LOGN) + ((size_t)tile_in << INNER_TLOG)));
    const char *key0 = (const char *)((ia.hoisted ? hk.evk[op] : ia.evk) + (((size_t)mi << LOGN) + ((size_t)tile << INNER_TLOG)));
    const char *d_limb = (const char *)((ia.hoisted && hk.d[op] ? hk.d[op] : ia.d + (((size_t)op * ia.d_stride) << LOGN)) + ((size_t)a << LOGN));
    const size_t raised_step = ((size_t)Ma << LOGN) * 8, comp_step = ((size_t)M << LOGN) * 8, key_step = 2 * comp_step;
    const unsigned lane16 = threadIdx.x * 16u;        // this thread's pair within a 512-pair row of the tile
    const unsigned lane_mid = (blk * 256u + t) * 8u;  // element t of block blk
    // pair i of the product phase: LDS words of the sources of its even and odd element (an aligned pair, in
    // either order), and whether the pair arrives swapped
    unsigned lsx[4], lsy[4], swm = 0;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const unsigned pos = (tile << INNER_TLOG) + pair8_at(i);
        const unsigned sr = g == 1 ? pos : galois_index(pos, g, LOGN);
        const unsigned sl = sr & (INNER_TILE - 2u), sw = sr & 1u;
        const unsigned w = (sl >> 8) * TILE_GROUP + (sl & 255u) + ((sl & 255u) >> 4);
        lsx[i] = w + sw, lsy[i] = w + 1 - sw;
        swm |= sw << i;
    }
    u64 r0[8], r1[8];
    if (m.qd != 0.0) {
        const ArithFp ar = make_fp(T, mi, LOGN);
        // The raised digit after the one being worked on is already on its way into LDS: each wave copies the two
        // blocks its lanes own, 4 x 1 KiB, with loads that write to LDS directly (lane i's 16 bytes land at
        // base + 16 i) and need no registers while they are in flight.
        const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        auto prefetch = [&](int j) {
            const char *src = raised0 + (size_t)j * raised_step + wave * 4096u + lane * 16u;
            // a digit that only this operation reads is streamed past the key slices that the batch shares in L2
            // (cache policy 2: nontemporal)
            if (ia.raised_stride != 0) {
#pragma unroll
                for (int c = 0; c < 4; c++)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + 1024 * c),
                                                     (__attribute__((address_space(3))) void *)(pre + wave * 512 + c * 128), 16, 0, 2);
            } else {
#pragma unroll
                for (int c = 0; c < 4; c++)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + 1024 * c),
                                                     (__attribute__((address_space(3))) void *)(pre + wave * 512 + c * 128), 16, 0, 0);
            }
        };
        {
            const int j0 = own == 0 ? 1 : 0;
            if (j0 < beta) prefetch(j0);
        }
        double *tw = tws + blk * 256;
        for (unsigned c = t; c < 255; c += 32) tw[c] = ar.twf[ArithFp::fwd16_twiddle(LOGN - 8, tile_in * INNER_BLOCKS + blk, c)];
        __syncthreads();
        const unsigned g2 = t & 7, r2 = t >> 3;
        u64 *l1 = lds + blk * TILE_GROUP + t + (t >> 4);
        u64 *l2 = lds + blk * TILE_GROUP + 34 * g2 + r2;
        u64 *l3 = lds + blk * TILE_GROUP + 4 * t + (t >> 2);
        double acc0[8], acc1[8];
#pragma unroll
        for (int k = 0; k < 8; k++) acc0[k] = acc1[k] = 0.0;
        for (int j = 0; j < beta; j++) {
            double dv[8];
            f64x2 e0[4], e1[4]; // key words of a floating-point limb are balanced doubles
            const char *kj = key0 + (size_t)j * key_step;
            if (j == own) {
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const unsigned pos = (tile << INNER_TLOG) + pair8_at(i);
                    const unsigned sr = g == 1 ? pos : galois_index(pos, g, LOGN);
                    const u64x2 v = ld_at<u64x2>(d_limb, (sr & ~1u) * 8u);
                    const bool sw = (swm >> i) & 1u;
                    dv[2 * i] = u2d(sw ? v.y : v.x), dv[2 * i + 1] = u2d(sw ? v.x : v.y);
                }
#pragma unroll
                for (int i = 0; i < 4; i++)
                    e0[i] = ld_at<f64x2>(kj + INNER_THREADS * 16 * i, lane16), e1[i] = ld_at<f64x2>(kj + comp_step + INNER_THREADS * 16 * i, lane16);
            } else {
                // this digit has arrived (nothing else of this wave is in flight here); once it is in registers the
                // buffer is free for the next one
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                const u64 *pw = pre + blk * 256 + t;
#pragma unroll
                for (int k = 0; k < 8; k++) dv[k] = ar.load_mid(pw[32 * k]);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                {
                    const int jn = j + 1 == own ? j + 2 : j + 1;
                    if (jn < beta) prefetch(jn);
                }
                // the key loads are issued before the block pass and complete behind it
#pragma unroll
                for (int i = 0; i < 4; i++)
                    e0[i] = ld_at<f64x2>(kj + INNER_THREADS * 16 * i, lane16), e1[i] = ld_at<f64x2>(kj + comp_step + INNER_THREADS * 16 * i, lane16);
                // ranges (in units of q): the column pass leaves up to 3.7; reduced, step 1 ends below 2.7 and
                // step 2 below 6.3; reduced again, step 3 ends below 1.9, small enough for exact products
                ar.fwd8_with(dv, true, [&](int sp, int gg) { return tw[(1 << sp) - 1 + gg]; });
#pragma unroll
                for (int k = 0; k < 8; k++) l1[34 * k] = ar.store_mid(dv[k]);
                block_sync();
#pragma unroll
                for (int k = 0; k < 8; k++) dv[k] = ar.load_mid(l2[4 * k + (k >> 2)]);
                ar.fwd8_with(dv, false, [&](int sp, int gg) { return tw[(8 << sp) - 1 + (g2 << sp) + gg]; });
#pragma unroll
                for (int k = 0; k < 8; k++) l2[4 * k + (k >> 2)] = ar.store_mid(dv[k]);
                block_sync();
#pragma unroll
                for (int k = 0; k < 8; k++) dv[k] = ar.load_mid(l3[136 * (k >> 2) + (k & 3)]);
                ar.fwd4x2_with(dv, true, [&](int h, int sp, int gg) { return tw[(64 << sp) - 1 + ((t + 32 * h) << sp) + gg]; });
#pragma unroll
                for (int k = 0; k < 8; k++) l3[136 * (k >> 2) + (k & 3)] = ar.store_mid(dv[k]);
                __syncthreads();
#pragma unroll
                for (int i = 0; i < 4; i++) dv[2 * i] = ar.load_mid(lds[lsx[i]]), dv[2 * i + 1] = ar.load_mid(lds[lsy[i]]);
                __syncthreads();
            }
#pragma unroll
            for (int i = 0; i < 4; i++) {
                acc0[2 * i] += ar.mulmod(dv[2 * i], e0[i].x);
                acc0[2 * i + 1] += ar.mulmod(dv[2 * i + 1], e0[i].y);
                acc1[2 * i] += ar.mulmod(dv[2 * i], e1[i].x);
                acc1[2 * i + 1] += ar.mulmod(dv[2 * i + 1], e1[i].y);
            }
            if ((j & 3) == 3) {
#pragma unroll
                for (int k = 0; k < 8; k++) acc0[k] = ar.reduce(acc0[k]), acc1[k] = ar.reduce(acc1[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < 8; k++) r0[k] = fp_canon(acc0[k], m.qd, m.qinvd), r1[k] = fp_canon(acc1[k], m.qd, m.qinvd);
    } else {
        // integer path: the raised digits arrive finished (NTT domain); read through the index map
        unsigned so[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const unsigned pos = (tile << INNER_TLOG) + pair8_at(i);
            so[i] = ((g == 1 ? pos : galois_index(pos, g, LOGN)) & ~1u) * 8u;
        }
        const char *fin0 = (const char *)(ia.raised + (((size_t)op * ia.raised_stride + a) << LOGN));
#pragma unroll
        for (int h = 0; h < 2; h++) { // two pairs at a time: the 128-bit accumulators of four would not fit
            U128 acc0[4], acc1[4];
#pragma unroll
            for (int k = 0; k < 4; k++) acc0[k] = acc1[k] = U128{0, 0};
            for (int j = 0; j < beta; j++) {
                const char *dj = j == own ? d_limb : fin0 + (size_t)j * raised_step;
                const char *kj = key0 + (size_t)j * key_step;
#pragma unroll
                for (int i = 0; i < 2; i++) {
                    const int ii = 2 * h + i;
                    const u64x2 v = ld_at<u64x2>(dj, so[ii]);
                    const bool sw = (swm >> ii) & 1u;
                    const u64 x = sw ? v.y : v.x, y = sw ? v.x : v.y;
                    const u64x2 ka = ld_at<u64x2>(kj + INNER_THREADS * 16 * ii, lane16), kb = ld_at<u64x2>(kj + comp_step + INNER_THREADS * 16 * ii, lane16);
                    mac128(acc0[2 * i], x, ka.x);
                    mac128(acc0[2 * i + 1], y, ka.y);
                    mac128(acc1[2 * i], x, kb.x);
                    mac128(acc1[2 * i + 1], y, kb.y);
                }
            }
#pragma unroll
            for (int k = 0; k < 4; k++) r0[4 * h + k] = reduce128(acc0[k], m), r1[4 * h + k] = reduce128(acc1[k], m);
        }
    }
    u64 *u0 = ia.u + ((((size_t)op * ia.u_stride + a) << LOGN)), *u1 = u0 + ((size_t)Ma << LOGN);
    if (ia.inv_special && a >= level) {
        if (m.qd != 0.0) {
            const ArithFp ar = make_fp(T, mi, LOGN);
            inv_blocks_from_pairs8<LOGN>(r0, u0, ar, lds, tile);
            inv_blocks_from_pairs8<LOGN>(r1, u1, ar, lds, tile);
        } else {
            const ArithInt ar = make_int(T, mi, LOGN);
            inv_blocks_from_pairs8<LOGN>(r0, u0, ar, lds, tile);
            inv_blocks_from_pairs8<LOGN>(r1, u1, ar, lds, tile);
        }
    } else {
        char *o0 = (char *)(u0 + ((size_t)tile << INNER_TLOG)), *o1 = (char *)(u1 + ((size_t)tile << INNER_TLOG));
#pragma unroll
        for (int i = 0; i < 4; i++) {
            __builtin_nontemporal_store(u64x2{r0[2 * i], r0[2 * i + 1]}, (u64x2 *)(o0 + INNER_THREADS * 16 * i + lane16));
            __builtin_nontemporal_store(u64x2{r1[2 * i], r1[2 * i + 1]}, (u64x2 *)(o1 + INNER_THREADS * 16 * i + lane16));
        }
    }
}
