// The inner product of key switching with the evaluation key.
#pragma once
#include "kernels_ntt.h"

// ---- inner product with the evaluation key, block pass of the raised digits' forward NTT fused in -----------
//
// u[c][a][n] = sum_j D_j[a][pi_g(n)] * evk[j][c][mod(a)][n] on every active limb a, where D_j[a] is the
// raised digit outside digit j and the NTT-domain input d[a] inside it.
// One work-group produces 4096 consecutive outputs (16 blocks of 256) of one active limb.  The index map of
// sigma_g sends aligned groups of 2^m consecutive NTT-domain indices to aligned groups (the low bits of
// (2 brv(k) + 1) g depend only on the low bits of brv(k), i.e. on the high bits of k), so the sources of
// these outputs are the 4096 indices of one input tile.  For a limb on the floating-point path the raised
// digits arrive as the column pass left them; each is finished here (stages logN-8 .. logN-1) into LDS
// and read back through the index map, so the transformed digits never travel to memory.  Limbs on
// the integer path read digits that the block-pass kernel has finished.  With inv_special the special
// limbs of u leave this kernel with the block pass of their inverse transform already applied.

typedef u64 u64x2 __attribute__((ext_vector_type(2)));

// Ownership in the product phase: thread t holds the pairs (4096 tile + 512 i + 2 t, + 1), i = 0..7, so that
// key loads and result stores are 16 bytes per lane and 1 KiB contiguous per wave.  sigma_g maps an aligned
// pair onto an aligned pair (possibly swapped): the source of k + 1 is the source of k with its lowest bit
// flipped, because k + 1 adds N to the exponent 2 brv(k) + 1 and g is odd.
__device__ __forceinline__ unsigned pair_at(unsigned i) { return 512u * i + 2u * threadIdx.x; }

template <int LOGN, class A>
__device__ __forceinline__ void inv_blocks_from_pairs(const u64 (&r)[16], u64 *limb, const A &ar, u64 *lds, unsigned bg)
{
    const unsigned blk = threadIdx.x >> 4, il = threadIdx.x & 15;
    typename A::V a[16];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const unsigned p = pair_at(i);
        lds[tile_at(p >> 8, p & 255u)] = r[2 * i];
        lds[tile_at(p >> 8, (p & 255u) + 1)] = r[2 * i + 1];
    }
    __syncthreads();
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
    __syncthreads();
}

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
#define HOIST_MAX 32
struct HoistKeys {
    const u64 *evk[HOIST_MAX];
    unsigned g[HOIST_MAX];
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
template <int LOGN> __global__ __launch_bounds__(256) void k_inner_blocks(InnerArgs ia, DevTables T, HoistKeys hk)
{
    __shared__ u64 lds[16 * TILE_GROUP];
    __shared__ double tws[16 * 15 + 256 * 15];
    const int level = ia.level, M = ia.L + ia.K, Ma = level + ia.K;
    const unsigned ntile = 1u << (LOGN - 12);
    const unsigned slot = blockIdx.x / XCDS, op = slot % (unsigned)ia.count;
    const unsigned tl = slot / (unsigned)ia.count * XCDS + blockIdx.x % XCDS;
    if (tl >= ntile * (unsigned)Ma) return; // padding of the last group of eight (whole work-group)
    const int a = Ma - 1 - (int)(tl / ntile); // special limbs (the slowest) first
    const unsigned tile = tl % ntile;
    const u64 *raised = ia.raised + (((size_t)op * ia.raised_stride) << LOGN);
    u64 *u = ia.u + (((size_t)op * ia.u_stride) << LOGN);
    const u64 *d = ia.d + (((size_t)op * ia.d_stride) << LOGN);
    const unsigned g = ia.hoisted ? hk.g[op] : ia.g;
    const u64 *evk = ia.hoisted ? hk.evk[op] : ia.evk;
    const int mi = active_mod(a, level, ia.L);
    const int own = a < level ? a / ia.alpha : -1;
    const ModConst m = T.mod[mi];
    const unsigned blk = threadIdx.x >> 4, il = threadIdx.x & 15;
    const unsigned bg = tile * 16 + blk;
    const unsigned tile_in = g == 1 ? tile : galois_index(tile << 12, g, LOGN) >> 12;
    const unsigned bg_in = tile_in * 16 + blk;
    unsigned src[8]; // source of the even element of pair i
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const unsigned pos = (tile << 12) + pair_at(i);
        src[i] = g == 1 ? pos : galois_index(pos, g, LOGN);
    }
    const size_t key_at = ((size_t)tile << 11) + threadIdx.x; // in pairs, inside one limb
    u64 r0[16], r1[16];
    if (m.qd != 0.0) {
        const ArithFp ar = make_fp(T, mi, LOGN);
        // Every digit's block pass uses the same twiddles (15 per block for its first four stages, 15 per
        // thread for the last four): fetched once and kept in LDS, so that no global load sits inside the
        // block pass and the key loads issued before it stay in flight until the products need them.
        double *tw_blk = tws, *tw_thr = tws + 16 * 15 + threadIdx.x * 15;
        if (il < 15) tw_blk[blk * 15 + il] = ar.twf[ArithFp::fwd16_twiddle(LOGN - 8, bg_in, il)];
#pragma unroll
        for (unsigned c = 0; c < 15; c++) tw_thr[c] = ar.twf[ArithFp::fwd16_twiddle(LOGN - 4, bg_in * 16 + il, c)];
        __syncthreads();
        tw_blk += blk * 15;
        double acc0[16], acc1[16];
#pragma unroll
        for (int k = 0; k < 16; k++) acc0[k] = acc1[k] = 0.0;
        for (int j = 0; j < ia.beta; j++) {
            double dv[16];
            u64x2 e0[8], e1[8];
            const u64x2 *k0 = (const u64x2 *)(evk + ((((size_t)j * 2 + 0) * M + mi) << LOGN)) + key_at;
            const u64x2 *k1 = (const u64x2 *)(evk + ((((size_t)j * 2 + 1) * M + mi) << LOGN)) + key_at;
            if (j == own) {
                const u64 *dj = d + ((size_t)a << LOGN);
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    const u64x2 v = *(const u64x2 *)(dj + (src[i] & ~1u));
                    const bool sw = src[i] & 1u;
                    dv[2 * i] = u2d(sw ? v.y : v.x), dv[2 * i + 1] = u2d(sw ? v.x : v.y);
                }
#pragma unroll
                for (int i = 0; i < 8; i++) e0[i] = k0[256 * i], e1[i] = k1[256 * i];
            } else {
                const u64 *mid = raised + (((size_t)j * Ma + a) << LOGN);
#pragma unroll
                for (int k = 0; k < 16; k++) dv[k] = ar.load_mid(mid[bg_in * 256 + il + 16 * k]);
                // the key loads are issued before the block pass and complete behind it
#pragma unroll
                for (int i = 0; i < 8; i++) e0[i] = k0[256 * i], e1[i] = k1[256 * i];
                ar.fwd16_with(dv, true, [&](int c) { return tw_blk[c]; });
#pragma unroll
                for (int k = 0; k < 16; k++) lds[tile_at(blk, il + 16 * k)] = ar.store_mid(dv[k]);
                block_sync();
#pragma unroll
                for (int k = 0; k < 16; k++) dv[k] = ar.load_mid(lds[tile_at(blk, 16 * il + k)]);
                ar.fwd16_with(dv, true, [&](int c) { return tw_thr[c]; });
#pragma unroll
                for (int k = 0; k < 16; k++) lds[tile_at(blk, 16 * il + k)] = ar.store_mid(ar.reduce(dv[k]));
                __syncthreads();
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    const unsigned s = src[i] & 4094u;
                    const double x = ar.load_mid(lds[tile_at(s >> 8, s & 255u)]);
                    const double y = ar.load_mid(lds[tile_at(s >> 8, (s & 255u) + 1)]);
                    const bool sw = src[i] & 1u;
                    dv[2 * i] = sw ? y : x, dv[2 * i + 1] = sw ? x : y;
                }
                __syncthreads();
            }
#pragma unroll
            for (int i = 0; i < 8; i++) {
                acc0[2 * i] += ar.mulmod(dv[2 * i], u2d(e0[i].x));
                acc0[2 * i + 1] += ar.mulmod(dv[2 * i + 1], u2d(e0[i].y));
                acc1[2 * i] += ar.mulmod(dv[2 * i], u2d(e1[i].x));
                acc1[2 * i + 1] += ar.mulmod(dv[2 * i + 1], u2d(e1[i].y));
            }
            if ((j & 3) == 3) {
#pragma unroll
                for (int k = 0; k < 16; k++) acc0[k] = ar.reduce(acc0[k]), acc1[k] = ar.reduce(acc1[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < 16; k++) r0[k] = fp_canon(acc0[k], m.qd, m.qinvd), r1[k] = fp_canon(acc1[k], m.qd, m.qinvd);
    } else {
#pragma unroll
        for (int h = 0; h < 2; h++) {
            U128 acc0[8], acc1[8];
#pragma unroll
            for (int k = 0; k < 8; k++) acc0[k] = acc1[k] = U128{0, 0};
            for (int j = 0; j < ia.beta; j++) {
                const u64 *dj = j == own ? d + ((size_t)a << LOGN) : raised + (((size_t)j * Ma + a) << LOGN);
                const u64x2 *k0 = (const u64x2 *)(evk + ((((size_t)j * 2 + 0) * M + mi) << LOGN)) + key_at;
                const u64x2 *k1 = (const u64x2 *)(evk + ((((size_t)j * 2 + 1) * M + mi) << LOGN)) + key_at;
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const unsigned s = src[4 * h + i];
                    const u64x2 v = *(const u64x2 *)(dj + (s & ~1u));
                    const bool sw = s & 1u;
                    const u64 x = sw ? v.y : v.x, y = sw ? v.x : v.y;
                    const u64x2 ka = k0[256 * (4 * h + i)], kb = k1[256 * (4 * h + i)];
                    mac128(acc0[2 * i], x, ka.x);
                    mac128(acc0[2 * i + 1], y, ka.y);
                    mac128(acc1[2 * i], x, kb.x);
                    mac128(acc1[2 * i + 1], y, kb.y);
                }
            }
#pragma unroll
            for (int k = 0; k < 8; k++) r0[8 * h + k] = reduce128(acc0[k], m), r1[8 * h + k] = reduce128(acc1[k], m);
        }
    }
    u64 *u0 = u + (((size_t)0 * Ma + a) << LOGN), *u1 = u + (((size_t)1 * Ma + a) << LOGN);
    if (ia.inv_special && a >= level) {
        if (m.qd != 0.0) {
            const ArithFp ar = make_fp(T, mi, LOGN);
            inv_blocks_from_pairs<LOGN>(r0, u0, ar, lds, bg);
            inv_blocks_from_pairs<LOGN>(r1, u1, ar, lds, bg);
        } else {
            const ArithInt ar = make_int(T, mi, LOGN);
            inv_blocks_from_pairs<LOGN>(r0, u0, ar, lds, bg);
            inv_blocks_from_pairs<LOGN>(r1, u1, ar, lds, bg);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; i++) {
            ((u64x2 *)u0)[key_at + 256 * i] = u64x2{r0[2 * i], r0[2 * i + 1]};
            ((u64x2 *)u1)[key_at + 256 * i] = u64x2{r1[2 * i], r1[2 * i + 1]};
        }
    }
}
