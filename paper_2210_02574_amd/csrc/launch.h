// Kernel launch plumbing shared by the translation units of the device library.
//
// The kernels are templates over the ring size; each ring size is instantiated in a translation unit of
// its own (dev_n12.hip, dev_n16_blocks.hip, dev_n17_blocks.hip, and dev_cols.hip once per ring size and
// prologue) so that the library builds in parallel, and device.hip reaches them through one table of launchers per ring size.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include "kernels_ks.h"

// ---- optional per-kernel timing with HIP events on the launch stream (he_profile_start/stop)
enum KernelId {
    KID_FWD_COLS, KID_FWD_COLS_MODUP, KID_FWD_COLS_MODDOWN, KID_FWD_COLS_RESCALE, KID_FWD_COLS_MODDOWN_RS, KID_FWD_BLOCKS,
    KID_FWD_BLOCKS_FIN,
    KID_INV_BLOCKS, KID_INV_COLS, KID_LIMBWISE, KID_CMULT, KID_TENSOR, KID_INNER, KID_COUNT
};

// Creates the event pair of one profiled launch and appends it to the context's record list.
bool prof_events(he_ctx *c, int kid, double bytes, ProfRecord &r);

// Launch wrapper: `bytes` = bytes the launch has to move by the definition of its step.  While profiling,
// the launch carries a start and a stop event that take the kernel's own begin and end timestamps.
#define KLAUNCH_T(c, st, kid, bytes, kernel, grid, threads, ...)                                                    \
    do {                                                                                                             \
        ProfRecord pr_;                                                                                              \
        if ((c)->prof_on && prof_events((c), (kid), (double)(bytes), pr_))                                           \
            hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(threads), 0, (st), (hipEvent_t)pr_.a, (hipEvent_t)pr_.b,   \
                                  0, __VA_ARGS__);                                                                   \
        else                                                                                                         \
            hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), 0, (st), __VA_ARGS__);                             \
    } while (0)
#define KLAUNCH(c, st, kid, bytes, kernel, grid, ...) KLAUNCH_T(c, st, kid, bytes, kernel, grid, 256, __VA_ARGS__)
// work-groups per limb of the block pass
#define BLK_TILES(c) ((int)((c)->N / (256 * BLK_PER_WG)))

// Launchers of one ring size.  `wide`: a base conversion has more than four source limbs.
struct DevLaunch {
    // forward column pass of the nb limbs of lb, one launcher per prologue (PRO_*)
    void (*fwd_cols[5])(he_ctx *c, hipStream_t st, int kid, double bytes, bool wide, u64 *data, const LimbBatch &lb, int nb,
                        const ConvArgs &cv);
    // the same with the corrected base conversions (entries of prologues without a conversion stay null)
    void (*fwd_cols_ex[5])(he_ctx *c, hipStream_t st, int kid, double bytes, bool wide, u64 *data, const LimbBatch &lb, int nb,
                           const ConvArgs &cv);
    // forward block pass of the first nb limbs of lb; fin: with the ModDown / rescale epilogue
    void (*fwd_blocks)(he_ctx *c, hipStream_t st, double bytes, bool fin, u64 *data, const LimbBatch &lb, int nb,
                       const FinArgs &fa, const HoistOuts &ho);
    void (*inv_blocks)(he_ctx *c, hipStream_t st, double bytes, const u64 *src, u64 *dst, const LimbBatch &lb, int nb);
    void (*inv_cols)(he_ctx *c, hipStream_t st, double bytes, int scale, u64 *dst, const LimbBatch &lb, int nb,
                     const ConvArgs &cv);
    void (*inner)(he_ctx *c, hipStream_t st, double bytes, unsigned grid, const InnerArgs &ia, const HoistKeys &hk);
};
// Each translation unit fills its part of a ring size's table: dev_launch_cols<logN>_<p> the forward
// column pass with prologue p (p = 5: the inverse column pass).
void dev_launch_n12(DevLaunch &t);
void dev_launch_n16_blocks(DevLaunch &t);
void dev_launch_n17_blocks(DevLaunch &t);
#define HE_DECL_COLS(n)                                                                                              \
    void dev_launch_cols##n##_0(DevLaunch &t);                                                                       \
    void dev_launch_cols##n##_1(DevLaunch &t);                                                                       \
    void dev_launch_cols##n##_2(DevLaunch &t);                                                                       \
    void dev_launch_cols##n##_3(DevLaunch &t);                                                                       \
    void dev_launch_cols##n##_4(DevLaunch &t);                                                                       \
    void dev_launch_cols##n##_5(DevLaunch &t);                                                                       \
    void dev_launch_cols_ex##n##_1(DevLaunch &t);                                                                    \
    void dev_launch_cols_ex##n##_2(DevLaunch &t);                                                                    \
    void dev_launch_cols_ex##n##_4(DevLaunch &t);
HE_DECL_COLS(16)
HE_DECL_COLS(17)
#undef HE_DECL_COLS

// ---- launcher bodies, instantiated by the per-ring-size translation units ------------------------------

template <int LOGN>
static void launch_fwd_blocks(he_ctx *c, hipStream_t st, double bytes, bool fin, u64 *data, const LimbBatch &lb, int nb,
                              const FinArgs &fa, const HoistOuts &ho)
{
    if (fin)
        KLAUNCH_T(c, st, KID_FWD_BLOCKS_FIN, bytes, (k_ntt_fwd_blocks<LOGN, EPI_FIN>), BLK_TILES(c) * nb, BLK_THREADS, data,
                  c->dev, lb, fa, ho);
    else
        KLAUNCH_T(c, st, KID_FWD_BLOCKS, bytes, (k_ntt_fwd_blocks<LOGN, EPI_STORE>), BLK_TILES(c) * nb, BLK_THREADS, data,
                  c->dev, lb, fa, ho);
}
template <int LOGN>
static void launch_inv_blocks(he_ctx *c, hipStream_t st, double bytes, const u64 *src, u64 *dst, const LimbBatch &lb, int nb)
{
    KLAUNCH_T(c, st, KID_INV_BLOCKS, bytes, (k_ntt_inv_blocks<LOGN>), BLK_TILES(c) * nb, BLK_THREADS, src, dst, c->dev, lb);
}
template <int LOGN>
static void launch_inner(he_ctx *c, hipStream_t st, double bytes, unsigned grid, const InnerArgs &ia, const HoistKeys &hk)
{
    KLAUNCH_T(c, st, KID_INNER, bytes, (k_inner_blocks8<LOGN>), grid, INNER_THREADS, ia, c->dev, hk);
}
