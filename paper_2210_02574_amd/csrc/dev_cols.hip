// Column-pass kernels of the ring sizes N = 2^16 and 2^17 and their launchers.  Compiled once per
// (HE_LOGN, HE_PRO, HE_EX): one object per ring size and prologue, HE_PRO = 5 for the inverse column pass, and
// a further one (HE_EX = 1) for each prologue with a base conversion in its corrected form, so that the large
// kernels build in parallel.
#include "launch.h"

#if HE_LOGN == 16
#define FWD_KERNEL k_ntt_fwd_cols16
#define INV_KERNEL k_ntt_inv_cols16
#define NS_WIDE 8
#else
#define FWD_KERNEL k_ntt_fwd_cols17
#define INV_KERNEL k_ntt_inv_cols17
#define NS_WIDE 4 // wider conversions are refused at N = 2^17 when the context is created
#endif
// the preprocessor sees the prologue as a number: tie the numbers used below to the enumeration
static_assert(PRO_LOAD == 0 && PRO_MODUP == 1 && PRO_MODDOWN == 2 && PRO_RESCALE == 3 && PRO_MODDOWN_RS == 4, "prologue numbering");
#ifndef HE_EX
#define HE_EX 0
#endif
#define PASTE3_(a, b, c) a##b##_##c
#define PASTE3(a, b, c) PASTE3_(a, b, c)

#if HE_PRO < 5
static void fwd_cols(he_ctx *c, hipStream_t st, int kid, double bytes, bool wide, u64 *data, const LimbBatch &lb, int nb,
                     const ConvArgs &cv)
{
#if HE_LOGN == 16 && HE_PRO == 1 /* PRO_MODUP */
    if (!wide) {
        KLAUNCH(c, st, kid, bytes, (k_ntt_fwd_cols16_modup2<4, HE_EX != 0>), 16 * ((nb + 1) / 2), data, c->dev, lb, cv, nb);
        return;
    }
#endif
#if HE_PRO == 0 || HE_PRO == 3 /* PRO_LOAD, PRO_RESCALE: no base conversion, one form */
    KLAUNCH(c, st, kid, bytes, (FWD_KERNEL<HE_PRO, 4, HE_EX != 0>), 16 * nb, data, c->dev, lb, cv);
#else
    if (wide)
        KLAUNCH(c, st, kid, bytes, (FWD_KERNEL<HE_PRO, NS_WIDE, HE_EX != 0>), 16 * nb, data, c->dev, lb, cv);
    else
        KLAUNCH(c, st, kid, bytes, (FWD_KERNEL<HE_PRO, 4, HE_EX != 0>), 16 * nb, data, c->dev, lb, cv);
#endif
}
#if HE_EX
void PASTE3(dev_launch_cols_ex, HE_LOGN, HE_PRO)(DevLaunch &t) { t.fwd_cols_ex[HE_PRO] = fwd_cols; }
#else
void PASTE3(dev_launch_cols, HE_LOGN, HE_PRO)(DevLaunch &t) { t.fwd_cols[HE_PRO] = fwd_cols; }
#endif
#else
static void inv_cols(he_ctx *c, hipStream_t st, double bytes, int scale, u64 *dst, const LimbBatch &lb, int nb,
                     const ConvArgs &cv)
{
    switch (scale) {
    case SCALE_NONE: KLAUNCH(c, st, KID_INV_COLS, bytes, (INV_KERNEL<SCALE_NONE>), 16 * nb, dst, c->dev, lb, cv); break;
    case SCALE_MODUP: KLAUNCH(c, st, KID_INV_COLS, bytes, (INV_KERNEL<SCALE_MODUP>), 16 * nb, dst, c->dev, lb, cv); break;
    default: KLAUNCH(c, st, KID_INV_COLS, bytes, (INV_KERNEL<SCALE_MODDOWN>), 16 * nb, dst, c->dev, lb, cv); break;
    }
}
void PASTE3(dev_launch_cols, HE_LOGN, HE_PRO)(DevLaunch &t) { t.inv_cols = inv_cols; }
#endif
