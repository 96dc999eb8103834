// Kernels of the ring size N = 2^12 and their launchers.
#include "launch.h"

template <int PRO, bool EX>
static void fwd_cols12(he_ctx *c, hipStream_t st, int kid, double bytes, bool wide, u64 *data, const LimbBatch &lb, int nb,
                       const ConvArgs &cv)
{
    if (wide && PRO != PRO_LOAD && PRO != PRO_RESCALE)
        KLAUNCH(c, st, kid, bytes, (k_ntt_fwd_cols12<PRO, 8, EX>), nb, data, c->dev, lb, cv);
    else
        KLAUNCH(c, st, kid, bytes, (k_ntt_fwd_cols12<PRO, 4, EX>), nb, data, c->dev, lb, cv);
}
static void inv_cols12(he_ctx *c, hipStream_t st, double bytes, int scale, u64 *dst, const LimbBatch &lb, int nb,
                       const ConvArgs &cv)
{
    switch (scale) {
    case SCALE_NONE: KLAUNCH(c, st, KID_INV_COLS, bytes, (k_ntt_inv_cols12<SCALE_NONE>), nb, dst, c->dev, lb, cv); break;
    case SCALE_MODUP: KLAUNCH(c, st, KID_INV_COLS, bytes, (k_ntt_inv_cols12<SCALE_MODUP>), nb, dst, c->dev, lb, cv); break;
    default: KLAUNCH(c, st, KID_INV_COLS, bytes, (k_ntt_inv_cols12<SCALE_MODDOWN>), nb, dst, c->dev, lb, cv); break;
    }
}
void dev_launch_n12(DevLaunch &t)
{
    t.fwd_cols[PRO_LOAD] = fwd_cols12<PRO_LOAD, false>;
    t.fwd_cols[PRO_MODUP] = fwd_cols12<PRO_MODUP, false>;
    t.fwd_cols[PRO_MODDOWN] = fwd_cols12<PRO_MODDOWN, false>;
    t.fwd_cols[PRO_RESCALE] = fwd_cols12<PRO_RESCALE, false>;
    t.fwd_cols[PRO_MODDOWN_RS] = fwd_cols12<PRO_MODDOWN_RS, false>;
    t.fwd_cols_ex[PRO_MODUP] = fwd_cols12<PRO_MODUP, true>;
    t.fwd_cols_ex[PRO_MODDOWN] = fwd_cols12<PRO_MODDOWN, true>;
    t.fwd_cols_ex[PRO_MODDOWN_RS] = fwd_cols12<PRO_MODDOWN_RS, true>;
    t.inv_cols = inv_cols12;
    t.fwd_blocks = launch_fwd_blocks<12>;
    t.inv_blocks = launch_inv_blocks<12>;
    t.inner = launch_inner<12>;
}
