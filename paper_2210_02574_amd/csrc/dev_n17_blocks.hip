// Block-pass and inner-product kernels of the ring size N = 2^17 and their launchers.
#include "launch.h"

void dev_launch_n17_blocks(DevLaunch &t)
{
    t.fwd_blocks = launch_fwd_blocks<17>;
    t.inv_blocks = launch_inv_blocks<17>;
    t.inner = launch_inner<17>;
}
