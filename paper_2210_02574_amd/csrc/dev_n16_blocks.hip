// Block-pass and inner-product kernels of the ring size N = 2^16 and their launchers.
#include "launch.h"

void dev_launch_n16_blocks(DevLaunch &t)
{
    t.fwd_blocks = launch_fwd_blocks<16>;
    t.inv_blocks = launch_inv_blocks<16>;
    t.inner = launch_inner<16>;
}
