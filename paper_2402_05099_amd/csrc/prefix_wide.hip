// The persistent 256-row shared-block kernel (Sec. 3.2) at head dimension 128, its host-side work partition
// (plan_prefix_wide) and the launcher for both head dimensions; the kernel's source is prefix_wide_impl.h.
#define HG_WIDE_D 128
#define HG_WIDE_KERNEL prefix_kernel_wide
#include "prefix_wide_impl.h"
