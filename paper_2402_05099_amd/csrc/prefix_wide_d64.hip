// The persistent 256-row shared-block kernel (Sec. 3.2) at head dimension 64: stages of 64 keys (the same 8 KiB per
// tensor and stage as 32 keys at D = 128), two 32-key score tiles per stage; the kernel's source is prefix_wide_impl.h.
#define HG_WIDE_D 64
#define HG_WIDE_KERNEL prefix_kernel_wide_d64
#include "prefix_wide_impl.h"
