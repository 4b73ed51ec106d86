// The general kernel for problems beyond the fast kernel's limits (more than 8 devices, 32 block types, 4 types on a
// device or 8 micro-batches per window; Table I bounds none of them): its instantiations for 16 and 32 devices, in a
// translation unit of their own so that they compile beside the rest of the library.  The kernel is defined in
// tessel_kernels.hip, which this file includes up to the point where the instantiations stand.
#define TESSEL_WIDE_INSTANTIATIONS
#include "tessel_kernels.hip"
