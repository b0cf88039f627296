// The plainly written forward and dQ kernels of burst_plain_mfma.h compiled for d = 128
// (namespace burst::d128p): 128 query rows per workgroup and two workgroups per CU, for calls
// whose query slice is too short to give every CU one of the 256-row workgroups of the
// hand-scheduled kernels, and for calls with block flags finer than those workgroups: here a
// wavefront skips the tiles the flags hide from its own 32 rows, which the hand-scheduled
// kernels cannot (their matrix phases admit no branch).  (The dK/dV side needs none: its
// workgroups own 128 keys either way, and the plain dK/dV kernel at d = 128 spills registers and
// is slower than the hand-scheduled one even on fine patterns.)
#define BURST_SMALL_D 128
#define BURST_SMALL_NS d128p
#define BURST_SMALL_NO_DKV
#include "burst_plain_mfma.h"
