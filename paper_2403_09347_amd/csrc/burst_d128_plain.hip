// The plainly written forward and dQ kernels of burst_d64_mfma.hip compiled for d = 128
// (namespace burst::d128p): 128 query rows per workgroup and two workgroups per CU, for calls
// whose query slice is too short to give every CU one of the 256-row workgroups of the
// hand-scheduled kernels.  (The dK/dV side needs none: its workgroups own 128 keys either way.)
#define BURST_SMALL_D 128
#define BURST_SMALL_NS d128p
#define BURST_SMALL_NO_DKV
#include "burst_d64_mfma.hip"
