// The plainly written kernels of burst_plain_mfma.h compiled for d = 128 (namespace burst::d128p).
// Forward and dQ: 128 query rows per workgroup and two workgroups per CU, for calls whose query
// slice is too short to give every CU one of the 256-row workgroups of the hand-scheduled kernels,
// and for calls with block flags finer than those workgroups: here a wavefront skips the tiles the
// flags hide from its own 32 rows, which the hand-scheduled kernels cannot (their accumulators are
// pinned to AGPRs through inline assembly, and a branch around the matrix phases makes the
// register allocator move all of them through VGPRs in every iteration).
// dK/dV: two wavefronts = 64 keys per workgroup, two workgroups per CU.  It runs only when this
// family is forced (burst_set_kernel_family): calls with 64-wide block flags, which it was built
// for, are served by the hand-scheduled dK/dV kernel's own 64-key shape, which is faster at every
// density.
#define BURST_SMALL_D 128
#define BURST_SMALL_NS d128p
#define BURST_SMALL_DKV_WAVES 2
#include "burst_plain_mfma.h"
