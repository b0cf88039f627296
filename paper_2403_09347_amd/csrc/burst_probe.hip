// Micro-benchmarks behind bench.py: what the chip sustains on the two resources the attention
// kernels live on, measured with the same instruction forms those kernels use.  Not part of the
// method; they exist so that the rates the kernels are compared with are numbers anyone can
// re-measure, not estimates.
//   burst_probe_mfma      v_mfma_f32_32x32x16_bf16 back to back, nothing else in the loop: operands
//                         held in registers, or the A operand read fresh from LDS for every MFMA /
//                         every second MFMA (128-bit reads, as the kernels' K / V / Q fragments are).
//                         The contents of the operands matter (the core clock under matrix load
//                         depends on how many bits toggle), so the caller supplies them.
//   burst_probe_atomic_dq the memory side of a backward that computed the block pair once
//                         (key-stationary, dQ partial sums leaving each workgroup through fp32
//                         atomics): exactly those atomic adds, in that pattern, and no arithmetic.
#include <hip/hip_runtime.h>
#include "burst_common.h"

namespace burst {
namespace {

// SHARE = 0: operands in registers; 1: a fresh A operand from LDS for every MFMA; 2: for every
// second MFMA.  Four accumulators per wavefront, so consecutive MFMAs are independent.
template <int SHARE>
__global__ void __launch_bounds__(512) probe_mfma_kernel(const bf16x8* __restrict__ operands, float* __restrict__ sink,
                                                         int iters) {
  __shared__ __attribute__((aligned(16))) char smem[65536];
  for (int i = threadIdx.x; i < 4096; i += blockDim.x) reinterpret_cast<bf16x8*>(smem)[i] = operands[i];
  __syncthreads();
  const int lane = threadIdx.x & 63;
  bf16x8 b[8], a_reg[8];
#pragma unroll
  for (int i = 0; i < 8; i++) {
    b[i] = operands[(threadIdx.x * 8 + i) & 4095];
    a_reg[i] = operands[(threadIdx.x * 8 + i + 2048) & 4095];
  }
  f32x16 c[4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) c[i][r] = 0.f;
  int base = (threadIdx.x >> 6) * 4096;
  for (int it = 0; it < iters; it++) {
    if constexpr (SHARE == 0) {
#pragma unroll
      for (int i = 0; i < 16; i++) c[i & 3] = mfma32(a_reg[i & 7], b[(i >> 1) & 7], c[i & 3]);
    } else {
      bf16x8 a[16 / SHARE];
#pragma unroll
      for (int j = 0; j < 16 / SHARE; j++) a[j] = lds_read_b128(smem, (base + j * 1024 + lane * 16) & 65535);
#pragma unroll
      for (int i = 0; i < 16; i++) c[i & 3] = mfma32(a[i / SHARE], b[i & 7], c[i & 3]);
      base += 16384;
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) s += c[i][r];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// One workgroup per (head, block of 128 keys), workgroup ids mapped so that a head stays on one
// XCD, as the backward kernels do.  It walks the head's 64-row query tiles and adds a [64][128]
// fp32 tile into dQ for each: wavefront w owns 32 of the 128 columns, a lane one column and 32
// rows, in the register layout an MFMA accumulator of dQ = dS K would have.  Workgroups of a head
// start at different tiles so that they do not all hit the same rows at once.
// MODE 1: atomic adds; 0: plain stores; 2: plain read-modify-write (load, add, store: what a
// workgroup that held a tile exclusively would do).
template <int MODE>
__global__ void __launch_bounds__(256) probe_atomic_dq_kernel(float* __restrict__ dq, int nq, int key_blocks) {
  const int bid = blockIdx.x, xcd = bid & 7, idx = bid >> 3;
  const int hx = idx / key_blocks, kb = idx - hx * key_blocks, head = hx * 8 + xcd;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
  float* base = dq + (size_t)head * nq * 128;
  const int tiles = nq / 64;
  for (int t = 0; t < tiles; t++) {
    const int qt = (t + kb * 2) % tiles;
#pragma unroll
    for (int rb = 0; rb < 2; rb++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int row = qt * 64 + rb * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
        float* p = base + (size_t)row * 128 + w * 32 + col;
        if constexpr (MODE == 1) unsafeAtomicAdd(p, 1.0f);
        else if constexpr (MODE == 2) __builtin_nontemporal_store(__builtin_nontemporal_load(p) + 1.0f, p);
        else *p = 1.0f;
      }
  }
}

}  // namespace
}  // namespace burst

extern "C" {

int burst_probe_mfma(int a_from_lds, int wavefronts_per_simd, const void* operands, float* sink, int iters,
                     void* stream) {
  using namespace burst;
  if (operands == nullptr || sink == nullptr) return BURST_ERR_NULL;
  if (a_from_lds < 0 || a_from_lds > 2 || (wavefronts_per_simd != 1 && wavefronts_per_simd != 2) || iters < 1 ||
      iters > (1 << 22)) return BURST_ERR_SHAPE;
  const dim3 grid(256), block(256 * wavefronts_per_simd);
  hipStream_t s = (hipStream_t)stream;
  const bf16x8* in = static_cast<const bf16x8*>(operands);
  if (a_from_lds == 0) hipLaunchKernelGGL(probe_mfma_kernel<0>, grid, block, 0, s, in, sink, iters);
  else if (a_from_lds == 1) hipLaunchKernelGGL(probe_mfma_kernel<1>, grid, block, 0, s, in, sink, iters);
  else hipLaunchKernelGGL(probe_mfma_kernel<2>, grid, block, 0, s, in, sink, iters);
  return hipGetLastError() == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
}

int burst_probe_atomic_dq(float* dQ, int heads, int Nq, int key_blocks, int mode, void* stream) {
  using namespace burst;
  if (dQ == nullptr) return BURST_ERR_NULL;
  if (heads < 8 || heads % 8 != 0 || heads > 4096 || Nq < 64 || Nq % 64 != 0 || Nq > (1 << 20) || key_blocks < 1 ||
      key_blocks > 4096 || mode < 0 || mode > 2) return BURST_ERR_SHAPE;
  const dim3 grid((unsigned)(heads * key_blocks)), block(256);
  hipStream_t s = (hipStream_t)stream;
  if (mode == 1) hipLaunchKernelGGL(probe_atomic_dq_kernel<1>, grid, block, 0, s, dQ, Nq, key_blocks);
  else if (mode == 2) hipLaunchKernelGGL(probe_atomic_dq_kernel<2>, grid, block, 0, s, dQ, Nq, key_blocks);
  else hipLaunchKernelGGL(probe_atomic_dq_kernel<0>, grid, block, 0, s, dQ, Nq, key_blocks);
  return hipGetLastError() == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
}

}  // extern "C"
