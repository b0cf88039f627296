// Shared device-side helpers for the gfx950 local-attention kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <mutex>
#include "../../include/burst.h"

namespace burst {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
#define BURST_NEG_INF (-__builtin_inff())

// Where the storage-type tensors lie in memory: element strides between batch entries, heads
// and rows of Q, dO, O (query side) and of K, V (key side); the last dimension is contiguous.
// fp32 tensors (state, lse, D, gradients) are always contiguous [B, H, rows, d] / [B, H, rows].
struct Layout {
  long long qs_b, qs_h, qs_r;
  long long ks_b, ks_h, ks_r;
  int heads, kv_heads;             // heads per batch entry on either side
  // element offset of row 0 of a head; `head` counts batch x heads
  __host__ __device__ size_t q_base(int head) const {
    const int b = head / heads;
    return (size_t)b * qs_b + (size_t)(head - b * heads) * qs_h;
  }
  __host__ __device__ size_t kv_base(int kvhead) const {
    const int b = kvhead / kv_heads;
    return (size_t)b * ks_b + (size_t)(kvhead - b * kv_heads) * ks_h;
  }
};

// Row r of the query-side tensors, r counting the rows of all (batch, head)s: element offset.
struct QRows {
  Layout lay;
  int Nq, d, dense;                // dense: contiguous [B, H, Nq, d], the offset is r * d
  __host__ __device__ size_t off(long long r) const {
    if (dense) return (size_t)r * d;
    const long long head = r / Nq;
    return lay.q_base((int)head) + (size_t)(r - head * Nq) * lay.qs_r;
  }
};

// Kernel-side copy of the call's parameters (plain data, passed by value).
struct KParams {
  Layout lay;
  int B, H, Nq, Nc, d;
  int causal;
  float scale;
  long long q_off, k_off;
  long long window;      // 0 = none
  const uint8_t* bmask;  // block mask [ceil(Nq/bsize)][bpitch] (nullptr = none), bpitch = ceil(Nc/bsize)
  int bsize, bpitch;
  long long bhstride;    // bytes between the flag matrices of consecutive (batch, query head)s; 0 = shared
  int group;             // query heads per key/value head (1 = every head has its own K, V)
  QRows q_rows() const {
    QRows q;
    q.lay = lay; q.Nq = Nq; q.d = d;
    q.dense = lay.qs_r == d && lay.qs_h == (long long)Nq * d && lay.qs_b == (long long)Nq * d * H;
    return q;
  }
};

// The opt-in to more than 64 KB of dynamic LDS is a per-device function attribute: launchers
// set it once per device (index = current device, or -1 if it cannot be determined), whichever
// host thread comes first.
constexpr int kMaxDevicesForAttr = 64;
inline int current_device_slot() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevicesForAttr) return -1;
  return dev;
}
struct DeviceOnce {
  std::once_flag flag[kMaxDevicesForAttr];
  int status[kMaxDevicesForAttr];
  template <typename F>
  int run(F&& setup) {                       // setup() returns a burst_status; it runs once per device
    const int dev = current_device_slot();
    if (dev < 0) return BURST_ERR_LAUNCH;
    std::call_once(flag[dev], [&] { status[dev] = setup(); });
    return status[dev];
  }
};

// An entry point that enqueues several kernels first walks its launchers with this flag set: they
// validate, set their function attributes and return without launching, so that an error can
// still be reported with nothing enqueued.
extern thread_local bool t_validate_only;
#define BURST_LAUNCH(...)                                          \
  do {                                                             \
    if (!::burst::t_validate_only) hipLaunchKernelGGL(__VA_ARGS__); \
  } while (0)
inline int launch_status() {
  if (t_validate_only) return BURST_OK;
  return hipGetLastError() == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Cross-half exchange.  v_permlane32_swap exchanges the upper 32 lanes of its first operand
// with the lower 32 lanes of its second; fed the same value twice, every lane ends up with
// (value of lane%32, value of lane%32 + 32).  The second operand goes through an opaque
// register copy: the optimizer otherwise treats the swap of two identical values as the
// identity and drops the combination of the two results.
struct HalfPair { float lo, hi; };
__device__ __forceinline__ HalfPair both_halves(float x) {
  int a = __builtin_bit_cast(int, x);
  int b;
  asm volatile("v_mov_b32 %0, %1\n\ts_nop 1" : "=v"(b) : "v"(a));   // nop: VALU write -> permlane read
  auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  HalfPair p;
  p.lo = __builtin_bit_cast(float, (int)r[0]);
  p.hi = __builtin_bit_cast(float, (int)r[1]);
  return p;
}
__device__ __forceinline__ float max_both_halves(float x) {
  HalfPair p = both_halves(x);
  return fmaxf(p.lo, p.hi);
}
__device__ __forceinline__ float sum_both_halves(float x) {
  HalfPair p = both_halves(x);
  return p.lo + p.hi;
}

// LDS tile layout for a [rows][128] bf16 tile: row pitch 256 B, the sixteen 16-byte
// granules of a row are permuted by XOR with a 4-bit code of the row.  The code is a linear
// map over GF(2) of the low four row bits (images 0x7, 0xb, 0x4, 0x9 of bits 0..3), picked by
// an exhaustive search over all 20160 invertible maps, timed on the GPU, for the two access
// patterns of the MFMA operand loads on gfx950: 128-bit reads of one granule column over 32
// consecutive rows (246 B/clk/CU, the LDS peak) and transposing 64-bit reads of 4
// consecutive rows x 2 granules (185 B/clk/CU; a plain bit rotation reaches only 116).
__device__ __forceinline__ int row_code(int row) {
  return ((row & 1) ? 0x7 : 0) ^ ((row & 2) ? 0xb : 0) ^ ((row & 4) ? 0x4 : 0) ^ ((row & 8) ? 0x9 : 0);
}
__device__ __forceinline__ int tile_off(int row, int granule) {
  return row * 256 + ((granule ^ row_code(row)) << 4);
}

__device__ __forceinline__ bf16x8 lds_read_b128(const char* lds, int byte_off) {
  return *reinterpret_cast<const bf16x8*>(lds + byte_off);
}
// Transposing LDS read: within each group of 16 lanes, lane j supplies the address of 4
// consecutive bf16 of matrix row (j/4), columns 4*(j%4)..+3; lane i receives column i of
// rows 0..3.
__device__ __forceinline__ bf16x4 lds_read_tr(const char* lds, int byte_off) {
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (lds_s16x4*)(__attribute__((address_space(3))) char*)(lds + byte_off));
  return __builtin_bit_cast(bf16x4, v);
}

// Raw buffer access: loads beyond `bytes` return 0 without touching memory, so ragged tile
// tails and prefetches past the end need no branch.  The whole offset goes into the VGPR
// operand (the range check covers it).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ i32x4 buffer_load_b128(__amdgpu_buffer_rsrc_t rsrc, int byte_off) {
  return __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, 0));
}

// HBM -> LDS DMA: one wave-wide 128-bit buffer load with the LDS modifier.  Lane i's 16
// bytes land at lds_base + 16*i (lds_base wave-uniform, passed through M0); offsets beyond
// the buffer's size write zeros.  Issued as inline assembly on purpose: the compiler then
// does not treat it as an LDS store that every later LDS read must wait for (it would drain
// the whole memory queue before each read).  Ordering against the readers is the caller's
// job: s_waitcnt vmcnt(n) followed by a workgroup barrier.
__device__ __forceinline__ void dma_b128_to_lds(__amdgpu_buffer_rsrc_t rsrc, unsigned lds_base, int voffset) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_base), "v"(voffset), "s"(rsrc) : "memory", "m0");
}
// Same with 32 bits per lane: lane i's dword lands at lds_base + 4*i.
__device__ __forceinline__ void dma_b32_to_lds(__amdgpu_buffer_rsrc_t rsrc, unsigned lds_base, int voffset) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, 0 offen lds"
               :: "s"(lds_base), "v"(voffset), "s"(rsrc) : "memory", "m0");
}
// LDS byte address of a pointer into the workgroup's dynamic shared memory.
__device__ __forceinline__ unsigned lds_addr(const void* p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const char*)(const char*)p;
}

// MFMA with the accumulator pinned to accumulation registers (AGPRs).  Used for the long-lived
// output accumulators so that the register allocator can never move them through VGPRs.
// As inline assembly the instruction is invisible to the compiler's hazard recognizer:
//  - a VGPR written by a vector instruction must not be read by an MFMA in the next two
//    cycles: the leading s_nop covers the operand copies the compiler may place right before;
//  - the accumulator must not be touched by other instructions until the MFMA has drained:
//    callers go through mfma_acc_fence() before reading or rewriting it.
__device__ __forceinline__ void mfma32_acc(f32x16& acc, bf16x8 a, bf16x8 b) {
  asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// Waits until every MFMA issued so far has written its accumulator (an MFMA takes at most
// 16 passes of 4 cycles; 3 x 16 idle cycles cover it with margin) and orders the listed
// accumulators after it.
__device__ __forceinline__ void mfma_acc_fence(f32x16 (&acc)[2][4]) {
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15"
               : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]),
                 "+a"(acc[1][0]), "+a"(acc[1][1]), "+a"(acc[1][2]), "+a"(acc[1][3]));
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

}  // namespace burst
