// C ABI (see include/burst.h): argument validation and dispatch to the kernels.
#include <hip/hip_runtime.h>
#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>
#include "burst_common.h"

namespace burst {
int launch_state_init(const KParams&, float*, float*, float*, hipStream_t);
int launch_finalize(const KParams&, int, const float*, const float*, const float*, void*, float*, hipStream_t);
int launch_merge_state(const KParams&, float*, float*, float*, const float*, const float*, const float*, hipStream_t);
int launch_bwd_prepare(const KParams&, int, const void*, const void*, float*, hipStream_t);
int launch_zero_fill(float*, long long, hipStream_t);
int launch_fwd_mfma(const KParams&, const void*, const void*, const void*, float*, float*, float*, hipStream_t);
int launch_fwd_generic(const KParams&, int, const void*, const void*, const void*, float*, float*, float*, hipStream_t);
int launch_bwd_dq_mfma(const KParams&, const void*, const void*, const void*, const void*, const float*,
                       const float*, float*, int, hipStream_t);
int launch_bwd_dkv_mfma(const KParams&, const void*, const void*, const void*, const void*, const float*,
                        const float*, float*, float*, int, hipStream_t, int key_waves);
int launch_bwd_dq_generic(const KParams&, int, const void*, const void*, const void*, const void*, const float*,
                          const float*, float*, int, hipStream_t);
int launch_bwd_dkv_generic(const KParams&, int, const void*, const void*, const void*, const void*, const float*,
                           const float*, float*, float*, int, hipStream_t);
namespace d64 {
int launch_fwd(const KParams&, const void*, const void*, const void*, float*, float*, float*, hipStream_t);
int launch_bwd_dq(const KParams&, const void*, const void*, const void*, const void*, const float*,
                  const float*, float*, int, hipStream_t);
int launch_bwd_dkv(const KParams&, const void*, const void*, const void*, const void*, const float*,
                   const float*, float*, float*, int, hipStream_t);
}  // namespace d64
namespace d128p {
int launch_fwd(const KParams&, const void*, const void*, const void*, float*, float*, float*, hipStream_t);
int launch_bwd_dq(const KParams&, const void*, const void*, const void*, const void*, const float*,
                  const float*, float*, int, hipStream_t);
int launch_bwd_dkv(const KParams&, const void*, const void*, const void*, const void*, const float*,
                   const float*, float*, float*, int, hipStream_t);
}  // namespace d128p
size_t materialized_workspace_bytes(const KParams&, int);
size_t materialized_bwd_workspace_bytes(const KParams&, int);
int launch_bwd_materialized(const KParams&, int, bool, const void*, const void*, const void*, const void*, const float*,
                            const float*, float*, float*, float*, int, int, void*, hipStream_t);
int launch_fwd_materialized(const KParams&, int, bool, const void*, const void*, const void*, float*, float*, float*,
                            void*, hipStream_t);
}  // namespace burst

namespace burst {
thread_local bool t_validate_only = false;
}

namespace {

using burst::KParams;

constexpr int kMaxDevices = 64;
int g_arch_ok[kMaxDevices];                 // 0 = unknown, 1 = gfx950, -1 = other
std::mutex g_mutex;

// Library-owned D buffers for burst_local_bwd(D = NULL): one per (device, stream), so that calls on
// different streams never share one.  A buffer that has become too small is replaced by one of at
// least twice its size and is NOT freed: kernels already enqueued may still read it, and hipFree
// would synchronise the device.  The retired blocks stay allocated until the process ends (less
// than the final size in total).  Calls with D = NULL hold g_bwd_mutex from the lookup to the last
// enqueue, so two host threads that share a stream cannot interleave their kernels around the
// shared buffer.
struct DScratch { int dev; hipStream_t stream; float* ptr; size_t elems; };
std::vector<DScratch> g_d_scratch;
std::mutex g_bwd_mutex;

// Static device scratch for burst_local_bwd_static (the entry point for callers that cannot
// allocate): D of one call, BURST_STATIC_MAX_ROWS floats = 8 MiB, held by every GPU the library runs
// on until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the device address is looked up once per device (each GPU has its own
// copy) and kept here, and that pointer, never the name, is what kernels are given.
static __device__ __align__(256) float scratch[BURST_STATIC_MAX_ROWS];
float* g_static_d[kMaxDevices];
burst::DeviceOnce g_static_d_once;

int static_d_buffer(float** out) {
  const int st = g_static_d_once.run([] {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return (int)BURST_ERR_LAUNCH;
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return (int)BURST_ERR_LAUNCH;
    g_static_d[dev] = static_cast<float*>(ptr);
    return (int)BURST_OK;
  });
  if (st != BURST_OK) return st;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BURST_ERR_LAUNCH;
  *out = g_static_d[dev];
  return BURST_OK;
}

int check_arch() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BURST_ERR_ARCH;
  std::lock_guard<std::mutex> lock(g_mutex);
  if (g_arch_ok[dev] == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return BURST_ERR_ARCH;
    g_arch_ok[dev] = (std::strncmp(prop.gcnArchName, "gfx950", 6) == 0) ? 1 : -1;
  }
  return g_arch_ok[dev] == 1 ? BURST_OK : BURST_ERR_ARCH;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Validates the parameter block; fills the kernel-side copy.
int check_params(const burst_params* p, KParams* k) {
  if (p == nullptr) return BURST_ERR_NULL;
  if (p->dtype != BURST_BF16 && p->dtype != BURST_F32) return BURST_ERR_DTYPE;
  if (p->B < 1 || p->H < 1 || p->Nq < 0 || p->Nc < 0 || p->d < 1 || p->d > 128) return BURST_ERR_SHAPE;
  if (!(p->scale > 0.f) || !std::isfinite(p->scale)) return BURST_ERR_SHAPE;
  if ((long long)p->B * p->H > 0x7fffffffLL) return BURST_ERR_SHAPE;
  // rows must be addressable with 16-byte aligned row starts for the vector kernels
  k->B = p->B; k->H = p->H; k->Nq = p->Nq; k->Nc = p->Nc; k->d = p->d;
  k->causal = p->causal != 0; k->scale = p->scale; k->q_off = p->q_off; k->k_off = p->k_off;
  if (p->window < 0) return BURST_ERR_SHAPE;
  k->window = p->window;
  k->group = 1;
  if (p->kv_heads != 0) {
    if (p->kv_heads < 0 || p->H % p->kv_heads != 0) return BURST_ERR_SHAPE;
    k->group = p->H / p->kv_heads;
  }
  // strides: all zero = contiguous [B, heads, rows, d]
  {
    const long long hk = p->H / k->group, d = p->d;
    burst::Layout& L = k->lay;
    L.heads = p->H; L.kv_heads = (int)hk;
    const int64_t* q = p->q_strides; const int64_t* kv = p->kv_strides;
    const long long unit = p->dtype == BURST_BF16 ? 8 : 4;     // 16-byte granules
    if (q[0] == 0 && q[1] == 0 && q[2] == 0) {
      L.qs_r = d; L.qs_h = (long long)p->Nq * d; L.qs_b = L.qs_h * p->H;
    } else {
      if (q[0] < 0 || q[1] < 0 || q[2] < d || q[0] % unit || q[1] % unit || q[2] % unit) return BURST_ERR_SHAPE;
      L.qs_b = q[0]; L.qs_h = q[1]; L.qs_r = q[2];
    }
    if (kv[0] == 0 && kv[1] == 0 && kv[2] == 0) {
      L.ks_r = d; L.ks_h = (long long)p->Nc * d; L.ks_b = L.ks_h * hk;
    } else {
      if (kv[0] < 0 || kv[1] < 0 || kv[2] < d || kv[0] % unit || kv[1] % unit || kv[2] % unit) return BURST_ERR_SHAPE;
      L.ks_b = kv[0]; L.ks_h = kv[1]; L.ks_r = kv[2];
    }
  }
  k->bmask = nullptr; k->bsize = 64; k->bpitch = 0; k->bhstride = 0;
  if (p->block_mask != nullptr) {
    if (p->block <= 0 || p->block % 64 != 0) return BURST_ERR_SHAPE;
    k->bmask = p->block_mask; k->bsize = p->block; k->bpitch = (p->Nc + p->block - 1) / p->block;
    k->bhstride = p->block_mask_stride;
    // one matrix per (batch, head): they must not overlap
    const long long matrix = (long long)((p->Nq + p->block - 1) / p->block) * k->bpitch;
    if (k->bhstride != 0 && k->bhstride < matrix) return BURST_ERR_SHAPE;
  }
  return BURST_OK;
}

#define REQUIRE_PTR(ptr)                                 \
  do {                                                   \
    if ((ptr) == nullptr) return BURST_ERR_NULL;         \
    if (!aligned16(ptr)) return BURST_ERR_ALIGN;         \
  } while (0)

// The MFMA kernels address a head's rows through 32-bit byte offsets (plus a few tiles of
// prefetch past the end; dK/dV: the rows of all query heads of a group, from the first head's
// row 0); longer or wider-strided slices or chunks take the generic kernels.
constexpr int kMaxMfmaRows = 4 * 1024 * 1024;
bool spans_fit(const burst_params* p, const KParams& k) {
  const long long q = ((long long)p->Nq + 1024) * k.lay.qs_r * 2 + (long long)(k.group - 1) * k.lay.qs_h * 2;
  const long long kv = ((long long)p->Nc + 1024) * k.lay.ks_r * 2;
  return q <= 0xffffffffLL && kv <= 0xffffffffLL;
}
// With block flags the MFMA kernels keep a list of visible tiles in LDS (8192 tiles of 64 keys or
// rows, or 16384 of 32 keys): longer masked slices or chunks take the generic kernels.
constexpr int kMaxMaskedRows = 8192 * 64;
bool use_mfma(const burst_params* p, const KParams& k) {
  return p->dtype == BURST_BF16 && p->d == 128 && p->Nq <= kMaxMfmaRows && p->Nc <= kMaxMfmaRows && spans_fit(p, k);
}
// bf16, d = 64 has MFMA kernels of its own.
bool use_d64(const burst_params* p, const KParams& k) {
  if (!(p->dtype == BURST_BF16 && p->d == 64 && p->Nq <= kMaxMfmaRows && p->Nc <= kMaxMfmaRows &&
        spans_fit(p, k))) return false;
  if (p->block_mask == nullptr) return true;
  // with block flags: lists of at most 4096 tiles (32 keys or rows each; rows of all heads of a group)
  const long long group = (p->kv_heads > 0) ? p->H / p->kv_heads : 1;
  return p->Nc <= 4096 * 32 && group * ((p->Nq + 31) / 32) <= 4096;
}
// The forward and dQ kernels for d = 128 run one 256-row workgroup per CU, so a call takes
// ceil(workgroups / 256) rounds on the chip's 256 CUs.  When the last round is at most half full
// (short query slices, or a workgroup count just above a multiple of 256) the plainly written
// kernels with 128 rows per workgroup and two workgroups per CU do better: 1.3-1.5x (forward)
// and 1.1-1.25x (backward) at up to 128 workgroups, 15 % at 320, 3-6 % (forward) at 384 .. 1152;
// they lose 3-6 % where the rounds are full, and the gain fades as the rounds grow in number.
std::atomic<int> g_kernel_family{0};            // burst_set_kernel_family
bool use_plain128(const burst_params* p, const KParams& k) {
  if (!use_mfma(p, k)) return false;
  const bool flags = p->block_mask != nullptr;
  if (flags && p->Nc > 4096 * 32) return false;    // their tile lists hold 4096 entries (32-key tiles in dQ)
  const int family = g_kernel_family.load(std::memory_order_relaxed);
  if (family != 0) return family == 2;
  // Block flags finer than the 256-row workgroups of the list-driven kernels: the plain kernels
  // skip per wavefront (32 rows x 64 or 32 keys), which is what such patterns need.
  if (flags) return p->block < 256;
  const long long wgs = (long long)p->B * p->H * ((p->Nq + 255) / 256);
  const long long last = wgs % 256;                // workgroups of the last round (0 = full)
  return last != 0 && last <= 128 && wgs <= 1536;
}
// The dK/dV MFMA kernel walks the query tiles of all heads of a group as one list: whole 64-row
// tiles per head and at most 8192 tiles in all; other grouped shapes take the generic kernel.
bool dkv_mfma_ok(const burst_params* p, const KParams& k) {
  if (k.group > 1) return p->Nq % 64 == 0 && (long long)k.group * (p->Nq / 64) <= 8192 && k.group <= 256 &&
                          (long long)k.group * p->Nq <= kMaxMfmaRows;
  return p->block_mask == nullptr || p->Nq <= kMaxMaskedRows;
}

// Entry points that enqueue several kernels: one pass over the launchers in validate-only mode
// (shape limits, function attributes), so that an error is reported with nothing enqueued, then
// the real pass.
template <typename F>
int validated(F&& enqueue) {
  burst::t_validate_only = true;
  const int e = enqueue();
  burst::t_validate_only = false;
  return e != BURST_OK ? e : enqueue();
}

// Block flags narrower than the 128 keys of a dK/dV workgroup: the hand-scheduled kernel runs in
// its shape with 64-key workgroups, whose tile lists hold what 64 keys need (its time then
// follows the density; a 128-key workgroup cannot skip what only half of its keys need).  Those
// lists hold 2048 entries of 64 query rows (all heads of a group).
int dkv_key_waves(const burst_params* p, const KParams& k) {
  if (p->block_mask == nullptr || p->block >= 128) return 4;
  if ((long long)k.group * ((p->Nq + 63) / 64) > 2048) return 4;
  return g_kernel_family.load(std::memory_order_relaxed) == 0 ? 2 : 4;
}
// The plainly written dK/dV kernel with 64-key workgroups runs when the plain family is forced.
// Its tile lists hold 4096 entries of 32 query rows (all heads of a group).
bool use_plain128_dkv(const burst_params* p, const KParams& k) {
  if (!use_mfma(p, k)) return false;
  const bool flags = p->block_mask != nullptr;
  if (flags && (long long)k.group * ((p->Nq + 31) / 32) > 4096) return false;
  return g_kernel_family.load(std::memory_order_relaxed) == 2;
}

// Caller holds g_bwd_mutex.
int get_d_scratch(hipStream_t stream, size_t elems, float** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return BURST_ERR_ALLOC;
  DScratch* slot = nullptr;
  for (DScratch& e : g_d_scratch)
    if (e.dev == dev && e.stream == stream) slot = &e;
  if (slot == nullptr) {
    g_d_scratch.push_back(DScratch{dev, stream, nullptr, 0});
    slot = &g_d_scratch.back();
  }
  if (slot->elems < elems) {
    const size_t want = elems > 2 * slot->elems ? elems : 2 * slot->elems;
    float* ptr = nullptr;
    if (hipMalloc(&ptr, want * sizeof(float)) != hipSuccess) return BURST_ERR_ALLOC;
    slot->ptr = ptr;                               // the old block, if any, is retired, not freed
    slot->elems = want;
  }
  *out = slot->ptr;
  return BURST_OK;
}

}  // namespace

extern "C" {

int burst_state_init(float* O_acc, float* m, float* l, const burst_params* p, void* stream) {
  KParams k;
  int st = check_params(p, &k);
  if (st != BURST_OK) return st;
  if ((long long)k.B * k.H * k.Nq == 0) return BURST_OK;
  REQUIRE_PTR(O_acc); REQUIRE_PTR(m); REQUIRE_PTR(l);
  if ((st = check_arch()) != BURST_OK) return st;
  return burst::launch_state_init(k, O_acc, m, l, (hipStream_t)stream);
}

int burst_local_fwd(const void* Q, const void* K_chunk, const void* V_chunk,
                    float* O_acc, float* m, float* l, const burst_params* p, void* stream) {
  KParams k;
  int st = check_params(p, &k);
  if (st != BURST_OK) return st;
  if ((long long)k.B * k.H * k.Nq == 0 || k.Nc == 0) return BURST_OK;   // an empty chunk is the identity
  REQUIRE_PTR(Q); REQUIRE_PTR(K_chunk); REQUIRE_PTR(V_chunk);
  REQUIRE_PTR(O_acc); REQUIRE_PTR(m); REQUIRE_PTR(l);
  if ((st = check_arch()) != BURST_OK) return st;
  if (use_d64(p, k)) return burst::d64::launch_fwd(k, Q, K_chunk, V_chunk, O_acc, m, l, (hipStream_t)stream);
  if (use_plain128(p, k)) return burst::d128p::launch_fwd(k, Q, K_chunk, V_chunk, O_acc, m, l, (hipStream_t)stream);
  if (use_mfma(p, k) && (p->block_mask == nullptr || p->Nc <= kMaxMaskedRows))
    return burst::launch_fwd_mfma(k, Q, K_chunk, V_chunk, O_acc, m, l, (hipStream_t)stream);
  return burst::launch_fwd_generic(k, p->dtype, Q, K_chunk, V_chunk, O_acc, m, l, (hipStream_t)stream);
}

int burst_set_kernel_family(int family) {
  if (family < 0 || family > 2) return BURST_ERR_SHAPE;
  g_kernel_family.store(family, std::memory_order_relaxed);
  return BURST_OK;
}

int burst_kernel_family_for(const burst_params* p) {
  KParams k;
  const int st = check_params(p, &k);
  if (st != BURST_OK) return st;
  if (use_plain128(p, k)) return 2;
  return use_mfma(p, k) && (p->block_mask == nullptr || p->Nc <= kMaxMaskedRows) ? 1 : 0;
}

size_t burst_workspace_bytes(const burst_params* p) {
  KParams k;
  if (check_params(p, &k) != BURST_OK) return 0;
  return (size_t)k.B * k.H * k.Nq * sizeof(float);
}

size_t burst_materialized_workspace_bytes(const burst_params* p) {
  KParams k;
  if (check_params(p, &k) != BURST_OK) return 0;
  return burst::materialized_workspace_bytes(k, p->dtype);
}

int burst_local_fwd_materialized(const void* Q, const void* K_chunk, const void* V_chunk,
                                 float* O_acc, float* m, float* l,
                                 void* workspace, size_t workspace_bytes,
                                 const burst_params* p, void* stream) {
  KParams k;
  int st = check_params(p, &k);
  if (st != BURST_OK) return st;
  if ((long long)k.B * k.H * k.Nq == 0 || k.Nc == 0) return BURST_OK;   // an empty chunk is the identity
  REQUIRE_PTR(Q); REQUIRE_PTR(K_chunk); REQUIRE_PTR(V_chunk);
  REQUIRE_PTR(O_acc); REQUIRE_PTR(m); REQUIRE_PTR(l);
  if (workspace == nullptr) return BURST_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return BURST_ERR_ALIGN;
  if (workspace_bytes < burst::materialized_workspace_bytes(k, p->dtype)) return BURST_ERR_SHAPE;
  if ((st = check_arch()) != BURST_OK) return st;
  return validated([&] {
    return burst::launch_fwd_materialized(k, p->dtype, use_mfma(p, k), Q, K_chunk, V_chunk, O_acc, m, l, workspace,
                                          (hipStream_t)stream);
  });
}

size_t burst_materialized_bwd_workspace_bytes(const burst_params* p) {
  KParams k;
  if (check_params(p, &k) != BURST_OK) return 0;
  return burst::materialized_bwd_workspace_bytes(k, p->dtype);
}

int burst_local_bwd_materialized(const void* Q, const void* K_chunk, const void* V_chunk,
                                 const void* dO, const float* lse, const float* D,
                                 float* dQ, float* dK_chunk, float* dV_chunk,
                                 int accumulate_dq, int accumulate_dkv,
                                 void* workspace, size_t workspace_bytes,
                                 const burst_params* p, void* stream) {
  KParams k;
  int st = check_params(p, &k);
  if (st != BURST_OK) return st;
  const long long bh = (long long)k.B * k.H;
  const bool have_q = bh * k.Nq > 0, have_k = bh * k.Nc > 0;
  if (!have_q && !have_k) return BURST_OK;
  if (have_q) { REQUIRE_PTR(Q); REQUIRE_PTR(dO); REQUIRE_PTR(lse); REQUIRE_PTR(D); REQUIRE_PTR(dQ); }
  if (have_k) { REQUIRE_PTR(K_chunk); REQUIRE_PTR(V_chunk); REQUIRE_PTR(dK_chunk); REQUIRE_PTR(dV_chunk); }
  if ((st = check_arch()) != BURST_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  if (!have_q || !have_k) {                        // nothing to contract over: the contribution is zero
    if (have_q && !accumulate_dq && (st = burst::launch_zero_fill(dQ, bh * k.Nq * k.d, s)) != BURST_OK) return st;
    if (have_k && !accumulate_dkv) {
      if ((st = burst::launch_zero_fill(dK_chunk, bh / k.group * k.Nc * k.d, s)) != BURST_OK) return st;
      if ((st = burst::launch_zero_fill(dV_chunk, bh / k.group * k.Nc * k.d, s)) != BURST_OK) return st;
    }
    return BURST_OK;
  }
  REQUIRE_PTR(workspace);
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return BURST_ERR_ALIGN;
  if (workspace_bytes < burst::materialized_bwd_workspace_bytes(k, p->dtype)) return BURST_ERR_SHAPE;
  return validated([&] {
    return burst::launch_bwd_materialized(k, p->dtype, use_mfma(p, k), Q, K_chunk, V_chunk, dO, lse, D, dQ, dK_chunk,
                                          dV_chunk, accumulate_dq != 0, accumulate_dkv != 0, workspace, s);
  });
}

int burst_finalize(const float* O_acc, const float* m, const float* l,
                   void* O_out, float* lse, const burst_params* p, void* stream) {
  KParams k;
  int st = check_params(p, &k);
  if (st != BURST_OK) return st;
  if ((long long)k.B * k.H * k.Nq == 0) return BURST_OK;
  REQUIRE_PTR(O_acc); REQUIRE_PTR(m); REQUIRE_PTR(l); REQUIRE_PTR(O_out); REQUIRE_PTR(lse);
  if ((st = check_arch()) != BURST_OK) return st;
  return burst::launch_finalize(k, p->dtype, O_acc, m, l, O_out, lse, (hipStream_t)stream);
}

int burst_merge_state(float* O_a, float* m_a, float* l_a,
                      const float* O_b, const float* m_b, const float* l_b,
                      const burst_params* p, void* stream) {
  KParams k;
  int st = check_params(p, &k);
  if (st != BURST_OK) return st;
  if ((long long)k.B * k.H * k.Nq == 0) return BURST_OK;
  REQUIRE_PTR(O_a); REQUIRE_PTR(m_a); REQUIRE_PTR(l_a);
  REQUIRE_PTR(O_b); REQUIRE_PTR(m_b); REQUIRE_PTR(l_b);
  if ((st = check_arch()) != BURST_OK) return st;
  return burst::launch_merge_state(k, O_a, m_a, l_a, O_b, m_b, l_b, (hipStream_t)stream);
}

int burst_bwd_prepare(const void* O, const void* dO, float* D, const burst_params* p, void* stream) {
  KParams k;
  int st = check_params(p, &k);
  if (st != BURST_OK) return st;
  if ((long long)k.B * k.H * k.Nq == 0) return BURST_OK;
  REQUIRE_PTR(O); REQUIRE_PTR(dO); REQUIRE_PTR(D);
  if ((st = check_arch()) != BURST_OK) return st;
  return burst::launch_bwd_prepare(k, p->dtype, O, dO, D, (hipStream_t)stream);
}

// Shared by the three backward entry points.  which: 1 = dQ, 2 = dK/dV, 3 = both.
// static_d: D == NULL takes the static device scratch instead of an allocated buffer.
static int local_bwd_impl(int which, const void* Q, const void* K_chunk, const void* V_chunk,
                          const void* O, const void* dO, const float* lse, const float* D,
                          float* dQ, float* dK_chunk, float* dV_chunk,
                          int accumulate_dq, int accumulate_dkv,
                          const burst_params* p, void* stream, bool static_d = false) {
  KParams k;
  int st = check_params(p, &k);
  if (st != BURST_OK) return st;
  const bool want_dq = (which & 1) != 0, want_dkv = (which & 2) != 0;
  const long long bh = (long long)k.B * k.H;
  const bool have_q = bh * k.Nq > 0, have_k = bh * k.Nc > 0;
  if (!(want_dq && have_q) && !(want_dkv && have_k)) return BURST_OK;
  if (have_q) { REQUIRE_PTR(Q); REQUIRE_PTR(dO); REQUIRE_PTR(lse); }
  if (have_k) { REQUIRE_PTR(K_chunk); REQUIRE_PTR(V_chunk); }
  if (want_dq && have_q) REQUIRE_PTR(dQ);
  if (want_dkv && have_k) { REQUIRE_PTR(dK_chunk); REQUIRE_PTR(dV_chunk); }
  if (D != nullptr && !aligned16(D)) return BURST_ERR_ALIGN;
  if (D == nullptr && have_q && have_k) REQUIRE_PTR(O);
  if (static_d && bh * k.Nq > (long long)BURST_STATIC_MAX_ROWS) return BURST_ERR_TOO_LARGE;
  if ((st = check_arch()) != BURST_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  // Degenerate sides: nothing to contract over, the contribution is zero.
  if (!have_q || !have_k) {
    if (want_dq && have_q && !accumulate_dq &&
        (st = burst::launch_zero_fill(dQ, bh * k.Nq * k.d, s)) != BURST_OK) return st;
    if (want_dkv && have_k && !accumulate_dkv) {
      if ((st = burst::launch_zero_fill(dK_chunk, bh / k.group * k.Nc * k.d, s)) != BURST_OK) return st;
      if ((st = burst::launch_zero_fill(dV_chunk, bh / k.group * k.Nc * k.d, s)) != BURST_OK) return st;
    }
    return BURST_OK;
  }
  // The kernels of this call: D (when it is not given), then the dQ half, then the dK/dV half.
  const bool mfma_dq = use_mfma(p, k) && (p->block_mask == nullptr || p->Nc <= kMaxMaskedRows);
  const bool mfma_dkv = use_mfma(p, k) && dkv_mfma_ok(p, k);
  const bool d64 = use_d64(p, k), plain128 = use_plain128(p, k), plain128_dkv = use_plain128_dkv(p, k);
  const bool adq = accumulate_dq != 0, adkv = accumulate_dkv != 0;
  auto enqueue = [&](const float* Duse, float* Dwrite) -> int {
    int e;
    if (Dwrite != nullptr && (e = burst::launch_bwd_prepare(k, p->dtype, O, dO, Dwrite, s)) != BURST_OK) return e;
    if (want_dq) {
      e = d64 ? burst::d64::launch_bwd_dq(k, Q, K_chunk, V_chunk, dO, lse, Duse, dQ, adq, s)
        : plain128 ? burst::d128p::launch_bwd_dq(k, Q, K_chunk, V_chunk, dO, lse, Duse, dQ, adq, s)
        : mfma_dq ? burst::launch_bwd_dq_mfma(k, Q, K_chunk, V_chunk, dO, lse, Duse, dQ, adq, s)
                  : burst::launch_bwd_dq_generic(k, p->dtype, Q, K_chunk, V_chunk, dO, lse, Duse, dQ, adq, s);
      if (e != BURST_OK) return e;
    }
    if (want_dkv) {
      e = d64 ? burst::d64::launch_bwd_dkv(k, Q, K_chunk, V_chunk, dO, lse, Duse, dK_chunk, dV_chunk, adkv, s)
        : plain128_dkv ? burst::d128p::launch_bwd_dkv(k, Q, K_chunk, V_chunk, dO, lse, Duse, dK_chunk, dV_chunk, adkv, s)
        : mfma_dkv ? burst::launch_bwd_dkv_mfma(k, Q, K_chunk, V_chunk, dO, lse, Duse, dK_chunk, dV_chunk, adkv, s,
                                                dkv_key_waves(p, k))
                   : burst::launch_bwd_dkv_generic(k, p->dtype, Q, K_chunk, V_chunk, dO, lse, Duse, dK_chunk,
                                                   dV_chunk, adkv, s);
      if (e != BURST_OK) return e;
    }
    return BURST_OK;
  };
  if (D != nullptr) return validated([&] { return enqueue(D, nullptr); });
  std::lock_guard<std::mutex> lock(g_bwd_mutex);
  float* dbuf = nullptr;
  if ((st = static_d ? static_d_buffer(&dbuf) : get_d_scratch(s, (size_t)(bh * k.Nq), &dbuf)) != BURST_OK) return st;
  return validated([&] { return enqueue(dbuf, dbuf); });
}

int burst_local_bwd(const void* Q, const void* K_chunk, const void* V_chunk,
                    const void* O, const void* dO, const float* lse, const float* D,
                    float* dQ, float* dK_chunk, float* dV_chunk,
                    int accumulate_dq, int accumulate_dkv,
                    const burst_params* p, void* stream) {
  return local_bwd_impl(3, Q, K_chunk, V_chunk, O, dO, lse, D, dQ, dK_chunk, dV_chunk,
                        accumulate_dq, accumulate_dkv, p, stream);
}

int burst_local_bwd_static(const void* Q, const void* K_chunk, const void* V_chunk,
                           const void* O, const void* dO, const float* lse,
                           float* dQ, float* dK_chunk, float* dV_chunk,
                           int accumulate_dq, int accumulate_dkv,
                           const burst_params* p, void* stream) {
  return local_bwd_impl(3, Q, K_chunk, V_chunk, O, dO, lse, nullptr, dQ, dK_chunk, dV_chunk,
                        accumulate_dq, accumulate_dkv, p, stream, /*static_d=*/true);
}

int burst_local_bwd_dq(const void* Q, const void* K_chunk, const void* V_chunk,
                       const void* dO, const float* lse, const float* D,
                       float* dQ, int accumulate_dq, const burst_params* p, void* stream) {
  if (D == nullptr) return BURST_ERR_NULL;
  return local_bwd_impl(1, Q, K_chunk, V_chunk, nullptr, dO, lse, D, dQ, nullptr, nullptr,
                        accumulate_dq, 0, p, stream);
}

int burst_local_bwd_dkv(const void* Q, const void* K_chunk, const void* V_chunk,
                        const void* dO, const float* lse, const float* D,
                        float* dK_chunk, float* dV_chunk, int accumulate_dkv,
                        const burst_params* p, void* stream) {
  if (D == nullptr) return BURST_ERR_NULL;
  return local_bwd_impl(2, Q, K_chunk, V_chunk, nullptr, dO, lse, D, nullptr, dK_chunk, dV_chunk,
                        0, accumulate_dkv, p, stream);
}

void* burst_event_create(void) {
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return (void*)e;
}
int burst_event_record(void* event, void* stream) {
  if (event == nullptr) return BURST_ERR_NULL;
  return hipEventRecord((hipEvent_t)event, (hipStream_t)stream) == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
}
int burst_event_elapsed_ms(void* start, void* stop, float* ms) {
  if (start == nullptr || stop == nullptr || ms == nullptr) return BURST_ERR_NULL;
  if (hipEventSynchronize((hipEvent_t)stop) != hipSuccess) return BURST_ERR_LAUNCH;
  return hipEventElapsedTime(ms, (hipEvent_t)start, (hipEvent_t)stop) == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
}
void burst_event_destroy(void* event) {
  if (event != nullptr) (void)hipEventDestroy((hipEvent_t)event);
}

const char* burst_strerror(int status) {
  switch (status) {
    case BURST_OK: return "ok";
    case BURST_ERR_NULL: return "a required pointer is NULL";
    case BURST_ERR_ALIGN: return "a pointer is not 16-byte aligned";
    case BURST_ERR_SHAPE: return "unsupported or inconsistent sizes or scale";
    case BURST_ERR_DTYPE: return "unknown dtype";
    case BURST_ERR_ARCH: return "current device is not gfx950";
    case BURST_ERR_LAUNCH: return "HIP runtime reported a launch error";
    case BURST_ERR_ALLOC: return "internal scratch allocation failed";
    case BURST_ERR_TOO_LARGE: return "B*H*Nq exceeds the static scratch of burst_local_bwd_static (BURST_STATIC_MAX_ROWS rows)";
    default: return "unknown status";
  }
}

int burst_version(void) { return 111; }

}  // extern "C"
