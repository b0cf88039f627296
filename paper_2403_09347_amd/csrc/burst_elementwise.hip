// HBM-bound steps of the path: state init, finalize, standalone merge (paper Alg. 1) and
// D = rowsum(dO o O) (paper Alg. 2 pre-step).  One thread handles 4 consecutive elements of
// a row (128-bit accesses); the d/4 threads of a row are consecutive lanes, so every
// wavefront touches whole rows and per-row scalars are read once per row.
#include "burst_common.h"

namespace burst {

__global__ void __launch_bounds__(256)
state_init_kernel(float* __restrict__ O_acc, float* __restrict__ m, float* __restrict__ l,
                  long long n_o4, long long n_rows) {
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  long long stride = (long long)gridDim.x * 256;
  f32x4 z = {0.f, 0.f, 0.f, 0.f};
  for (long long k = i; k < n_o4; k += stride) reinterpret_cast<f32x4*>(O_acc)[k] = z;
  for (long long k = i; k < n_rows; k += stride) { m[k] = BURST_NEG_INF; l[k] = 0.f; }
}

// Scalar tail-safe variant for d not a multiple of 4 is handled by VEC = 1.
template <typename OutT, int VEC>
__global__ void __launch_bounds__(256)
finalize_kernel(const float* __restrict__ O_acc, const float* __restrict__ m, const float* __restrict__ l,
                OutT* __restrict__ O_out, float* __restrict__ lse, long long n_rows, int d, QRows qr) {
  const int per_row = d / VEC;
  long long total = n_rows * per_row;
  long long stride = (long long)gridDim.x * 256;
  for (long long k = (long long)blockIdx.x * 256 + threadIdx.x; k < total; k += stride) {
    long long row = k / per_row;
    int c = (int)(k - row * per_row);
    float lv = l[row];
    float inv = lv > 0.f ? 1.0f / lv : 0.f;
    if (c == 0) lse[row] = lv > 0.f ? m[row] + __logf(lv) : BURST_NEG_INF;
    const float* src = O_acc + row * d + c * VEC;
    OutT* dst = O_out + qr.off(row) + c * VEC;
    if (VEC == 4) {
      f32x4 v = *reinterpret_cast<const f32x4*>(src);
      if (sizeof(OutT) == 4) {
        f32x4 r;
        for (int t = 0; t < 4; t++) r[t] = lv > 0.f ? v[t] * inv : 0.f;
        *reinterpret_cast<f32x4*>(dst) = r;
      } else {
        bf16x4 r;
        for (int t = 0; t < 4; t++) r[t] = (bf16)(lv > 0.f ? v[t] * inv : 0.f);
        *reinterpret_cast<bf16x4*>(dst) = r;
      }
    } else {
      dst[0] = (OutT)(lv > 0.f ? src[0] * inv : 0.f);
    }
  }
}

// Standalone merge.  The state is updated in place, so every thread of a row must read the
// row's old (m, l) before the new ones are written.  Both kernels keep a row inside ONE
// wavefront: its loads of (m, l) precede the store in program order.
//   packed: d/4 lanes per row (d/4 divides 64), 128-bit accesses
__global__ void __launch_bounds__(256)
merge_state_packed_kernel(float* __restrict__ O_a, float* __restrict__ m_a, float* __restrict__ l_a,
                          const float* __restrict__ O_b, const float* __restrict__ m_b,
                          const float* __restrict__ l_b, long long n_rows, int d) {
  const int per_row = d >> 2;
  long long total = n_rows * per_row;
  long long stride = (long long)gridDim.x * 256;
  for (long long k = (long long)blockIdx.x * 256 + threadIdx.x; k < total; k += stride) {
    long long row = k / per_row;
    int c = (int)(k - row * per_row);
    float ma = m_a[row], mb = m_b[row], la = l_a[row], lb = l_b[row];
    float mn = fmaxf(ma, mb);
    float ref = (mn == BURST_NEG_INF) ? 0.f : mn;
    float fa = __expf(ma - ref), fb = __expf(mb - ref);   // exp(-inf) = 0
    float* pa = O_a + row * d + c * 4;
    f32x4 va = *reinterpret_cast<const f32x4*>(pa);
    f32x4 vb = *reinterpret_cast<const f32x4*>(O_b + row * d + c * 4);
    f32x4 r;
    for (int t = 0; t < 4; t++)
      r[t] = (fa == 0.f ? 0.f : fa * va[t]) + (fb == 0.f ? 0.f : fb * vb[t]);
    *reinterpret_cast<f32x4*>(pa) = r;
    if (c == 0) {
      m_a[row] = mn;
      l_a[row] = (fa == 0.f ? 0.f : fa * la) + (fb == 0.f ? 0.f : fb * lb);
    }
  }
}
//   generic: one wavefront per row, any d
__global__ void __launch_bounds__(256)
merge_state_row_kernel(float* __restrict__ O_a, float* __restrict__ m_a, float* __restrict__ l_a,
                       const float* __restrict__ O_b, const float* __restrict__ m_b,
                       const float* __restrict__ l_b, long long n_rows, int d) {
  const int lane = threadIdx.x & 63;
  long long wave = ((long long)blockIdx.x * 256 + threadIdx.x) >> 6;
  long long nwaves = ((long long)gridDim.x * 256) >> 6;
  for (long long row = wave; row < n_rows; row += nwaves) {
    float ma = m_a[row], mb = m_b[row], la = l_a[row], lb = l_b[row];
    float mn = fmaxf(ma, mb);
    float ref = (mn == BURST_NEG_INF) ? 0.f : mn;
    float fa = __expf(ma - ref), fb = __expf(mb - ref);
    for (int c = lane; c < d; c += 64) {
      float* pa = O_a + row * d + c;
      pa[0] = (fa == 0.f ? 0.f : fa * pa[0]) + (fb == 0.f ? 0.f : fb * O_b[row * d + c]);
    }
    if (lane == 0) {
      m_a[row] = mn;
      l_a[row] = (fa == 0.f ? 0.f : fa * la) + (fb == 0.f ? 0.f : fb * lb);
    }
  }
}

// D = rowsum(dO o O): the threads of a row are `per_row` consecutive lanes (a power of two
// <= 64 for the vector path), reduced with lane shuffles.
template <typename T>
__global__ void __launch_bounds__(256)
bwd_prepare_kernel(const T* __restrict__ O, const T* __restrict__ dO, float* __restrict__ D,
                   long long n_rows, int d, QRows qr) {
  // one wavefront per row, lanes stride over the row in chunks of 4 elements when possible
  const int lane = threadIdx.x & 63;
  long long wave = ((long long)blockIdx.x * 256 + threadIdx.x) >> 6;
  long long nwaves = ((long long)gridDim.x * 256) >> 6;
  const bool vec = (d % 4) == 0;
  for (long long row = wave; row < n_rows; row += nwaves) {
    const T* o = O + qr.off(row);
    const T* g = dO + qr.off(row);
    float acc = 0.f;
    if (vec) {
      for (int c = lane * 4; c < d; c += 256) {
        if (sizeof(T) == 4) {
          f32x4 a = *reinterpret_cast<const f32x4*>(o + c);
          f32x4 b = *reinterpret_cast<const f32x4*>(g + c);
          for (int t = 0; t < 4; t++) acc += a[t] * b[t];
        } else {
          bf16x4 a = *reinterpret_cast<const bf16x4*>(o + c);
          bf16x4 b = *reinterpret_cast<const bf16x4*>(g + c);
          for (int t = 0; t < 4; t++) acc += (float)a[t] * (float)b[t];
        }
      }
    } else {
      for (int c = lane; c < d; c += 64) acc += (float)o[c] * (float)g[c];
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) D[row] = acc;
  }
}

// Row-packed variant for d = 128 (32 lanes x 4 elements per row, two rows per wavefront):
// fully coalesced 8-byte (bf16) or 16-byte (fp32) loads.
template <typename T>
__global__ void __launch_bounds__(256)
bwd_prepare_d128_kernel(const T* __restrict__ O, const T* __restrict__ dO, float* __restrict__ D,
                        long long n_rows, QRows qr) {
  long long stride = (long long)gridDim.x * 256;
  long long total = n_rows * 32;
  long long total_pad = (total + 63) & ~63LL;      // keep whole wavefronts in the loop for the shuffles
  for (long long k = (long long)blockIdx.x * 256 + threadIdx.x; k < total_pad; k += stride) {
    float acc = 0.f;
    long long row = k >> 5;
    if (k < total) {
      const size_t c = qr.off(row) + (size_t)(k & 31) * 4;
      if (sizeof(T) == 4) {
        f32x4 a = *reinterpret_cast<const f32x4*>(O + c);
        f32x4 b = *reinterpret_cast<const f32x4*>(dO + c);
        for (int t = 0; t < 4; t++) acc += a[t] * b[t];
      } else {
        bf16x4 a = *reinterpret_cast<const bf16x4*>(O + c);
        bf16x4 b = *reinterpret_cast<const bf16x4*>(dO + c);
        for (int t = 0; t < 4; t++) acc += (float)a[t] * (float)b[t];
      }
    }
    for (int off = 16; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (k < total && (k & 31) == 0) D[row] = acc;
  }
}

__global__ void __launch_bounds__(256)
zero_fill_kernel(float* __restrict__ p, long long n) {
  long long stride = (long long)gridDim.x * 256;
  long long n4 = n >> 2;
  f32x4 z = {0.f, 0.f, 0.f, 0.f};
  for (long long k = (long long)blockIdx.x * 256 + threadIdx.x; k < n4; k += stride)
    reinterpret_cast<f32x4*>(p)[k] = z;
  for (long long k = (n4 << 2) + (long long)blockIdx.x * 256 + threadIdx.x; k < n; k += stride) p[k] = 0.f;
}

static inline unsigned grid_for(long long work_items, int per_block = 256, unsigned cap = 256 * 16) {
  long long b = (work_items + per_block - 1) / per_block;
  if (b < 1) b = 1;
  if (b > cap) b = cap;
  return (unsigned)b;
}


int launch_state_init(const KParams& p, float* O_acc, float* m, float* l, hipStream_t s) {
  long long rows = (long long)p.B * p.H * p.Nq;
  long long n_o = rows * p.d;
  if (rows == 0) return BURST_OK;
  if (n_o % 4 != 0) {  // odd sizes: scalar fill through the generic zero kernel + row init
    BURST_LAUNCH(zero_fill_kernel, dim3(grid_for(n_o)), dim3(256), 0, s, O_acc, n_o);
    BURST_LAUNCH(state_init_kernel, dim3(grid_for(rows)), dim3(256), 0, s, O_acc, m, l, 0LL, rows);
  } else {
    BURST_LAUNCH(state_init_kernel, dim3(grid_for(n_o / 4)), dim3(256), 0, s, O_acc, m, l, n_o / 4, rows);
  }
  return launch_status();
}

int launch_finalize(const KParams& p, int dtype, const float* O_acc, const float* m, const float* l,
                    void* O_out, float* lse, hipStream_t s) {
  long long rows = (long long)p.B * p.H * p.Nq;
  if (rows == 0) return BURST_OK;
  bool vec = (p.d % 4) == 0;
  unsigned g = grid_for(rows * (vec ? p.d / 4 : p.d));
  if (dtype == BURST_BF16) {
    if (vec) BURST_LAUNCH((finalize_kernel<bf16, 4>), dim3(g), dim3(256), 0, s, O_acc, m, l, (bf16*)O_out, lse, rows, p.d, p.q_rows());
    else BURST_LAUNCH((finalize_kernel<bf16, 1>), dim3(g), dim3(256), 0, s, O_acc, m, l, (bf16*)O_out, lse, rows, p.d, p.q_rows());
  } else {
    if (vec) BURST_LAUNCH((finalize_kernel<float, 4>), dim3(g), dim3(256), 0, s, O_acc, m, l, (float*)O_out, lse, rows, p.d, p.q_rows());
    else BURST_LAUNCH((finalize_kernel<float, 1>), dim3(g), dim3(256), 0, s, O_acc, m, l, (float*)O_out, lse, rows, p.d, p.q_rows());
  }
  return launch_status();
}

int launch_merge_state(const KParams& p, float* O_a, float* m_a, float* l_a,
                       const float* O_b, const float* m_b, const float* l_b, hipStream_t s) {
  long long rows = (long long)p.B * p.H * p.Nq;
  if (rows == 0) return BURST_OK;
  if (p.d % 4 == 0 && 64 % (p.d / 4) == 0) {
    BURST_LAUNCH(merge_state_packed_kernel, dim3(grid_for(rows * (p.d / 4))), dim3(256), 0, s,
                       O_a, m_a, l_a, O_b, m_b, l_b, rows, p.d);
  } else {
    BURST_LAUNCH(merge_state_row_kernel, dim3(grid_for(rows * 64)), dim3(256), 0, s,
                       O_a, m_a, l_a, O_b, m_b, l_b, rows, p.d);
  }
  return launch_status();
}

int launch_bwd_prepare(const KParams& p, int dtype, const void* O, const void* dO, float* D, hipStream_t s) {
  long long rows = (long long)p.B * p.H * p.Nq;
  if (rows == 0) return BURST_OK;
  if (p.d == 128) {
    unsigned g = grid_for(rows * 32);
    if (dtype == BURST_BF16) BURST_LAUNCH((bwd_prepare_d128_kernel<bf16>), dim3(g), dim3(256), 0, s, (const bf16*)O, (const bf16*)dO, D, rows, p.q_rows());
    else BURST_LAUNCH((bwd_prepare_d128_kernel<float>), dim3(g), dim3(256), 0, s, (const float*)O, (const float*)dO, D, rows, p.q_rows());
  } else {
    unsigned g = grid_for(rows * 64);
    if (dtype == BURST_BF16) BURST_LAUNCH((bwd_prepare_kernel<bf16>), dim3(g), dim3(256), 0, s, (const bf16*)O, (const bf16*)dO, D, rows, p.d, p.q_rows());
    else BURST_LAUNCH((bwd_prepare_kernel<float>), dim3(g), dim3(256), 0, s, (const float*)O, (const float*)dO, D, rows, p.d, p.q_rows());
  }
  return launch_status();
}

int launch_zero_fill(float* ptr, long long n, hipStream_t s) {
  if (n <= 0) return BURST_OK;
  BURST_LAUNCH(zero_fill_kernel, dim3(grid_for(n / 4 + 1)), dim3(256), 0, s, ptr, n);
  return launch_status();
}

}  // namespace burst
