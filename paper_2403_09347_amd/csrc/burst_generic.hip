// Generic (any dtype, any d <= 128, any Nq / Nc) kernels in plain fp32 FMA arithmetic.
// They serve the shapes the MFMA kernels do not cover (fp32 inputs, d != 128); the work per
// call is small there, so they are written for clarity: one wavefront per output row, keys
// (or queries) spread over the 64 lanes, dot products over d done per lane, reductions and
// broadcasts through lane shuffles.  Same mathematics as the tiled kernels: paper Alg. 1 loop
// body + merge for the forward, Alg. 2 block pair for the backward.
#include "burst_common.h"

namespace burst {

struct GenArgs {
  const void* Q; const void* K; const void* V; const void* dO;
  float* O_acc; float* m; float* l;               // forward state
  const float* lse; const float* D;               // backward inputs
  float* dQ; float* dK; float* dV;
  int Nq, Nc, d, BH;
  int causal;
  float scale;
  long long q_off, k_off;
  long long window;
  const uint8_t* bmask; int bsize, bpitch;        // block mask (nullptr = none)
  long long bhstride;                             // bytes between heads' flag matrices (0 = shared)
  Layout lay;                                     // strides of Q, dO and of K, V
  int group;                                      // query heads per key/value head
  int acc_dq, acc_dkv;
};

// Visibility of key `key` of the chunk from query row `row` of the slice (both in range).
__device__ __forceinline__ bool visible(const GenArgs& a, int head, int row, int key) {
  const long long qpos = a.q_off + row, kpos = a.k_off + key;
  if (a.causal && kpos > qpos) return false;
  if (a.window != 0 && kpos <= qpos - a.window) return false;
  if (a.bmask != nullptr && a.bmask[(size_t)head * a.bhstride + (size_t)(row / a.bsize) * a.bpitch + key / a.bsize] == 0) return false;
  return true;
}

template <typename T> __device__ __forceinline__ float ld(const T* p) { return (float)(*p); }

__device__ __forceinline__ float wave_max(float v) {
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// ---------------------------------------------------------------------------- forward
template <typename T>
__global__ void __launch_bounds__(256)
fwd_generic_kernel(GenArgs a) {
  __shared__ float qrow[4][128];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  long long wave = (long long)blockIdx.x * 4 + w;
  long long total = (long long)a.BH * a.Nq;
  const bool live = wave < total;
  if (!live) wave = 0;                             // keep every wavefront up to the barrier
  const int head = (int)(wave / a.Nq), row = (int)(wave % a.Nq);
  const T* Qr = (const T*)a.Q + a.lay.q_base(head) + (size_t)row * a.lay.qs_r;
  const T* Kh = (const T*)a.K + a.lay.kv_base(head / a.group);
  const T* Vh = (const T*)a.V + a.lay.kv_base(head / a.group);
  for (int t = lane; t < a.d; t += 64) qrow[w][t] = ld(Qr + t);
  __syncthreads();
  if (!live) return;
  const long long qpos = a.q_off + row;
  float m_run = BURST_NEG_INF, l_run = 0.f, o0 = 0.f, o1 = 0.f;   // dims lane and lane + 64
  for (int k0 = 0; k0 < a.Nc; k0 += 64) {
    int key = k0 + lane;
    bool vis = key < a.Nc && visible(a, head, row, key);
    float s = BURST_NEG_INF;
    if (vis) {
      float acc = 0.f;
      const T* kr = Kh + (size_t)key * a.lay.ks_r;
      for (int t = 0; t < a.d; t++) acc = __builtin_fmaf(qrow[w][t], ld(kr + t), acc);
      s = acc * a.scale;
    }
    float m_tile = wave_max(s);
    float m_new = fmaxf(m_run, m_tile);
    float ref = (m_new == BURST_NEG_INF) ? 0.f : m_new;
    float p = expf(s - ref);                       // exp(-inf) = 0 for masked keys
    float alpha = expf(m_run - ref);
    l_run = l_run * alpha + wave_sum(p);
    o0 *= alpha; o1 *= alpha;
    m_run = m_new;
    int nk = min(64, a.Nc - k0);
    for (int k = 0; k < nk; k++) {
      float pk = __shfl(p, k);
      const T* vr = Vh + (size_t)(k0 + k) * a.lay.ks_r;
      if (lane < a.d) o0 = __builtin_fmaf(pk, ld(vr + lane), o0);
      if (lane + 64 < a.d) o1 = __builtin_fmaf(pk, ld(vr + lane + 64), o1);
    }
  }
  if (m_run == BURST_NEG_INF) return;              // the row saw no key: state untouched
  // merge into the stored state (Alg. 1 merge step)
  size_t r = (size_t)head * a.Nq + row;
  float m_old = a.m[r], l_old = a.l[r];
  float m_new = fmaxf(m_old, m_run);
  float fa = expf(m_old - m_new), fb = expf(m_run - m_new);
  float* orow = a.O_acc + r * a.d;
  if (lane < a.d) orow[lane] = (fa == 0.f ? 0.f : fa * orow[lane]) + fb * o0;
  if (lane + 64 < a.d) orow[lane + 64] = (fa == 0.f ? 0.f : fa * orow[lane + 64]) + fb * o1;
  if (lane == 0) {
    a.m[r] = m_new;
    a.l[r] = (fa == 0.f ? 0.f : fa * l_old) + fb * l_run;
  }
}

// ---------------------------------------------------------------------------- backward, dQ
// One wavefront per query row; lanes = keys of a 64-key tile.
template <typename T>
__global__ void __launch_bounds__(256)
bwd_dq_generic_kernel(GenArgs a) {
  __shared__ float qrow[4][128];
  __shared__ float grow[4][128];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  long long wave = (long long)blockIdx.x * 4 + w;
  long long total = (long long)a.BH * a.Nq;
  const bool live = wave < total;
  if (!live) wave = 0;
  const int head = (int)(wave / a.Nq), row = (int)(wave % a.Nq);
  size_t r = (size_t)head * a.Nq + row;
  const T* Qr = (const T*)a.Q + a.lay.q_base(head) + (size_t)row * a.lay.qs_r;
  const T* Gr = (const T*)a.dO + a.lay.q_base(head) + (size_t)row * a.lay.qs_r;
  const T* Kh = (const T*)a.K + a.lay.kv_base(head / a.group);
  const T* Vh = (const T*)a.V + a.lay.kv_base(head / a.group);
  for (int t = lane; t < a.d; t += 64) { qrow[w][t] = ld(Qr + t); grow[w][t] = ld(Gr + t); }
  __syncthreads();
  if (!live) return;
  const float lse = a.lse[r], Dr = a.D[r];
  const long long qpos = a.q_off + row;
  float q0 = 0.f, q1 = 0.f;
  for (int k0 = 0; k0 < a.Nc; k0 += 64) {
    int key = k0 + lane;
    bool vis = key < a.Nc && lse != BURST_NEG_INF && visible(a, head, row, key);
    float ds = 0.f;
    if (vis) {
      float sa = 0.f, dp = 0.f;
      const T* kr = Kh + (size_t)key * a.lay.ks_r;
      const T* vr = Vh + (size_t)key * a.lay.ks_r;
      for (int t = 0; t < a.d; t++) {
        sa = __builtin_fmaf(qrow[w][t], ld(kr + t), sa);
        dp = __builtin_fmaf(grow[w][t], ld(vr + t), dp);
      }
      float p = expf(sa * a.scale - lse);
      ds = p * (dp - Dr);
    }
    int nk = min(64, a.Nc - k0);
    for (int k = 0; k < nk; k++) {
      float dsk = __shfl(ds, k);
      const T* kr = Kh + (size_t)(k0 + k) * a.lay.ks_r;
      if (lane < a.d) q0 = __builtin_fmaf(dsk, ld(kr + lane), q0);
      if (lane + 64 < a.d) q1 = __builtin_fmaf(dsk, ld(kr + lane + 64), q1);
    }
  }
  float* out = a.dQ + r * a.d;
  if (lane < a.d) out[lane] = (a.acc_dq ? out[lane] : 0.f) + a.scale * q0;
  if (lane + 64 < a.d) out[lane + 64] = (a.acc_dq ? out[lane + 64] : 0.f) + a.scale * q1;
}

// ---------------------------------------------------------------------------- backward, dK dV
// One wavefront per key row; lanes = query rows of a 64-row tile.
template <typename T>
__global__ void __launch_bounds__(256)
bwd_dkv_generic_kernel(GenArgs a) {
  __shared__ float krow[4][128];
  __shared__ float vrow[4][128];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  long long wave = (long long)blockIdx.x * 4 + w;
  long long total = (long long)(a.BH / a.group) * a.Nc;      // one wavefront per key row of a key/value head
  const bool live = wave < total;
  if (!live) wave = 0;
  const int kvhead = (int)(wave / a.Nc), key = (int)(wave % a.Nc);
  size_t kr_i = (size_t)kvhead * a.Nc + key;
  const T* Kr = (const T*)a.K + a.lay.kv_base(kvhead) + (size_t)key * a.lay.ks_r;
  const T* Vr = (const T*)a.V + a.lay.kv_base(kvhead) + (size_t)key * a.lay.ks_r;
  for (int t = lane; t < a.d; t += 64) { krow[w][t] = ld(Kr + t); vrow[w][t] = ld(Vr + t); }
  __syncthreads();
  if (!live) return;
  float k0a = 0.f, k1a = 0.f, v0a = 0.f, v1a = 0.f;
  for (int g = 0; g < a.group; g++) {                        // the query heads that share this key/value head
    const int head = kvhead * a.group + g;
    const T* Qh = (const T*)a.Q + a.lay.q_base(head);
    const T* Gh = (const T*)a.dO + a.lay.q_base(head);
    const float* lseh = a.lse + (size_t)head * a.Nq;
    const float* Dh = a.D + (size_t)head * a.Nq;
    for (int r0 = 0; r0 < a.Nq; r0 += 64) {
      int row = r0 + lane;
      float p = 0.f, ds = 0.f;
      if (row < a.Nq && visible(a, head, row, key)) {
        float lse = lseh[row];
        if (lse != BURST_NEG_INF) {
          float sa = 0.f, dp = 0.f;
          const T* qr = Qh + (size_t)row * a.lay.qs_r;
          const T* gr = Gh + (size_t)row * a.lay.qs_r;
          for (int t = 0; t < a.d; t++) {
            sa = __builtin_fmaf(ld(qr + t), krow[w][t], sa);
            dp = __builtin_fmaf(ld(gr + t), vrow[w][t], dp);
          }
          p = expf(sa * a.scale - lse);
          ds = p * (dp - Dh[row]);
        }
      }
      int nr = min(64, a.Nq - r0);
      for (int j = 0; j < nr; j++) {
        float pj = __shfl(p, j), dsj = __shfl(ds, j);
        const T* qr = Qh + (size_t)(r0 + j) * a.lay.qs_r;
        const T* gr = Gh + (size_t)(r0 + j) * a.lay.qs_r;
        if (lane < a.d) { v0a = __builtin_fmaf(pj, ld(gr + lane), v0a); k0a = __builtin_fmaf(dsj, ld(qr + lane), k0a); }
        if (lane + 64 < a.d) { v1a = __builtin_fmaf(pj, ld(gr + lane + 64), v1a); k1a = __builtin_fmaf(dsj, ld(qr + lane + 64), k1a); }
      }
    }
  }
  float* dk = a.dK + kr_i * a.d;
  float* dv = a.dV + kr_i * a.d;
  if (lane < a.d) {
    dk[lane] = (a.acc_dkv ? dk[lane] : 0.f) + a.scale * k0a;
    dv[lane] = (a.acc_dkv ? dv[lane] : 0.f) + v0a;
  }
  if (lane + 64 < a.d) {
    dk[lane + 64] = (a.acc_dkv ? dk[lane + 64] : 0.f) + a.scale * k1a;
    dv[lane + 64] = (a.acc_dkv ? dv[lane + 64] : 0.f) + v1a;
  }
}

static GenArgs make_args(const KParams& p) {
  GenArgs a = {};
  a.Nq = p.Nq; a.Nc = p.Nc; a.d = p.d; a.BH = p.B * p.H;
  a.causal = p.causal; a.scale = p.scale; a.q_off = p.q_off; a.k_off = p.k_off; a.window = p.window;
  a.bmask = p.bmask; a.bsize = p.bsize; a.bpitch = p.bpitch; a.bhstride = p.bhstride; a.group = p.group;
  a.lay = p.lay;
  return a;
}

int launch_fwd_generic(const KParams& p, int dtype, const void* Q, const void* K, const void* V,
                       float* O_acc, float* m, float* l, hipStream_t s) {
  long long waves = (long long)p.B * p.H * p.Nq;
  if (waves == 0 || p.Nc == 0) return BURST_OK;
  long long blocks = (waves + 3) / 4;
  if (blocks > 0x7fffffffLL) return BURST_ERR_SHAPE;
  GenArgs a = make_args(p);
  a.Q = Q; a.K = K; a.V = V; a.O_acc = O_acc; a.m = m; a.l = l;
  if (dtype == BURST_BF16) BURST_LAUNCH((fwd_generic_kernel<bf16>), dim3((unsigned)blocks), dim3(256), 0, s, a);
  else BURST_LAUNCH((fwd_generic_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, s, a);
  return launch_status();
}

int launch_bwd_dq_generic(const KParams& p, int dtype, const void* Q, const void* K, const void* V,
                          const void* dO, const float* lse, const float* D, float* dQ, int acc_dq, hipStream_t s) {
  GenArgs a = make_args(p);
  a.Q = Q; a.K = K; a.V = V; a.dO = dO; a.lse = lse; a.D = D; a.dQ = dQ; a.acc_dq = acc_dq;
  long long wq = (long long)p.B * p.H * p.Nq;
  if (wq == 0) return BURST_OK;
  if ((wq + 3) / 4 > 0x7fffffffLL) return BURST_ERR_SHAPE;
  unsigned blocks = (unsigned)((wq + 3) / 4);
  if (dtype == BURST_BF16) BURST_LAUNCH((bwd_dq_generic_kernel<bf16>), dim3(blocks), dim3(256), 0, s, a);
  else BURST_LAUNCH((bwd_dq_generic_kernel<float>), dim3(blocks), dim3(256), 0, s, a);
  return launch_status();
}

int launch_bwd_dkv_generic(const KParams& p, int dtype, const void* Q, const void* K, const void* V,
                           const void* dO, const float* lse, const float* D, float* dK, float* dV,
                           int acc_dkv, hipStream_t s) {
  GenArgs a = make_args(p);
  a.Q = Q; a.K = K; a.V = V; a.dO = dO; a.lse = lse; a.D = D; a.dK = dK; a.dV = dV; a.acc_dkv = acc_dkv;
  long long wk = (long long)p.B * p.H / p.group * p.Nc;
  if (wk == 0) return BURST_OK;
  if ((wk + 3) / 4 > 0x7fffffffLL) return BURST_ERR_SHAPE;
  unsigned blocks = (unsigned)((wk + 3) / 4);
  if (dtype == BURST_BF16) BURST_LAUNCH((bwd_dkv_generic_kernel<bf16>), dim3(blocks), dim3(256), 0, s, a);
  else BURST_LAUNCH((bwd_dkv_generic_kernel<float>), dim3(blocks), dim3(256), 0, s, a);
  return launch_status();
}

}  // namespace burst
