// Local attention WITHOUT the tiling of paper Sec. 2.4 (the "w/o LAO" row of the paper's
// ablation): the chunk step of Alg. 1 exactly as printed, with S_ij and P_ij of the whole
// block pair stored in HBM between the steps.
//   1. S_ij = scale Q_i K_j^T                      -> workspace (fp32, Nq x Nc per head)
//   2. m_ij = rowmax(S_ij), P_ij = exp(S_ij - m_ij),
//      l_ij = rowsum(P_ij)                         -> workspace (P in the input type)
//   3. O_ij = P_ij V_j, merged into (O_i, m_i, l_i) (Alg. 1 merge step)
// It exists to measure what the tiling buys (memory B Z N^2 / G^2 per device and the HBM round
// trips of S and P), not to be fast: nothing is skipped (masked scores are computed and
// discarded) and steps 1 and 3 read their operands with plain loads.
#include "burst_common.h"

namespace burst {

struct MatArgs {
  const void* Q; const void* K; const void* V;
  float* S; void* P; float* m_c; float* l_c;
  float* O_acc; float* m; float* l;
  int Nq, Nc, Ncp, d;      // Ncp = Nc rounded up to 8: row pitch of S and P
  long long BH;
  int causal;
  float scale;
  long long q_off, k_off, window;
  const uint8_t* bmask; int bsize, bpitch;   // block mask (nullptr = none)
  long long bhstride;                        // bytes between heads' flag matrices (0 = shared)
  Layout lay;                                // strides of Q and of K, V
  int group;                                 // query heads per key/value head
};

// ---- step 1, bf16, d = 128: one wavefront = a 32 x 32 block of S (8 MFMAs over d)
__global__ void __launch_bounds__(256)
mat_scores_mfma_kernel(MatArgs a) {
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, lr = lane & 31, h = lane >> 5;
  const int head = blockIdx.z;
  const int q0 = blockIdx.y * 32;
  const int k0 = (blockIdx.x * 4 + w) * 32;
  if (k0 >= a.Ncp) return;
  const bf16* Qh = (const bf16*)a.Q + a.lay.q_base(head);
  const bf16* Kh = (const bf16*)a.K + a.lay.kv_base(head / a.group);
  const int qrow = q0 + lr, krow = k0 + lr;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; r++) acc[r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < 8; ks++) {
    bf16x8 qa, kb;
#pragma unroll
    for (int t = 0; t < 8; t++) { qa[t] = (bf16)0.0f; kb[t] = (bf16)0.0f; }
    if (qrow < a.Nq) qa = *reinterpret_cast<const bf16x8*>(Qh + (size_t)qrow * a.lay.qs_r + ks * 16 + h * 8);
    if (krow < a.Nc) kb = *reinterpret_cast<const bf16x8*>(Kh + (size_t)krow * a.lay.ks_r + ks * 16 + h * 8);
    acc = mfma32(qa, kb, acc);          // rows of the product = query rows, columns = keys
  }
  // register r of lane (lr, h) holds query row 8*(r/4) + 4h + r%4, key lr of the block
  float* Sh = a.S + (size_t)head * a.Nq * a.Ncp;
  if (krow < a.Ncp) {
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int qr = q0 + 8 * (r >> 2) + 4 * h + (r & 3);
      if (qr < a.Nq) Sh[(size_t)qr * a.Ncp + krow] = acc[r] * a.scale;
    }
  }
}

// ---- step 1, any type and d: one thread per score
template <typename T>
__global__ void __launch_bounds__(256)
mat_scores_generic_kernel(MatArgs a) {
  const long long total = a.BH * a.Nq * a.Ncp;
  for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
    const int c = (int)(idx % a.Ncp);
    const long long hr = idx / a.Ncp;
    const int r = (int)(hr % a.Nq);
    const long long head = hr / a.Nq;
    float s = 0.f;
    if (c < a.Nc) {
      const T* q = (const T*)a.Q + a.lay.q_base((int)head) + (size_t)r * a.lay.qs_r;
      const T* k = (const T*)a.K + a.lay.kv_base((int)(head / a.group)) + (size_t)c * a.lay.ks_r;
      for (int t = 0; t < a.d; t++) s = __builtin_fmaf((float)q[t], (float)k[t], s);
    }
    a.S[idx] = s * a.scale;
  }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// ---- step 2: one wavefront per query row.  Causal and window leave one interval of the chunk
// visible (up to the row's position; from position - window + 1); a block mask thins it further.
template <typename T>
__global__ void __launch_bounds__(256)
mat_softmax_kernel(MatArgs a) {
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + w;
  if (row >= a.BH * a.Nq) return;
  const int r = (int)(row % a.Nq);
  const float* Srow = a.S + (size_t)row * a.Ncp;
  T* Prow = (T*)a.P + (size_t)row * a.Ncp;
  const long long qpos = a.q_off + r;
  long long hi = a.Nc, lo = 0;
  if (a.causal) hi = qpos - a.k_off + 1 < hi ? qpos - a.k_off + 1 : hi;
  if (a.window > 0) lo = qpos - a.window + 1 - a.k_off > 0 ? qpos - a.window + 1 - a.k_off : 0;
  if (hi < 0) hi = 0;
  if (lo > hi) lo = hi;
  const uint8_t* brow = a.bmask == nullptr ? nullptr : a.bmask + (size_t)(row / a.Nq) * a.bhstride + (size_t)(r / a.bsize) * a.bpitch;
  auto seen = [&](long long c) { return c >= lo && c < hi && (brow == nullptr || brow[c / a.bsize] != 0); };
  float mx = BURST_NEG_INF;
  for (long long c = lo + lane; c < hi; c += 64)
    if (seen(c)) mx = fmaxf(mx, Srow[c]);
  mx = wave_max(mx);
  const float ref = (mx == BURST_NEG_INF) ? 0.f : mx;
  float sum = 0.f;
  for (int c = lane; c < a.Ncp; c += 64) {
    float p = seen(c) ? fast_exp2((Srow[c] - ref) * kLog2e) : 0.f;
    T pt = (T)p;
    Prow[c] = pt;
    sum += (float)pt;                   // the sum of what step 3 multiplies with
  }
  sum = wave_sum(sum);
  if (lane == 0) { a.m_c[row] = mx; a.l_c[row] = sum; }
}

// ---- step 3, bf16, d = 128: one workgroup = 128 query rows (32 per wavefront); V tiles of 32
// keys go through LDS (two buffers, filled by DMA) and are read transposed, P comes straight
// from the workspace.  O^T (128 x 32 per wavefront) += V^T P^T.
constexpr int MAT_VTILE_BYTES = 32 * 256;

__global__ void __launch_bounds__(256)
mat_pv_merge_mfma_kernel(MatArgs a) {
  __shared__ __attribute__((aligned(16))) char smem[2 * MAT_VTILE_BYTES];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, lr = lane & 31, h = lane >> 5;
  const int head = blockIdx.y;
  const int q0 = blockIdx.x * 128 + w * 32;
  const bf16* Vh = (const bf16*)a.V + a.lay.kv_base(head / a.group);
  const unsigned vpitch = (unsigned)a.lay.ks_r * 2u;         // bytes between rows of V
  const bf16* Ph = (const bf16*)a.P + (size_t)head * a.Nq * a.Ncp;
  const __amdgpu_buffer_rsrc_t vrs = make_rsrc(Vh, a.Nc > 0 ? (unsigned)(a.Nc - 1) * vpitch + 256u : 0u);
  const int ntiles = (a.Nc + 31) / 32;
  const int wu = __builtin_amdgcn_readfirstlane(w);
  const unsigned lds0 = lds_addr(smem);
  int goff[2];
#pragma unroll
  for (int il = 0; il < 2; il++) {
    const int row = 8 * w + 4 * il + (lane >> 4);
    goff[il] = (int)(row * vpitch + (((lane & 15) ^ row_code(row)) << 4));
  }
  // transposing reads: 16-lane group (h, dh) reads tile rows kg*16 + 8h + 4s + (0..3), columns
  // db*32 + dh*16 + (0..15); lane lr = dh*16 + j16 ends up with column lr of the d block
  int vaddr[2][4][2];
  {
    const int j16 = lane & 15, dh = (lane >> 4) & 1;
#pragma unroll
    for (int kg = 0; kg < 2; kg++)
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int s = 0; s < 2; s++)
          vaddr[kg][db][s] = tile_off(kg * 16 + 8 * h + 4 * s + (j16 >> 2), db * 4 + 2 * dh + ((j16 & 3) >> 1)) + (j16 & 1) * 8;
  }
  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; db++)
#pragma unroll
    for (int r = 0; r < 16; r++) o[db][r] = 0.f;

  const int prow = q0 + lr;
  auto load_p = [&](int t, int kg) __attribute__((always_inline)) {
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; e++) v[e] = (bf16)0.0f;
    const int key = t * 32 + kg * 16 + 8 * h;
    if (prow < a.Nq && key < a.Ncp) v = *reinterpret_cast<const bf16x8*>(Ph + (size_t)prow * a.Ncp + key);
    return v;
  };

#pragma unroll
  for (int il = 0; il < 2; il++) dma_b128_to_lds(vrs, lds0 + (unsigned)(wu * 2 + il) * 1024u, goff[il]);
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __builtin_amdgcn_s_barrier();
  for (int t = 0; t < ntiles; t++) {
    const char* vl = smem + (t & 1) * MAT_VTILE_BYTES;
    if (t + 1 < ntiles) {
#pragma unroll
      for (int il = 0; il < 2; il++)
        dma_b128_to_lds(vrs, lds0 + (unsigned)(((t + 1) & 1) * MAT_VTILE_BYTES) + (unsigned)(wu * 2 + il) * 1024u,
                        (int)((t + 1) * 32 * vpitch) + goff[il]);
    }
    bf16x8 pf[2];
    pf[0] = load_p(t, 0);
    pf[1] = load_p(t, 1);
#pragma unroll
    for (int kg = 0; kg < 2; kg++)
#pragma unroll
      for (int db = 0; db < 4; db++) {
        const bf16x4 va = lds_read_tr(vl, vaddr[kg][db][0]), vb = lds_read_tr(vl, vaddr[kg][db][1]);
        bf16x8 vf;
        vf[0] = va[0]; vf[1] = va[1]; vf[2] = va[2]; vf[3] = va[3];
        vf[4] = vb[0]; vf[5] = vb[1]; vf[6] = vb[2]; vf[7] = vb[3];
        o[db] = mfma32(vf, pf[kg], o[db]);
      }
    __builtin_amdgcn_s_waitcnt(0x0070);            // vmcnt(0), lgkmcnt(0): next tile landed, reads done
    __builtin_amdgcn_s_barrier();
  }

  // merge (Alg. 1): lane (lr, h) holds row lr, columns db*32 + 8*q4 + 4h + (0..3)
  if (prow < a.Nq) {
    const size_t srow = (size_t)head * a.Nq + prow;
    const float m_ij = a.m_c[srow];
    if (m_ij != BURST_NEG_INF) {                   // rows that saw no key keep their state bit for bit
      const float l_ij = a.l_c[srow];
      const float m_old = a.m[srow], l_old = a.l[srow];
      const float m_new = fmaxf(m_old, m_ij);
      const float fa = fast_exp2((m_old - m_new) * kLog2e);
      const float fb = fast_exp2((m_ij - m_new) * kLog2e);
      float* orow = a.O_acc + srow * 128;
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          float* ptr = orow + db * 32 + 8 * q4 + 4 * h;
          f32x4 old = *reinterpret_cast<f32x4*>(ptr);
          f32x4 nw;
#pragma unroll
          for (int b = 0; b < 4; b++) {
            float keep = (fa == 0.f) ? 0.f : old[b] * fa;   // a fresh state may hold anything
            nw[b] = keep + fb * o[db][4 * q4 + b];
          }
          *reinterpret_cast<f32x4*>(ptr) = nw;
        }
      if (h == 0) {
        a.m[srow] = m_new;
        a.l[srow] = ((fa == 0.f) ? 0.f : fa * l_old) + fb * l_ij;
      }
    }
  }
}

// ---- step 3, any type and d: one thread per element of O; m and l are merged by a second
// kernel once every element of the row has used the old m.
template <typename T>
__global__ void __launch_bounds__(256)
mat_pv_merge_generic_kernel(MatArgs a) {
  const long long total = a.BH * a.Nq * a.d;
  for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
    const int col = (int)(idx % a.d);
    const long long srow = idx / a.d;
    const long long head = srow / a.Nq;
    const float m_ij = a.m_c[srow];
    if (m_ij == BURST_NEG_INF) continue;
    const T* p = (const T*)a.P + (size_t)srow * a.Ncp;
    const T* v = (const T*)a.V + a.lay.kv_base((int)(head / a.group)) + col;
    float acc = 0.f;
    for (int c = 0; c < a.Nc; c++) acc = __builtin_fmaf((float)p[c], (float)v[(size_t)c * a.lay.ks_r], acc);
    const float m_old = a.m[srow];
    const float m_new = fmaxf(m_old, m_ij);
    const float fa = fast_exp2((m_old - m_new) * kLog2e);
    const float fb = fast_exp2((m_ij - m_new) * kLog2e);
    const float keep = (fa == 0.f) ? 0.f : a.O_acc[idx] * fa;
    a.O_acc[idx] = keep + fb * acc;
  }
}
__global__ void __launch_bounds__(256)
mat_ml_merge_kernel(MatArgs a) {
  const long long srow = (long long)blockIdx.x * 256 + threadIdx.x;
  if (srow >= a.BH * a.Nq) return;
  const float m_ij = a.m_c[srow];
  if (m_ij == BURST_NEG_INF) return;
  const float m_old = a.m[srow], l_old = a.l[srow];
  const float m_new = fmaxf(m_old, m_ij);
  const float fa = fast_exp2((m_old - m_new) * kLog2e);
  const float fb = fast_exp2((m_ij - m_new) * kLog2e);
  a.m[srow] = m_new;
  a.l[srow] = ((fa == 0.f) ? 0.f : fa * l_old) + fb * a.l_c[srow];
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Bytes of workspace one call needs: S (fp32) and P (input type), Nq x Ncp per head each, and
// the chunk's row statistics.
size_t materialized_workspace_bytes(const KParams& p, int dtype) {
  const size_t rows = (size_t)p.B * p.H * p.Nq;
  const size_t ncp = ((size_t)p.Nc + 7) & ~(size_t)7;
  const size_t esize = dtype == BURST_BF16 ? 2 : 4;
  return align256(rows * ncp * 4) + align256(rows * ncp * esize) + 2 * align256(rows * 4);
}

int launch_fwd_materialized(const KParams& p, int dtype, bool mfma, const void* Q, const void* K, const void* V,
                            float* O_acc, float* m, float* l, void* workspace, hipStream_t s) {
  MatArgs a;
  a.Q = Q; a.K = K; a.V = V; a.O_acc = O_acc; a.m = m; a.l = l;
  a.Nq = p.Nq; a.Nc = p.Nc; a.Ncp = (p.Nc + 7) & ~7; a.d = p.d; a.BH = (long long)p.B * p.H;
  a.causal = p.causal; a.scale = p.scale; a.q_off = p.q_off; a.k_off = p.k_off; a.window = p.window;
  a.bmask = p.bmask; a.bsize = p.bsize; a.bpitch = p.bpitch; a.bhstride = p.bhstride; a.group = p.group;
  a.lay = p.lay;
  const size_t rows = (size_t)a.BH * a.Nq;
  const size_t esize = dtype == BURST_BF16 ? 2 : 4;
  char* ws = (char*)workspace;
  a.S = (float*)ws;                 ws += align256(rows * a.Ncp * 4);
  a.P = (void*)ws;                  ws += align256(rows * a.Ncp * esize);
  a.m_c = (float*)ws;               ws += align256(rows * 4);
  a.l_c = (float*)ws;

  const long long row_blocks = ((long long)rows + 3) / 4;
  if (row_blocks > 0x7fffffffLL) return BURST_ERR_SHAPE;
  auto grid1d = [](long long items) { long long b = (items + 255) / 256; return (unsigned)(b < 1 ? 1 : (b > (1 << 20) ? (1 << 20) : b)); };
  if (mfma) {
    const long long kb = (a.Ncp + 127) / 128, qb = (a.Nq + 31) / 32, qb128 = (a.Nq + 127) / 128;
    if (qb > 65535 || a.BH > 65535 || kb > 0x7fffffffLL) return BURST_ERR_SHAPE;
    hipLaunchKernelGGL(mat_scores_mfma_kernel, dim3((unsigned)kb, (unsigned)qb, (unsigned)a.BH), dim3(256), 0, s, a);
    hipLaunchKernelGGL((mat_softmax_kernel<bf16>), dim3((unsigned)row_blocks), dim3(256), 0, s, a);
    hipLaunchKernelGGL(mat_pv_merge_mfma_kernel, dim3((unsigned)qb128, (unsigned)a.BH), dim3(256), 0, s, a);
  } else if (dtype == BURST_BF16) {
    hipLaunchKernelGGL((mat_scores_generic_kernel<bf16>), dim3(grid1d((long long)rows * a.Ncp)), dim3(256), 0, s, a);
    hipLaunchKernelGGL((mat_softmax_kernel<bf16>), dim3((unsigned)row_blocks), dim3(256), 0, s, a);
    hipLaunchKernelGGL((mat_pv_merge_generic_kernel<bf16>), dim3(grid1d((long long)rows * a.d)), dim3(256), 0, s, a);
    hipLaunchKernelGGL(mat_ml_merge_kernel, dim3((unsigned)(((long long)rows + 255) / 256)), dim3(256), 0, s, a);
  } else {
    hipLaunchKernelGGL((mat_scores_generic_kernel<float>), dim3(grid1d((long long)rows * a.Ncp)), dim3(256), 0, s, a);
    hipLaunchKernelGGL((mat_softmax_kernel<float>), dim3((unsigned)row_blocks), dim3(256), 0, s, a);
    hipLaunchKernelGGL((mat_pv_merge_generic_kernel<float>), dim3(grid1d((long long)rows * a.d)), dim3(256), 0, s, a);
    hipLaunchKernelGGL(mat_ml_merge_kernel, dim3((unsigned)(((long long)rows + 255) / 256)), dim3(256), 0, s, a);
  }
  return hipGetLastError() == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
}

}  // namespace burst
