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
//
// The backward of the same variant is the loop body of Alg. 2 as printed, every matrix of the
// block pair stored in HBM:
//   1. S_ij = scale Q_i K_j^T -> workspace (fp32);  2. P_ij = exp(S_ij - lse_i) -> workspace
//   3. dV_j += P_ij^T dO_i;   4. dP_ij = dO_i V_j^T -> workspace (fp32, over S_ij)
//   5. dS_ij = P_ij o (dP_ij - D_i) -> workspace;   6. dQ_i += scale dS_ij K_j
//   7. dK_j += scale dS_ij^T Q_i
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
  // backward only
  const float* lse; const float* D;
  float* out;                                // gradient written by the product kernels
  float alpha;                               // ... as alpha * product (+ out if acc)
  int acc;
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

// EPI = 0: the merge of Alg. 1 as above.  EPI = 1 (backward, dQ_i += scale dS_ij K_j): the same
// product with dS_ij in the place of P_ij and K_j in the place of V_j, added to a.out.
template <int EPI>
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

  // lane (lr, h) holds row lr, columns db*32 + 8*q4 + 4h + (0..3)
  if constexpr (EPI == 1) {
    if (prow < a.Nq) {
      float* orow = a.out + ((size_t)head * a.Nq + prow) * 128;
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          float* ptr = orow + db * 32 + 8 * q4 + 4 * h;
          f32x4 nw = {0.f, 0.f, 0.f, 0.f};
          if (a.acc) nw = *reinterpret_cast<f32x4*>(ptr);
#pragma unroll
          for (int b = 0; b < 4; b++) nw[b] += a.alpha * o[db][4 * q4 + b];
          *reinterpret_cast<f32x4*>(ptr) = nw;
        }
    }
    return;
  }
  // merge (Alg. 1)
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


// ------------------------------------------------------------------------------ backward
// Visible interval of the chunk for one query row (causal: up to the row's position; window:
// from position - window + 1) and the row's block flags.
struct RowView {
  long long lo, hi;
  const uint8_t* brow;
  int bsize;
  __device__ bool seen(long long c) const { return c >= lo && c < hi && (brow == nullptr || brow[c / bsize] != 0); }
};
__device__ __forceinline__ RowView row_view(const MatArgs& a, long long row) {
  const int r = (int)(row % a.Nq);
  const long long qpos = a.q_off + r;
  RowView v;
  v.hi = a.Nc; v.lo = 0;
  if (a.causal) v.hi = qpos - a.k_off + 1 < v.hi ? qpos - a.k_off + 1 : v.hi;
  if (a.window > 0) v.lo = qpos - a.window + 1 - a.k_off > 0 ? qpos - a.window + 1 - a.k_off : 0;
  if (v.hi < 0) v.hi = 0;
  if (v.lo > v.hi) v.lo = v.hi;
  v.brow = a.bmask == nullptr ? nullptr : a.bmask + (size_t)(row / a.Nq) * a.bhstride + (size_t)(r / a.bsize) * a.bpitch;
  v.bsize = a.bsize;
  return v;
}

// ---- step 2: P_ij = exp(S_ij - lse_i), hidden entries and rows that saw nothing 0.  One wavefront per row.
template <typename T>
__global__ void __launch_bounds__(256)
mat_bwd_p_kernel(MatArgs a) {
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + w;
  if (row >= a.BH * a.Nq) return;
  const RowView v = row_view(a, row);
  const float lse = a.lse[row];
  const float* Srow = a.S + (size_t)row * a.Ncp;
  T* Prow = (T*)a.P + (size_t)row * a.Ncp;
  for (int c = lane; c < a.Ncp; c += 64)
    Prow[c] = (T)((lse != BURST_NEG_INF && v.seen(c)) ? fast_exp2((Srow[c] - lse) * kLog2e) : 0.f);
}

// ---- step 5: dS_ij = P_ij o (dP_ij - D_i) (dP_ij lies where S_ij was).  One wavefront per row.
template <typename T>
__global__ void __launch_bounds__(256)
mat_bwd_ds_kernel(MatArgs a, T* dS) {
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + w;
  if (row >= a.BH * a.Nq) return;
  const float Dv = a.D[row];
  const float* dProw = a.S + (size_t)row * a.Ncp;
  const T* Prow = (const T*)a.P + (size_t)row * a.Ncp;
  T* out = dS + (size_t)row * a.Ncp;
  for (int c = lane; c < a.Ncp; c += 64) {
    const float p = (float)Prow[c];
    out[c] = (T)(p == 0.f ? 0.f : p * (dProw[c] - Dv));
  }
}

// ---- steps 3 and 7, bf16, d = 128: out_j (+)= alpha X^T Y with X = P_ij or dS_ij ([Nq][Ncp] per
// query head, in the workspace: a.P) and Y = dO_i or Q_i (a.Q).  One workgroup = 128 keys of one
// key/value head (32 per wavefront); it walks the rows of every query head of the group in
// tiles of 32.  Both operands are contracted over rows, which is the slow direction of their
// storage: the tiles go through LDS (two buffers, filled by DMA) and are read transposed.
// out^T (128 x 32 per wavefront) += Y^T X.
constexpr int MAT_XT_TILE = 32 * 256;     // 32 rows x 128 keys (X) or x 128 columns (Y), bf16
__device__ __forceinline__ bf16x8 cat_tr(bf16x4 a, bf16x4 b) {
  bf16x8 v;
  v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
  v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
  return v;
}

__global__ void __launch_bounds__(256)
mat_xty_mfma_kernel(MatArgs a) {
  __shared__ __attribute__((aligned(16))) char smem[4 * MAT_XT_TILE];    // X0 X1 Y0 Y1
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, lr = lane & 31, h = lane >> 5;
  const int kvhead = blockIdx.y;
  const int key_wg = blockIdx.x * 128;
  const int tiles = (a.Nq + 31) / 32;
  const int nwalk = tiles * a.group;
  const unsigned xpitch = (unsigned)a.Ncp * 2u, ypitch = (unsigned)a.lay.qs_r * 2u;
  const int wu = __builtin_amdgcn_readfirstlane(w);
  const unsigned lds0 = lds_addr(smem);
  int xoff[2], yoff[2];
#pragma unroll
  for (int il = 0; il < 2; il++) {
    const int row = 8 * w + 4 * il + (lane >> 4);
    const unsigned g = (unsigned)(((lane & 15) ^ row_code(row)) << 4);
    xoff[il] = (int)(row * xpitch + g);
    yoff[il] = (int)(row * ypitch + g);
  }
  // the tile of walk position n (head g of the group, rows t*32 ..) into buffer buf
  auto fetch = [&](int n, int buf) __attribute__((always_inline)) {
    const int g = n / tiles, t = n - g * tiles;
    const int head = kvhead * a.group + g;
    // X: rows of this head's matrix from column key_wg on; a row's 256 bytes may run past the
    // matrix's row end into the next row (keys past the chunk: their products are dropped)
    const bf16* Xh = (const bf16*)a.P + (size_t)head * a.Nq * a.Ncp + key_wg;
    const __amdgpu_buffer_rsrc_t xrs = make_rsrc(Xh, (unsigned)a.Nq * xpitch - (unsigned)key_wg * 2u);
    const bf16* Yh = (const bf16*)a.Q + a.lay.q_base(head);
    const __amdgpu_buffer_rsrc_t yrs = make_rsrc(Yh, (unsigned)(a.Nq - 1) * ypitch + 256u);
#pragma unroll
    for (int il = 0; il < 2; il++) {
      dma_b128_to_lds(xrs, lds0 + (unsigned)(buf * MAT_XT_TILE) + (unsigned)(wu * 2 + il) * 1024u, (int)(t * 32 * xpitch) + xoff[il]);
      dma_b128_to_lds(yrs, lds0 + (unsigned)((2 + buf) * MAT_XT_TILE) + (unsigned)(wu * 2 + il) * 1024u, (int)(t * 32 * ypitch) + yoff[il]);
    }
  };
  // transposing reads of a 32-row tile: 16-lane group (h, dh) reads rows kg*16 + 8h + 4s + (0..3),
  // columns cb*32 + dh*16 + (0..15); lane lr = dh*16 + j16 ends up with column lr of block cb
  int yaddr[2][4][2], xaddr[2][2];
  {
    const int j16 = lane & 15, dh = (lane >> 4) & 1;
#pragma unroll
    for (int kg = 0; kg < 2; kg++)
#pragma unroll
      for (int sx = 0; sx < 2; sx++) {
        const int row = kg * 16 + 8 * h + 4 * sx + (j16 >> 2);
#pragma unroll
        for (int cb = 0; cb < 4; cb++) yaddr[kg][cb][sx] = tile_off(row, cb * 4 + 2 * dh + ((j16 & 3) >> 1)) + (j16 & 1) * 8;
        xaddr[kg][sx] = tile_off(row, w * 4 + 2 * dh + ((j16 & 3) >> 1)) + (j16 & 1) * 8;
      }
  }
  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; db++)
#pragma unroll
    for (int r = 0; r < 16; r++) o[db][r] = 0.f;

  if (nwalk > 0) {
    fetch(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    for (int n = 0; n < nwalk; n++) {
      const char* xl = smem + (n & 1) * MAT_XT_TILE;
      const char* yl = smem + (2 + (n & 1)) * MAT_XT_TILE;
      if (n + 1 < nwalk) fetch(n + 1, (n + 1) & 1);
#pragma unroll
      for (int kg = 0; kg < 2; kg++) {
        const bf16x8 xf = cat_tr(lds_read_tr(xl, xaddr[kg][0]), lds_read_tr(xl, xaddr[kg][1]));
#pragma unroll
        for (int db = 0; db < 4; db++) {
          const bf16x8 yf = cat_tr(lds_read_tr(yl, yaddr[kg][db][0]), lds_read_tr(yl, yaddr[kg][db][1]));
          o[db] = mfma32(yf, xf, o[db]);
        }
      }
      __builtin_amdgcn_s_waitcnt(0x0070);          // vmcnt(0), lgkmcnt(0): next tile landed, reads done
      __builtin_amdgcn_s_barrier();
    }
  }
  // lane (lr, h) holds key lr of the wavefront's 32, columns db*32 + 8*q4 + 4h + (0..3)
  const int key = key_wg + w * 32 + lr;
  if (key < a.Nc) {
    float* orow = a.out + ((size_t)kvhead * a.Nc + key) * 128;
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        float* ptr = orow + db * 32 + 8 * q4 + 4 * h;
        f32x4 nw = {0.f, 0.f, 0.f, 0.f};
        if (a.acc) nw = *reinterpret_cast<f32x4*>(ptr);
#pragma unroll
        for (int b = 0; b < 4; b++) nw[b] += a.alpha * o[db][4 * q4 + b];
        *reinterpret_cast<f32x4*>(ptr) = nw;
      }
  }
}

// ---- steps 3 and 7, any type and d: one thread per element of out_j
template <typename T>
__global__ void __launch_bounds__(256)
mat_xty_generic_kernel(MatArgs a) {
  const long long total = (a.BH / a.group) * a.Nc * a.d;
  for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
    const int col = (int)(idx % a.d);
    const long long kr = idx / a.d;
    const int key = (int)(kr % a.Nc);
    const long long kvhead = kr / a.Nc;
    float acc = 0.f;
    for (int g = 0; g < a.group; g++) {
      const long long head = kvhead * a.group + g;
      const T* x = (const T*)a.P + (size_t)head * a.Nq * a.Ncp + key;
      const T* y = (const T*)a.Q + a.lay.q_base((int)head) + col;
      for (int r = 0; r < a.Nq; r++) acc = __builtin_fmaf((float)x[(size_t)r * a.Ncp], (float)y[(size_t)r * a.lay.qs_r], acc);
    }
    a.out[idx] = (a.acc ? a.out[idx] : 0.f) + a.alpha * acc;
  }
}

// ---- step 6, any type and d: one thread per element of dQ_i (X = dS_ij in a.P, Y = K_j in a.V)
template <typename T>
__global__ void __launch_bounds__(256)
mat_xy_generic_kernel(MatArgs a) {
  const long long total = a.BH * a.Nq * a.d;
  for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
    const int col = (int)(idx % a.d);
    const long long srow = idx / a.d;
    const long long head = srow / a.Nq;
    const T* x = (const T*)a.P + (size_t)srow * a.Ncp;
    const T* y = (const T*)a.V + a.lay.kv_base((int)(head / a.group)) + col;
    float acc = 0.f;
    for (int c = 0; c < a.Nc; c++) acc = __builtin_fmaf((float)x[c], (float)y[(size_t)c * a.lay.ks_r], acc);
    a.out[idx] = (a.acc ? a.out[idx] : 0.f) + a.alpha * acc;
  }
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
    BURST_LAUNCH(mat_scores_mfma_kernel, dim3((unsigned)kb, (unsigned)qb, (unsigned)a.BH), dim3(256), 0, s, a);
    BURST_LAUNCH((mat_softmax_kernel<bf16>), dim3((unsigned)row_blocks), dim3(256), 0, s, a);
    BURST_LAUNCH(mat_pv_merge_mfma_kernel<0>, dim3((unsigned)qb128, (unsigned)a.BH), dim3(256), 0, s, a);
  } else if (dtype == BURST_BF16) {
    BURST_LAUNCH((mat_scores_generic_kernel<bf16>), dim3(grid1d((long long)rows * a.Ncp)), dim3(256), 0, s, a);
    BURST_LAUNCH((mat_softmax_kernel<bf16>), dim3((unsigned)row_blocks), dim3(256), 0, s, a);
    BURST_LAUNCH((mat_pv_merge_generic_kernel<bf16>), dim3(grid1d((long long)rows * a.d)), dim3(256), 0, s, a);
    BURST_LAUNCH(mat_ml_merge_kernel, dim3((unsigned)(((long long)rows + 255) / 256)), dim3(256), 0, s, a);
  } else {
    BURST_LAUNCH((mat_scores_generic_kernel<float>), dim3(grid1d((long long)rows * a.Ncp)), dim3(256), 0, s, a);
    BURST_LAUNCH((mat_softmax_kernel<float>), dim3((unsigned)row_blocks), dim3(256), 0, s, a);
    BURST_LAUNCH((mat_pv_merge_generic_kernel<float>), dim3(grid1d((long long)rows * a.d)), dim3(256), 0, s, a);
    BURST_LAUNCH(mat_ml_merge_kernel, dim3((unsigned)(((long long)rows + 255) / 256)), dim3(256), 0, s, a);
  }
  return launch_status();
}

// Bytes of workspace one backward call needs: S / dP (fp32), P and dS (input type), Nq x Ncp
// per head each.
size_t materialized_bwd_workspace_bytes(const KParams& p, int dtype) {
  const size_t rows = (size_t)p.B * p.H * p.Nq;
  const size_t ncp = ((size_t)p.Nc + 7) & ~(size_t)7;
  const size_t esize = dtype == BURST_BF16 ? 2 : 4;
  return align256(rows * ncp * 4) + 2 * align256(rows * ncp * esize);
}

int launch_bwd_materialized(const KParams& p, int dtype, bool mfma, const void* Q, const void* K, const void* V,
                            const void* dO, const float* lse, const float* D, float* dQ, float* dK, float* dV,
                            int acc_dq, int acc_dkv, void* workspace, hipStream_t s) {
  MatArgs a = {};
  a.Q = Q; a.K = K; a.V = V; a.lse = lse; a.D = D;
  a.Nq = p.Nq; a.Nc = p.Nc; a.Ncp = (p.Nc + 7) & ~7; a.d = p.d; a.BH = (long long)p.B * p.H;
  a.causal = p.causal; a.scale = p.scale; a.q_off = p.q_off; a.k_off = p.k_off; a.window = p.window;
  a.bmask = p.bmask; a.bsize = p.bsize; a.bpitch = p.bpitch; a.bhstride = p.bhstride; a.group = p.group;
  a.lay = p.lay;
  const size_t rows = (size_t)a.BH * a.Nq;
  const size_t esize = dtype == BURST_BF16 ? 2 : 4;
  char* ws = (char*)workspace;
  a.S = (float*)ws;                 ws += align256(rows * a.Ncp * 4);
  a.P = (void*)ws;                  ws += align256(rows * a.Ncp * esize);
  void* dS = (void*)ws;
  if (rows == 0 || a.Nc == 0) return BURST_OK;     // (the callers have cleared what is not accumulated)

  const long long row_blocks = ((long long)rows + 3) / 4;
  if (row_blocks > 0x7fffffffLL) return BURST_ERR_SHAPE;
  // the MFMA product kernels address one head's Nq x Ncp matrix through 32-bit byte offsets
  if (mfma && (long long)a.Nq * a.Ncp * 2 + 64LL * a.Ncp * 2 > 0xffffffffLL) mfma = false;
  auto grid1d = [](long long items) { long long b = (items + 255) / 256; return (unsigned)(b < 1 ? 1 : (b > (1 << 20) ? (1 << 20) : b)); };
  const long long kvh = a.BH / a.group;
  const long long kb = (a.Ncp + 127) / 128, qb = (a.Nq + 31) / 32, qb128 = (a.Nq + 127) / 128, kb128 = (a.Nc + 127) / 128;
  if (mfma && (qb > 65535 || a.BH > 65535 || kb > 0x7fffffffLL || kb128 > 0x7fffffffLL)) return BURST_ERR_SHAPE;

  // X^T Y into `out` (dV_j or dK_j), X = what a.P points at
  auto xty = [&](MatArgs b, const void* X, const void* Y, float* out, float alpha) {
    b.P = const_cast<void*>(X); b.Q = Y; b.out = out; b.alpha = alpha; b.acc = acc_dkv;
    if (mfma) BURST_LAUNCH(mat_xty_mfma_kernel, dim3((unsigned)kb128, (unsigned)kvh), dim3(256), 0, s, b);
    else if (dtype == BURST_BF16) BURST_LAUNCH((mat_xty_generic_kernel<bf16>), dim3(grid1d(kvh * a.Nc * a.d)), dim3(256), 0, s, b);
    else BURST_LAUNCH((mat_xty_generic_kernel<float>), dim3(grid1d(kvh * a.Nc * a.d)), dim3(256), 0, s, b);
  };
  // scale * A B^T into a.S
  auto scores = [&](MatArgs b, const void* A, const void* Bm, float scale) {
    b.Q = A; b.K = Bm; b.scale = scale;
    if (mfma) BURST_LAUNCH(mat_scores_mfma_kernel, dim3((unsigned)kb, (unsigned)qb, (unsigned)a.BH), dim3(256), 0, s, b);
    else if (dtype == BURST_BF16) BURST_LAUNCH((mat_scores_generic_kernel<bf16>), dim3(grid1d((long long)rows * a.Ncp)), dim3(256), 0, s, b);
    else BURST_LAUNCH((mat_scores_generic_kernel<float>), dim3(grid1d((long long)rows * a.Ncp)), dim3(256), 0, s, b);
  };

  scores(a, Q, K, p.scale);                                                        // 1
  if (dtype == BURST_BF16) BURST_LAUNCH((mat_bwd_p_kernel<bf16>), dim3((unsigned)row_blocks), dim3(256), 0, s, a);   // 2
  else BURST_LAUNCH((mat_bwd_p_kernel<float>), dim3((unsigned)row_blocks), dim3(256), 0, s, a);
  if (dV != nullptr) xty(a, a.P, dO, dV, 1.0f);                                    // 3
  scores(a, dO, V, 1.0f);                                                          // 4
  if (dtype == BURST_BF16) BURST_LAUNCH((mat_bwd_ds_kernel<bf16>), dim3((unsigned)row_blocks), dim3(256), 0, s, a, (bf16*)dS);   // 5
  else BURST_LAUNCH((mat_bwd_ds_kernel<float>), dim3((unsigned)row_blocks), dim3(256), 0, s, a, (float*)dS);
  if (dQ != nullptr) {                                                             // 6
    MatArgs b = a;
    b.P = dS; b.V = K; b.out = dQ; b.alpha = p.scale; b.acc = acc_dq;
    if (mfma) BURST_LAUNCH(mat_pv_merge_mfma_kernel<1>, dim3((unsigned)qb128, (unsigned)a.BH), dim3(256), 0, s, b);
    else if (dtype == BURST_BF16) BURST_LAUNCH((mat_xy_generic_kernel<bf16>), dim3(grid1d((long long)rows * a.d)), dim3(256), 0, s, b);
    else BURST_LAUNCH((mat_xy_generic_kernel<float>), dim3(grid1d((long long)rows * a.d)), dim3(256), 0, s, b);
  }
  if (dK != nullptr) xty(a, dS, Q, dK, p.scale);                                   // 7
  return launch_status();
}

}  // namespace burst
