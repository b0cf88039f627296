// Forward of one chunk (paper Alg. 1 loop body, tiled as in Sec. 2.4) for bf16, d = 128.
//
// One workgroup = 4 wavefronts = 256 query rows of one (batch, head); each wavefront owns
// 64 query rows (two 32-row blocks) and walks the chunk in tiles of 64 keys.
//   S^T tile  = K_tile Q^T           (32x32x16 bf16 MFMA, A = K from LDS, B = Q in registers)
//   softmax   : each lane owns ONE query row (shared with lane^32, which holds the other
//               half of the keys), so row max / row sum are in-register reductions plus
//               one cross-half exchange; running max, sum and O rescale stay in registers
//   O^T tile += V_tile^T P^T         (A = V^T through transposing LDS reads, B = P from the
//               S^T accumulators, which already have the B-operand layout)
// The chunk-local (O_ij, m_ij, l_ij) is merged into the state in HBM in the epilogue
// (Alg. 1: m_new = max, rescale, add).  No S or P tile ever leaves registers.
#include "burst_common.h"

namespace burst {

constexpr int FWD_BR = 256;   // query rows per workgroup
constexpr int FWD_BC = 64;    // keys per tile
constexpr int FWD_TILE_BYTES = FWD_BC * 256;

struct FwdArgs {
  const bf16* Q; const bf16* K; const bf16* V;
  float* O_acc; float* m; float* l;
  int Nq, Nc, H;
  int causal;
  float c;               // scale * log2(e)
  long long q_off, k_off;
  int q_blocks;          // ceil(Nq / FWD_BR)
};

// Global -> registers for one 64x128 bf16 tile (K or V): 4 granules of 16 B per thread.
__device__ __forceinline__ void load_tile_regs(const bf16* __restrict__ base, int row0, int nrows,
                                               int tid, i32x4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int gi = i * 256 + tid;
    int row = gi >> 4, g = gi & 15;
    i32x4 v = {0, 0, 0, 0};
    if (row0 + row < nrows)
      v = *reinterpret_cast<const i32x4*>(base + (size_t)(row0 + row) * 128 + g * 8);
    r[i] = v;
  }
}
__device__ __forceinline__ void store_tile_lds(char* lds, int tid, const i32x4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int gi = i * 256 + tid;
    int row = gi >> 4, g = gi & 15;
    *reinterpret_cast<i32x4*>(lds + tile_off(row, g)) = r[i];
  }
}

__global__ void __launch_bounds__(256, 1)
burst_fwd_mfma_kernel(FwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // buffer b: K tile at (2b) * FWD_TILE_BYTES, V tile at (2b + 1) * FWD_TILE_BYTES

  const int tid = threadIdx.x;
  const int w = tid >> 6, lane = tid & 63, lr = lane & 31, h = lane >> 5;

  // XCD-aware mapping: consecutive workgroup ids go round-robin to the 8 XCDs, so all
  // query blocks of one head are given ids that are congruent mod 8 (same XCD, same L2).
  // (a.H counts batch x heads; the id space is padded to a multiple of 8 heads.)
  int head, qb;
  {
    int bid = blockIdx.x;
    int xcd = bid & 7, idx = bid >> 3;
    int hx = idx / a.q_blocks;
    qb = idx - hx * a.q_blocks;
    head = hx * 8 + xcd;
    if (head >= a.H) return;                       // whole workgroup exits together
  }

  const int q0 = qb * FWD_BR + w * 64;             // first query row of this wave
  const bf16* Qh = a.Q + (size_t)head * a.Nq * 128;
  const bf16* Kh = a.K + (size_t)head * a.Nc * 128;
  const bf16* Vh = a.V + (size_t)head * a.Nc * 128;

  // Number of key tiles this workgroup must visit (causal: stop after the last tile that
  // any of its rows can see).
  int ntiles = (a.Nc + FWD_BC - 1) / FWD_BC;
  const long long wg_last_q = a.q_off + min(qb * FWD_BR + FWD_BR, a.Nq) - 1;
  if (a.causal) {
    long long lim = wg_last_q - a.k_off;           // last visible key index in this chunk
    if (lim < 0) return;                           // nothing visible: state unchanged
    long long t = lim / FWD_BC + 1;
    if (t < ntiles) ntiles = (int)t;
  }
  if (ntiles <= 0) return;

  // Q fragments (B operand): lane holds row lr of each 32-row block, 8 consecutive d.
  bf16x8 qf[2][8];
#pragma unroll
  for (int rb = 0; rb < 2; rb++) {
    int row = q0 + rb * 32 + lr;
#pragma unroll
    for (int ks = 0; ks < 8; ks++) {
      bf16x8 v;
#pragma unroll
      for (int t = 0; t < 8; t++) v[t] = (bf16)0.0f;
      if (row < a.Nq) v = *reinterpret_cast<const bf16x8*>(Qh + (size_t)row * 128 + ks * 16 + h * 8);
      qf[rb][ks] = v;
    }
  }

  f32x16 o[2][4];          // O^T accumulators: [row block][32-wide d block]
#pragma unroll
  for (int rb = 0; rb < 2; rb++)
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int r = 0; r < 16; r++) o[rb][db][r] = 0.f;
  float m2[2] = {BURST_NEG_INF, BURST_NEG_INF};   // running max, log2 units, per row block
  float lsum[2] = {0.f, 0.f};                     // running sum over this lane's keys only

  // per-lane LDS byte offsets; tile-relative constants are added at the use site
  // K reads (128-bit): row = kb*32 + lr, granule = 2*ks + h
  int kaddr[8];
#pragma unroll
  for (int ks = 0; ks < 8; ks++) kaddr[ks] = tile_off(lr, 2 * ks + h);
  // V reads (transposing): row = kg*16 + 8*s + 4*h + j16/4 ; granule = db*4 + 2*dh + (j16&3)/2 ;
  // plus 8 bytes for odd j16.  The row code of rows kg*16 + x equals that of x.
  int vaddr[4][2];
  {
    const int j16 = lane & 15, dh = (lane >> 4) & 1;
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int sx = 0; sx < 2; sx++)
        vaddr[db][sx] = tile_off(8 * sx + 4 * h + (j16 >> 2), db * 4 + 2 * dh + ((j16 & 3) >> 1)) + (j16 & 1) * 8;
  }

  i32x4 kreg[4], vreg[4];
  load_tile_regs(Kh, 0, a.Nc, tid, kreg);
  load_tile_regs(Vh, 0, a.Nc, tid, vreg);
  store_tile_lds(smem, tid, kreg);
  store_tile_lds(smem + FWD_TILE_BYTES, tid, vreg);
  if (ntiles > 1) {
    load_tile_regs(Kh, FWD_BC, a.Nc, tid, kreg);
    load_tile_regs(Vh, FWD_BC, a.Nc, tid, vreg);
  }
  __syncthreads();

  const long long wave_first_q = a.q_off + q0;
  const long long wave_last_q = a.q_off + q0 + 63;

  for (int kt = 0; kt < ntiles; kt++) {
    const int cur = kt & 1;
    if (kt + 1 < ntiles) {
      store_tile_lds(smem + (cur ^ 1) * 2 * FWD_TILE_BYTES, tid, kreg);
      store_tile_lds(smem + ((cur ^ 1) * 2 + 1) * FWD_TILE_BYTES, tid, vreg);
      if (kt + 2 < ntiles) {
        load_tile_regs(Kh, (kt + 2) * FWD_BC, a.Nc, tid, kreg);
        load_tile_regs(Vh, (kt + 2) * FWD_BC, a.Nc, tid, vreg);
      }
    }
    const long long tile_first_k = a.k_off + (long long)kt * FWD_BC;
    const bool wave_skips = (a.causal && tile_first_k > wave_last_q) || (q0 >= a.Nq);
    if (!wave_skips) {
      const char* kl = smem + cur * 2 * FWD_TILE_BYTES;
      const char* vl = kl + FWD_TILE_BYTES;
      // ---- S^T = K Q^T
      f32x16 s[2][2];      // [key block][row block]
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int rb = 0; rb < 2; rb++)
#pragma unroll
          for (int r = 0; r < 16; r++) s[kb][rb][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ks++) {
#pragma unroll
        for (int kb = 0; kb < 2; kb++) {
          bf16x8 kf = lds_read_b128(kl, kb * 32 * 256 + kaddr[ks]);
#pragma unroll
          for (int rb = 0; rb < 2; rb++) s[kb][rb] = mfma32(kf, qf[rb][ks], s[kb][rb]);
        }
      }
      // ---- masking (diagonal tiles, ragged key tail)
      const bool need_mask = (a.causal && tile_first_k + FWD_BC - 1 > wave_first_q) ||
                             ((kt + 1) * FWD_BC > a.Nc);
      if (need_mask) {
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
          for (int rb = 0; rb < 2; rb++) {
            long long qpos = a.q_off + q0 + rb * 32 + lr;
#pragma unroll
            for (int r = 0; r < 16; r++) {
              int kidx = kt * FWD_BC + kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
              bool vis = (kidx < a.Nc) && (!a.causal || (a.k_off + kidx <= qpos));
              if (!vis) s[kb][rb][r] = BURST_NEG_INF;
            }
          }
      }
      // ---- online softmax, one query row per lane
      bf16x8 pf[2][4];     // P^T fragments (B operand): [row block][16-key group]
#pragma unroll
      for (int rb = 0; rb < 2; rb++) {
        float mx = s[0][rb][0];
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
          for (int r = 0; r < 16; r++) mx = fmaxf(mx, s[kb][rb][r]);
        mx = max_both_halves(mx);
        float m_new = fmaxf(m2[rb], mx * a.c);
        float ref = (m_new == BURST_NEG_INF) ? 0.f : m_new;
        float alpha = fast_exp2(m2[rb] - ref);
        m2[rb] = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; kb++) {
          float p[16];
#pragma unroll
          for (int r = 0; r < 16; r++) {
            p[r] = fast_exp2(__builtin_fmaf(s[kb][rb][r], a.c, -ref));
            psum += p[r];
          }
#pragma unroll
          for (int u = 0; u < 2; u++) {
            bf16x8 f;
#pragma unroll
            for (int t = 0; t < 8; t++) f[t] = (bf16)p[8 * u + t];
            pf[rb][2 * kb + u] = f;
          }
        }
        lsum[rb] = lsum[rb] * alpha + psum;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
          for (int r = 0; r < 16; r++) o[rb][db][r] *= alpha;
      }
      // ---- O^T += V^T P^T
#pragma unroll
      for (int kg = 0; kg < 4; kg++) {
#pragma unroll
        for (int db = 0; db < 4; db++) {
          bf16x4 va = lds_read_tr(vl, kg * 16 * 256 + vaddr[db][0]);
          bf16x4 vb = lds_read_tr(vl, kg * 16 * 256 + vaddr[db][1]);
          bf16x8 vf;
          vf[0] = va[0]; vf[1] = va[1]; vf[2] = va[2]; vf[3] = va[3];
          vf[4] = vb[0]; vf[5] = vb[1]; vf[6] = vb[2]; vf[7] = vb[3];
#pragma unroll
          for (int rb = 0; rb < 2; rb++) o[rb][db] = mfma32(vf, pf[rb][kg], o[rb][db]);
        }
      }
    }
    __syncthreads();
  }

  // ---- epilogue: merge the chunk result into the state in HBM (Alg. 1 merge step)
  float* Oh = a.O_acc + (size_t)head * a.Nq * 128;
  float* mh = a.m + (size_t)head * a.Nq;
  float* lh = a.l + (size_t)head * a.Nq;
#pragma unroll
  for (int rb = 0; rb < 2; rb++) {
    int row = q0 + rb * 32 + lr;
    float l_chunk = sum_both_halves(lsum[rb]);
    if (row < a.Nq && m2[rb] != BURST_NEG_INF) {   // rows that saw no key keep their state bit for bit
      float m_old2 = mh[row] * kLog2e;             // stored in natural-log units
      float l_old = lh[row];
      float m_new = fmaxf(m_old2, m2[rb]);
      float ref = (m_new == BURST_NEG_INF) ? 0.f : m_new;
      float fa = fast_exp2(m_old2 - ref);          // weight of the stored state
      float fb = fast_exp2(m2[rb] - ref);          // weight of this chunk
      float* orow = Oh + (size_t)row * 128;
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
            nw[b] = keep + fb * o[rb][db][4 * q4 + b];
          }
          *reinterpret_cast<f32x4*>(ptr) = nw;
        }
      if (h == 0) {
        mh[row] = m_new * kLn2;
        lh[row] = ((fa == 0.f) ? 0.f : fa * l_old) + fb * l_chunk;
      }
    }
  }
}

int launch_fwd_mfma(const KParams& p, const void* Q, const void* K, const void* V,
                    float* O_acc, float* m, float* l, hipStream_t stream) {
  FwdArgs a;
  a.Q = (const bf16*)Q; a.K = (const bf16*)K; a.V = (const bf16*)V;
  a.O_acc = O_acc; a.m = m; a.l = l;
  a.Nq = p.Nq; a.Nc = p.Nc; a.H = p.B * p.H;
  a.causal = p.causal;
  a.c = p.scale * kLog2e;
  a.q_off = p.q_off; a.k_off = p.k_off;
  a.q_blocks = (p.Nq + FWD_BR - 1) / FWD_BR;
  int heads8 = ((a.H + 7) / 8) * 8;                // pad the head count to a multiple of 8 ids
  long long nblocks = (long long)heads8 * a.q_blocks;
  if (nblocks > 0x7fffffffLL) return BURST_ERR_SHAPE;
  hipLaunchKernelGGL(burst_fwd_mfma_kernel, dim3((unsigned)nblocks), dim3(256), 4 * FWD_TILE_BYTES, stream, a);
  return hipGetLastError() == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
}

}  // namespace burst
