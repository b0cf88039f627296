// Backward of one block pair (paper Alg. 2 loop body) for bf16, d = 128, as two kernels.
//
// Alg. 2 accumulates dK_i, dV_i over query rows and dQ_j over keys.  On this GPU a single
// kernel that keeps one side in registers has to push the other side through fp32 atomics,
// whose rate (about one per clock per L2 channel) is far below what d = 128 needs.  So the
// block pair is done twice, each time with the reduction side held in registers:
//   * bwd_dq:  query rows stationary (64 per wavefront), keys streamed in 32-key tiles:
//              S^T = K Q^T, dP^T = V dO^T, dS^T = P^T o (dP^T - D), dQ^T += K^T dS^T
//   * bwd_dkv: keys stationary (64 per wavefront), query rows streamed in 32-row tiles:
//              S = Q K^T, dP = dO V^T, P, dS, dV += P^T dO, dK += dS^T Q
// Both recompute P = exp(S - lse) from the saved log-sum-exp; neither stores S, P or dS.
// No atomics: results are deterministic.
#include "burst_bwd_common.h"

namespace burst {

// 32 rows x 128 bf16 tile: 512 granules of 16 B, 2 per thread.
__device__ __forceinline__ void load_tile32_regs(const bf16* __restrict__ base, int row0, int nrows,
                                                 int tid, i32x4 (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; i++) {
    int gi = i * 256 + tid;
    int row = gi >> 4, g = gi & 15;
    i32x4 v = {0, 0, 0, 0};
    if (row0 + row < nrows)
      v = *reinterpret_cast<const i32x4*>(base + (size_t)(row0 + row) * 128 + g * 8);
    r[i] = v;
  }
}
__device__ __forceinline__ void store_tile32_lds(char* lds, int tid, const i32x4 (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; i++) {
    int gi = i * 256 + tid;
    int row = gi >> 4, g = gi & 15;
    *reinterpret_cast<i32x4*>(lds + tile_off(row, g)) = r[i];
  }
}

// ------------------------------------------------------------------------------------ dK, dV
constexpr int DKV_BC = 256;           // keys per workgroup (4 wavefronts x 64)
constexpr int DKV_BR = 32;            // query rows per tile
constexpr int DKV_QTILE_BYTES = DKV_BR * 256;
// LDS: V block | K block (256 rows x 256 B each) | Q tile | dO tile | lse2 | D
// The K/V blocks stay for the whole kernel (they are the B operands of every step); the
// Q / dO tile is single-buffered in LDS and double-buffered through registers.
constexpr int DKV_LDS_V = 0;
constexpr int DKV_LDS_K = DKV_BC * 256;
constexpr int DKV_LDS_Q = 2 * DKV_BC * 256;
constexpr int DKV_LDS_G = DKV_LDS_Q + DKV_QTILE_BYTES;
constexpr int DKV_LDS_L = DKV_LDS_G + DKV_QTILE_BYTES;
constexpr int DKV_LDS_D = DKV_LDS_L + DKV_BR * 4;
constexpr int DKV_LDS_BYTES = DKV_LDS_D + DKV_BR * 4;

__global__ void __launch_bounds__(256, 1)
burst_bwd_dkv_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x;
  const int w = tid >> 6, lane = tid & 63, lr = lane & 31, h = lane >> 5;
  int head, kblk;
  {
    int bid = blockIdx.x;
    int xcd = bid & 7, idx = bid >> 3;
    int hx = idx / a.blocks_per_head;
    kblk = idx - hx * a.blocks_per_head;
    head = hx * 8 + xcd;
    if (head >= a.H) return;
  }
  const int key_wg = kblk * DKV_BC;
  const int key0 = key_wg + w * 64;                // first key of this wavefront
  const bf16* Qh = a.Q + (size_t)head * a.Nq * 128;
  const bf16* Gh = a.dO + (size_t)head * a.Nq * 128;
  const bf16* Kh = a.K + (size_t)head * a.Nc * 128;
  const bf16* Vh = a.V + (size_t)head * a.Nc * 128;
  const float* lseh = a.lse + (size_t)head * a.Nq;
  const float* Dh = a.D + (size_t)head * a.Nq;

  // query tiles to visit: causal rows before the first key of the workgroup see none of it
  const int ntiles_all = (a.Nq + DKV_BR - 1) / DKV_BR;
  int t_begin = 0;
  if (a.causal) {
    long long first_row = a.k_off + key_wg - a.q_off;      // first row index that sees key_wg
    if (first_row > 0) t_begin = (int)min((long long)ntiles_all, first_row / DKV_BR);
  }

  f32x16 dk[2][4], dv[2][4];
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int r = 0; r < 16; r++) { dk[kb][db][r] = 0.f; dv[kb][db][r] = 0.f; }

  if (t_begin < ntiles_all) {
    // K and V blocks of the workgroup -> LDS (4096 granules each, 16 per thread)
#pragma unroll 4
    for (int i = 0; i < 16; i++) {
      int gi = i * 256 + tid;
      int row = gi >> 4, g = gi & 15;
      i32x4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
      if (key_wg + row < a.Nc) {
        kv = *reinterpret_cast<const i32x4*>(Kh + (size_t)(key_wg + row) * 128 + g * 8);
        vv = *reinterpret_cast<const i32x4*>(Vh + (size_t)(key_wg + row) * 128 + g * 8);
      }
      *reinterpret_cast<i32x4*>(smem + DKV_LDS_K + tile_off(row, g)) = kv;
      *reinterpret_cast<i32x4*>(smem + DKV_LDS_V + tile_off(row, g)) = vv;
    }
    // A / B operand reads (128-bit): row = base row + lr, granule 2*ks + h.  Since 2*ks and
    // (h ^ row code) occupy different bits, the address of step ks is base ^ (ks << 5).
    const int abase = lr * 256 + ((h ^ row_code(lr)) << 4);
    const int kvbase = (w * 64) * 256 + abase;     // + kb * 32 * 256 at the use site
    int taddr[4][2];     // Q / dO as B operand through transposing reads (rows = q, cols = d)
    {
      const int j16 = lane & 15, dh = (lane >> 4) & 1;
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int sx = 0; sx < 2; sx++)
          taddr[db][sx] = tile_off(8 * sx + 4 * h + (j16 >> 2), db * 4 + 2 * dh + ((j16 & 3) >> 1)) + (j16 & 1) * 8;
    }

    // lse2 (threads 0..31) and D (threads 32..63) of a tile travel with the Q / dO prefetch
    auto load_rowstat = [&](int t) -> float {
      float v = 0.f;
      if (tid < 64) {
        int row = t * DKV_BR + (tid & 31);
        if (tid < 32) {
          float lv = row < a.Nq ? lseh[row] : BURST_NEG_INF;
          v = (lv == BURST_NEG_INF) ? __builtin_inff() : lv * kLog2e;      // +inf => P = 0
        } else {
          v = row < a.Nq ? Dh[row] : 0.f;
        }
      }
      return v;
    };
    auto store_rowstat = [&](float v) {
      if (tid < 32) reinterpret_cast<float*>(smem + DKV_LDS_L)[tid] = v;
      else if (tid < 64) reinterpret_cast<float*>(smem + DKV_LDS_D)[tid - 32] = v;
    };

    i32x4 qreg[2], greg[2];
    float rstat;
    load_tile32_regs(Qh, t_begin * DKV_BR, a.Nq, tid, qreg);
    load_tile32_regs(Gh, t_begin * DKV_BR, a.Nq, tid, greg);
    rstat = load_rowstat(t_begin);

    const long long wave_first_k = a.k_off + key0;
    const long long wave_last_k = a.k_off + key0 + 63;
    for (int t = t_begin; t < ntiles_all; t++) {
      // registers (tile t) -> LDS; the previous step's readers are past the closing barrier
      store_tile32_lds(smem + DKV_LDS_Q, tid, qreg);
      store_tile32_lds(smem + DKV_LDS_G, tid, greg);
      store_rowstat(rstat);
      if (t + 1 < ntiles_all) {
        load_tile32_regs(Qh, (t + 1) * DKV_BR, a.Nq, tid, qreg);
        load_tile32_regs(Gh, (t + 1) * DKV_BR, a.Nq, tid, greg);
        rstat = load_rowstat(t + 1);
      }
      __syncthreads();
      const long long tile_first_q = a.q_off + (long long)t * DKV_BR;
      const long long tile_last_q = tile_first_q + DKV_BR - 1;
      const bool wave_skips = (a.causal && wave_first_k > tile_last_q) || (key0 >= a.Nc);
      if (!wave_skips) {
        const char* ql = smem + DKV_LDS_Q;
        const char* gl = smem + DKV_LDS_G;
        f32x16 s[2], dp[2];
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
          for (int r = 0; r < 16; r++) { s[kb][r] = 0.f; dp[kb][r] = 0.f; }
        // S = Q K^T, dP = dO V^T: operand fragments are fetched one k-step ahead; the
        // scheduling barriers keep the compiler from hoisting all 48 LDS reads (which would
        // not fit in registers next to the 256 accumulators).
        bf16x8 qa, ga, kf0, kf1, vf0, vf1;
        qa = lds_read_b128(ql, abase);
        ga = lds_read_b128(gl, abase);
        kf0 = lds_read_b128(smem + DKV_LDS_K, kvbase);
        kf1 = lds_read_b128(smem + DKV_LDS_K, 32 * 256 + kvbase);
        vf0 = lds_read_b128(smem + DKV_LDS_V, kvbase);
        vf1 = lds_read_b128(smem + DKV_LDS_V, 32 * 256 + kvbase);
#pragma unroll
        for (int ks = 0; ks < 8; ks++) {
          bf16x8 qa_n, ga_n, kf0_n, kf1_n, vf0_n, vf1_n;
          if (ks < 7) {
            const int x = (ks + 1) << 5;
            qa_n = lds_read_b128(ql, abase ^ x);
            ga_n = lds_read_b128(gl, abase ^ x);
            kf0_n = lds_read_b128(smem + DKV_LDS_K, kvbase ^ x);
            kf1_n = lds_read_b128(smem + DKV_LDS_K, 32 * 256 + (kvbase ^ x));
            vf0_n = lds_read_b128(smem + DKV_LDS_V, kvbase ^ x);
            vf1_n = lds_read_b128(smem + DKV_LDS_V, 32 * 256 + (kvbase ^ x));
          }
          s[0] = mfma32(qa, kf0, s[0]);
          dp[0] = mfma32(ga, vf0, dp[0]);
          s[1] = mfma32(qa, kf1, s[1]);
          dp[1] = mfma32(ga, vf1, dp[1]);
          __builtin_amdgcn_sched_barrier(0);
          if (ks < 7) { qa = qa_n; ga = ga_n; kf0 = kf0_n; kf1 = kf1_n; vf0 = vf0_n; vf1 = vf1_n; }
        }
        // P = exp2(S c - lse2), dS = P o (dP - D).  Register r of a lane belongs to query row
        // 8*(r/4) + 4*h + (r%4) of the tile; the row statistics are broadcast reads from LDS.
        const bool need_mask = a.causal && (wave_last_k > tile_first_q);
        bf16x8 pf[2][2], dsf[2][2];
        const float* lp = reinterpret_cast<const float*>(smem + DKV_LDS_L);
        const float* dp_ = reinterpret_cast<const float*>(smem + DKV_LDS_D);
#pragma unroll
        for (int u = 0; u < 2; u++) {
          float lse2v[8], Dvv[8];
#pragma unroll
          for (int q2 = 0; q2 < 2; q2++) {
            f32x4 lv = *reinterpret_cast<const f32x4*>(lp + 16 * u + 8 * q2 + 4 * h);
            f32x4 dv4 = *reinterpret_cast<const f32x4*>(dp_ + 16 * u + 8 * q2 + 4 * h);
#pragma unroll
            for (int b = 0; b < 4; b++) { lse2v[4 * q2 + b] = lv[b]; Dvv[4 * q2 + b] = dv4[b]; }
          }
#pragma unroll
          for (int kb = 0; kb < 2; kb++) {
            long long kpos = a.k_off + key0 + kb * 32 + lr;
            bf16x8 f, g;
#pragma unroll
            for (int t8 = 0; t8 < 8; t8++) {
              const int r = 8 * u + t8;
              float p = fast_exp2(__builtin_fmaf(s[kb][r], a.c, -lse2v[t8]));
              if (need_mask) {
                long long qpos = tile_first_q + 8 * (r >> 2) + 4 * h + (r & 3);
                if (kpos > qpos) p = 0.f;
              }
              f[t8] = (bf16)p;
              g[t8] = (bf16)(p * (dp[kb][r] - Dvv[t8]));
            }
            pf[kb][u] = f; dsf[kb][u] = g;
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        // dV += P^T dO ; dK += dS^T Q   (B operands through transposing reads, one step ahead)
        bf16x4 g0 = lds_read_tr(gl, taddr[0][0]), g1 = lds_read_tr(gl, taddr[0][1]);
        bf16x4 q0 = lds_read_tr(ql, taddr[0][0]), q1 = lds_read_tr(ql, taddr[0][1]);
#pragma unroll
        for (int it = 0; it < 8; it++) {
          const int u = it >> 2, db = it & 3;
          bf16x4 g0n, g1n, q0n, q1n;
          if (it < 7) {
            const int un = (it + 1) >> 2, dbn = (it + 1) & 3;
            g0n = lds_read_tr(gl, un * 16 * 256 + taddr[dbn][0]);
            g1n = lds_read_tr(gl, un * 16 * 256 + taddr[dbn][1]);
            q0n = lds_read_tr(ql, un * 16 * 256 + taddr[dbn][0]);
            q1n = lds_read_tr(ql, un * 16 * 256 + taddr[dbn][1]);
          }
          bf16x8 gt = cat4(g0, g1), qt = cat4(q0, q1);
          dv[0][db] = mfma32(pf[0][u], gt, dv[0][db]);
          dk[0][db] = mfma32(dsf[0][u], qt, dk[0][db]);
          dv[1][db] = mfma32(pf[1][u], gt, dv[1][db]);
          dk[1][db] = mfma32(dsf[1][u], qt, dk[1][db]);
          __builtin_amdgcn_sched_barrier(0);
          if (it < 7) { g0 = g0n; g1 = g1n; q0 = q0n; q1 = q1n; }
        }
      }
      __syncthreads();           // everyone is done with this Q / dO tile
    }
  }
  // epilogue: keys are owned by this wavefront alone. C layout: lane = d column, regs = keys.
  float* dKh = a.dK + (size_t)head * a.Nc * 128;
  float* dVh = a.dV + (size_t)head * a.Nc * 128;
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      int key = key0 + kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
      if (key < a.Nc) {
#pragma unroll
        for (int db = 0; db < 4; db++) {
          size_t off = (size_t)key * 128 + db * 32 + lr;
          float k_old = 0.f, v_old = 0.f;
          if (a.acc_dkv) { k_old = dKh[off]; v_old = dVh[off]; }
          dKh[off] = k_old + a.scale * dk[kb][db][r];
          dVh[off] = v_old + dv[kb][db][r];
        }
      }
    }
}

static int set_dkv_lds_attr() {
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)burst_bwd_dkv_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                            DKV_LDS_BYTES) != hipSuccess) return BURST_ERR_LAUNCH;
    attr_set = true;
  }
  return BURST_OK;
}

int launch_bwd_dkv_mfma(const KParams& p, const void* Q, const void* K, const void* V,
                        const void* dO, const float* lse, const float* D, float* dK, float* dV,
                        int acc_dkv, hipStream_t stream) {
  if (p.Nc <= 0) return BURST_OK;
  int st = set_dkv_lds_attr();
  if (st != BURST_OK) return st;
  BwdArgs a = make_bwd_args(p, Q, K, V, dO, lse, D, nullptr, dK, dV, 0, acc_dkv);
  int heads8 = ((a.H + 7) / 8) * 8;
  a.blocks_per_head = (p.Nc + DKV_BC - 1) / DKV_BC;
  long long nb = (long long)heads8 * a.blocks_per_head;
  if (nb > 0x7fffffffLL) return BURST_ERR_SHAPE;
  hipLaunchKernelGGL(burst_bwd_dkv_kernel, dim3((unsigned)nb), dim3(256), DKV_LDS_BYTES, stream, a);
  return hipGetLastError() == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
}

}  // namespace burst
