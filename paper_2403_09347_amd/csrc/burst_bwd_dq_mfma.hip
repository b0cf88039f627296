// Backward, dQ side of one block pair (paper Alg. 2 loop body) for bf16, d = 128.
//
// Alg. 2 accumulates dK_i, dV_i over query rows and dQ_j over keys.  On this GPU a single
// kernel that keeps one side in registers has to push the other side through fp32 atomics,
// whose rate (about one per clock per L2 channel) is far below what d = 128 needs.  So the
// block pair is done twice, each time with the reduction side held in registers; this file
// is the query-stationary half:
//     S^T = K Q^T,  dP^T = V dO^T,  P^T = exp(S^T - lse),  dS^T = P^T o (dP^T - D),
//     dQ^T += K^T dS^T
// P is recomputed from the saved log-sum-exp; neither S, P nor dS is ever stored.
//
// One workgroup = 4 wavefronts = 256 query rows of one (batch, head); a wavefront owns 64
// rows (their Q fragments stay in registers as B operands, their dO rows stay in LDS for the
// whole kernel) and walks the chunk in tiles of 32 keys.  With S^T = K Q^T every lane owns one query row, so lse and D are
// per-lane scalars, and the dS^T accumulators already have the B-operand layout that
// dQ^T += K^T dS^T needs (K^T comes through transposing LDS reads).  Same machinery as the
// forward kernel: dQ^T accumulators pinned in AGPRs, two (S, dP) buffers that swap roles
// each tile, the 48 MFMAs of a tile hand-interleaved with the vector work, K/V tiles DMA-ed
// from HBM into LDS rings two tiles ahead, one barrier per tile.
#include "burst_bwd_common.h"

namespace burst {

constexpr int DQ_BR = 256;            // query rows per workgroup (4 wavefronts x 64)
constexpr int DQ_BC = 32;             // keys per tile
constexpr int DQ_TILE_BYTES = DQ_BC * 256;
constexpr int DQ_KSLOTS = 4;          // K of tile t is read in steps t-1 (S) and t (dQ)
constexpr int DQ_VSLOTS = 3;
constexpr int DQ_GBASE = (DQ_KSLOTS + DQ_VSLOTS) * DQ_TILE_BYTES;   // dO block of the workgroup: 256 rows
constexpr int DQ_LDS_BYTES = DQ_GBASE + DQ_BR * 256;

// WINDOW = false compiles the sliding-window code away: this kernel uses every register of the
// file, and the few values the window logic keeps alive would otherwise push others to scratch.
template <bool WINDOW>
__global__ void __launch_bounds__(256, 1)
burst_bwd_dq_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const long long window = WINDOW ? a.window : 0;
  const int tid = threadIdx.x;
  const int w = tid >> 6, lane = tid & 63, lr = lane & 31, h = lane >> 5;
  int head, qb;
  {
    int bid = blockIdx.x;
    int xcd = bid & 7, idx = bid >> 3;
    int hx = idx / a.blocks_per_head;
    qb = idx - hx * a.blocks_per_head;
    head = hx * 8 + xcd;
    if (head >= a.H) return;
  }
  const int q0 = qb * DQ_BR + w * 64;
  const bf16* Qh = a.Q + (size_t)head * a.Nq * 128;
  const bf16* Gh = a.dO + (size_t)head * a.Nq * 128;
  const bf16* Kh = a.K + (size_t)head * a.Nc * 128;
  const bf16* Vh = a.V + (size_t)head * a.Nc * 128;
  const float* lseh = a.lse + (size_t)head * a.Nq;
  const float* Dh = a.D + (size_t)head * a.Nq;
  float* dQh = a.dQ + (size_t)head * a.Nq * 128;

  // Sliding window: key tiles before the first one that the workgroup's first row can see are
  // skipped by moving the start of the chunk (pointers, length, global offset) forward by whole
  // tiles; everything below works on that shortened chunk.
  int Nc = a.Nc;
  long long k_off = a.k_off;
  if (window > 0) {
    long long lo = a.q_off + (long long)qb * DQ_BR - window + 1 - a.k_off;   // first visible key index
    if (lo >= a.Nc) Nc = 0;                        // nothing visible: contribution 0
    else if (lo > 0) {
      const int skip = (int)(lo / DQ_BC) * DQ_BC;
      Kh += (size_t)skip * 128; Vh += (size_t)skip * 128;
      Nc -= skip; k_off += skip;
    }
  }
  int ntiles = (Nc + DQ_BC - 1) / DQ_BC;
  if (a.causal) {
    long long lim = a.q_off + min(qb * DQ_BR + DQ_BR, a.Nq) - 1 - k_off;
    long long t = lim < 0 ? 0 : lim / DQ_BC + 1;
    if (t < ntiles) ntiles = (int)t;
  }

  f32x16 dq[2][4];         // dQ^T accumulators [row block][32-wide d block], pinned in AGPRs
#pragma unroll
  for (int rb = 0; rb < 2; rb++)
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int r = 0; r < 16; r++) dq[rb][db][r] = 0.f;

  if (ntiles > 0) {
    bf16x8 qf[2][8];
    float nlse2[2], Dv[2];
#pragma unroll
    for (int rb = 0; rb < 2; rb++) {
      int row = q0 + rb * 32 + lr;
      bool ok = row < a.Nq;
      float lv = ok ? lseh[row] : BURST_NEG_INF;
      nlse2[rb] = (lv == BURST_NEG_INF) ? BURST_NEG_INF : -lv * kLog2e;   // -inf => P = exp2(-inf) = 0
      Dv[rb] = ok ? Dh[row] : 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ks++) {
        bf16x8 z;
#pragma unroll
        for (int t = 0; t < 8; t++) z[t] = (bf16)0.0f;
        qf[rb][ks] = ok ? *reinterpret_cast<const bf16x8*>(Qh + (size_t)row * 128 + ks * 16 + h * 8) : z;
      }
    }
    // LDS addressing.  A-operand reads (128-bit): row lr, granule 2*ks + h; since 2*ks and
    // (h ^ row code) occupy different bits the address of step ks is abase ^ (ks << 5).
    const int abase = lr * 256 + ((h ^ row_code(lr)) << 4);
    int taddr[4][2];       // K^T through transposing reads (rows = keys, cols = d)
    {
      const int j16 = lane & 15, dh = (lane >> 4) & 1;
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int sx = 0; sx < 2; sx++)
          taddr[db][sx] = tile_off(8 * sx + 4 * h + (j16 >> 2), db * 4 + 2 * dh + ((j16 & 3) >> 1)) + (j16 & 1) * 8;
    }
    // DMA: a 32-key tile is 8 wave-loads of 4 rows; wavefront w issues loads 2w and 2w + 1
    const __amdgpu_buffer_rsrc_t krs = make_rsrc(Kh, (unsigned)Nc * 256u);
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc(Vh, (unsigned)Nc * 256u);
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const unsigned lds0 = lds_addr(smem);
    int goff[2];
#pragma unroll
    for (int il = 0; il < 2; il++) {
      int row = 8 * w + 4 * il + (lane >> 4);
      goff[il] = row * 256 + (((lane & 15) ^ row_code(row)) << 4);
    }
    auto dma_tile = [&](__amdgpu_buffer_rsrc_t rs, unsigned lds_tile, int il, int tile) __attribute__((always_inline)) {
      dma_b128_to_lds(rs, lds_tile + (unsigned)(wu * 2 + il) * 1024u, tile * DQ_TILE_BYTES + goff[il]);
    };
    constexpr int VBASE = DQ_KSLOTS * DQ_TILE_BYTES;
    // dO rows of the workgroup -> LDS once (64 wave-loads of 4 rows, 16 per wavefront); rows
    // past Nq read as zeros
    {
      const __amdgpu_buffer_rsrc_t grs = make_rsrc(Gh, (unsigned)a.Nq * 256u);
#pragma unroll
      for (int il = 0; il < 16; il++) {
        int row = 64 * w + 4 * il + (lane >> 4);
        int off = row * 256 + (((lane & 15) ^ row_code(row)) << 4);
        dma_b128_to_lds(grs, lds0 + DQ_GBASE + (unsigned)(wu * 16 + il) * 1024u, qb * DQ_BR * 256 + off);
      }
    }
    const char* gl = smem + DQ_GBASE + w * 64 * 256;         // this wavefront's 64 dO rows
#pragma unroll
    for (int t = 0; t < 3; t++)
#pragma unroll
      for (int il = 0; il < 2; il++) {
        dma_tile(krs, lds0 + t * DQ_TILE_BYTES, il, t);
        dma_tile(vrs, lds0 + VBASE + t * DQ_TILE_BYTES, il, t);
      }
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wavefront's DMA has landed
    __builtin_amdgcn_s_barrier();

    // S^T and dP^T of a tile: [row block] accumulators of 32 keys x 32 rows
    auto sdp_tile = [&](const char* kl, const char* vl, f32x16 (&s)[2], f32x16 (&dp)[2]) __attribute__((always_inline)) {
#pragma unroll
      for (int rb = 0; rb < 2; rb++)
#pragma unroll
        for (int r = 0; r < 16; r++) { s[rb][r] = 0.f; dp[rb][r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ks++) {
        bf16x8 kf = lds_read_b128(kl, abase ^ (ks << 5));
        bf16x8 vf = lds_read_b128(vl, abase ^ (ks << 5));
#pragma unroll
        for (int rb = 0; rb < 2; rb++) {
          bf16x8 gfr = lds_read_b128(gl, rb * 32 * 256 + (abase ^ (ks << 5)));
          s[rb] = mfma32(kf, qf[rb][ks], s[rb]);
          dp[rb] = mfma32(vf, gfr, dp[rb]);
        }
      }
    };
    f32x16 sA[2], dpA[2], sB[2], dpB[2];
    sdp_tile(smem, smem + VBASE, sA, dpA);

    const long long wave_first_q = a.q_off + q0;

    // One tile: (sc, dpc) hold S^T, dP^T of tile kt; (sx, dpx) receive those of tile kt + 1.
    auto step = [&](f32x16 (&sc)[2], f32x16 (&dpc)[2], f32x16 (&sx)[2], f32x16 (&dpx)[2], int kt, int kslot,
                    int vslot) __attribute__((always_inline)) {
      const int kslot1 = (kslot + 1) & 3;                       // K of tile kt + 1
      const int kslot3 = (kslot + 3) & 3;                       // K of tile kt + 3 replaces K of tile kt - 1
      const int vslot1 = (vslot == DQ_VSLOTS - 1) ? 0 : vslot + 1;   // V of tile kt + 1; V of kt + 3 replaces V of kt
      const char* kl_next = smem + kslot1 * DQ_TILE_BYTES;
      const char* vl_next = smem + VBASE + vslot1 * DQ_TILE_BYTES;
      const char* kl = smem + kslot * DQ_TILE_BYTES;
      const unsigned k_dst = lds0 + kslot3 * DQ_TILE_BYTES;
      const unsigned v_dst = lds0 + VBASE + vslot * DQ_TILE_BYTES;
      // Operand queue for the first 32 slices, one LDS read per slice, LEAD slices ahead of its
      // use.  Read j = 4*ks + m: m = 0 K fragment (A of S^T, slices 4ks, 4ks+1), m = 1 V fragment
      // (A of dP^T, slices 4ks+2, 4ks+3), m = 2 / 3 dO fragments of row block 0 / 1 (B of dP^T).
      constexpr int LEAD = 4, RING = LEAD + 3;
      bf16x8 fq[RING];
      auto issue_read = [&](int j) __attribute__((always_inline)) {
        const int ks = j >> 2, m = j & 3;
        const int off = abase ^ (ks << 5);
        fq[j % RING] = (m == 0) ? lds_read_b128(kl_next, off)
                     : (m == 1) ? lds_read_b128(vl_next, off)
                                : lds_read_b128(gl, (m - 2) * 32 * 256 + off);
      };
#pragma unroll
      for (int j = 0; j < LEAD; j++) issue_read(j);
      // ---- masking (diagonal tiles, ragged key tail): rare.  A masked score becomes -inf,
      // its P and dS become 0.
      const long long tile_first_k = k_off + (long long)kt * DQ_BC;
      const bool need_mask = (a.causal && tile_first_k + DQ_BC - 1 > wave_first_q) ||
                             (window > 0 && tile_first_k < wave_first_q + 63 - window + 1) ||
                             ((kt + 1) * DQ_BC > Nc);
      if (need_mask) {
#pragma unroll
        for (int rb = 0; rb < 2; rb++) {
          // score register r holds key index kt*32 + 4h + (8*(r/4) + r%4) of the chunk; with
          // dd = (row position) - (position of key kt*32 + 4h) the key of register r is visible
          // iff cpart <= dd (causal), cpart > dd - window, and it exists (ragged tail).
          // Computed here, in the rare path, so that nothing of it stays live in the main loop.
          const int ln = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));   // lane id, recomputed
          const int mlr = ln & 31, mh = ln >> 5;
          const long long dd = (a.q_off - k_off) + (q0 + rb * 32 + mlr) - ((long long)kt * DQ_BC + 4 * mh);
          const int tail = Nc - 1 - (kt * DQ_BC + 4 * mh);
          int lim = a.causal ? (int)(dd < -1 ? -1 : (dd > 64 ? 64 : dd)) : 64;
          lim = lim < tail ? lim : tail;
          const long long dl = dd - window + 1;
          const int lim_lo = window > 0 ? (int)(dl < -1 ? -1 : (dl > 64 ? 64 : dl)) : -1;
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int cpart = 8 * (r >> 2) + (r & 3);
            sc[rb][r] = (cpart <= lim && cpart >= lim_lo) ? sc[rb][r] : BURST_NEG_INF;
          }
        }
      }
      bf16x8 dsf[2][2];    // dS^T fragments (B operand): [row block][16-key group]
      constexpr int TRING = 3;                     // K^T fragments: LEAD / 2 = 2 ahead
      bf16x4 tq[TRING][2];
      auto ds_pair = [&](int pidx) __attribute__((always_inline)) {   // pidx = kg * 8 + rb * 4 + t / 2
        const int kg = pidx >> 3, srb = (pidx >> 2) & 1, t = (pidx & 3) * 2;
        const int r = 8 * kg + t;
        float p0 = fast_exp2(__builtin_fmaf(sc[srb][r], a.c, nlse2[srb]));
        float p1 = fast_exp2(__builtin_fmaf(sc[srb][r + 1], a.c, nlse2[srb]));
        float d0 = p0 * (dpc[srb][r] - Dv[srb]);
        float d1 = p1 * (dpc[srb][r + 1] - Dv[srb]);
        dsf[srb][kg][t] = (bf16)d0;
        dsf[srb][kg][t + 1] = (bf16)d1;
      };
#pragma unroll
      for (int rb = 0; rb < 2; rb++)
#pragma unroll
        for (int r = 0; r < 16; r++) { sx[rb][r] = 0.f; dpx[rb][r] = 0.f; }
      __builtin_amdgcn_sched_barrier(0);
      // ---- slices 0..31: S^T and dP^T of the next tile, with the 16 dS pairs of this tile.
      // After the last tile the products read stale buffers and are discarded.
#pragma unroll
      for (int i = 0; i < 32; i++) {
        const int ks = i >> 2, m = i & 3, rb = i & 1;
        if (i + LEAD < 32) issue_read(i + LEAD);
        if (i + LEAD >= 32 && ((i + LEAD) & 1) == 0) {   // first K^T fragments of the last 16 slices
          const int tn = (i + LEAD - 32) >> 1;
          tq[tn][0] = lds_read_tr(kl, taddr[tn & 3][0]);
          tq[tn][1] = lds_read_tr(kl, taddr[tn & 3][1]);
        }
        if (m < 2) sx[rb] = mfma32(fq[(4 * ks) % RING], qf[rb][ks], sx[rb]);
        else dpx[rb] = mfma32(fq[(4 * ks + 1) % RING], fq[(4 * ks + m) % RING], dpx[rb]);
        if (i & 1) ds_pair(i >> 1);
        __builtin_amdgcn_sched_barrier(0);
      }
      // ---- slices 32..47: dQ^T += K^T dS^T, with the DMA of tiles kt + 3
#pragma unroll
      for (int i = 0; i < 16; i++) {
        const int tf = i >> 1;                     // K^T fragment: kg = tf / 4, db = tf % 4
        const int kg = tf >> 2, db = tf & 3, rb = i & 1;
        if ((i & 1) == 0 && tf + 2 < 8) {
          const int tn = tf + 2;
          tq[tn % TRING][0] = lds_read_tr(kl, (tn >> 2) * 16 * 256 + taddr[tn & 3][0]);
          tq[tn % TRING][1] = lds_read_tr(kl, (tn >> 2) * 16 * 256 + taddr[tn & 3][1]);
        }
        if ((i & 3) == 1) {
          const int j = i >> 2;                    // 0, 1 -> K of tile kt + 3; 2, 3 -> V of tile kt + 3
          if (j < 2) dma_tile(krs, k_dst, j, kt + 3);
          else dma_tile(vrs, v_dst, j - 2, kt + 3);
        }
        mfma32_acc(dq[rb][db], cat4(tq[tf % TRING][0], tq[tf % TRING][1]), dsf[rb][kg]);
        __builtin_amdgcn_sched_barrier(0);
      }
      // The 4 DMA loads just issued may stay in flight; older ones must have landed.
      __builtin_amdgcn_s_waitcnt(0x0F74);          // vmcnt(4)
      __builtin_amdgcn_s_barrier();
    };

    int kslot = 0, vslot = 0;
    for (int kt = 0; kt < ntiles; kt += 2) {
      step(sA, dpA, sB, dpB, kt, kslot, vslot);
      kslot = (kslot + 1) & 3;
      vslot = (vslot == DQ_VSLOTS - 1) ? 0 : vslot + 1;
      if (kt + 1 >= ntiles) break;
      step(sB, dpB, sA, dpA, kt + 1, kslot, vslot);
      kslot = (kslot + 1) & 3;
      vslot = (vslot == DQ_VSLOTS - 1) ? 0 : vslot + 1;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): no DMA may outlive the loop
  }
  mfma_acc_fence(dq);
  // epilogue: dQ rows are owned by this wavefront alone
#pragma unroll
  for (int rb = 0; rb < 2; rb++) {
    int row = q0 + rb * 32 + lr;
    if (row < a.Nq) {
      float* orow = dQh + (size_t)row * 128;
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          float* ptr = orow + db * 32 + 8 * q4 + 4 * h;
          f32x4 v = {0.f, 0.f, 0.f, 0.f};
          if (a.acc_dq) v = *reinterpret_cast<f32x4*>(ptr);
#pragma unroll
          for (int b = 0; b < 4; b++) v[b] += a.scale * dq[rb][db][4 * q4 + b];
          *reinterpret_cast<f32x4*>(ptr) = v;
        }
    }
  }
}

int launch_bwd_dq_mfma(const KParams& p, const void* Q, const void* K, const void* V,
                       const void* dO, const float* lse, const float* D, float* dQ, int acc_dq,
                       hipStream_t stream) {
  if (p.Nq <= 0) return BURST_OK;
  BwdArgs a = make_bwd_args(p, Q, K, V, dO, lse, D, dQ, nullptr, nullptr, acc_dq, 0);
  int heads8 = ((a.H + 7) / 8) * 8;
  a.blocks_per_head = (p.Nq + DQ_BR - 1) / DQ_BR;
  long long nb = (long long)heads8 * a.blocks_per_head;
  if (nb > 0x7fffffffLL) return BURST_ERR_SHAPE;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)burst_bwd_dq_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            DQ_LDS_BYTES) != hipSuccess ||
        hipFuncSetAttribute((const void*)burst_bwd_dq_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            DQ_LDS_BYTES) != hipSuccess) return BURST_ERR_LAUNCH;
    attr_set = true;
  }
  if (a.window > 0)
    hipLaunchKernelGGL(burst_bwd_dq_kernel<true>, dim3((unsigned)nb), dim3(256), DQ_LDS_BYTES, stream, a);
  else
    hipLaunchKernelGGL(burst_bwd_dq_kernel<false>, dim3((unsigned)nb), dim3(256), DQ_LDS_BYTES, stream, a);
  return hipGetLastError() == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
}

}  // namespace burst
