// Plainly written MFMA kernels for the forward chunk step (paper Alg. 1 loop body, tiled as in
// Sec. 2.4) and the two halves of the backward block pair (Alg. 2 loop body), bf16, with the head
// dimension a compile-time constant.  This header is the source of two kernel families; each is
// built by a small translation unit that defines BURST_SMALL_D (head dimension), BURST_SMALL_NS
// (namespace) and, optionally, BURST_SMALL_DKV_WAVES before including it:
//   burst_d64_mfma.hip    d = 64, namespace burst::d64, all three kernels
//   burst_d128_plain.hip  d = 128, namespace burst::d128p, all three kernels, the dK/dV one with
//                         two wavefronts (64 keys) per workgroup (BURST_SMALL_DKV_WAVES = 2)
//
// Same mathematics, operand orientations and register layouts as the hand-scheduled d = 128
// kernels (S^T = K Q^T with one query row per lane for the forward and dQ side, S = Q K^T with one
// key per lane for the dK/dV side; P and dS leave the accumulators already in the layout the next
// MFMA wants), but written plainly: one wavefront owns 32 rows (or keys), a step runs its phases
// one after the other with compiler-scheduled MFMAs in VGPR accumulators, tiles are
// double-buffered in LDS by DMA with one barrier per tile, and two workgroups share a CU so that
// one's vector work overlaps the other's matrix work.  At d = 64 a tile has half the matrix work
// per score of d = 128 and the same softmax work, so these kernels are bound by the vector unit;
// the hand-interleaved schedules of the d = 128 kernels would buy little here.
//
// LDS tile layout at d = 64: rows of 128 bytes (8 granules of 16 bytes); granule g of row r sits
// at slot g ^ ((r >> 1) & 7), which makes the 128-bit operand reads of 32 consecutive rows
// conflict-free.  At d = 128: the layout of burst_common.h.
#pragma once
#if !defined(BURST_SMALL_D) || !defined(BURST_SMALL_NS)
#error "define BURST_SMALL_D and BURST_SMALL_NS before including burst_plain_mfma.h"
#endif
#include "burst_bwd_common.h"

namespace burst {
namespace BURST_SMALL_NS {

constexpr int S_D = BURST_SMALL_D;
constexpr int S_ROWB = S_D * 2;                   // bytes per row
constexpr int S_KS = S_D / 16;                    // k-steps of a contraction over d
constexpr int S_DB = S_D / 32;                    // 32-wide blocks of d
constexpr int S_RPL = 1024 / S_ROWB;              // tile rows per wave-wide DMA load
constexpr int S_GPR = S_ROWB / 16;                // granules per row
constexpr float S_LAZY = 8.0f;                    // log2 of the largest P allowed before the max is raised

struct FwdArgsLite {
  const bf16* Q; const bf16* K; const bf16* V;
  float* O_acc; float* m; float* l;
  int Nq, Nc, H, group;
  int causal;
  float c;               // scale * log2(e)
  long long q_off, k_off, window;
  const uint8_t* bmask; int bsize, bpitch;       // block flags (nullptr = none)
  long long bhstride;                            // bytes between heads' flag matrices (0 = shared)
  int blocks_per_head;
  Layout lay;                                    // strides of Q and of K, V
};

__device__ __forceinline__ int s_swz(int row) { return S_D == 64 ? ((row >> 1) & 7) : row_code(row); }
__device__ __forceinline__ int s_off(int row, int granule) {
  return row * S_ROWB + ((granule ^ s_swz(row)) << 4);
}
// DMA of `rows8` groups of 8 tile rows: one wave-wide load moves 8 rows (1024 bytes); lane i
// fills LDS slot i & 7 of row i >> 3 of the group and asks for the granule that belongs there.
// (pitch: bytes between rows of the tensor in HBM)
__device__ __forceinline__ int s_dma_off(int group, int lane, unsigned pitch) {
  const int row = group * S_RPL + lane / S_GPR;
  return (int)(row * pitch + (((lane % S_GPR) ^ s_swz(row)) << 4));
}
// bytes a buffer descriptor must cover for `rows` rows `pitch` bytes apart
__device__ __forceinline__ unsigned s_span(int rows, unsigned pitch) {
  return rows > 0 ? (unsigned)(rows - 1) * pitch + (unsigned)S_ROWB : 0u;
}
// addresses of the transposing reads of a 16-row group (see the d = 128 forward kernel): the
// 16-lane group (h, dh) reads rows 8*sx + 4*h + (0..3), columns db*32 + dh*16 + (0..15)
__device__ __forceinline__ void s_taddr(int lane, int (&taddr)[S_DB][2]) {
  const int j16 = lane & 15, dh = (lane >> 4) & 1, h = lane >> 5;
#pragma unroll
  for (int db = 0; db < S_DB; db++)
#pragma unroll
    for (int sx = 0; sx < 2; sx++)
      taddr[db][sx] = s_off(8 * sx + 4 * h + (j16 >> 2), db * 4 + 2 * dh + ((j16 & 3) >> 1)) + (j16 & 1) * 8;
}
__device__ __forceinline__ bf16x8 s_load8(const bf16* p, bool ok) {
  bf16x8 z;
#pragma unroll
  for (int t = 0; t < 8; t++) z[t] = (bf16)0.0f;
  return ok ? *reinterpret_cast<const bf16x8*>(p) : z;
}
__device__ __forceinline__ void s_head_block(int bid, int blocks_per_head, int& head, int& blk) {
  // consecutive workgroup ids go round-robin to the 8 XCDs: all blocks of a head share an XCD
  const int xcd = bid & 7, idx = bid >> 3;
  const int hx = idx / blocks_per_head;
  blk = idx - hx * blocks_per_head;
  head = hx * 8 + xcd;
}

// Calls with block flags (paper Sec. 2.6) run the SPARSE instantiations: wavefront 0 first writes
// the list of tiles that at least one wavefront of the workgroup can see into LDS (tile index plus
// one bit per wavefront, list[0] = count, two end entries that name a tile past the data), the
// loop then walks that list, and a wavefront whose bit is clear hides the whole tile.
constexpr int S_MAX_LIST = 4096;                  // entries; longer masked calls take the generic kernels
template <typename F>
__device__ __forceinline__ int s_build_list(int* list, int w, int lane, int t_lo, int t_hi, int end_tile, F bits_of) {
  if (w == 0) {
    int n = 0;
    for (int base = t_lo; base < t_hi; base += 64) {
      const int t = base + lane;
      int bits = 0;
      if (t < t_hi) bits = bits_of(t);
      const unsigned long long bal = __builtin_amdgcn_ballot_w64(bits != 0);
      if (bits != 0) {
        const int pos = n + __builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0u));
        list[1 + pos] = t | (bits << 20);
      }
      n += __builtin_popcountll(bal);
    }
    if (lane < 2) list[1 + n + lane] = end_tile;
    if (lane == 0) list[0] = n;
  }
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(list[0]);
}

// ------------------------------------------------------------------------------- forward
constexpr int SF_BR = 128;                        // query rows per workgroup (4 wavefronts x 32)
constexpr int SF_BC = 64;                         // keys per tile
constexpr int SF_TILE = SF_BC * S_ROWB;

template <bool SPARSE>
__global__ void __launch_bounds__(256, 2)
burst_fwd_d64_kernel(FwdArgsLite a) {
  __shared__ __attribute__((aligned(16))) char smem[4 * SF_TILE];   // K[2], V[2]
  extern __shared__ int s_list[];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, lr = lane & 31, h = lane >> 5;
  int head, qb;
  s_head_block(blockIdx.x, a.blocks_per_head, head, qb);
  if (head >= a.H) return;
  if (a.causal) qb = a.blocks_per_head - 1 - qb;   // later blocks see more keys: the long ones start first
  const int q0 = qb * SF_BR + w * 32;
  const bf16* Qh = a.Q + a.lay.q_base(head);
  const bf16* Kh = a.K + a.lay.kv_base(head / a.group);
  const bf16* Vh = a.V + a.lay.kv_base(head / a.group);
  const unsigned kpitch = (unsigned)a.lay.ks_r * 2u;             // bytes between key rows

  int Nc = a.Nc;
  long long k_off = a.k_off;
  int t_lo = 0;
  if (a.window > 0) {                              // skip whole tiles before the window of the first row
    long long lo = a.q_off + (long long)qb * SF_BR - a.window + 1 - a.k_off;
    if (lo >= a.Nc) return;
    if (lo > 0) {
      const int skip = (int)(lo / SF_BC) * SF_BC;
      if constexpr (SPARSE) {
        t_lo = skip / SF_BC;
      } else {
        Kh += (size_t)skip * a.lay.ks_r; Vh += (size_t)skip * a.lay.ks_r;
        Nc -= skip; k_off += skip;
      }
    }
  }
  int ntiles = (Nc + SF_BC - 1) / SF_BC;
  if (a.causal) {                                  // stop after the last tile any row of the workgroup sees
    long long lim = a.q_off + min(qb * SF_BR + SF_BR, a.Nq) - 1 - k_off;
    if (lim < 0) return;
    long long t = lim / SF_BC + 1;
    if (t < ntiles) ntiles = (int)t;
  }
  if (ntiles <= 0) return;
  if constexpr (SPARSE) {
    ntiles = s_build_list(s_list, w, lane, t_lo, ntiles, (Nc + SF_BC - 1) / SF_BC, [&](int t) {
      int bits = 0;
#pragma unroll
      for (int ww = 0; ww < 4; ww++) {
        const int row0 = qb * SF_BR + ww * 32;
        if (row0 < a.Nq && (a.bmask + (size_t)head * a.bhstride)[(size_t)(row0 / a.bsize) * a.bpitch + (t * SF_BC) / a.bsize] != 0) bits |= 1 << ww;
      }
      return bits;
    });
    if (ntiles == 0) return;
  }
  auto entry_at = [&](int j) __attribute__((always_inline)) {      // walk position -> tile | wavefront bits << 20
    if constexpr (SPARSE) return __builtin_amdgcn_readfirstlane(s_list[1 + j]);
    else return j | (0xf << 20);
  };

  bf16x8 qf[S_KS];
#pragma unroll
  for (int ks = 0; ks < S_KS; ks++) qf[ks] = s_load8(Qh + (size_t)(q0 + lr) * a.lay.qs_r + ks * 16 + h * 8, q0 + lr < a.Nq);
  f32x16 o[S_DB];
#pragma unroll
  for (int db = 0; db < S_DB; db++)
#pragma unroll
    for (int r = 0; r < 16; r++) o[db][r] = 0.f;
  float m2 = BURST_NEG_INF, lsum = 0.f;            // reference max (log2 units), sum over this lane's keys

  int kaddr[S_KS], taddr[S_DB][2];
#pragma unroll
  for (int ks = 0; ks < S_KS; ks++) kaddr[ks] = s_off(lr, 2 * ks + h);
  s_taddr(lane, taddr);
  const __amdgpu_buffer_rsrc_t krs = make_rsrc(Kh, s_span(Nc, kpitch));
  const __amdgpu_buffer_rsrc_t vrs = make_rsrc(Vh, s_span(Nc, kpitch));
  const int wu = __builtin_amdgcn_readfirstlane(w);
  const unsigned lds0 = lds_addr(smem);
  constexpr int NL = SF_BC / S_RPL / 4;           // wave-wide loads per wavefront and tile
  int goff[NL];
#pragma unroll
  for (int il = 0; il < NL; il++) goff[il] = s_dma_off(w * NL + il, lane, kpitch);
  auto dma_tile = [&](int t, int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int il = 0; il < NL; il++) {
      dma_b128_to_lds(krs, lds0 + buf * SF_TILE + (unsigned)(wu * NL + il) * 1024u, (int)(t * SF_BC * kpitch) + goff[il]);
      dma_b128_to_lds(vrs, lds0 + (2 + buf) * SF_TILE + (unsigned)(wu * NL + il) * 1024u, (int)(t * SF_BC * kpitch) + goff[il]);
    }
  };
  const long long wave_first_q = a.q_off + q0, wave_last_q = wave_first_q + 31;
  bf16x2 ones;
  ones[0] = (bf16)1.0f; ones[1] = (bf16)1.0f;

  dma_tile(entry_at(0) & 0xfffff, 0);
  for (int j = 0; j < ntiles; j++) {               // j = walk position, kt = tile
    const int e = entry_at(j);
    const int kt = e & 0xfffff;
    const bool mine = ((e >> (20 + wu)) & 1) != 0;
    __builtin_amdgcn_s_waitcnt(0x0070);            // vmcnt(0), lgkmcnt(0): the tile landed, reads of the one before are done
    __builtin_amdgcn_s_barrier();
    if (j + 1 < ntiles) dma_tile(entry_at(j + 1) & 0xfffff, (j + 1) & 1);
    if (!mine) continue;                           // block flags hide the tile from this wavefront's rows
    const char* kl = smem + (j & 1) * SF_TILE;
    const char* vl = smem + (2 + (j & 1)) * SF_TILE;
    // S^T = K Q^T: register r of key block kb = key kt*64 + kb*32 + 8*(r/4) + 4h + r%4
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int r = 0; r < 16; r++) s[kb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < S_KS; ks++)
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
        s[kb] = mfma32(lds_read_b128(kl, kb * 32 * S_ROWB + kaddr[ks]), qf[ks], s[kb]);
    const long long tile_first_k = k_off + (long long)kt * SF_BC;
    const bool need_mask = (a.causal && tile_first_k + SF_BC - 1 > wave_first_q) ||
                           (a.window > 0 && tile_first_k < wave_last_q - a.window + 1) ||
                           ((kt + 1) * SF_BC > Nc);
    if (need_mask) {
      const long long dd = (a.q_off - k_off) + (q0 + lr) - ((long long)kt * SF_BC + 4 * h);
      const int tail = Nc - 1 - (kt * SF_BC + 4 * h);
      int lim = a.causal ? (int)(dd < -1 ? -1 : (dd > 64 ? 64 : dd)) : 64;
      lim = lim < tail ? lim : tail;
      const long long dl = dd - a.window + 1;
      const int lim_lo = a.window > 0 ? (int)(dl < -1 ? -1 : (dl > 64 ? 64 : dl)) : -1;
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int cpart = kb * 32 + 8 * (r >> 2) + (r & 3);
          if (!(cpart <= lim && cpart >= lim_lo)) s[kb][r] = BURST_NEG_INF;
        }
    }
    float v = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int r = 0; r < 16; r++) v = fmaxf(v, s[kb][r]);
    const float mx = max_both_halves(v) * a.c;
    if (__builtin_amdgcn_ballot_w64(mx > m2 + S_LAZY) != 0) {   // raise the reference max (rare after the first tiles)
      const float m_new = fmaxf(m2, mx);
      const float ref = (m_new == BURST_NEG_INF) ? 0.f : m_new;
      const float alpha = fast_exp2(m2 - ref);
      m2 = m_new;
      lsum *= alpha;
#pragma unroll
      for (int db = 0; db < S_DB; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) o[db][r] *= alpha;
    }
    const float nref = (m2 == BURST_NEG_INF) ? 0.f : -m2;
    bf16x8 pf[4];                                  // P^T fragments per 16-key group
#pragma unroll
    for (int kg = 0; kg < 4; kg++)
#pragma unroll
      for (int t = 0; t < 8; t += 2) {
        const int kb = kg >> 1, r = 8 * (kg & 1) + t;
        bf16x2 pk;
        pk[0] = (bf16)fast_exp2(__builtin_fmaf(s[kb][r], a.c, nref));
        pk[1] = (bf16)fast_exp2(__builtin_fmaf(s[kb][r + 1], a.c, nref));
        lsum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, lsum, false);   // sums what the MFMA multiplies
        pf[kg][t] = pk[0]; pf[kg][t + 1] = pk[1];
      }
    // O^T += V^T P^T
#pragma unroll
    for (int kg = 0; kg < 4; kg++)
#pragma unroll
      for (int db = 0; db < S_DB; db++) {
        const bf16x4 va = lds_read_tr(vl, kg * 16 * S_ROWB + taddr[db][0]);
        const bf16x4 vb = lds_read_tr(vl, kg * 16 * S_ROWB + taddr[db][1]);
        o[db] = mfma32(cat4(va, vb), pf[kg], o[db]);
      }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);

  // merge into the state (Alg. 1): lane (lr, h) holds row lr, columns db*32 + 8*q4 + 4h + (0..3)
  const int row = q0 + lr;
  const float l_chunk = sum_both_halves(lsum);
  if (row < a.Nq && m2 != BURST_NEG_INF) {
    const size_t srow = (size_t)head * a.Nq + row;
    const float m_old2 = a.m[srow] * kLog2e, l_old = a.l[srow];
    const float m_new = fmaxf(m_old2, m2);
    const float fa = fast_exp2(m_old2 - m_new), fb = fast_exp2(m2 - m_new);
    float* orow = a.O_acc + srow * S_D;
#pragma unroll
    for (int db = 0; db < S_DB; db++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        float* ptr = orow + db * 32 + 8 * q4 + 4 * h;
        f32x4 old = *reinterpret_cast<f32x4*>(ptr), nw;
#pragma unroll
        for (int b = 0; b < 4; b++) nw[b] = ((fa == 0.f) ? 0.f : old[b] * fa) + fb * o[db][4 * q4 + b];
        *reinterpret_cast<f32x4*>(ptr) = nw;
      }
    if (h == 0) {
      a.m[srow] = m_new * kLn2;
      a.l[srow] = ((fa == 0.f) ? 0.f : fa * l_old) + fb * l_chunk;
    }
  }
}

// ------------------------------------------------------------------------------- backward, dQ
constexpr int SQ_BR = 128;                        // query rows per workgroup
constexpr int SQ_BC = 32;                         // keys per tile
constexpr int SQ_TILE = SQ_BC * S_ROWB;

template <bool SPARSE>
__global__ void __launch_bounds__(256, 2)
burst_bwd_dq_d64_kernel(BwdArgs a) {
  __shared__ __attribute__((aligned(16))) char smem[4 * SQ_TILE];   // K[2], V[2]
  extern __shared__ int s_list[];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, lr = lane & 31, h = lane >> 5;
  int head, qb;
  s_head_block(blockIdx.x, a.blocks_per_head, head, qb);
  if (head >= a.H) return;
  if (a.causal) qb = a.blocks_per_head - 1 - qb;   // later blocks see more keys: the long ones start first
  const int q0 = qb * SQ_BR + w * 32;
  const int row = q0 + lr;
  const bool ok = row < a.Nq;
  const size_t srow = (size_t)head * a.Nq + (ok ? row : 0);
  const bf16* Kh = a.K + a.lay.kv_base(head / a.group);
  const bf16* Vh = a.V + a.lay.kv_base(head / a.group);
  const unsigned kpitch = (unsigned)a.lay.ks_r * 2u;             // bytes between key rows

  int Nc = a.Nc;
  long long k_off = a.k_off;
  bool nothing = false;
  int t_lo = 0;
  if (a.window > 0) {
    long long lo = a.q_off + (long long)qb * SQ_BR - a.window + 1 - a.k_off;
    if (lo >= a.Nc) nothing = true;
    else if (lo > 0) {
      const int skip = (int)(lo / SQ_BC) * SQ_BC;
      if constexpr (SPARSE) {
        t_lo = skip / SQ_BC;
      } else {
        Kh += (size_t)skip * a.lay.ks_r; Vh += (size_t)skip * a.lay.ks_r;
        Nc -= skip; k_off += skip;
      }
    }
  }
  int ntiles = nothing ? 0 : (Nc + SQ_BC - 1) / SQ_BC;
  if (a.causal) {
    long long lim = a.q_off + min(qb * SQ_BR + SQ_BR, a.Nq) - 1 - k_off;
    long long t = lim < 0 ? 0 : lim / SQ_BC + 1;
    if (t < ntiles) ntiles = (int)t;
  }

  if constexpr (SPARSE) {
    ntiles = s_build_list(s_list, w, lane, t_lo, ntiles, (Nc + SQ_BC - 1) / SQ_BC, [&](int t) {
      int bits = 0;
#pragma unroll
      for (int ww = 0; ww < 4; ww++) {
        const int row0 = qb * SQ_BR + ww * 32;
        if (row0 < a.Nq && (a.bmask + (size_t)head * a.bhstride)[(size_t)(row0 / a.bsize) * a.bpitch + (t * SQ_BC) / a.bsize] != 0) bits |= 1 << ww;
      }
      return bits;
    });
  }
  auto entry_at = [&](int j) __attribute__((always_inline)) {
    if constexpr (SPARSE) return __builtin_amdgcn_readfirstlane(s_list[1 + j]);
    else return j | (0xf << 20);
  };

  f32x16 dq[S_DB];
#pragma unroll
  for (int db = 0; db < S_DB; db++)
#pragma unroll
    for (int r = 0; r < 16; r++) dq[db][r] = 0.f;

  if (ntiles > 0) {                                // (uniform over the workgroup)
    bf16x8 qf[S_KS], gf[S_KS];
#pragma unroll
    for (int ks = 0; ks < S_KS; ks++) {
      const size_t qrow = a.lay.q_base(head) + (size_t)(ok ? row : 0) * a.lay.qs_r;
      qf[ks] = s_load8(a.Q + qrow + ks * 16 + h * 8, ok);
      gf[ks] = s_load8(a.dO + qrow + ks * 16 + h * 8, ok);
    }
    const float lv = ok ? a.lse[srow] : BURST_NEG_INF;
    const float nlse2 = (lv == BURST_NEG_INF) ? BURST_NEG_INF : -lv * kLog2e;   // -inf: P = 0
    const float Dv = ok ? a.D[srow] : 0.f;
    int kaddr[S_KS], taddr[S_DB][2];
#pragma unroll
    for (int ks = 0; ks < S_KS; ks++) kaddr[ks] = s_off(lr, 2 * ks + h);
    s_taddr(lane, taddr);
    const __amdgpu_buffer_rsrc_t krs = make_rsrc(Kh, s_span(Nc, kpitch));
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc(Vh, s_span(Nc, kpitch));
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const unsigned lds0 = lds_addr(smem);
    constexpr int NL = SQ_BC / S_RPL / 4;         // wave-wide loads per wavefront and tile
    int goff[NL];
#pragma unroll
    for (int il = 0; il < NL; il++) goff[il] = s_dma_off(w * NL + il, lane, kpitch);
    auto dma_tile = [&](int t, int buf) __attribute__((always_inline)) {
#pragma unroll
      for (int il = 0; il < NL; il++) {
        dma_b128_to_lds(krs, lds0 + buf * SQ_TILE + (unsigned)(wu * NL + il) * 1024u, (int)(t * SQ_BC * kpitch) + goff[il]);
        dma_b128_to_lds(vrs, lds0 + (2 + buf) * SQ_TILE + (unsigned)(wu * NL + il) * 1024u, (int)(t * SQ_BC * kpitch) + goff[il]);
      }
    };
    const long long wave_first_q = a.q_off + q0;

    dma_tile(entry_at(0) & 0xfffff, 0);
    for (int j = 0; j < ntiles; j++) {             // j = walk position, kt = tile
      const int e = entry_at(j);
      const int kt = e & 0xfffff;
      const bool mine = ((e >> (20 + wu)) & 1) != 0;
      __builtin_amdgcn_s_waitcnt(0x0070);
      __builtin_amdgcn_s_barrier();
      if (j + 1 < ntiles) dma_tile(entry_at(j + 1) & 0xfffff, (j + 1) & 1);
      if (!mine) continue;                         // block flags hide the tile from this wavefront's rows
      const char* kl = smem + (j & 1) * SQ_TILE;
      const char* vl = smem + (2 + (j & 1)) * SQ_TILE;
      // S^T = K Q^T, dP^T = V dO^T: register r = key kt*32 + 8*(r/4) + 4h + r%4
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < S_KS; ks++) {
        s = mfma32(lds_read_b128(kl, kaddr[ks]), qf[ks], s);
        dp = mfma32(lds_read_b128(vl, kaddr[ks]), gf[ks], dp);
      }
      const long long tile_first_k = k_off + (long long)kt * SQ_BC;
      const bool need_mask = (a.causal && tile_first_k + SQ_BC - 1 > wave_first_q) ||
                             (a.window > 0 && tile_first_k < wave_first_q + 31 - a.window + 1) ||
                             ((kt + 1) * SQ_BC > Nc);
      if (need_mask) {
        const long long dd = (a.q_off - k_off) + (q0 + lr) - ((long long)kt * SQ_BC + 4 * h);
        const int tail = Nc - 1 - (kt * SQ_BC + 4 * h);
        int lim = a.causal ? (int)(dd < -1 ? -1 : (dd > 64 ? 64 : dd)) : 64;
        lim = lim < tail ? lim : tail;
        const long long dl = dd - a.window + 1;
        const int lim_lo = a.window > 0 ? (int)(dl < -1 ? -1 : (dl > 64 ? 64 : dl)) : -1;
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int cpart = 8 * (r >> 2) + (r & 3);
          if (!(cpart <= lim && cpart >= lim_lo)) s[r] = BURST_NEG_INF;
        }
      }
      bf16x8 dsf[2];                               // dS^T fragments per 16-key group
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const float p = fast_exp2(__builtin_fmaf(s[r], a.c, nlse2));
        dsf[r >> 3][r & 7] = (bf16)(p * (dp[r] - Dv));
      }
      // dQ^T += K^T dS^T
#pragma unroll
      for (int kg = 0; kg < 2; kg++)
#pragma unroll
        for (int db = 0; db < S_DB; db++) {
          const bf16x4 ta = lds_read_tr(kl, kg * 16 * S_ROWB + taddr[db][0]);
          const bf16x4 tb = lds_read_tr(kl, kg * 16 * S_ROWB + taddr[db][1]);
          dq[db] = mfma32(cat4(ta, tb), dsf[kg], dq[db]);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  if (ok) {
    float* orow = a.dQ + srow * S_D;
#pragma unroll
    for (int db = 0; db < S_DB; db++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        float* ptr = orow + db * 32 + 8 * q4 + 4 * h;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (a.acc_dq) v = *reinterpret_cast<f32x4*>(ptr);
#pragma unroll
        for (int b = 0; b < 4; b++) v[b] += a.scale * dq[db][4 * q4 + b];
        *reinterpret_cast<f32x4*>(ptr) = v;
      }
  }
}

// ------------------------------------------------------------------------------- backward, dK / dV
// Wavefronts per dK/dV workgroup, 32 keys each.  Four by default.  With two (BURST_SMALL_DKV_WAVES
// = 2: the d = 128 build) a workgroup owns 64 keys, the finest block edge a call's flags can have,
// so its list of visible tiles is exactly the tiles those 64 keys are needed for, and two such
// workgroups share a CU at one wavefront per SIMD (the kernel needs more than 256 registers at
// d = 128).
#ifndef BURST_SMALL_DKV_WAVES
#define BURST_SMALL_DKV_WAVES 4
#endif
constexpr int SK_WAVES = BURST_SMALL_DKV_WAVES;
constexpr int SK_BC = 32 * SK_WAVES;              // keys per workgroup
constexpr int SK_BR = 32;                         // query rows per tile
constexpr int SK_TILE = SK_BR * S_ROWB;
constexpr int SK_STAT = 4 * SK_TILE;              // per buffer: 32 x (-lse log2 e), 32 x D

template <bool SPARSE>
__global__ void __launch_bounds__(64 * SK_WAVES, SK_WAVES == 4 ? 2 : 1)   // (second figure: wavefronts per SIMD)
burst_bwd_dkv_d64_kernel(BwdArgs a) {
  __shared__ __attribute__((aligned(16))) char smem[4 * SK_TILE + 2 * 64 * 4];   // Q[2], dO[2], statistics[2]
  extern __shared__ int s_list[];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, lr = lane & 31, h = lane >> 5;
  int kvhead, kblk;
  s_head_block(blockIdx.x, a.blocks_per_head, kvhead, kblk);
  if (kvhead >= a.H) return;                       // a.H counts key/value heads here
  const int key_wg = kblk * SK_BC, key0 = key_wg + w * 32;
  const bf16* Kh = a.K + a.lay.kv_base(kvhead);
  const bf16* Vh = a.V + a.lay.kv_base(kvhead);
  const unsigned qpitch = (unsigned)a.lay.qs_r * 2u;             // bytes between query rows

  // query tiles of one head to visit (causal: rows before the first key see nothing; window:
  // rows too far behind the last key neither), then the same range for every head of the group
  int t_end = (a.Nq + SK_BR - 1) / SK_BR, t_begin = 0;
  if (a.causal) {
    long long first_row = a.k_off + key_wg - a.q_off;
    if (first_row > 0) t_begin = (int)min((long long)t_end, first_row / SK_BR);
  }
  if (a.window > 0) {
    long long last_row = a.k_off + min(key_wg + SK_BC, a.Nc) - 1 + a.window - 1 - a.q_off;
    t_end = last_row < 0 ? 0 : (int)min((long long)t_end, last_row / SK_BR + 1);
  }
  const int per_head = t_end > t_begin ? t_end - t_begin : 0;
  int nwalk = per_head * a.group;
  if constexpr (SPARSE) {                          // entries count tiles over all heads of the group
    nwalk = s_build_list(s_list, w, lane, 0, nwalk, 0, [&](int n) {
      const int g = n / (per_head > 0 ? per_head : 1);
      const int t = t_begin + n % (per_head > 0 ? per_head : 1);
      const uint8_t* mrow = a.bmask + (size_t)(kvhead * a.group + g) * a.bhstride + (size_t)((t * SK_BR) / a.bsize) * a.bpitch;
      int bits = 0;
#pragma unroll
      for (int ww = 0; ww < SK_WAVES; ww++) {
        const int k0 = key_wg + ww * 32;
        if (k0 < a.Nc && mrow[k0 / a.bsize] != 0) bits |= 1 << ww;
      }
      return bits;
    });
  }
  // walk position -> (query head of the group, tile, this wavefront's bit)
  auto locate = [&](int j, int& g, int& t) __attribute__((always_inline)) {
    int n = j, bits = 0xf;
    if constexpr (SPARSE) {
      const int e = __builtin_amdgcn_readfirstlane(s_list[1 + j]);
      n = e & 0xfffff; bits = e >> 20;
    }
    if (a.group == 1) {                            // (no division in the common case: a scalar divide is some forty instructions)
      g = 0;
      t = t_begin + n;
    } else {
      g = n / per_head;
      t = t_begin + (n - g * per_head);
    }
    return bits;
  };

  f32x16 dk[S_DB], dv[S_DB];
#pragma unroll
  for (int db = 0; db < S_DB; db++)
#pragma unroll
    for (int r = 0; r < 16; r++) { dk[db][r] = 0.f; dv[db][r] = 0.f; }

  if (nwalk > 0) {
    bf16x8 kf[S_KS], vf[S_KS];
#pragma unroll
    for (int ks = 0; ks < S_KS; ks++) {
      kf[ks] = s_load8(Kh + (size_t)(key0 + lr) * a.lay.ks_r + ks * 16 + h * 8, key0 + lr < a.Nc);
      vf[ks] = s_load8(Vh + (size_t)(key0 + lr) * a.lay.ks_r + ks * 16 + h * 8, key0 + lr < a.Nc);
    }
    int qaddr[S_KS], taddr[S_DB][2];
#pragma unroll
    for (int ks = 0; ks < S_KS; ks++) qaddr[ks] = s_off(lr, 2 * ks + h);
    s_taddr(lane, taddr);
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const unsigned lds0 = lds_addr(smem);
    constexpr int NL = SK_BR / S_RPL / SK_WAVES;  // wave-wide loads per wavefront and tile
    static_assert(NL >= 1 && NL * SK_WAVES * S_RPL == SK_BR, "a tile's rows must divide evenly among the wavefronts");
    int goff[NL];
#pragma unroll
    for (int il = 0; il < NL; il++) goff[il] = s_dma_off(w * NL + il, lane, qpitch);
    float* const stat = reinterpret_cast<float*>(smem + SK_STAT);
    // walk position n -> (query head, tile); every wavefront DMAs its 8 rows of Q and dO.  The
    // first wavefront also fetches the 32 rows' statistics with plain loads issued BEFORE the
    // DMA (the wait the compiler places before their first use then does not cover the DMA) and
    // writes them to LDS at the end of the step (stat_commit).
    float stat_x = 0.f;
    auto fetch = [&](int n, int buf) __attribute__((always_inline)) {
      int g, t;
      locate(n, g, t);
      const size_t hrow = (size_t)(kvhead * a.group + g) * a.Nq;
      if (tid < 64) {
        const int r = t * SK_BR + (tid & 31);
        if (tid < 32) stat_x = r < a.Nq ? a.lse[hrow + r] : BURST_NEG_INF;
        else stat_x = r < a.Nq ? a.D[hrow + r] : 0.f;
      }
      const size_t hbase = a.lay.q_base(kvhead * a.group + g);
      const __amdgpu_buffer_rsrc_t qrs = make_rsrc(a.Q + hbase, s_span(a.Nq, qpitch));
      const __amdgpu_buffer_rsrc_t grs = make_rsrc(a.dO + hbase, s_span(a.Nq, qpitch));
#pragma unroll
      for (int il = 0; il < NL; il++) {
        dma_b128_to_lds(qrs, lds0 + buf * SK_TILE + (unsigned)(wu * NL + il) * 1024u, (int)(t * SK_BR * qpitch) + goff[il]);
        dma_b128_to_lds(grs, lds0 + (2 + buf) * SK_TILE + (unsigned)(wu * NL + il) * 1024u, (int)(t * SK_BR * qpitch) + goff[il]);
      }
    };
    auto stat_commit = [&](int buf) __attribute__((always_inline)) {
      if (tid < 32) stat[buf * 64 + tid] = (stat_x == BURST_NEG_INF) ? BURST_NEG_INF : -stat_x * kLog2e;   // -inf: P = 0
      else if (tid < 64) stat[buf * 64 + tid] = stat_x;
    };
    const long long wave_first_k = a.k_off + key0, wave_last_k = wave_first_k + 31;
    const long long kpos = wave_first_k + lr;

    fetch(0, 0);
    stat_commit(0);
    for (int n = 0; n < nwalk; n++) {
      __builtin_amdgcn_s_waitcnt(0x0070);
      __builtin_amdgcn_s_barrier();
      if (n + 1 < nwalk) fetch(n + 1, (n + 1) & 1);
      const int buf = n & 1;
      const char* ql = smem + buf * SK_TILE;
      const char* gl = smem + (2 + buf) * SK_TILE;
      int g_unused, t;
      const bool mine = ((locate(n, g_unused, t) >> wu) & 1) != 0;
      if (mine) {                                  // (else: block flags hide this wavefront's keys from the tile)
        // S = Q K^T, dP = dO V^T: lane = key lr, register r = row t*32 + 8*(r/4) + 4h + r%4
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
        if constexpr (SK_WAVES == 2) {
          // One wavefront per SIMD: nobody else hides an LDS read's latency, and left alone the
          // compiler reads one fragment, waits, multiplies, sixteen times over.  All sixteen
          // fragments are requested first (the registers are there), then the MFMAs run.
          bf16x8 qa[S_KS], ga[S_KS];
#pragma unroll
          for (int ks = 0; ks < S_KS; ks++) { qa[ks] = lds_read_b128(ql, qaddr[ks]); ga[ks] = lds_read_b128(gl, qaddr[ks]); }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int ks = 0; ks < S_KS; ks++) { s = mfma32(qa[ks], kf[ks], s); dp = mfma32(ga[ks], vf[ks], dp); }
        } else {
#pragma unroll
          for (int ks = 0; ks < S_KS; ks++) {
            s = mfma32(lds_read_b128(ql, qaddr[ks]), kf[ks], s);
            dp = mfma32(lds_read_b128(gl, qaddr[ks]), vf[ks], dp);
          }
        }
        const long long tile_first_q = a.q_off + (long long)t * SK_BR;
        const bool need_mask = (a.causal && wave_last_k > tile_first_q) ||
                               (a.window > 0 && tile_first_q + SK_BR - 1 >= wave_first_k + a.window);
        if (need_mask) {
          // visible iff key position <= row position (constant part >= lim) and row position <
          // key position + window (constant part <= lim2)
          const long long d = kpos - (tile_first_q + 4 * h);
          const int lim = a.causal ? (int)(d < -1 ? -1 : (d > 64 ? 64 : d)) : -1;
          const long long d2 = d + a.window - 1;
          const int lim2 = a.window > 0 ? (int)(d2 < -1 ? -1 : (d2 > 64 ? 64 : d2)) : 64;
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int cpart = 8 * (r >> 2) + (r & 3);
            if (!(cpart >= lim && cpart <= lim2)) s[r] = BURST_NEG_INF;
          }
        }
        // (two wavefronts per workgroup: the transposed dO and Q fragments of the last phase are
        // requested here, so that they arrive while the exponentials run)
        bf16x4 tg[2][S_DB][2], tq[2][S_DB][2];
        if constexpr (SK_WAVES == 2) {
#pragma unroll
          for (int u = 0; u < 2; u++)
#pragma unroll
            for (int db = 0; db < S_DB; db++)
#pragma unroll
              for (int sx = 0; sx < 2; sx++) {
                tg[u][db][sx] = lds_read_tr(gl, u * 16 * S_ROWB + taddr[db][sx]);
                tq[u][db][sx] = lds_read_tr(ql, u * 16 * S_ROWB + taddr[db][sx]);
              }
          __builtin_amdgcn_sched_barrier(0);
        }
        bf16x8 pf[2], dsf[2];                        // per 16-row group: A operands of dV, dK
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          const f32x4 nl = *reinterpret_cast<const f32x4*>(stat + buf * 64 + 8 * q4 + 4 * h);
          const f32x4 dr = *reinterpret_cast<const f32x4*>(stat + buf * 64 + 32 + 8 * q4 + 4 * h);
#pragma unroll
          for (int j = 0; j < 4; j++) {
            const int r = 4 * q4 + j;
            const float p = fast_exp2(__builtin_fmaf(s[r], a.c, nl[j]));
            pf[r >> 3][r & 7] = (bf16)p;
            dsf[r >> 3][r & 7] = (bf16)(p * (dp[r] - dr[j]));
          }
        }
        // dV += P^T dO, dK += dS^T Q (dO and Q through transposing reads)
#pragma unroll
        for (int u = 0; u < 2; u++)
#pragma unroll
          for (int db = 0; db < S_DB; db++) {
            bf16x8 bg, bq;
            if constexpr (SK_WAVES == 2) {
              bg = cat4(tg[u][db][0], tg[u][db][1]);
              bq = cat4(tq[u][db][0], tq[u][db][1]);
            } else {
              bg = cat4(lds_read_tr(gl, u * 16 * S_ROWB + taddr[db][0]), lds_read_tr(gl, u * 16 * S_ROWB + taddr[db][1]));
              bq = cat4(lds_read_tr(ql, u * 16 * S_ROWB + taddr[db][0]), lds_read_tr(ql, u * 16 * S_ROWB + taddr[db][1]));
            }
            dv[db] = mfma32(pf[u], bg, dv[db]);
            dk[db] = mfma32(dsf[u], bq, dk[db]);
          }
      }
      if (n + 1 < nwalk) stat_commit((n + 1) & 1);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  // lane = d column, registers = keys
  float* dKh = a.dK + (size_t)kvhead * a.Nc * S_D;
  float* dVh = a.dV + (size_t)kvhead * a.Nc * S_D;
#pragma unroll
  for (int r = 0; r < 16; r++) {
    const int key = key0 + 8 * (r >> 2) + 4 * h + (r & 3);
    if (key < a.Nc) {
#pragma unroll
      for (int db = 0; db < S_DB; db++) {
        const size_t off = (size_t)key * S_D + db * 32 + lr;
        float k_old = 0.f, v_old = 0.f;
        if (a.acc_dkv) { k_old = dKh[off]; v_old = dVh[off]; }
        dKh[off] = k_old + a.scale * dk[db][r];
        dVh[off] = v_old + dv[db][r];
      }
    }
  }
}



// ------------------------------------------------------------------------------- launchers
// Tile lists are dynamic LDS behind up to 64 KB of static tiles: the kernels that take one opt
// in to the larger total once per device.
template <typename K>
static int allow_list(K kernel, DeviceOnce& once) {
  return once.run([kernel] {
    return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (S_MAX_LIST + 4) * 4) ==
                   hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
  });
}

int launch_fwd(const KParams& p, const void* Q, const void* K, const void* V,
                   float* O_acc, float* m, float* l, hipStream_t stream) {
  FwdArgsLite a;
  a.Q = (const bf16*)Q; a.K = (const bf16*)K; a.V = (const bf16*)V;
  a.O_acc = O_acc; a.m = m; a.l = l;
  a.Nq = p.Nq; a.Nc = p.Nc; a.H = p.B * p.H; a.group = p.group;
  a.causal = p.causal; a.c = p.scale * kLog2e;
  a.q_off = p.q_off; a.k_off = p.k_off; a.window = p.window;
  a.bmask = p.bmask; a.bsize = p.bsize; a.bpitch = p.bpitch; a.bhstride = p.bhstride;
  a.lay = p.lay;
  a.blocks_per_head = (p.Nq + SF_BR - 1) / SF_BR;
  const long long nb = (long long)((a.H + 7) / 8 * 8) * a.blocks_per_head;
  if (nb > 0x7fffffffLL) return BURST_ERR_SHAPE;
  if (a.bmask != nullptr) {
    const int entries = (p.Nc + SF_BC - 1) / SF_BC;
    if (entries > S_MAX_LIST) return BURST_ERR_SHAPE;
    static DeviceOnce done;
    if (int st = allow_list(burst_fwd_d64_kernel<true>, done); st != BURST_OK) return st;
    BURST_LAUNCH(burst_fwd_d64_kernel<true>, dim3((unsigned)nb), dim3(256), (entries + 4) * 4, stream, a);
  } else {
    BURST_LAUNCH(burst_fwd_d64_kernel<false>, dim3((unsigned)nb), dim3(256), 0, stream, a);
  }
  return launch_status();
}

int launch_bwd_dq(const KParams& p, const void* Q, const void* K, const void* V,
                      const void* dO, const float* lse, const float* D, float* dQ, int acc_dq,
                      hipStream_t stream) {
  if (p.Nq <= 0) return BURST_OK;
  BwdArgs a = make_bwd_args(p, Q, K, V, dO, lse, D, dQ, nullptr, nullptr, acc_dq, 0);
  a.blocks_per_head = (p.Nq + SQ_BR - 1) / SQ_BR;
  const long long nb = (long long)((a.H + 7) / 8 * 8) * a.blocks_per_head;
  if (nb > 0x7fffffffLL) return BURST_ERR_SHAPE;
  if (a.bmask != nullptr) {
    const int entries = (p.Nc + SQ_BC - 1) / SQ_BC;
    if (entries > S_MAX_LIST) return BURST_ERR_SHAPE;
    static DeviceOnce done;
    if (int st = allow_list(burst_bwd_dq_d64_kernel<true>, done); st != BURST_OK) return st;
    BURST_LAUNCH(burst_bwd_dq_d64_kernel<true>, dim3((unsigned)nb), dim3(256), (entries + 4) * 4, stream, a);
  } else {
    BURST_LAUNCH(burst_bwd_dq_d64_kernel<false>, dim3((unsigned)nb), dim3(256), 0, stream, a);
  }
  return launch_status();
}

int launch_bwd_dkv(const KParams& p, const void* Q, const void* K, const void* V,
                       const void* dO, const float* lse, const float* D, float* dK, float* dV,
                       int acc_dkv, hipStream_t stream) {
  if (p.Nc <= 0) return BURST_OK;
  BwdArgs a = make_bwd_args(p, Q, K, V, dO, lse, D, nullptr, dK, dV, 0, acc_dkv);
  a.H = p.B * p.H / p.group;                       // workgroups are laid out over key/value heads
  a.blocks_per_head = (p.Nc + SK_BC - 1) / SK_BC;
  const long long nb = (long long)((a.H + 7) / 8 * 8) * a.blocks_per_head;
  if (nb > 0x7fffffffLL) return BURST_ERR_SHAPE;
  if (a.bmask != nullptr) {
    const long long entries = (long long)p.group * ((p.Nq + SK_BR - 1) / SK_BR);
    if (entries > S_MAX_LIST) return BURST_ERR_SHAPE;
    static DeviceOnce done;
    if (int st = allow_list(burst_bwd_dkv_d64_kernel<true>, done); st != BURST_OK) return st;
    BURST_LAUNCH(burst_bwd_dkv_d64_kernel<true>, dim3((unsigned)nb), dim3(64 * SK_WAVES), ((int)entries + 4) * 4, stream, a);
  } else {
    BURST_LAUNCH(burst_bwd_dkv_d64_kernel<false>, dim3((unsigned)nb), dim3(64 * SK_WAVES), 0, stream, a);
  }
  return launch_status();
}

}  // namespace BURST_SMALL_NS
}  // namespace burst
