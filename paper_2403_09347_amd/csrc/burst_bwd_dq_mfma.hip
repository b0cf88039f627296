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
// rows (their Q fragments stay in VGPRs and their dO fragments in AGPRs as B operands for the
// whole kernel) and walks the chunk in tiles of 32 keys.  With S^T = K Q^T every lane owns one
// query row, so lse and D are per-lane scalars, and the dS^T accumulators already have the B-operand layout that
// dQ^T += K^T dS^T needs (K^T comes through transposing LDS reads).  dQ^T accumulators are
// pinned in AGPRs; K/V tiles are DMA-ed from HBM into LDS rings three tiles ahead, one barrier
// per tile.  The 48 MFMAs of a tile run in three phases of 16, each carrying the vector work of
// a neighbouring phase so that no phase waits for it:
//   1: S^T of tile t          2: dP^T of tile t + exp2 of tile t (P^T replaces S^T in place)
//   3: dQ^T products of tile t-1 (its dS^T fragments were finished a step ago) + dS^T of tile t
// Only the 16-register dS^T fragment sets exist twice; everything fits the register file
// without shuttling accumulators through AGPRs.
#include "burst_bwd_common.h"

namespace burst {

constexpr int DQ_BR = 256;            // query rows per workgroup (4 wavefronts x 64)
constexpr int DQ_BC = 32;             // keys per tile
constexpr int DQ_TILE_BYTES = DQ_BC * 256;
constexpr int DQ_KSLOTS = 5;          // K of tiles t-1 (dQ), t (S), t+1, t+2 (landed), t+3 (in flight)
constexpr int DQ_VSLOTS = 4;          // V of tiles t (dP), t+1, t+2, t+3
constexpr int DQ_LDS_BYTES = (DQ_KSLOTS + DQ_VSLOTS) * DQ_TILE_BYTES;
constexpr int DQ_MAX_LIST = 16384;    // block-sparse calls: most key tiles of one chunk (512K keys)
constexpr int DQ_LIST_BYTES = (DQ_MAX_LIST + 8) * 4;

// dP^T MFMA: accumulator in VGPRs (the vector unit reads it next), B operand (a dO fragment of
// the wavefront's own rows, resident for the whole kernel) in AGPRs, which this kernel otherwise
// leaves half empty.  As inline assembly the instruction is invisible to the compiler's hazard
// recognizer: the leading s_nop covers register copies the compiler may place right before (a
// vector write must not be read by an MFMA within two cycles), the caller separates the last one
// from the first vector read of the accumulator (mfma_vgpr_fence) and never issues two in a row
// on the same accumulator.
// The resident operand is declared read-write although the instruction only reads it: its value
// then lives in AGPRs from one statement to the next, like the pinned accumulators; as a plain
// input the compiler keeps its home in VGPRs and copies it over before every use.
// First k-step: the accumulator starts at `start` (16 registers holding -D of the lane's row).
__device__ __forceinline__ void mfma32_dp_first(f32x16& acc, bf16x8 a, bf16x8& b_resident, const f32x16& start) {
  asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %2, %1, %3"
               : "=&v"(acc), "+a"(b_resident) : "v"(a), "v"(start));   // early clobber: the result must not share registers with an operand
}
__device__ __forceinline__ void mfma32_dp(f32x16& acc, bf16x8 a, bf16x8& b_resident) {
  asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %2, %1, %0" : "+v"(acc), "+a"(b_resident) : "v"(a));
}
// The same MFMAs with the slice's own vector work inside the same asm statement: two independent
// vector instructions in front (whatever register copies the compiler puts before the statement
// are then at least two instructions away from the MFMA, and no s_nop is needed), the rest behind.
// Nothing the compiler can see consumes a result right after the statement, so it adds no wait
// state of its own either (after an asm statement it cannot look into it assumes the worst: a
// transcendental result, one wait state before its first use).
// x0 <- exp2(x0 * c + n), x1 <- exp2(x1 * c + n) in place (two scores become two probabilities), with
// the dP^T MFMA between the multiply-adds and the exponentials.  The exponentials' results are
// first read a phase later.
__device__ __forceinline__ void exp2_mfma32_dp(f32x16& acc, bf16x8 a, bf16x8& b_resident, float& x0, float& x1,
                                               float c, float n) {
  asm volatile("v_fma_f32 %2, %2, %5, %6\n\tv_fma_f32 %3, %3, %5, %6\n\tv_mfma_f32_32x32x16_bf16 %0, %4, %1, %0\n\t"
               "v_exp_f32 %2, %2\n\tv_exp_f32 %3, %3"
               : "+v"(acc), "+a"(b_resident), "+v"(x0), "+v"(x1) : "v"(a), "s"(c), "v"(n));
}
__device__ __forceinline__ void exp2_mfma32_dp_first(f32x16& acc, bf16x8 a, bf16x8& b_resident, const f32x16& start,
                                                     float& x0, float& x1, float c, float n) {
  asm volatile("v_fma_f32 %2, %2, %6, %7\n\tv_fma_f32 %3, %3, %6, %7\n\tv_mfma_f32_32x32x16_bf16 %0, %4, %1, %5\n\t"
               "v_exp_f32 %2, %2\n\tv_exp_f32 %3, %3"
               : "=&v"(acc), "+a"(b_resident), "+v"(x0), "+v"(x1) : "v"(a), "v"(start), "s"(c), "v"(n));
}
// ds = pack_bf16(p0 * q0, p1 * q1) (two dS values), with a dQ^T MFMA on an AGPR accumulator between
// the products and the conversion.
__device__ __forceinline__ void ds2_mfma32_acc(f32x16& acc, bf16x8 a, bf16x8 b, unsigned& ds,
                                               float p0, float q0, float p1, float q1) {
  float tmp;
  asm volatile("v_mul_f32 %1, %5, %6\n\tv_mul_f32 %2, %7, %8\n\tv_mfma_f32_32x32x16_bf16 %0, %3, %4, %0\n\t"
               "v_cvt_pk_bf16_f32 %1, %1, %2"
               : "+a"(acc), "=&v"(ds), "=&v"(tmp) : "v"(a), "v"(b), "v"(p0), "v"(q0), "v"(p1), "v"(q1));
}
__device__ __forceinline__ void mfma_vgpr_fence(f32x16 (&acc)[2]) {
  asm volatile("s_nop 15\n\ts_nop 3" : "+v"(acc[0]), "+v"(acc[1]));
}

// MODE 0 compiles the sliding-window code away: this kernel uses every register of the file, and
// the few values the window logic keeps alive would otherwise push others to scratch.  MODE 1
// has it.  MODE 2 (the call carries block flags, paper Sec. 2.6) has it too and walks a list of
// the key tiles that at least one wavefront of the workgroup can see, built in LDS at the start
// (tile index plus one bit per wavefront); a wavefront whose bit is clear hides the whole tile
// in the masking path.  Entries past the end name a tile beyond the chunk: its DMA reads zeros
// and the ragged-tail mask hides it.
template <int MODE>
__global__ void __launch_bounds__(256, 1)
burst_bwd_dq_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr bool WINDOW = MODE != 0, SPARSE = MODE == 2;
  const long long window = WINDOW ? a.window : 0;
  const int tid = threadIdx.x;
  const int w = tid >> 6, lane = tid & 63, lr = lane & 31, h = lane >> 5;
  int head, qb;
  {
    int bid = blockIdx.x;
    int xcd = bid & 7, idx = bid >> 3;
    int hx = idx / a.blocks_per_head;
    qb = idx - hx * a.blocks_per_head;
    if (a.causal) qb = a.blocks_per_head - 1 - qb;   // longest blocks of a head first (see the forward kernel)
    head = hx * 8 + xcd;
    if (head >= a.H) return;
  }
  const int q0 = qb * DQ_BR + w * 64;
  const bf16* Qh = a.Q + a.lay.q_base(head);
  const bf16* Gh = a.dO + a.lay.q_base(head);
  const bf16* Kh = a.K + a.lay.kv_base(head / a.group);
  const bf16* Vh = a.V + a.lay.kv_base(head / a.group);
  const unsigned kpitch = (unsigned)a.lay.ks_r * 2u;             // bytes between key rows
  const unsigned ktile = kpitch * DQ_BC;                         // ... between key tiles
  const float* lseh = a.lse + (size_t)head * a.Nq;
  const float* Dh = a.D + (size_t)head * a.Nq;
  float* dQh = a.dQ + (size_t)head * a.Nq * 128;

  // Sliding window: key tiles before the first one that the workgroup's first row can see are
  // skipped by moving the start of the chunk (pointers, length, global offset) forward by whole
  // tiles; everything below works on that shortened chunk.
  int Nc = a.Nc;
  long long k_off = a.k_off;
  int t_lo = 0;                                    // SPARSE: first tile of the list (the chunk is not shifted)
  bool nothing = false;
  if (window > 0) {
    long long lo = a.q_off + (long long)qb * DQ_BR - window + 1 - a.k_off;   // first visible key index
    if (lo >= a.Nc) nothing = true;                // nothing visible: contribution 0
    else if (lo > 0) {
      const int skip = (int)(lo / DQ_BC) * DQ_BC;
      if constexpr (SPARSE) {
        t_lo = skip / DQ_BC;
      } else {
        Kh += (size_t)skip * a.lay.ks_r; Vh += (size_t)skip * a.lay.ks_r;
        Nc -= skip; k_off += skip;
      }
    }
  }
  int ntiles = nothing ? 0 : (Nc + DQ_BC - 1) / DQ_BC;
  if (a.causal) {
    long long lim = a.q_off + min(qb * DQ_BR + DQ_BR, a.Nq) - 1 - k_off;
    long long t = lim < 0 ? 0 : lim / DQ_BC + 1;
    if (t < ntiles) ntiles = (int)t;
  }
  // SPARSE: the list of visible tiles, built by wavefront 0 (64 candidate tiles per round).
  // list[0] = number of entries, list[1 + j] = tile | (wavefront bits << 20), then 6 end entries.
  int* const list = reinterpret_cast<int*>(smem + DQ_LDS_BYTES);
  if constexpr (SPARSE) {
    const int end_tile = (Nc + DQ_BC - 1) / DQ_BC;               // a tile past the chunk
    if (w == 0) {
      const uint8_t* const bm = a.bmask + (size_t)head * a.bhstride;
      int n = 0;
      for (int base = t_lo; base < ntiles; base += 64) {
        const int kt = base + lane;
        int bits = 0;
        if (kt < ntiles) {
          const int col = (kt * DQ_BC) / a.bsize;
#pragma unroll
          for (int ww = 0; ww < 4; ww++) {
            const int row0 = qb * DQ_BR + ww * 64;
            if (row0 < a.Nq && bm[(size_t)(row0 / a.bsize) * a.bpitch + col] != 0) bits |= 1 << ww;
          }
        }
        const unsigned long long bal = __builtin_amdgcn_ballot_w64(bits != 0);
        if (bits != 0) {
          const int pos = n + __builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0u));
          list[1 + pos] = kt | (bits << 20);
        }
        n += __builtin_popcountll(bal);
      }
      if (lane < 6) list[1 + n + lane] = end_tile;
      if (lane == 0) list[0] = n;
    }
    __syncthreads();
    ntiles = __builtin_amdgcn_readfirstlane(list[0]);            // from here on: number of list entries
  }
  auto tile_at = [&](int j) __attribute__((always_inline)) {      // tile index of list entry j
    if constexpr (SPARSE) return __builtin_amdgcn_readfirstlane(list[1 + j]) & 0xfffff;
    else return j;
  };

  f32x16 dq[2][4];         // dQ^T accumulators [row block][32-wide d block], pinned in AGPRs
#pragma unroll
  for (int rb = 0; rb < 2; rb++)
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int r = 0; r < 16; r++) dq[rb][db][r] = 0.f;

  if (ntiles > 0) {
    bf16x8 qf[2][8];       // Q fragments of the wavefront's rows (B operand of S^T), VGPRs
    bf16x8 gfr[2][8];      // dO fragments of the same rows (B operand of dP^T), AGPRs
    float nlse2[2];
    f32x16 negD[2];        // -D of the lane's row in all 16 registers: start value of the dP^T accumulators,
                           // so that dS^T = P^T o (dP^T - D) needs no subtraction per score
#pragma unroll
    for (int rb = 0; rb < 2; rb++) {
      int row = q0 + rb * 32 + lr;
      bool ok = row < a.Nq;
      float lv = ok ? lseh[row] : BURST_NEG_INF;
      nlse2[rb] = (lv == BURST_NEG_INF) ? BURST_NEG_INF : -lv * kLog2e;   // -inf => P = exp2(-inf) = 0
      {
        const float nd = ok ? -Dh[row] : 0.f;
#pragma unroll
        for (int r = 0; r < 16; r++) negD[rb][r] = nd;
      }
#pragma unroll
      for (int ks = 0; ks < 8; ks++) {
        bf16x8 z;
#pragma unroll
        for (int t = 0; t < 8; t++) z[t] = (bf16)0.0f;
        qf[rb][ks] = ok ? *reinterpret_cast<const bf16x8*>(Qh + (size_t)row * a.lay.qs_r + ks * 16 + h * 8) : z;
        gfr[rb][ks] = ok ? *reinterpret_cast<const bf16x8*>(Gh + (size_t)row * a.lay.qs_r + ks * 16 + h * 8) : z;
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
    const unsigned kbytes = Nc > 0 ? (unsigned)(Nc - 1) * kpitch + 256u : 0u;   // up to the end of the last row
    const __amdgpu_buffer_rsrc_t krs = make_rsrc(Kh, kbytes);
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc(Vh, kbytes);
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const unsigned lds0 = lds_addr(smem);
    int goff[2];
#pragma unroll
    for (int il = 0; il < 2; il++) {
      int row = 8 * w + 4 * il + (lane >> 4);
      goff[il] = (int)(row * kpitch + (((lane & 15) ^ row_code(row)) << 4));
    }
    auto dma_tile = [&](__amdgpu_buffer_rsrc_t rs, unsigned lds_tile, int il, int tile) __attribute__((always_inline)) {
      dma_b128_to_lds(rs, lds_tile + (unsigned)(wu * 2 + il) * 1024u, (int)(tile * ktile) + goff[il]);
    };
    constexpr int VBASE = DQ_KSLOTS * DQ_TILE_BYTES;
#pragma unroll
    for (int t = 0; t < 3; t++) {
      const int src = tile_at(t);
#pragma unroll
      for (int il = 0; il < 2; il++) {
        dma_tile(krs, lds0 + t * DQ_TILE_BYTES, il, src);
        dma_tile(vrs, lds0 + VBASE + t * DQ_TILE_BYTES, il, src);
      }
    }
    {
      // the slot of "tile -1" feeds the first, all-zero dQ^T products: clear it
      const i32x4 z = {0, 0, 0, 0};
      *reinterpret_cast<i32x4*>(smem + (DQ_KSLOTS - 1) * DQ_TILE_BYTES + tid * 32) = z;
      *reinterpret_cast<i32x4*>(smem + (DQ_KSLOTS - 1) * DQ_TILE_BYTES + tid * 32 + 16) = z;
    }
    __builtin_amdgcn_s_waitcnt(0x0070);            // vmcnt(0), lgkmcnt(0): this wavefront's DMA and stores are done
    __builtin_amdgcn_s_barrier();

    const long long wave_first_q = a.q_off + q0;
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 s[2], dp[2];      // S^T (then P^T, in place) and dP^T of the current tile: [row block], 32 keys x 32 rows
    bf16x8 kfq[3];           // K fragments (A of S^T), read two k-steps ahead; the first two of a tile
                             // are fetched at the end of the previous step
    kfq[0] = lds_read_b128(smem, abase);
    kfq[1] = lds_read_b128(smem, abase ^ (1 << 5));

    // dQ^T += K^T dS^T of one tile: 16 MFMAs (K^T fragment tf = kg*4 + db feeds both row blocks).
    // `extra(i)` is called once per slice after the MFMA (vector work / DMA that rides along).
    auto dq_phase = [&](const char* kl_prev, const bf16x8 (&dsp)[2][2], auto extra) __attribute__((always_inline)) {
      constexpr int TRING = 3;
      bf16x4 tq[TRING][2];
#pragma unroll
      for (int tn = 0; tn < 2; tn++) {
        tq[tn][0] = lds_read_tr(kl_prev, taddr[tn & 3][0]);
        tq[tn][1] = lds_read_tr(kl_prev, taddr[tn & 3][1]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 16; i++) {
        const int tf = i >> 1, kg = tf >> 2, db = tf & 3, rb = i & 1;
        if ((i & 1) == 0 && tf + 2 < 8) {
          const int tn = tf + 2;
          tq[tn % TRING][0] = lds_read_tr(kl_prev, (tn >> 2) * 16 * 256 + taddr[tn & 3][0]);
          tq[tn % TRING][1] = lds_read_tr(kl_prev, (tn >> 2) * 16 * 256 + taddr[tn & 3][1]);
        }
        extra(i, dq[rb][db], cat4(tq[tf % TRING][0], tq[tf % TRING][1]), dsp[rb][kg]);
        __builtin_amdgcn_sched_barrier(0);
      }
    };

    // One step = tile kt: S^T(kt), then dP^T(kt) with the exponentials riding along, then the
    // dQ^T products of tile kt - 1 (whose dS^T fragments `dsp` were finished one step ago) with the
    // dS of tile kt riding along into `dsc`.  kslot / vslot: ring slots of tile kt.
    // jt = position of the tile in the walk (dense: jt = kt).
    auto step = [&](const bf16x8 (&dsp)[2][2], bf16x8 (&dsc)[2][2], int jt, int kslot, int vslot) __attribute__((always_inline)) {
      int kt = jt, kt3 = jt + 3;                   // this tile, and the tile whose K / V are fetched now
      bool mine = true;                            // SPARSE: this wavefront's rows can see the tile
      if constexpr (SPARSE) {
        const int e = __builtin_amdgcn_readfirstlane(list[1 + jt]);
        kt = e & 0xfffff;
        mine = ((e >> (20 + wu)) & 1) != 0;
        kt3 = tile_at(jt + 3);
      }
      const char* kl = smem + kslot * DQ_TILE_BYTES;
      const int kprev = (kslot == 0) ? DQ_KSLOTS - 1 : kslot - 1;
      const int knext = (kslot == DQ_KSLOTS - 1) ? 0 : kslot + 1;
      const char* kl_prev = smem + kprev * DQ_TILE_BYTES;                    // K of tile kt - 1
      const char* kl_next = smem + knext * DQ_TILE_BYTES;                    // K of tile kt + 1 (landed a step ago)
      const char* vl = smem + VBASE + vslot * DQ_TILE_BYTES;
      int k3 = kslot + 3; if (k3 >= DQ_KSLOTS) k3 -= DQ_KSLOTS;             // K of tile kt + 3 replaces K of tile kt - 2
      const int v3 = (vslot + 3) & 3;                                        // V of tile kt + 3 replaces V of tile kt - 1
      const unsigned k_dst = lds0 + k3 * DQ_TILE_BYTES;
      const unsigned v_dst = lds0 + VBASE + v3 * DQ_TILE_BYTES;
      bf16x8 vfq[3];           // V fragments (A of dP^T), read two k-steps ahead
      // ---- slices 0..15: S^T = K Q^T (k-step ks = i / 2, row block i % 2)
#pragma unroll
      for (int i = 0; i < 16; i++) {
        const int ks = i >> 1, rb = i & 1;
        if (rb == 0 && ks + 2 < 8) kfq[(ks + 2) % 3] = lds_read_b128(kl, abase ^ ((ks + 2) << 5));
        if (i == 13) vfq[0] = lds_read_b128(vl, abase);
        if (i == 15) vfq[1] = lds_read_b128(vl, abase ^ (1 << 5));
        s[rb] = mfma32(kfq[ks % 3], qf[rb][ks], ks == 0 ? zero16 : s[rb]);
        __builtin_amdgcn_sched_barrier(0);
      }
      // The exponents below are computed inside asm statements, where the compiler does not see
      // that they read S^T: the last MFMA that wrote s[0] is one MFMA (32 cycles) and the mask test
      // (some twenty instructions) ahead of the first such read, s[1] is first read eight slices
      // later; the four idle cycles here are a margin on top of that.
      asm volatile("s_nop 3" : "+v"(s[0]), "+v"(s[1]));
      // ---- masking (diagonal tiles, window edge, ragged key tail): rare.  A masked score becomes
      // -inf, its P and dS become 0.
      const long long tile_first_k = k_off + (long long)kt * DQ_BC;
      const bool need_mask = (a.causal && tile_first_k + DQ_BC - 1 > wave_first_q) ||
                             (window > 0 && tile_first_k < wave_first_q + 63 - window + 1) ||
                             ((kt + 1) * DQ_BC > Nc) || !mine;
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
          if (!mine) lim = -1;
          const long long dl = dd - window + 1;
          const int lim_lo = window > 0 ? (int)(dl < -1 ? -1 : (dl > 64 ? 64 : dl)) : -1;
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int cpart = 8 * (r >> 2) + (r & 3);
            s[rb][r] = (cpart <= lim && cpart >= lim_lo) ? s[rb][r] : BURST_NEG_INF;
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      // ---- slices 16..31: dP^T = V dO^T; P^T = exp2(c S^T - lse log2 e) of score pair i replaces S^T
#pragma unroll
      for (int i = 0; i < 16; i++) {
        const int ks = i >> 1, rb = i & 1;
        if (rb == 0 && ks + 2 < 8) vfq[(ks + 2) % 3] = lds_read_b128(vl, abase ^ ((ks + 2) << 5));
        {
          // the slice's MFMA with the exponents of score pair i computed right in front of it and
          // the exponentials right behind, all in one asm statement
          const int prb = i >> 3, r = 2 * (i & 7);
          float x0 = s[prb][r], x1 = s[prb][r + 1];
          if (ks == 0) exp2_mfma32_dp_first(dp[rb], vfq[0], gfr[rb][0], negD[rb], x0, x1, a.c, nlse2[prb]);
          else exp2_mfma32_dp(dp[rb], vfq[ks % 3], gfr[rb][ks], x0, x1, a.c, nlse2[prb]);
          s[prb][r] = x0;
          s[prb][r + 1] = x1;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      mfma_vgpr_fence(dp);     // the last dP^T MFMAs have written their accumulators
      // ---- slices 32..47: dQ^T(kt - 1) += K^T dS^T; dS^T = P^T o (dP^T - D) of score pair i of
      // tile kt rides along, and so do the DMA of tile kt + 3 and the first K reads of tile kt + 1
      dq_phase(kl_prev, dsp, [&](int i, f32x16& acc, bf16x8 fa, bf16x8 fb) __attribute__((always_inline)) {
        const int prb = i >> 3, r = 2 * (i & 7), kg = r >> 3, t = r & 7;
        // the slice's MFMA with the two dS products of score pair i right in front of it and
        // their conversion to packed bf16 right behind, all in one asm statement
        unsigned pu;
        ds2_mfma32_acc(acc, fa, fb, pu, s[prb][r], dp[prb][r], s[prb][r + 1], dp[prb][r + 1]);
        const bf16x2 pk = __builtin_bit_cast(bf16x2, pu);
        dsc[prb][kg][t] = pk[0]; dsc[prb][kg][t + 1] = pk[1];
        if ((i & 3) == 1) {
          const int j = i >> 2;                    // 0, 1 -> K of tile kt + 3; 2, 3 -> V of tile kt + 3
          if (j < 2) dma_tile(krs, k_dst, j, kt3);
          else dma_tile(vrs, v_dst, j - 2, kt3);
        }
        if (i == 14) kfq[0] = lds_read_b128(kl_next, abase);
        if (i == 15) kfq[1] = lds_read_b128(kl_next, abase ^ (1 << 5));
      });
      // The 4 DMA loads just issued may stay in flight; older ones (tile kt + 2) must have landed.
      __builtin_amdgcn_s_waitcnt(0x0F74);          // vmcnt(4)
      __builtin_amdgcn_s_barrier();
    };

    // dS^T fragments (B operands of dQ^T): [row block][16-key group], two sets that swap roles
    bf16x8 dsA[2][2], dsB[2][2];
#pragma unroll
    for (int rb = 0; rb < 2; rb++)
#pragma unroll
      for (int kg = 0; kg < 2; kg++)
#pragma unroll
        for (int t = 0; t < 8; t++) { dsA[rb][kg][t] = (bf16)0.0f; dsB[rb][kg][t] = (bf16)0.0f; }
    // tiles are taken in pairs; an odd count is rounded up (the extra tile lies past the end of the
    // chunk: its K / V read as zeros and every score of it is masked)
    const int ntiles2 = (ntiles + 1) & ~1;
    int kslot = 0, vslot = 0;
    for (int kt = 0; kt < ntiles2; kt += 2) {
      step(dsB, dsA, kt, kslot, vslot);
      kslot = (kslot == DQ_KSLOTS - 1) ? 0 : kslot + 1;
      vslot = (vslot + 1) & 3;
      step(dsA, dsB, kt + 1, kslot, vslot);
      kslot = (kslot == DQ_KSLOTS - 1) ? 0 : kslot + 1;
      vslot = (vslot + 1) & 3;
    }
    // the dQ^T products of the last tile
    {
      const int kprev = (kslot == 0) ? DQ_KSLOTS - 1 : kslot - 1;
      dq_phase(smem + kprev * DQ_TILE_BYTES, dsB, [&](int, f32x16& acc, bf16x8 fa, bf16x8 fb) __attribute__((always_inline)) {
        mfma32_acc(acc, fa, fb);
      });
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): no DMA may outlive the loop
    // The fence stands here, inside the block, on purpose: behind the join with the path that
    // skipped the loop the compiler may move the accumulators to other registers, and those moves
    // are vector instructions that would read them while the last MFMAs are still in flight.
    mfma_acc_fence(dq);
  }
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
  static DeviceOnce lds_opt_in;
  const int st = lds_opt_in.run([] {
    return hipFuncSetAttribute((const void*)burst_bwd_dq_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               DQ_LDS_BYTES) == hipSuccess &&
           hipFuncSetAttribute((const void*)burst_bwd_dq_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               DQ_LDS_BYTES) == hipSuccess &&
           hipFuncSetAttribute((const void*)burst_bwd_dq_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               DQ_LDS_BYTES + DQ_LIST_BYTES) == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
  });
  if (st != BURST_OK) return st;
  if (a.bmask != nullptr) {
    if ((p.Nc + DQ_BC - 1) / DQ_BC > DQ_MAX_LIST) return BURST_ERR_SHAPE;
    BURST_LAUNCH(burst_bwd_dq_kernel<2>, dim3((unsigned)nb), dim3(256), DQ_LDS_BYTES + DQ_LIST_BYTES, stream, a);
  } else if (a.window > 0) {
    BURST_LAUNCH(burst_bwd_dq_kernel<1>, dim3((unsigned)nb), dim3(256), DQ_LDS_BYTES, stream, a);
  } else {
    BURST_LAUNCH(burst_bwd_dq_kernel<0>, dim3((unsigned)nb), dim3(256), DQ_LDS_BYTES, stream, a);
  }
  return launch_status();
}

}  // namespace burst
