// Backward, dK / dV side of one block pair (paper Alg. 2 loop body) for bf16, d = 128.
//
// Key-stationary half of the split backward (see burst_bwd_dq_mfma.hip for why it is split):
//     S = Q K^T,  dP = dO V^T,  P = exp(S - lse),  dS = P o (dP - D),
//     dV += P^T dO,  dK += dS^T Q
// P is recomputed from the saved log-sum-exp; neither S, P nor dS is ever stored.
//
// One workgroup = 4 wavefronts = 128 keys of one (batch, head); a wavefront owns 32 keys:
// their K and V fragments (B operands of S and dP) and the dK / dV accumulators stay in
// registers for the whole kernel, the accumulators pinned in AGPRs.  Query rows stream through
// in tiles of 64 rows (two 32-row blocks): Q and dO tiles are DMA-ed from HBM into LDS rings two
// tiles ahead.  With S = Q K^T a lane owns one key and its registers run over query rows, so P
// and dS already have the A-operand layout of P^T dO and dS^T Q (contraction over rows); the B
// operands dO and Q come through transposing LDS reads.  lse and D are per-row, i.e. per
// register: they are staged (already scaled) in a small LDS ring and read as broadcasts.
// The 64 MFMAs of a tile run in four phases of 16, software-pipelined across the two row
// blocks so that the vector work of one block rides on the MFMAs of the other:
//   1: S, dP of block 0            2: S, dP of block 1   + P, dS of block 0
//   3: dV, dK of block 0 + P, dS of block 1              4: dV, dK of block 1 + DMA of tile t+2
// No atomics: every key row is owned by one wavefront, results are bitwise reproducible.
//
// A second shape of the same kernel has 2 wavefronts = 64 keys per workgroup and two workgroups
// per CU (NW = 2), for block flags 64 keys wide (paper Sec. 2.6): a workgroup's tile list then
// holds what its own 64 keys need and nothing else, which the 128-key shape cannot offer (a tile
// that half of its keys need costs the full time).  Two workgroups share the CU's LDS, so the
// tile ring has two slots instead of three and a tile is fetched one step ahead instead of two.
#include "burst_bwd_common.h"

namespace burst {

constexpr int DKV_BR = 64;            // query rows per tile
constexpr int DKV_TILE_BYTES = DKV_BR * 256;
constexpr int DKV_STAT_SLOTS = 4;     // row statistics run one tile further ahead than the tiles
// Sizes and LDS layout for NW wavefronts per workgroup.
template <int NW>
struct DkvShape {
  static constexpr int BC = 32 * NW;                 // keys per workgroup
  static constexpr int SLOTS = NW == 4 ? 3 : 2;      // tile ring
  static constexpr int LPW = 16 / NW;                // DMA wave-loads per tensor and tile that a wavefront issues
  static constexpr int LDS_Q = 0;
  static constexpr int LDS_G = SLOTS * DKV_TILE_BYTES;
  static constexpr int LDS_L = 2 * SLOTS * DKV_TILE_BYTES;             // -lse / scale per row
  static constexpr int LDS_D = LDS_L + DKV_STAT_SLOTS * DKV_BR * 4;    // -D per row
  static constexpr int LDS_DUMMY = LDS_D + DKV_STAT_SLOTS * DKV_BR * 4;  // sink of the padding DMA (256 B)
  static constexpr int LDS_BYTES = LDS_DUMMY + 256;
  // block-sparse calls: most query tiles of one slice (512K rows; 128K rows where two workgroups
  // share the LDS)
  static constexpr int MAX_LIST = NW == 4 ? 8192 : 2048;
  static constexpr int LIST_BYTES = (MAX_LIST + 8) * 4;
};

// SPARSE: the call carries block flags (paper Sec. 2.6) or several query heads share a key/value
// head (a.group > 1: the tiles of all heads of the group are walked, `head` is then the key/value
// head and Q, dO, lse, D of the group are addressed as one tensor of group * Nq rows, which needs
// Nq to be a multiple of the tile).  The workgroup first writes the list of
// query tiles that at least one of its wavefronts' keys are visible to (tile index plus one bit per
// wavefront) into LDS and then walks that list instead of t_begin, t_begin + 1, ...; a wavefront
// whose bit is clear hides the whole tile in the masking path.  Entries past the end name a tile
// beyond the slice: its Q, dO and statistics read as zeros and contribute nothing.
template <bool SPARSE, int NW>
__global__ void __launch_bounds__(64 * NW, 1)
burst_bwd_dkv_kernel(BwdArgs a) {
  using Shape = DkvShape<NW>;
  constexpr int DKV_BC = Shape::BC, DKV_SLOTS = Shape::SLOTS, LPW = Shape::LPW;
  constexpr int DKV_LDS_Q = Shape::LDS_Q, DKV_LDS_G = Shape::LDS_G, DKV_LDS_L = Shape::LDS_L, DKV_LDS_D = Shape::LDS_D;
  constexpr int DKV_LDS_DUMMY = Shape::LDS_DUMMY, DKV_LDS_BYTES = Shape::LDS_BYTES;
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
  const int key0 = key_wg + w * 32;                // first key of this wavefront
  const int group = SPARSE ? a.group : 1;          // query heads that share this key/value head
  const int q_rows = group * a.Nq;                 // rows of the group's Q / dO / lse / D
  const bf16* Qh = a.Q + a.lay.q_base(head * group);    // first query head of the group
  const bf16* Gh = a.dO + a.lay.q_base(head * group);
  const bf16* Kh = a.K + a.lay.kv_base(head);
  const bf16* Vh = a.V + a.lay.kv_base(head);
  const unsigned qpitch = (unsigned)a.lay.qs_r * 2u;             // bytes between query rows
  const unsigned qtile = qpitch * DKV_BR;                        // ... between query tiles
  const float* lseh = a.lse + (size_t)head * q_rows;
  const float* Dh = a.D + (size_t)head * q_rows;

  // query tiles to visit: causal rows before the first key of the workgroup see none of it
  int ntiles_all = (a.Nq + DKV_BR - 1) / DKV_BR;
  int t_begin = 0;
  if (a.causal) {
    long long first_row = a.k_off + key_wg - a.q_off;      // first row index that sees key_wg
    if (first_row > 0) t_begin = (int)min((long long)ntiles_all, first_row / DKV_BR);
  }
  if (a.window > 0) {
    // sliding window: rows at positions >= key position + window no longer see the key
    long long last_row = a.k_off + min(key_wg + DKV_BC, a.Nc) - 1 + a.window - 1 - a.q_off;
    ntiles_all = last_row < 0 ? 0 : (int)min((long long)ntiles_all, last_row / DKV_BR + 1);
  }

  f32x16 dk[4], dv[4];     // [32-wide d block]: rows = the wavefront's 32 keys; pinned in AGPRs
#pragma unroll
  for (int db = 0; db < 4; db++)
#pragma unroll
    for (int r = 0; r < 16; r++) { dk[db][r] = 0.f; dv[db][r] = 0.f; }

  // K, V fragments (B operands: lane = key lr, 8 consecutive d), requested before the tile list is
  // built so that the two latencies overlap
  bf16x8 kf[8], vf[8];
  {
    const int key = key0 + lr;
#pragma unroll
    for (int ks = 0; ks < 8; ks++) {
      bf16x8 z;
#pragma unroll
      for (int t = 0; t < 8; t++) z[t] = (bf16)0.0f;
      kf[ks] = key < a.Nc ? *reinterpret_cast<const bf16x8*>(Kh + (size_t)key * a.lay.ks_r + ks * 16 + h * 8) : z;
      vf[ks] = key < a.Nc ? *reinterpret_cast<const bf16x8*>(Vh + (size_t)key * a.lay.ks_r + ks * 16 + h * 8) : z;
    }
  }
  int nwalk = ntiles_all - t_begin;                // tiles to walk
  // SPARSE: the list of visible tiles, built by wavefront 0 (64 candidate tiles per round).
  // list[0] = number of entries, list[1 + j] = tile | (wavefront bits << 16), then 4 end entries.
  int* const list = reinterpret_cast<int*>(smem + DKV_LDS_BYTES);
  const int tiles_per_head = (a.Nq + DKV_BR - 1) / DKV_BR;
  if constexpr (SPARSE) {
    const int end_tile = (q_rows + DKV_BR - 1) / DKV_BR;        // a tile past the group's rows
    if (w == 0) {
      int n = 0;
      for (int g = 0; g < group; g++)
        for (int base = t_begin; base < ntiles_all; base += 64) {
          const int t = base + lane;
          int bits = 0;
          if (t < ntiles_all) {
            if (a.bmask == nullptr) {
              bits = (1 << NW) - 1;
            } else {
              const uint8_t* mrow = a.bmask + (size_t)(head * group + g) * a.bhstride + (size_t)((t * DKV_BR) / a.bsize) * a.bpitch;
#pragma unroll
              for (int ww = 0; ww < NW; ww++) {
                const int k0 = key_wg + ww * 32;
                if (k0 < a.Nc && mrow[k0 / a.bsize] != 0) bits |= 1 << ww;
              }
            }
          }
          const unsigned long long bal = __builtin_amdgcn_ballot_w64(bits != 0);
          if (bits != 0) {
            const int pos = n + __builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0u));
            list[1 + pos] = (g * tiles_per_head + t) | (bits << 16) | (g << 20);
          }
          n += __builtin_popcountll(bal);
        }
      if (lane < 4) list[1 + n + lane] = end_tile;
      if (lane == 0) list[0] = n;
    }
    __syncthreads();
    nwalk = __builtin_amdgcn_readfirstlane(list[0]);
  }
  // walk position j -> its entry: the tile index in the low 16 bits and, SPARSE, the wavefront
  // bits (16..19) and the head of the group (20..27)
  auto entry_at = [&](int j) __attribute__((always_inline)) {
    if constexpr (SPARSE) return __builtin_amdgcn_readfirstlane(list[1 + j]);
    else return t_begin + j;
  };
  auto tile_of = [&](int e) __attribute__((always_inline)) {
    if constexpr (SPARSE) return e & 0xffff;
    else return e;
  };

  if (nwalk > 0) {
    // LDS addressing inside a 64-row tile.  A operands (128-bit): row rb*32 + lr, granule
    // 2*ks + h -> rb*8192 + (abase ^ (ks << 5)).  B operands through transposing reads:
    // rows = query rows rb*32 + u*16 + ..., cols = d.
    const int abase = lr * 256 + ((h ^ row_code(lr)) << 4);
    int taddr[4][2];
    {
      const int j16 = lane & 15, dh = (lane >> 4) & 1;
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int sx = 0; sx < 2; sx++)
          taddr[db][sx] = tile_off(8 * sx + 4 * h + (j16 >> 2), db * 4 + 2 * dh + ((j16 & 3) >> 1)) + (j16 & 1) * 8;
    }
    // DMA: a 64-row tile is 16 wave-loads of 4 rows; wavefront w issues loads LPW*w .. LPW*w + LPW-1
    // (the rows of the group's heads lie (head stride) apart: a tile of head g of the group starts
    // g * gfix bytes away from where it would in one tensor of group * Nq rows)
    const unsigned hbytes = (unsigned)a.lay.qs_h * 2u;
    const unsigned gfix = hbytes - (unsigned)tiles_per_head * qtile;
    const unsigned qbytes = a.Nq > 0 ? (unsigned)(group - 1) * hbytes + (unsigned)(a.Nq - 1) * qpitch + 256u : 0u;
    const __amdgpu_buffer_rsrc_t qrs = make_rsrc(Qh, qbytes);
    const __amdgpu_buffer_rsrc_t grs = make_rsrc(Gh, qbytes);
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const unsigned lds0 = lds_addr(smem);
    int goff[LPW];
#pragma unroll
    for (int il = 0; il < LPW; il++) {
      int row = 4 * LPW * w + 4 * il + (lane >> 4);
      goff[il] = (int)(row * qpitch + (((lane & 15) ^ row_code(row)) << 4));
    }
    // `e`: an entry (see entry_at)
    auto dma_tile = [&](__amdgpu_buffer_rsrc_t rs, unsigned lds_tile, int il, int e) __attribute__((always_inline)) {
      unsigned tile = (unsigned)tile_of(e) * qtile;
      if constexpr (SPARSE) tile += (unsigned)((e >> 20) & 0xff) * gfix;
      dma_b128_to_lds(rs, lds_tile + (unsigned)(wu * LPW + il) * 1024u, (int)tile + goff[il]);
    };
    // Per-row statistics of a tile travel like the tiles: wavefront 0 DMAs the 64 lse values,
    // wavefront 1 the 64 D values (rows past Nq read as 0; their Q and dO rows are 0 too, so they
    // contribute nothing).  Two steps before use, wavefront 0 rewrites lse in place as
    // -lse/scale, or -inf for a row that saw nothing (then P = exp2(-inf) = 0), and wavefront
    // 1 rewrites D as -D: the S and dP accumulators START at these values, so that
    // P = exp2(c (Q K^T - lse/scale)) and dS = P o (dO V^T - D) need no subtraction in the
    // per-element vector work.  (Multiplying K by c beforehand would also remove the multiply,
    // but rounds c K to bf16 again; with few visible keys per row P is then visibly off.)  No
    // compiler-visible global load is left in the loop: its wait would drain the DMA queue.
    const __amdgpu_buffer_rsrc_t lrs = make_rsrc(lseh, (unsigned)q_rows * 4u);
    const __amdgpu_buffer_rsrc_t drs = make_rsrc(Dh, (unsigned)q_rows * 4u);
    auto dma_rowstat = [&](int t, int slot) __attribute__((always_inline)) {
      // every wavefront issues exactly one such load per tile (the wait counts below rely on
      // it): 0 -> lse, 1 -> D, 2 and 3 -> a dummy copy of lse that nobody reads
      const unsigned dst = (wu == 0) ? lds0 + DKV_LDS_L + slot * DKV_BR * 4
                         : (wu == 1) ? lds0 + DKV_LDS_D + slot * DKV_BR * 4 : lds0 + DKV_LDS_DUMMY;
      dma_b32_to_lds(wu == 1 ? drs : lrs, dst, (t * DKV_BR + lane) * 4);
    };
    const float inv_scale = 1.0f / a.scale;
    // The same in two parts for the main loop, so that the LDS round trip hides behind MFMAs:
    // wavefronts 0 / 1 fetch their 64 values at one point of the step and write them back later.
    float stat_tmp = 0.f;
    auto rowstat_fetch = [&](int slot) __attribute__((always_inline)) {
      if (tid < 64) stat_tmp = *(reinterpret_cast<const float*>(smem + DKV_LDS_L) + slot * DKV_BR + tid);
      else if (tid < 128) stat_tmp = *(reinterpret_cast<const float*>(smem + DKV_LDS_D) + slot * DKV_BR + (tid - 64));
    };
    auto rowstat_store = [&](int slot) __attribute__((always_inline)) {
      if (tid < 64)
        *(reinterpret_cast<float*>(smem + DKV_LDS_L) + slot * DKV_BR + tid) =
            (stat_tmp == BURST_NEG_INF) ? BURST_NEG_INF : -stat_tmp * inv_scale;
      else if (tid < 128)
        *(reinterpret_cast<float*>(smem + DKV_LDS_D) + slot * DKV_BR + (tid - 64)) = -stat_tmp;
    };
    auto scale_rowstat = [&](int slot) __attribute__((always_inline)) {
      if (tid < 64) {
        float* ptr = reinterpret_cast<float*>(smem + DKV_LDS_L) + slot * DKV_BR + tid;
        float lv = *ptr;
        *ptr = (lv == BURST_NEG_INF) ? BURST_NEG_INF : -lv * inv_scale;
      } else if (tid < 128) {
        float* ptr = reinterpret_cast<float*>(smem + DKV_LDS_D) + slot * DKV_BR + (tid - 64);
        *ptr = -*ptr;
      }
    };

    // ---- prologue: tiles t_begin, t_begin + 1 into tile slots 0, 1 (two slots: the first tile
    // alone); the statistics of tiles t_begin .. t_begin + 2 into statistic slots 0 .. 2, the
    // first two scaled right away
#pragma unroll
    for (int t = 0; t < DKV_SLOTS - 1; t++) {
      const int src = entry_at(t);
#pragma unroll
      for (int il = 0; il < LPW; il++) {
        dma_tile(qrs, lds0 + DKV_LDS_Q + t * DKV_TILE_BYTES, il, src);
        dma_tile(grs, lds0 + DKV_LDS_G + t * DKV_TILE_BYTES, il, src);
      }
    }
#pragma unroll
    for (int t = 0; t < 3; t++) dma_rowstat(tile_of(entry_at(t)), t);
    __builtin_amdgcn_s_waitcnt(0x0070);            // vmcnt(0), lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    scale_rowstat(0);
    scale_rowstat(1);
    __builtin_amdgcn_s_waitcnt(0x0070);
    __builtin_amdgcn_s_barrier();

    const long long wave_first_k = a.k_off + key0;
    const long long wave_last_k = wave_first_k + 31;
    const long long kpos = wave_first_k + lr;
    constexpr int LEAD = 6, RING = LEAD + 2;       // A-operand reads run LEAD slices ahead
    constexpr int TLEAD = 5, TRING = TLEAD + 1;    // transposed fragments run TLEAD slices ahead
                                                   // (SQ counters showed 7 % of the wave time waiting for LDS at 4 / 3)

    // S and dP accumulators of the two row blocks.  They start at -lse/scale and -D of their
    // rows (register r of a block = row 8*(r/4) + 4h + r%4: four 128-bit broadcast reads per
    // block and statistic, straight into the accumulator registers).  Block 0 of the next tile is
    // loaded while the current tile's last phases run.
    f32x16 s[2], dp[2];
    auto load_init = [&](int rb, const float* lrow, const float* drow) __attribute__((always_inline)) {
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        const f32x4 lv = *reinterpret_cast<const f32x4*>(lrow + rb * 32 + 8 * q4 + 4 * h);
        const f32x4 dv = *reinterpret_cast<const f32x4*>(drow + rb * 32 + 8 * q4 + 4 * h);
#pragma unroll
        for (int j = 0; j < 4; j++) { s[rb][4 * q4 + j] = lv[j]; dp[rb][4 * q4 + j] = dv[j]; }
      }
    };
    load_init(0, reinterpret_cast<const float*>(smem + DKV_LDS_L), reinterpret_cast<const float*>(smem + DKV_LDS_D));

    int slot = 0;
    for (int n = 0; n < nwalk; n++) {                  // n = walk position; statistic slot n & 3 holds its tile
      // this tile, the entry of the tile whose rows are fetched now, the tile whose statistics are
      int t = t_begin + n, t2 = t + DKV_SLOTS - 1, t3 = t + 3, t_in_head = t;
      bool mine = true;                                // SPARSE: this wavefront's keys are visible to the tile
      if constexpr (SPARSE) {
        const int e = __builtin_amdgcn_readfirstlane(list[1 + n]);
        t = e & 0xffff;
        t_in_head = t - ((e >> 20) & 0xff) * tiles_per_head;
        mine = ((e >> (16 + wu)) & 1) != 0;
        t2 = entry_at(n + DKV_SLOTS - 1);
        t3 = tile_of(entry_at(n + 3));
      }
      const int slot1 = (slot == DKV_SLOTS - 1) ? 0 : slot + 1;
      // where the tile fetched in this step goes: the slot after the next tile's, or (two slots) the next tile's
      const int slot2 = DKV_SLOTS == 2 ? slot1 : (slot1 == DKV_SLOTS - 1) ? 0 : slot1 + 1;
      const char* ql = smem + DKV_LDS_Q + slot * DKV_TILE_BYTES;
      const char* gl = smem + DKV_LDS_G + slot * DKV_TILE_BYTES;
      const float* lp = reinterpret_cast<const float*>(smem + DKV_LDS_L) + (n & 3) * DKV_BR;
      const float* dp_ = reinterpret_cast<const float*>(smem + DKV_LDS_D) + (n & 3) * DKV_BR;
      const float* lp_next = reinterpret_cast<const float*>(smem + DKV_LDS_L) + ((n + 1) & 3) * DKV_BR;
      const float* dp_next = reinterpret_cast<const float*>(smem + DKV_LDS_D) + ((n + 1) & 3) * DKV_BR;
      // (t counts tiles over all heads of the group; the position restarts with every head)
      const long long tile_first_q = a.q_off + (long long)t_in_head * DKV_BR;
      // (no branch around the MFMA phases: the AGPR-pinned accumulators must not become phi
      // values, the allocator would shuttle them through VGPRs every iteration)
      const bool need_mask = (a.causal && wave_last_k > tile_first_q) ||
                             (a.window > 0 && tile_first_q + DKV_BR - 1 >= wave_first_k + a.window) || !mine;
      {
        // A-operand read j (0..31): rb = j / 16, ks = (j / 2) % 8, even: Q fragment (for S), odd:
        // dO fragment (for dP).  S and dP alternate so that no MFMA waits for its predecessor.
        bf16x8 fq[RING];
        auto issue_read = [&](int j) __attribute__((always_inline)) {
          const int rb = j >> 4, isg = j & 1, ks = (j >> 1) & 7;
          fq[j % RING] = lds_read_b128(isg ? gl : ql, rb * 32 * 256 + (abase ^ (ks << 5)));
        };
        // transposed fragment j (0..31): rb = j / 16, u = (j / 8) % 2, db = (j / 2) % 4, then
        // 0: dO (for dV), 1: Q (for dK)
        bf16x4 tq[TRING][2];
        auto issue_tread = [&](int j) __attribute__((always_inline)) {
          const int rb = j >> 4, u = (j >> 3) & 1, db = (j >> 1) & 3, isq = j & 1;
          const char* base = isq ? ql : gl;
          const int off = (rb * 32 + u * 16) * 256;
          tq[j % TRING][0] = lds_read_tr(base, off + taddr[db][0]);
          tq[j % TRING][1] = lds_read_tr(base, off + taddr[db][1]);
        };
        bf16x8 pf[2][2], dsf[2][2];   // [row block][16-row group]: A operands of dV, dK
        // P and dS of two scores: register pair (r, r+1) of row block rb = rows 8*(r/4)+4h+r%4.
        // The work is cut in two halves, one per MFMA slice: an in-order wavefront hides only
        // what it issues between two of its own MFMAs.
        float ph0, ph1;
        auto pds_half0 = [&](int rb, int pidx) __attribute__((always_inline)) {  // pidx 0..7
          const int r = 2 * pidx;
          ph0 = fast_exp2(s[rb][r] * a.c);
          ph1 = fast_exp2(s[rb][r + 1] * a.c);
          asm volatile("" : "+v"(ph0), "+v"(ph1));   // keep the arithmetic in this slice
        };
        auto pds_half1 = [&](int rb, int pidx) __attribute__((always_inline)) {
          const int r = 2 * pidx, u = r >> 3, t8 = r & 7;
          float d0 = ph0 * dp[rb][r];
          float d1 = ph1 * dp[rb][r + 1];
          bf16x2 pk, dk2;
          pk[0] = (bf16)ph0; pk[1] = (bf16)ph1;
          dk2[0] = (bf16)d0; dk2[1] = (bf16)d1;
          // (the only consumers are MFMAs two phases later; without an anchor the compiler sinks
          // the arithmetic there, behind the mask branches)
          unsigned pu = __builtin_bit_cast(unsigned, pk), du = __builtin_bit_cast(unsigned, dk2);
          asm volatile("" : "+v"(pu), "+v"(du));
          pk = __builtin_bit_cast(bf16x2, pu); dk2 = __builtin_bit_cast(bf16x2, du);
          pf[rb][u][t8] = pk[0]; pf[rb][u][t8 + 1] = pk[1];
          dsf[rb][u][t8] = dk2[0]; dsf[rb][u][t8 + 1] = dk2[1];
        };
        // mask of one row block (rare: tiles that straddle the diagonal or the far edge of the
        // sliding window).  Register r belongs to row tile_first_q + rb*32 + 4h + (8*(r/4) + r%4);
        // causal: the key is visible iff its position <= the row's, i.e. iff the constant part is
        // >= lim; window: iff the row's position < the key's + window, i.e. constant part <= lim2.
        // A masked score becomes -inf, its P and dS become 0.
        auto mask_block = [&](int rb) __attribute__((always_inline)) {
          const long long d = kpos - (tile_first_q + rb * 32 + 4 * h);
          const int lim = !mine ? 65 : a.causal ? (int)(d < -1 ? -1 : (d > 64 ? 64 : d)) : -1;
          const long long d2 = d + a.window - 1;
          const int lim2 = a.window > 0 ? (int)(d2 < -1 ? -1 : (d2 > 64 ? 64 : d2)) : 64;
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int cpart = 8 * (r >> 2) + (r & 3);
            s[rb][r] = (cpart >= lim && cpart <= lim2) ? s[rb][r] : BURST_NEG_INF;
          }
        };
#pragma unroll
        for (int j = 0; j < LEAD; j++) issue_read(j);
        __builtin_amdgcn_sched_barrier(0);
        // ---- phases 1, 2: S and dP (slice i: rb = i / 16, ks = (i / 2) % 8, even S, odd dP); in
        // phase 2 the P / dS pairs of row block 0 ride along (one pair every second slice)
#pragma unroll
        for (int i = 0; i < 32; i++) {
          const int rb = i >> 4, isg = i & 1, ks = (i >> 1) & 7;
          if (i == 16 && need_mask) mask_block(0);
          if (i + LEAD < 32) issue_read(i + LEAD);
          if (i + TLEAD >= 32) issue_tread(i + TLEAD - 32);
          if (i == 2) load_init(1, lp, dp_);
          if constexpr (DKV_SLOTS == 2) {
            // two slots: the slot of tile t - 1 is free since the last barrier; tile t + 1 and the
            // statistics of tile t + 3 are requested here and awaited at the end of the step
            if (i == 0) dma_rowstat(t3, (n + 3) & 3);
            if (i < 2 * LPW) {
              if (i & 1) dma_tile(grs, lds0 + DKV_LDS_G + slot2 * DKV_TILE_BYTES, i >> 1, t2);
              else dma_tile(qrs, lds0 + DKV_LDS_Q + slot2 * DKV_TILE_BYTES, i >> 1, t2);
            }
          }
          if (isg) dp[rb] = mfma32(fq[i % RING], vf[ks], dp[rb]);
          else s[rb] = mfma32(fq[i % RING], kf[ks], s[rb]);
          if (i >= 16) { if (i & 1) pds_half1(0, (i - 16) >> 1); else pds_half0(0, (i - 16) >> 1); }
          __builtin_amdgcn_sched_barrier(0);
        }
        // ---- phases 3, 4: dV += P^T dO, dK += dS^T Q (slice i: rb = i / 16, u = (i / 8) % 2,
        // db = (i / 2) % 4, even: dV, odd: dK); in phase 3 the pairs of row block 1 ride along
#pragma unroll
        for (int i = 0; i < 32; i++) {
          const int rb = i >> 4, u = (i >> 3) & 1, db = (i >> 1) & 3, isk = i & 1;
          if (i == 0 && need_mask) mask_block(1);
          if (i + TLEAD < 32) issue_tread(i + TLEAD);
          if (i == 4) load_init(0, lp_next, dp_next);     // block 0 of tile t + 1
          // the loads of the previous step (tile t + 1, statistics of tile t + 2) are most of a
          // step old: wait for them here, before this step's loads are issued, and rewrite those
          // statistics (fetch now, store a few slices later)
          // (two slots: they were awaited at the end of the previous step)
          if (i == 12) { if constexpr (DKV_SLOTS == 3) __builtin_amdgcn_s_waitcnt(0x0F70); rowstat_fetch((n + 2) & 3); }
          if (i == 22) rowstat_store((n + 2) & 3);
          // phase 4 has no vector work: the DMA of tile t + 2 (into the slot of tile t - 1, free
          // since the last barrier) and of the statistics of tile t + 3 is issued here
          if (DKV_SLOTS == 3 && i == 16) dma_rowstat(t3, (n + 3) & 3);
          if (DKV_SLOTS == 3 && i > 16 && (i & 1)) {
            const int j = (i - 17) >> 1;                  // 0..7: Q rows, then dO rows
            if (j < 4) dma_tile(qrs, lds0 + DKV_LDS_Q + slot2 * DKV_TILE_BYTES, j, t2);
            else dma_tile(grs, lds0 + DKV_LDS_G + slot2 * DKV_TILE_BYTES, j - 4, t2);
          }
          const bf16x8 bt = cat4(tq[i % TRING][0], tq[i % TRING][1]);
          if (isk) mfma32_acc(dk[db], dsf[rb][u], bt);
          else mfma32_acc(dv[db], pf[rb][u], bt);
          if (i < 16) { if (i & 1) pds_half1(1, i >> 1); else pds_half0(1, i >> 1); }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // ---- three slots: the 9 loads of this step stay in flight across the barrier; two: the 17
      // loads, issued most of a step ago, must have landed.  The LDS stores of the rewritten
      // statistics must be done.
      slot = slot1;
      if constexpr (DKV_SLOTS == 3) __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0)
      else __builtin_amdgcn_s_waitcnt(0x0070);                                   // vmcnt(0), lgkmcnt(0)
      __builtin_amdgcn_s_barrier();
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): no DMA may outlive the loop
    // wait for the last MFMAs before anything else touches the accumulators (inside the block:
    // behind the join with the path that skipped the loop the compiler may already move them)
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15"
                 : "+a"(dk[0]), "+a"(dk[1]), "+a"(dk[2]), "+a"(dk[3]),
                   "+a"(dv[0]), "+a"(dv[1]), "+a"(dv[2]), "+a"(dv[3]));
  }
  // epilogue: keys are owned by this wavefront alone. C layout: lane = d column, regs = keys.
  float* dKh = a.dK + (size_t)head * a.Nc * 128;
  float* dVh = a.dV + (size_t)head * a.Nc * 128;
#pragma unroll
  for (int r = 0; r < 16; r++) {
    int key = key0 + 8 * (r >> 2) + 4 * h + (r & 3);
    if (key < a.Nc) {
#pragma unroll
      for (int db = 0; db < 4; db++) {
        size_t off = (size_t)key * 128 + db * 32 + lr;
        float k_old = 0.f, v_old = 0.f;
        if (a.acc_dkv) { k_old = dKh[off]; v_old = dVh[off]; }
        dKh[off] = k_old + a.scale * dk[db][r];
        dVh[off] = v_old + dv[db][r];
      }
    }
  }
}

// key_waves: 4 (128-key workgroups) or 2 (64-key workgroups, calls with block flags only).
int launch_bwd_dkv_mfma(const KParams& p, const void* Q, const void* K, const void* V,
                        const void* dO, const float* lse, const float* D, float* dK, float* dV,
                        int acc_dkv, hipStream_t stream, int key_waves) {
  if (p.Nc <= 0) return BURST_OK;
  static DeviceOnce lds_opt_in;
  const int st = lds_opt_in.run([] {
    return hipFuncSetAttribute((const void*)burst_bwd_dkv_kernel<false, 4>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               DkvShape<4>::LDS_BYTES) == hipSuccess &&
           hipFuncSetAttribute((const void*)burst_bwd_dkv_kernel<true, 4>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               DkvShape<4>::LDS_BYTES + DkvShape<4>::LIST_BYTES) == hipSuccess &&
           hipFuncSetAttribute((const void*)burst_bwd_dkv_kernel<true, 2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               DkvShape<2>::LDS_BYTES + DkvShape<2>::LIST_BYTES) == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
  });
  if (st != BURST_OK) return st;
  BwdArgs a = make_bwd_args(p, Q, K, V, dO, lse, D, nullptr, dK, dV, 0, acc_dkv);
  a.H = p.B * p.H / p.group;                       // workgroups are laid out over key/value heads
  int heads8 = ((a.H + 7) / 8) * 8;
  const bool listed = a.bmask != nullptr || a.group > 1;
  if (key_waves != 4 && !(key_waves == 2 && listed)) return BURST_ERR_SHAPE;
  const int bc = 32 * key_waves;
  a.blocks_per_head = (p.Nc + bc - 1) / bc;
  long long nb = (long long)heads8 * a.blocks_per_head;
  if (nb > 0x7fffffffLL) return BURST_ERR_SHAPE;
  if (listed) {
    const int max_list = key_waves == 4 ? DkvShape<4>::MAX_LIST : DkvShape<2>::MAX_LIST;
    if ((long long)a.group * ((p.Nq + DKV_BR - 1) / DKV_BR) > max_list) return BURST_ERR_SHAPE;
    if (a.group > 1 && p.Nq % DKV_BR != 0) return BURST_ERR_SHAPE;
    if (key_waves == 4)
      BURST_LAUNCH((burst_bwd_dkv_kernel<true, 4>), dim3((unsigned)nb), dim3(256),
                   DkvShape<4>::LDS_BYTES + DkvShape<4>::LIST_BYTES, stream, a);
    else
      BURST_LAUNCH((burst_bwd_dkv_kernel<true, 2>), dim3((unsigned)nb), dim3(128),
                   DkvShape<2>::LDS_BYTES + DkvShape<2>::LIST_BYTES, stream, a);
  } else {
    BURST_LAUNCH((burst_bwd_dkv_kernel<false, 4>), dim3((unsigned)nb), dim3(256), DkvShape<4>::LDS_BYTES, stream, a);
  }
  return launch_status();
}

}  // namespace burst
