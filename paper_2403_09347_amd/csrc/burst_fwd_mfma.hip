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
// The wavefront runs at one wave per SIMD (512 registers).  The loop is software-pipelined: the
// S^T MFMAs of tile j+1 are issued in between the exp / sum / convert of tile j, so that neither
// kind of instruction ever waits for a result of the other (measured: a wavefront's own matrix
// and vector instructions do not execute concurrently, the gain is in the absent stalls).  K and
// V tiles are DMA-ed from HBM straight into LDS (buffer loads with the LDS modifier, no staging
// registers) into two rings of three tiles each, two tiles ahead of their use (one barrier per
// tile).  The running max is only raised when a row's new maximum exceeds it by more than 2^8
// (P stays <= 2^8, exact in fp32/bf16 range), so the O rescale is rare.
// The chunk-local (O_ij, m_ij, l_ij) is merged into the state in HBM in the epilogue
// (Alg. 1: m_new = max, rescale, add).  No S or P tile ever leaves registers.
#include "burst_common.h"

namespace burst {

constexpr int FWD_BR = 256;   // query rows per workgroup
constexpr int FWD_BC = 64;    // keys per tile
constexpr int FWD_TILE_BYTES = FWD_BC * 256;
constexpr int FWD_NBUF = 3;
constexpr float FWD_LAZY = 8.0f;   // log2 of the largest P allowed before the max is raised
constexpr int FWD_MAX_LIST = 8192;  // block-sparse calls: most key tiles of one chunk (512K keys)
constexpr int FWD_LIST_BYTES = (FWD_MAX_LIST + 8) * 4;

struct FwdArgs {
  const bf16* Q; const bf16* K; const bf16* V;
  float* O_acc; float* m; float* l;
  int Nq, Nc, H;
  int causal;
  float c;               // scale * log2(e)
  long long q_off, k_off;
  long long window;      // 0 = none; else keys at positions <= query position - window are hidden
  int q_blocks;          // ceil(Nq / FWD_BR)
  const uint8_t* bmask;  // block flags [ceil(Nq / bsize)][bpitch], nullptr = none (paper Sec. 2.6)
  int bsize, bpitch;     // bsize: a multiple of 64, so a wavefront's 64 rows and a key tile lie in one block
  long long bhstride;    // bytes between the flag matrices of consecutive heads (0 = shared)
  int group;             // query heads per key/value head (grouped-query attention; 1 = none)
  Layout lay;            // strides of Q and of K, V
};


// MFMA on an AGPR accumulator (see mfma32_acc) preceded, inside one asm statement, by two
// independent vector instructions of the caller's own work: whatever register copies the compiler
// puts before the statement are then at least two instructions away from the MFMA, which is what
// the leading s_nop of mfma32_acc is for.  t0 = x0 * c + n, t1 = x1 * c + n ...
__device__ __forceinline__ void fma2_mfma32_acc(f32x16& acc, bf16x8 a, bf16x8 b, float& t0, float& t1,
                                                float x0, float x1, float c, float n) {
  asm volatile("v_fma_f32 %1, %5, %7, %8\n\tv_fma_f32 %2, %6, %7, %8\n\tv_mfma_f32_32x32x16_bf16 %0, %3, %4, %0"
               : "+a"(acc), "=&v"(t0), "=&v"(t1) : "v"(a), "v"(b), "v"(x0), "v"(x1), "s"(c), "v"(n));
}
// ... or m0 = max(m0, x00, x01), m1 = max(m1, x10, x11).
__device__ __forceinline__ void max3x2_mfma32_acc(f32x16& acc, bf16x8 a, bf16x8 b, float& m0, float x00, float x01,
                                                  float& m1, float x10, float x11) {
  asm volatile("v_max3_f32 %1, %1, %5, %6\n\tv_max3_f32 %2, %2, %7, %8\n\tv_mfma_f32_32x32x16_bf16 %0, %3, %4, %0"
               : "+a"(acc), "+v"(m0), "+v"(m1) : "v"(a), "v"(b), "v"(x00), "v"(x01), "v"(x10), "v"(x11));
}

// HBM -> LDS for one 64x128 bf16 tile (K or V) without staging registers.  One wave-wide
// load writes 1024 contiguous LDS bytes (4 tile rows), lane i filling the 16 bytes at i*16;
// which global granule a lane fetches is free, so lane i asks for the granule that the XOR
// layout places at its slot.  Each wavefront issues 4 such loads per tile (16 rows).
// goff[il] is the lane's byte offset inside the tile for load il.
// (pitch: bytes between rows of the tensor in HBM)
__device__ __forceinline__ void tile_dma_offsets(int w, int lane, unsigned pitch, int (&goff)[4]) {
#pragma unroll
  for (int il = 0; il < 4; il++) {
    int row = 16 * w + 4 * il + (lane >> 4);
    goff[il] = (int)(row * pitch + (((lane & 15) ^ row_code(row)) << 4));
  }
}
__device__ __forceinline__ void tile_dma(__amdgpu_buffer_rsrc_t rsrc, unsigned lds_tile, int w_uniform, int il,
                                         int voffset) {
  dma_b128_to_lds(rsrc, lds_tile + (unsigned)(w_uniform * 4 + il) * 1024u, voffset);
}

// S^T (64 keys x 64 rows) = K_tile Q^T into s[key block][row block].
__device__ __forceinline__ void qk_tile(const char* kl, const int (&kaddr)[8], const bf16x8 (&qf)[2][8],
                                        f32x16 (&s)[2][2]) {
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
}

// SPARSE: the call carries block flags.  The workgroup first writes the list of key tiles that at
// least one of its wavefronts can see (tile index plus one bit per wavefront) into LDS and then
// walks that list instead of 0, 1, 2, ...; a wavefront whose bit is clear hides the whole tile
// in the masking path.  Entries past the end name a tile beyond the chunk: its DMA reads zeros
// and the ragged-tail mask hides it.
template <bool SPARSE>
__global__ void __launch_bounds__(256, 1)
burst_fwd_mfma_kernel(FwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];

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
    // causal: the later a query block, the more key tiles it sees; the blocks of a head start
    // in descending order so that the long ones do not end up in the last round
    if (a.causal) qb = a.q_blocks - 1 - qb;
    head = hx * 8 + xcd;
    if (head >= a.H) return;                       // whole workgroup exits together
  }

  const int q0 = qb * FWD_BR + w * 64;             // first query row of this wave
  const bf16* Qh = a.Q + a.lay.q_base(head);
  const bf16* Kh = a.K + a.lay.kv_base(head / a.group);
  const bf16* Vh = a.V + a.lay.kv_base(head / a.group);
  const unsigned kpitch = (unsigned)a.lay.ks_r * 2u;             // bytes between key rows
  const unsigned ktile = kpitch * FWD_BC;                        // ... between key tiles

  // Sliding window: key tiles before the first one that the workgroup's first row can see are
  // skipped by moving the start of the chunk (pointers, length, global offset) forward by whole
  // tiles; everything below works on that shortened chunk.
  int Nc = a.Nc;
  long long k_off = a.k_off;
  int t_lo = 0;                                    // SPARSE: first tile of the list (the chunk is not shifted)
  if (a.window > 0) {
    long long lo = a.q_off + (long long)qb * FWD_BR - a.window + 1 - a.k_off;   // first visible key index
    if (lo >= a.Nc) return;                        // nothing visible: state unchanged
    if (lo > 0) {
      const int skip = (int)(lo / FWD_BC) * FWD_BC;
      if constexpr (SPARSE) {
        t_lo = skip / FWD_BC;
      } else {
        Kh += (size_t)skip * a.lay.ks_r; Vh += (size_t)skip * a.lay.ks_r;
        Nc -= skip; k_off += skip;
      }
    }
  }

  // Number of key tiles this workgroup must visit (causal: stop after the last tile that
  // any of its rows can see).
  int ntiles = (Nc + FWD_BC - 1) / FWD_BC;
  const long long wg_last_q = a.q_off + min(qb * FWD_BR + FWD_BR, a.Nq) - 1;
  if (a.causal) {
    long long lim = wg_last_q - k_off;             // last visible key index in this chunk
    if (lim < 0) return;                           // nothing visible: state unchanged
    long long t = lim / FWD_BC + 1;
    if (t < ntiles) ntiles = (int)t;
  }
  if (ntiles <= 0) return;

  // SPARSE: the list of visible tiles, built by wavefront 0 (64 candidate tiles per round).
  // list[0] = number of entries, list[1 + j] = tile | (wavefront bits << 16), then 4 end entries.
  int* const list = reinterpret_cast<int*>(smem + 2 * FWD_NBUF * FWD_TILE_BYTES);
  if constexpr (SPARSE) {
    const int end_tile = (Nc + FWD_BC - 1) / FWD_BC;             // a tile past the chunk
    if (w == 0) {
      const uint8_t* const bm = a.bmask + (size_t)head * a.bhstride;
      int n = 0;
      for (int base = t_lo; base < ntiles; base += 64) {
        const int kt = base + lane;
        int bits = 0;
        if (kt < ntiles) {
          const int col = (kt * FWD_BC) / a.bsize;
#pragma unroll
          for (int ww = 0; ww < 4; ww++) {
            const int row0 = qb * FWD_BR + ww * 64;
            if (row0 < a.Nq && bm[(size_t)(row0 / a.bsize) * a.bpitch + col] != 0) bits |= 1 << ww;
          }
        }
        const unsigned long long bal = __builtin_amdgcn_ballot_w64(bits != 0);
        if (bits != 0) {
          const int pos = n + __builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0u));
          list[1 + pos] = kt | (bits << 16);
        }
        n += __builtin_popcountll(bal);
      }
      if (lane < 4) list[1 + n + lane] = end_tile;
      if (lane == 0) list[0] = n;
    }
    __syncthreads();
    ntiles = __builtin_amdgcn_readfirstlane(list[0]);            // from here on: number of list entries
    if (ntiles == 0) return;
  }
  auto tile_at = [&](int j) __attribute__((always_inline)) {      // tile index of list entry j
    if constexpr (SPARSE) return __builtin_amdgcn_readfirstlane(list[1 + j]) & 0xffff;
    else return j;
  };

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
      if (row < a.Nq) v = *reinterpret_cast<const bf16x8*>(Qh + (size_t)row * a.lay.qs_r + ks * 16 + h * 8);
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
  float m2[2] = {BURST_NEG_INF, BURST_NEG_INF};   // reference max, log2 units, per row block
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

  // ---- prologue: K tiles 0..2 and V tiles 0..1 into LDS, S of tile 0.
  // LDS: K ring = tiles 0..2 of the buffer, V ring = tiles 3..5; tile t lives in slot t % 3.
  // Tiles past the end of the chunk read as zeros (buffer range check) and are never used.
  const unsigned kbytes = Nc > 0 ? (unsigned)(Nc - 1) * kpitch + 256u : 0u;   // up to the end of the last row
  const __amdgpu_buffer_rsrc_t krs = make_rsrc(Kh, kbytes);
  const __amdgpu_buffer_rsrc_t vrs = make_rsrc(Vh, kbytes);
  const int wu = __builtin_amdgcn_readfirstlane(w);
  const unsigned lds0 = lds_addr(smem);
  int goff[4];
  tile_dma_offsets(w, lane, kpitch, goff);
#pragma unroll
  for (int t = 0; t < 3; t++) {
    const int src = tile_at(t);
#pragma unroll
    for (int il = 0; il < 4; il++) {
      tile_dma(krs, lds0 + t * FWD_TILE_BYTES, wu, il, (int)(src * ktile) + goff[il]);
      if (t < 2) tile_dma(vrs, lds0 + (3 + t) * FWD_TILE_BYTES, wu, il, (int)(src * ktile) + goff[il]);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): this wavefront's DMA has landed
  __builtin_amdgcn_s_barrier();                    // ... and everyone else's
  // Two score buffers that swap roles every tile (the loop body is unrolled twice, so no
  // register copies): while one holds the tile being exponentiated, the other receives the
  // S^T of the next tile.
  f32x16 sA[2][2], sB[2][2];   // [key block][row block]
  qk_tile(smem, kaddr, qf, sA);
  float mx[2];                 // row maximum (both lane halves, log2 units) of the tile in flight
  bool raise = false;          // some row's maximum exceeds the reference max by more than 2^LAZY
#pragma unroll
  for (int rb = 0; rb < 2; rb++) {
    float v = sA[0][rb][0];
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int r = 0; r < 16; r++) v = fmaxf(v, sA[kb][rb][r]);
    mx[rb] = max_both_halves(v) * a.c;
    raise = raise || (mx[rb] > m2[rb] + FWD_LAZY);
  }
  __builtin_amdgcn_s_barrier();   // K tile 0 is consumed by every wavefront before its slot is refilled

  const long long wave_first_q = a.q_off + q0;
  const long long wave_last_q = wave_first_q + 63;
  bf16x2 ones;
  ones[0] = (bf16)1.0f; ones[1] = (bf16)1.0f;
  constexpr int PF = 4;          // operand fragments are fetched PF MFMA pairs ahead

  // One tile: `sc` holds S^T of tile kt (unmasked), `sx` receives S^T of the next tile.
  // jt = position of the tile in the walk (dense: jt = kt), slot = jt % 3 its LDS ring slot.
  auto step = [&](f32x16 (&sc)[2][2], f32x16 (&sx)[2][2], int jt, int slot) __attribute__((always_inline)) {
    int kt = jt, kt2 = jt + 2, kt3 = jt + 3;       // this tile, and the tiles whose V / K are fetched now
    bool mine = true;                              // SPARSE: this wavefront's rows can see the tile
    if constexpr (SPARSE) {
      const int e = __builtin_amdgcn_readfirstlane(list[1 + jt]);
      kt = e & 0xffff;
      mine = ((e >> (16 + wu)) & 1) != 0;
      kt2 = tile_at(jt + 2);
      kt3 = tile_at(jt + 3);
    }
    const int slot1 = (slot == FWD_NBUF - 1) ? 0 : slot + 1;     // tile kt + 1
    const int slot2 = (slot1 == FWD_NBUF - 1) ? 0 : slot1 + 1;   // tile kt + 2
    const char* kl_next = smem + slot1 * FWD_TILE_BYTES;         // K of tile kt + 1
    const char* vl = smem + (3 + slot) * FWD_TILE_BYTES;         // V of tile kt
    const unsigned k_dst = lds0 + slot * FWD_TILE_BYTES;         // K of tile kt + 3 replaces K of tile kt
    const unsigned v_dst = lds0 + (3 + slot2) * FWD_TILE_BYTES;  // V of tile kt + 2 replaces V of tile kt - 1
    // first K fragments of the next tile: in flight while the rare-path checks run
    bf16x8 kfq[PF + 1];
#pragma unroll
    for (int pn = 0; pn < PF; pn++) kfq[pn] = lds_read_b128(kl_next, (pn & 1) * 32 * 256 + kaddr[pn >> 1]);
    const long long tile_first_k = k_off + (long long)kt * FWD_BC;
    // ---- masking (diagonal tiles, ragged key tail): rare; redo the row maxima afterwards
    const bool need_mask = (a.causal && tile_first_k + FWD_BC - 1 > wave_first_q) ||
                           (a.window > 0 && tile_first_k < wave_last_q - a.window + 1) ||
                           ((kt + 1) * FWD_BC > Nc) || !mine;
    if (need_mask) {
      raise = false;
#pragma unroll
      for (int rb = 0; rb < 2; rb++) {
        // score register r of key block kb holds key index kt*64 + 4h + (kb*32 + 8*(r/4) + r%4)
        // of the chunk; with dd = (row position) - (position of key kt*64 + 4h) the key of
        // register r is visible iff cpart <= dd (causal), cpart > dd - window, and it exists
        // (ragged tail).  Computed here, in the rare path: nothing of it stays live in the loop.
        const int ln = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));   // lane id, recomputed
        const int mlr = ln & 31, mh = ln >> 5;
        const long long dd = (a.q_off - k_off) + (q0 + rb * 32 + mlr) - ((long long)kt * FWD_BC + 4 * mh);
        const int tail = Nc - 1 - (kt * FWD_BC + 4 * mh);
        int lim = a.causal ? (int)(dd < -1 ? -1 : (dd > 64 ? 64 : dd)) : 64;
        lim = lim < tail ? lim : tail;
        if (!mine) lim = -1;
        const long long dl = dd - a.window + 1;
        const int lim_lo = a.window > 0 ? (int)(dl < -1 ? -1 : (dl > 64 ? 64 : dl)) : -1;
        float v = BURST_NEG_INF;
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int cpart = kb * 32 + 8 * (r >> 2) + (r & 3);
            float x = (cpart <= lim && cpart >= lim_lo) ? sc[kb][rb][r] : BURST_NEG_INF;
            sc[kb][rb][r] = x;
            v = fmaxf(v, x);
          }
        mx[rb] = max_both_halves(v) * a.c;
        raise = raise || (mx[rb] > m2[rb] + FWD_LAZY);
      }
    }
    // ---- raise the reference max only when it is exceeded by 2^LAZY
    if (__builtin_amdgcn_ballot_w64(raise) != 0) {             // wave-uniform, rare after the first tiles
      mfma_acc_fence(o);
#pragma unroll
      for (int rb = 0; rb < 2; rb++) {
        float m_new = fmaxf(m2[rb], mx[rb]);
        float ref = (m_new == BURST_NEG_INF) ? 0.f : m_new;
        float alpha = fast_exp2(m2[rb] - ref);                 // exp2(-inf) = 0 for a fresh row
        m2[rb] = m_new;
        lsum[rb] *= alpha;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
          for (int r = 0; r < 16; r++) o[rb][db][r] *= alpha;
      }
      mfma_acc_fence(o);
    }
    float nref[2];
#pragma unroll
    for (int rb = 0; rb < 2; rb++) nref[rb] = (m2[rb] == BURST_NEG_INF) ? 0.f : -m2[rb];

    // The 64 MFMAs of a tile (32 for S^T of the next tile, then 32 for O^T += V^T P^T) are
    // hand-interleaved with the vector work, one MFMA per slice, scheduling barriers between
    // slices, so that every MFMA finds its operands ready and every vector instruction its
    // inputs, whatever the latencies.  Vector work per tile: 32 "pairs"
    // (two scores: 2 fma, 2 exp, convert to packed bf16, row sum by dot product with ones),
    // ordered by key group so that P is ready when its MFMA comes; 20 pairs ride on the first
    // 32 slices, 12 on the next 12, then the row maxima of the next tile.
    bf16x8 pf[2][4];       // P^T fragments (B operand): [row block][16-key group]
    bf16x4 vfq[PF + 1][2]; // V^T fragment halves
    // second half of a pair whose exponents t0, t1 are already there
    auto softmax_pair_tail = [&](int pidx, float t0, float t1) __attribute__((always_inline)) {
      const int kg = pidx >> 3, srb = (pidx >> 2) & 1, t = (pidx & 3) * 2;
      float p0 = fast_exp2(t0), p1 = fast_exp2(t1);
      bf16x2 pk;
      pk[0] = (bf16)p0; pk[1] = (bf16)p1;
      lsum[srb] = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, lsum[srb], false);
      pf[srb][kg][t] = pk[0];
      pf[srb][kg][t + 1] = pk[1];
    };
    auto softmax_pair = [&](int pidx) __attribute__((always_inline)) {           // pidx = kg * 8 + rb * 4 + t / 2
      const int kg = pidx >> 3, srb = (pidx >> 2) & 1, t = (pidx & 3) * 2;
      const int skb = kg >> 1, r = 8 * (kg & 1) + t;
      float p0 = fast_exp2(__builtin_fmaf(sc[skb][srb][r], a.c, nref[srb]));
      float p1 = fast_exp2(__builtin_fmaf(sc[skb][srb][r + 1], a.c, nref[srb]));
      bf16x2 pk;
      pk[0] = (bf16)p0; pk[1] = (bf16)p1;
      lsum[srb] = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, lsum[srb], false);
      pf[srb][kg][t] = pk[0];
      pf[srb][kg][t + 1] = pk[1];
    };
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int rb = 0; rb < 2; rb++)
#pragma unroll
        for (int r = 0; r < 16; r++) sx[kb][rb][r] = 0.f;
    __builtin_amdgcn_sched_barrier(0);
    // ---- slices 0..31: S^T of the next tile.  After the last tile the product reads a stale
    // buffer and is discarded.
#pragma unroll
    for (int i = 0; i < 32; i++) {
      const int pair = i >> 1;                     // K fragment index: ks = pair / 2, kb = pair % 2
      const int ks = pair >> 1, kb = pair & 1, rb = i & 1;
      if ((i & 1) == 0 && pair + PF < 16) {
        const int pn = pair + PF;
        kfq[pn % (PF + 1)] = lds_read_b128(kl_next, (pn & 1) * 32 * 256 + kaddr[pn >> 1]);
      }
      if ((i & 1) == 0 && pair + PF >= 16) {       // first V fragments of the second half
        const int pn = pair + PF - 16;
        vfq[pn][0] = lds_read_tr(vl, vaddr[pn & 3][0]);
        vfq[pn][1] = lds_read_tr(vl, vaddr[pn & 3][1]);
      }
      sx[kb][rb] = mfma32(kfq[pair % (PF + 1)], qf[rb][ks], sx[kb][rb]);
      // 20 pairs over 32 slices: 5 in every 8
      {
        const int i8 = i & 7;
        if (i8 == 0 || i8 == 2 || i8 == 3 || i8 == 5 || i8 == 6) {
          const int within = (i8 == 0) ? 0 : (i8 == 2) ? 1 : (i8 == 3) ? 2 : (i8 == 5) ? 3 : 4;
          softmax_pair((i >> 3) * 5 + within);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---- slices 32..63: O^T += V^T P^T, with the DMA of tile kt + 3 (K) and kt + 2 (V), the
    // last 12 softmax pairs and the row maxima of the next tile
    float nmax0 = sx[0][0][0], nmax1 = sx[0][1][0];
#pragma unroll
    for (int i = 0; i < 32; i++) {
      const int pair = i >> 1;                     // V fragment index: kg = pair / 4, db = pair % 4
      const int kg = pair >> 2, db = pair & 3, rb = i & 1;
      if ((i & 1) == 0 && pair + PF < 16) {
        const int pn = pair + PF;
        vfq[pn % (PF + 1)][0] = lds_read_tr(vl, (pn >> 2) * 16 * 256 + vaddr[pn & 3][0]);
        vfq[pn % (PF + 1)][1] = lds_read_tr(vl, (pn >> 2) * 16 * 256 + vaddr[pn & 3][1]);
      }
      if ((i & 3) == 1) {                          // 8 slots: one DMA of 4 tile rows each
        const int j = i >> 2;                      // 0..3 -> K of tile kt + 3, 4..7 -> V of tile kt + 2
        if (j < 4) tile_dma(krs, k_dst, wu, j, (int)(kt3 * ktile) + goff[j]);
        else tile_dma(vrs, v_dst, wu, j - 4, (int)(kt2 * ktile) + goff[j - 4]);
      }
      {
        bf16x8 vf;
        const bf16x4 va = vfq[pair % (PF + 1)][0], vb = vfq[pair % (PF + 1)][1];
        vf[0] = va[0]; vf[1] = va[1]; vf[2] = va[2]; vf[3] = va[3];
        vf[4] = vb[0]; vf[5] = vb[1]; vf[6] = vb[2]; vf[7] = vb[3];
        // The MFMA of the slice with two vector instructions of the slice's own work in front
        // of it inside the same asm statement (the exponents of a score pair, or the running row
        // maxima of the next tile): they take the place of the two idle cycles an asm MFMA
        // otherwise needs after whatever register copies the compiler put before the statement.
        if (i < 12) {
          const int pidx = 20 + i, pkg = pidx >> 3, srb = (pidx >> 2) & 1, t = (pidx & 3) * 2;
          const int skb = pkg >> 1, r = 8 * (pkg & 1) + t;
          float t0, t1;
          fma2_mfma32_acc(o[rb][db], vf, pf[rb][kg], t0, t1, sc[skb][srb][r], sc[skb][srb][r + 1], a.c, nref[srb]);
          softmax_pair_tail(pidx, t0, t1);
        } else if (i < 28) {                       // row maxima of the next tile: 16 slices x 4 scores
          const int e = i - 12;                    // 0..15
          const int kb2 = e >> 3, r = (e & 7) * 2;
          max3x2_mfma32_acc(o[rb][db], vf, pf[rb][kg], nmax0, sx[kb2][0][r], sx[kb2][0][r + 1],
                            nmax1, sx[kb2][1][r], sx[kb2][1][r + 1]);
        } else {
          mfma32_acc(o[rb][db], vf, pf[rb][kg]);
        }
      }
      if (i == 28) mx[0] = max_both_halves(nmax0) * a.c;
      if (i == 29) mx[1] = max_both_halves(nmax1) * a.c;
      if (i == 30) raise = (mx[0] > m2[0] + FWD_LAZY) || (mx[1] > m2[1] + FWD_LAZY);
      __builtin_amdgcn_sched_barrier(0);
    }
    // The 8 DMA loads just issued may stay in flight; everything older (the tiles the next
    // step reads) must have landed before the barrier publishes it.
    __builtin_amdgcn_s_waitcnt(0x0F78);            // vmcnt(8), lgkmcnt / expcnt unconstrained
    __builtin_amdgcn_s_barrier();
  };

  int slot = 0;
  for (int kt = 0; kt < ntiles; kt += 2) {
    step(sA, sB, kt, slot);
    slot = (slot == FWD_NBUF - 1) ? 0 : slot + 1;
    if (kt + 1 >= ntiles) break;
    step(sB, sA, kt + 1, slot);
    slot = (slot == FWD_NBUF - 1) ? 0 : slot + 1;
  }

  __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): no DMA may outlive the loop
  mfma_acc_fence(o);
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
      float fa = fast_exp2(m_old2 - m_new);        // weight of the stored state
      float fb = fast_exp2(m2[rb] - m_new);        // weight of this chunk
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
  a.q_off = p.q_off; a.k_off = p.k_off; a.window = p.window;
  a.q_blocks = (p.Nq + FWD_BR - 1) / FWD_BR;
  a.bmask = p.bmask; a.bsize = p.bsize; a.bpitch = p.bpitch; a.bhstride = p.bhstride; a.group = p.group;
  a.lay = p.lay;
  int heads8 = ((a.H + 7) / 8) * 8;                // pad the head count to a multiple of 8 ids
  long long nblocks = (long long)heads8 * a.q_blocks;
  if (nblocks > 0x7fffffffLL) return BURST_ERR_SHAPE;
  static DeviceOnce lds_opt_in;
  const int st = lds_opt_in.run([] {
    return hipFuncSetAttribute((const void*)burst_fwd_mfma_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               2 * FWD_NBUF * FWD_TILE_BYTES) == hipSuccess &&
           hipFuncSetAttribute((const void*)burst_fwd_mfma_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               2 * FWD_NBUF * FWD_TILE_BYTES + FWD_LIST_BYTES) == hipSuccess ? BURST_OK : BURST_ERR_LAUNCH;
  });
  if (st != BURST_OK) return st;
  if (a.bmask != nullptr) {
    if ((p.Nc + FWD_BC - 1) / FWD_BC > FWD_MAX_LIST) return BURST_ERR_SHAPE;
    BURST_LAUNCH(burst_fwd_mfma_kernel<true>, dim3((unsigned)nblocks), dim3(256),
                       2 * FWD_NBUF * FWD_TILE_BYTES + FWD_LIST_BYTES, stream, a);
  } else {
    BURST_LAUNCH(burst_fwd_mfma_kernel<false>, dim3((unsigned)nblocks), dim3(256),
                       2 * FWD_NBUF * FWD_TILE_BYTES, stream, a);
  }
  return launch_status();
}

}  // namespace burst
