// Arguments shared by the two backward kernels (paper Alg. 2 loop body, bf16, d = 128).
#pragma once
#include "burst_common.h"

namespace burst {

struct BwdArgs {
  const bf16* Q; const bf16* K; const bf16* V; const bf16* dO;
  const float* lse; const float* D;
  float* dQ; float* dK; float* dV;
  int Nq, Nc, H;
  int causal;
  float c;               // scale * log2(e)
  float scale;
  long long q_off, k_off;
  long long window;      // 0 = none; else keys at positions <= query position - window are hidden
  const uint8_t* bmask;  // block flags [ceil(Nq / bsize)][bpitch], nullptr = none (paper Sec. 2.6)
  int bsize, bpitch;     // bsize: a multiple of 64
  long long bhstride;    // bytes between the flag matrices of consecutive query heads (0 = shared)
  int group;             // query heads per key/value head (grouped-query attention; 1 = none)
  int blocks_per_head;
  int acc_dq, acc_dkv;
  Layout lay;            // strides of Q, dO and of K, V
};

inline BwdArgs make_bwd_args(const KParams& p, const void* Q, const void* K, const void* V,
                             const void* dO, const float* lse, const float* D,
                             float* dQ, float* dK, float* dV, int acc_dq, int acc_dkv) {
  BwdArgs a;
  a.Q = (const bf16*)Q; a.K = (const bf16*)K; a.V = (const bf16*)V; a.dO = (const bf16*)dO;
  a.lse = lse; a.D = D; a.dQ = dQ; a.dK = dK; a.dV = dV;
  a.Nq = p.Nq; a.Nc = p.Nc; a.H = p.B * p.H;
  a.causal = p.causal; a.c = p.scale * kLog2e; a.scale = p.scale;
  a.q_off = p.q_off; a.k_off = p.k_off; a.window = p.window;
  a.bmask = p.bmask; a.bsize = p.bsize; a.bpitch = p.bpitch; a.bhstride = p.bhstride; a.group = p.group;
  a.blocks_per_head = 0; a.acc_dq = acc_dq; a.acc_dkv = acc_dkv;
  a.lay = p.lay;
  return a;
}

__device__ __forceinline__ bf16x8 cat4(bf16x4 a, bf16x4 b) {
  bf16x8 v;
  v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
  v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
  return v;
}

}  // namespace burst
