// The library used from a plain host program: no Python, no PyTorch, only the C ABI of
// include/burst.h and the HIP runtime for memory.  One device's share of the ring (paper Alg. 1 and
// Alg. 2 with the ring step replaced by taking the next chunk already in device memory):
//   state_init, G x local_fwd, finalize, then G x local_bwd_static (D is computed by the call into
//   the library's static scratch: this program allocates nothing after its set-up).
// Inputs are pseudo-random bf16 values made here; inputs and results are written to a binary file so
// that a test can hold the results against the CPU oracle (tests/test_gpu_c_example.py).
//
//   ring_walk H Nq Nc G causal seed out.bin
//
// File layout (little endian): int32 H, Nq, Nc, G, causal; float scale; then bf16 Q[H][Nq][128],
// K[G][H][Nc][128], V[G][H][Nc][128], dO[H][Nq][128]; bf16 O[H][Nq][128]; fp32 lse[H][Nq],
// dQ[H][Nq][128], dK[G][H][Nc][128], dV[G][H][Nc][128].
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include "burst.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define BURST_CALL(x) do { int s_ = (x); if (s_ != BURST_OK) { std::fprintf(stderr, "%s: %s\n", #x, burst_strerror(s_)); return 3; } } while (0)

static uint16_t to_bf16(float f) {                 // round to nearest even
  uint32_t u; std::memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
// approximately N(0,1): sum of twelve uniforms minus six, from a 64-bit LCG
static float next_normal(uint64_t& state) {
  float s = 0.f;
  for (int i = 0; i < 12; i++) {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    s += (float)((state >> 40) & 0xffffff) / 16777216.0f;
  }
  return s - 6.0f;
}

int main(int argc, char** argv) {
  if (argc != 8) { std::fprintf(stderr, "usage: ring_walk H Nq Nc G causal seed out.bin\n"); return 1; }
  const int H = std::atoi(argv[1]), Nq = std::atoi(argv[2]), Nc = std::atoi(argv[3]), G = std::atoi(argv[4]);
  const int causal = std::atoi(argv[5]), d = 128;
  uint64_t rng = 0x9e3779b97f4a7c15ull ^ (uint64_t)std::atoll(argv[6]);
  if (H < 1 || Nq < 1 || Nc < 1 || G < 1) return 1;
  const size_t nq = (size_t)H * Nq * d, nk = (size_t)H * Nc * d;
  std::vector<uint16_t> hQ(nq), hdO(nq), hK((size_t)G * nk), hV((size_t)G * nk);
  for (auto& x : hQ) x = to_bf16(next_normal(rng));
  for (auto& x : hK) x = to_bf16(next_normal(rng));
  for (auto& x : hV) x = to_bf16(next_normal(rng));
  for (auto& x : hdO) x = to_bf16(next_normal(rng));

  void *Q, *dO, *K, *V, *O;
  float *O_acc, *m, *l, *lse, *dQ, *dK, *dV;
  HIP_OK(hipMalloc(&Q, nq * 2)); HIP_OK(hipMalloc(&dO, nq * 2)); HIP_OK(hipMalloc(&O, nq * 2));
  HIP_OK(hipMalloc(&K, (size_t)G * nk * 2)); HIP_OK(hipMalloc(&V, (size_t)G * nk * 2));
  HIP_OK(hipMalloc((void**)&O_acc, nq * 4)); HIP_OK(hipMalloc((void**)&dQ, nq * 4));
  HIP_OK(hipMalloc((void**)&m, (size_t)H * Nq * 4)); HIP_OK(hipMalloc((void**)&l, (size_t)H * Nq * 4));
  HIP_OK(hipMalloc((void**)&lse, (size_t)H * Nq * 4));
  HIP_OK(hipMalloc((void**)&dK, (size_t)G * nk * 4)); HIP_OK(hipMalloc((void**)&dV, (size_t)G * nk * 4));
  HIP_OK(hipMemcpy(Q, hQ.data(), nq * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dO, hdO.data(), nq * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(K, hK.data(), (size_t)G * nk * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(V, hV.data(), (size_t)G * nk * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemset(dQ, 0, nq * 4));                 // dQ accumulates over the chunks
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));

  burst_params p;
  std::memset(&p, 0, sizeof p);
  p.B = 1; p.H = H; p.Nq = Nq; p.Nc = Nc; p.d = d; p.dtype = BURST_BF16; p.causal = causal;
  p.scale = 1.0f / std::sqrt((float)d);
  p.q_off = causal ? (int64_t)(G - 1) * Nc : 0;     // causal: the slice of the last rank, diagonal chunk last
  BURST_CALL(burst_state_init(O_acc, m, l, &p, stream));
  for (int j = 0; j < G; j++) {
    p.k_off = (int64_t)j * Nc;
    BURST_CALL(burst_local_fwd(Q, (char*)K + (size_t)j * nk * 2, (char*)V + (size_t)j * nk * 2, O_acc, m, l, &p, stream));
  }
  BURST_CALL(burst_finalize(O_acc, m, l, O, lse, &p, stream));
  for (int j = 0; j < G; j++) {
    p.k_off = (int64_t)j * Nc;
    BURST_CALL(burst_local_bwd_static(Q, (char*)K + (size_t)j * nk * 2, (char*)V + (size_t)j * nk * 2, O, dO, lse,
                                      dQ, dK + (size_t)j * nk, dV + (size_t)j * nk, 1, 0, &p, stream));
  }
  HIP_OK(hipStreamSynchronize(stream));

  std::vector<uint16_t> hO(nq);
  std::vector<float> hlse((size_t)H * Nq), hdQ(nq), hdK((size_t)G * nk), hdV((size_t)G * nk);
  HIP_OK(hipMemcpy(hO.data(), O, nq * 2, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(hlse.data(), lse, hlse.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(hdQ.data(), dQ, nq * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(hdK.data(), dK, hdK.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(hdV.data(), dV, hdV.size() * 4, hipMemcpyDeviceToHost));
  FILE* f = std::fopen(argv[7], "wb");
  if (f == nullptr) { std::perror(argv[7]); return 4; }
  const int32_t head[5] = {H, Nq, Nc, G, causal};
  std::fwrite(head, 4, 5, f); std::fwrite(&p.scale, 4, 1, f);
  std::fwrite(hQ.data(), 2, hQ.size(), f); std::fwrite(hK.data(), 2, hK.size(), f);
  std::fwrite(hV.data(), 2, hV.size(), f); std::fwrite(hdO.data(), 2, hdO.size(), f);
  std::fwrite(hO.data(), 2, hO.size(), f); std::fwrite(hlse.data(), 4, hlse.size(), f);
  std::fwrite(hdQ.data(), 4, hdQ.size(), f); std::fwrite(hdK.data(), 4, hdK.size(), f);
  std::fwrite(hdV.data(), 4, hdV.size(), f);
  std::fclose(f);
  std::printf("ring_walk: H=%d Nq=%d G=%d x Nc=%d causal=%d done, library version %d\n", H, Nq, G, Nc, causal, burst_version());
  return 0;
}
