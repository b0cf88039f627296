// Host-side argument validation of the C ABI, run under AddressSanitizer and
// UndefinedBehaviorSanitizer (host code only) by tests/test_host_sanitizers.py.  No call here
// reaches the device: every one is rejected (or found empty) by the checks in front of it.
#include "burst.h"
#include <cstdio>
#include <cstring>
int main() {
  burst_params p; std::memset(&p, 0, sizeof p);
  p.B = 1; p.H = 2; p.Nq = 16; p.Nc = 16; p.d = 128; p.dtype = BURST_BF16; p.scale = 0.5f;
  int bad = 0;
  bad += burst_state_init(nullptr, nullptr, nullptr, &p, nullptr) != BURST_ERR_NULL;
  p.d = 300; bad += burst_local_fwd(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, &p, nullptr) != BURST_ERR_SHAPE;
  p.d = 128; p.dtype = 9; bad += burst_finalize(nullptr, nullptr, nullptr, nullptr, nullptr, &p, nullptr) != BURST_ERR_DTYPE;
  p.dtype = BURST_BF16; p.window = -1; bad += burst_bwd_prepare(nullptr, nullptr, nullptr, &p, nullptr) != BURST_ERR_SHAPE;
  p.window = 0; p.kv_heads = 3; bad += burst_local_bwd(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0, &p, nullptr) != BURST_ERR_SHAPE;
  p.kv_heads = 0; p.Nq = 0; bad += burst_state_init(nullptr, nullptr, nullptr, &p, nullptr) != BURST_OK;
  p.Nq = 5; p.Nc = 9; p.d = 8; p.H = 2;
  bad += burst_materialized_workspace_bytes(&p) != 768 + 512 + 2 * 256;
  bad += burst_materialized_workspace_bytes(nullptr) != 0;
  // the entry point that allocates nothing: over its static scratch, then a missing O
  {
    burst_params q; std::memset(&q, 0, sizeof q);
    q.B = 1; q.H = 32; q.Nq = BURST_STATIC_MAX_ROWS / 32 + 1; q.Nc = 64; q.d = 128; q.dtype = BURST_BF16; q.scale = 0.5f;
    void* a = reinterpret_cast<void*>(4096);           // never dereferenced: rejected before any device call
    float* fa = static_cast<float*>(a);
    bad += burst_local_bwd_static(a, a, a, a, a, fa, fa, fa, fa, 1, 0, &q, nullptr) != BURST_ERR_TOO_LARGE;
    q.Nq = 64;
    bad += burst_local_bwd_static(a, a, a, nullptr, a, fa, fa, fa, fa, 1, 0, &q, nullptr) != BURST_ERR_NULL;
    bad += std::strstr(burst_strerror(BURST_ERR_TOO_LARGE), "static scratch") == nullptr;
  }
  // the measurement probes reject bad arguments on the host
  bad += burst_probe_mfma(3, 1, &p, reinterpret_cast<float*>(&p), 1, nullptr) != BURST_ERR_SHAPE;
  bad += burst_probe_mfma(0, 1, nullptr, nullptr, 1, nullptr) != BURST_ERR_NULL;
  bad += burst_probe_atomic_dq(reinterpret_cast<float*>(&p), 7, 64, 1, 1, nullptr) != BURST_ERR_SHAPE;
  bad += burst_workspace_bytes(&p) != (size_t)1 * 2 * 5 * 4;
  bad += std::strcmp(burst_strerror(0), "ok") != 0;
  bad += burst_version() < 100;
  std::printf("host checks failed: %d\n", bad);
  return bad;
}
