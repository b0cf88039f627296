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
  bad += std::strcmp(burst_strerror(0), "ok") != 0;
  bad += burst_version() < 100;
  std::printf("host checks failed: %d\n", bad);
  return bad;
}
