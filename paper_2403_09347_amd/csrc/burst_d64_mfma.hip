// bf16, d = 64: the plainly written forward, dQ and dK/dV kernels (namespace burst::d64).
#define BURST_SMALL_D 64
#define BURST_SMALL_NS d64
#include "burst_plain_mfma.h"
