// Declarations shared by the two backward kernels' translation units (not installed).
#pragma once
#include "fcp_device.h"

namespace fcp {

struct BwdParams {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  const uint16_t* d_o;
  const float* lse;
  const float* delta;
  const int32_t* q_limit;    // [tq] last key position each local query row sees, NULL = its own position (causal)
  const int32_t* k_from;     // [tkv] first query position that sees each pool key, NULL = its own position
  const float* stats;        // two planes [hq][tq]: -LSE * log2 e (-inf for a row without keys), then -delta
  SchedHeader* hdr;          // schedule region of the kernel being launched
  const Tile* tiles;
  float* dq;
  float* dk;
  float* dv;
  // Direct mode (all three set, or all NULL): a unit that owns its rows / keys in this launch (the scheduler's
  // exclusivity flags) writes its final bf16 result here and leaves the fp32 accumulator alone.
  uint16_t* dq_out;
  uint16_t* dk_out;
  uint16_t* dv_out;
  int32_t tq, hq, hkv;
  float scale, scale_log2;
};

// dK / dV over key tiles (csrc/fcp_attn_dkv.hip).  `units` = upper bound of (key tile, KV head) units.
int launch_dkv(const BwdParams& p, int head_dim, int64_t units, int n_cu, hipStream_t stream);

}  // namespace fcp
