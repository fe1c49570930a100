// Host-side construction of the per-launch dropout constants.
#pragma once
#include "device_common.h"
#include "kernels.h"

namespace lynx {

// Philox stream = step * 2^32 + layer_id * 4 + site; an element is dropped
// when its 16 random bits are below floor(p * 65536).
inline DropoutKey make_dropout_key(const DropoutParams& dp, int site) {
  DropoutKey k;
  k.key0 = static_cast<uint32_t>(dp.seed);
  k.key1 = static_cast<uint32_t>(dp.seed >> 32);
  k.stream0 = (dp.layer_id << 2) | static_cast<uint32_t>(site);
  k.stream1 = static_cast<uint32_t>(dp.step);
  k.threshold = static_cast<uint32_t>(static_cast<double>(dp.p) * 65536.0);
  k.scale = 1.0f / (1.0f - dp.p);
  return k;
}

}  // namespace lynx
