// bf16 MFMA flash-style attention for gfx950 (forward and backward).
#pragma once
#include "common.h"

namespace varuna {

inline bool attn_mfma_supported(int s, int d) { (void)s; (void)d; return false; }

inline hipError_t launch_attention_fwd_mfma(const bf16*, bf16*, float*, int, int, int, int, int, hipStream_t) {
  return hipErrorInvalidConfiguration;
}
inline hipError_t launch_attention_bwd_mfma(const bf16*, const bf16*, const float*, const bf16*, bf16*, float*, int, int,
                                            int, int, int, hipStream_t) {
  return hipErrorInvalidConfiguration;
}

}  // namespace varuna
