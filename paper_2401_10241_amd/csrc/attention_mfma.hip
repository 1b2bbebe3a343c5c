// MFMA attention kernels (bf16).  Shapes they do not take fall through to the generic kernels.
#include "zb_common.h"

namespace zb {

template <typename T> hipError_t launch_attention_fwd_mfma(const AttnArgs& a, hipStream_t s, bool* taken) {
  *taken = false;
  return hipSuccess;
}
template <typename T> hipError_t launch_attention_bwd_mfma(const AttnArgs& a, hipStream_t s, bool* taken) {
  *taken = false;
  return hipSuccess;
}
template hipError_t launch_attention_fwd_mfma<float>(const AttnArgs&, hipStream_t, bool*);
template hipError_t launch_attention_fwd_mfma<bf16_t>(const AttnArgs&, hipStream_t, bool*);
template hipError_t launch_attention_bwd_mfma<float>(const AttnArgs&, hipStream_t, bool*);
template hipError_t launch_attention_bwd_mfma<bf16_t>(const AttnArgs&, hipStream_t, bool*);

}  // namespace zb
