// Attention of the decode step with bf16 storage of the KV cache, and the entry points that pick the
// storage type (the kernels are templates in attn_kernels.hpp).
#include "attn_kernels.hpp"

namespace skv {

template hipError_t launch_attention_eb<2>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_keys_eb<2>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_values_eb<2>(const AttnArgs&, hipStream_t);
extern template hipError_t launch_attention_eb<1>(const AttnArgs&, hipStream_t);
extern template hipError_t launch_attention_keys_eb<1>(const AttnArgs&, hipStream_t);
extern template hipError_t launch_attention_values_eb<1>(const AttnArgs&, hipStream_t);

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
  return a.kv_bytes == 1 ? launch_attention_eb<1>(a, st) : launch_attention_eb<2>(a, st);
}
hipError_t launch_attention_keys(const AttnArgs& a, hipStream_t st) {
  return a.kv_bytes == 1 ? launch_attention_keys_eb<1>(a, st) : launch_attention_keys_eb<2>(a, st);
}
hipError_t launch_attention_values(const AttnArgs& a, hipStream_t st) {
  return a.kv_bytes == 1 ? launch_attention_values_eb<1>(a, st) : launch_attention_values_eb<2>(a, st);
}

}  // namespace skv
