// Attention of the decode step with FP8 (E5M2) storage of the KV cache: the instantiation of the
// templates in attn_kernels.hpp for one-byte elements.
#include "attn_kernels.hpp"

namespace skv {

template hipError_t launch_attention_eb<1>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_keys_eb<1>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_values_eb<1>(const AttnArgs&, hipStream_t);

}  // namespace skv
