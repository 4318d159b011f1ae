// Launcher of the attention kernel (attention_kernel.h) and its head-dimension-128 instantiations.
#include "attention_kernel.h"

namespace us {

hipError_t attn_dispatch_d128(const AttnArgs &a, hipStream_t stream) { return attn_dispatch_t<128>(a, stream); }

hipError_t launch_attention(const AttnArgs &a, hipStream_t stream)
{
    switch (a.head_dim) {
        case 64: return attn_dispatch_d64(a, stream);
        case 128: return attn_dispatch_d128(a, stream);
        case 256: return attn_dispatch_d256(a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace us
