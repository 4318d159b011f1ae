// The attention kernel's head-dimension-256 instantiations (a translation unit of their own: they compile in parallel).
#include "attention_kernel.h"

namespace us {

hipError_t attn_dispatch_d256(const AttnArgs &a, hipStream_t stream) { return attn_dispatch_t<256>(a, stream); }

}  // namespace us
