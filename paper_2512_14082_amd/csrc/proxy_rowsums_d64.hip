// One-sweep form of the compressed-space score kernel (proxy_kernel.h) at head dimension 64.
#include "proxy_kernel.h"

namespace us {

hipError_t proxy_rowsums_dispatch_d64(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream)
{
    return proxy_dispatch_t<64, true>(a, g, grid, stream);
}

}  // namespace us
