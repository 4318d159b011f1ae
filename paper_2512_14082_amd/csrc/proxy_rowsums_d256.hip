// One-sweep form of the compressed-space score kernel (proxy_kernel.h) at head dimension 256.
#include "proxy_kernel.h"

namespace us {

hipError_t proxy_rowsums_dispatch_d256(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream)
{
    return proxy_dispatch_t<256, true>(a, g, grid, stream);
}

}  // namespace us
