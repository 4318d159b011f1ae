// Launcher of the compressed-space score kernel (proxy_kernel.h) and its head-dimension-128 instantiations.
#include "proxy_kernel.h"

namespace us {

static int proxy_pick_hg(int G)
{
    if (G % 4 == 0) return 4;
    if (G % 2 == 0) return 2;
    return 1;
}

hipError_t proxy_dispatch_d128(const ProxyArgs &a, const ProxyGeom &g, dim3 grid, hipStream_t stream)
{
    return proxy_dispatch_t<128, false>(a, g, grid, stream);
}

hipError_t launch_proxy_scores(const ProxyArgs &a, hipStream_t stream)
{
    ProxyGeom g;
    const int G = a.n_heads_q / a.n_heads_kv;
    g.HG = proxy_pick_hg(G);
    g.RC = 4 / g.HG;
    g.GS = G / g.HG;
    // Workgroups of 4 wavefronts x 64 rows; a problem that yields fewer than four workgroups per CU (few composite
    // queries: high compression ratios, compressed heads) is cut into wavefronts of 32 rows instead, twice as many
    // workgroups of half the length, which the causal triangle needs to balance.
    int64_t nblk = 0;
    for (g.QT = 2; g.QT >= 1; --g.QT) {
        const int rows_per_tile = 32 * g.QT * g.RC;
        g.n_tiles = 0;
        for (int b = 0; b < a.st.num_seqs; ++b) {
            int lq = a.cu_cq[b + 1] - a.cu_cq[b];
            g.n_tiles += (lq + rows_per_tile - 1) / rows_per_tile;
        }
        nblk = (int64_t)a.n_heads_kv * g.GS * g.n_tiles;
        const bool want_one = a.tiles == 1 || (a.tiles == 0 && nblk < 4 * (int64_t)a.n_cu);
        if (!(want_one && g.QT == 2 && proxy_has_single_tile(a.head_dim, a.S / a.c_q))) break;
    }
    if (nblk == 0) return hipSuccess;
    dim3 grid((unsigned)nblk);
    const bool rowsums = a.u != nullptr;                    // one-sweep form: U and the row weights instead of Score
    if (rowsums && a.w == nullptr) return hipErrorInvalidValue;
    switch (a.head_dim) {
        case 64: return rowsums ? proxy_rowsums_dispatch_d64(a, g, grid, stream) : proxy_dispatch_d64(a, g, grid, stream);
        case 128: return rowsums ? proxy_rowsums_dispatch_d128(a, g, grid, stream) : proxy_dispatch_d128(a, g, grid, stream);
        case 256: return rowsums ? proxy_rowsums_dispatch_d256(a, g, grid, stream) : proxy_dispatch_d256(a, g, grid, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace us
