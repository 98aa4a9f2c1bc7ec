// Instantiates the tile kernels for ONE tile shape; compiled once per shape with
// -DLINREC_TILE_ID=<id> so that the shapes build in parallel.
#include "linrec_device.h"

#ifndef LINREC_TILE_ID
#error "compile with -DLINREC_TILE_ID=<id>"
#endif

namespace linrec {

template <class G>
static hipError_t launch_for(Kind kind, bool bwd, bool hp_late, const Args &A, hipStream_t s)
{
    const dim3 grid((unsigned)(A.K * A.G)), block(G::THREADS);
    switch (kind) {
    case KIND_REDUCE:
        if (bwd) hipLaunchKernelGGL((k_reduce<G, true>), grid, block, 0, s, A);
        else hipLaunchKernelGGL((k_reduce<G, false>), grid, block, 0, s, A);
        break;
    case KIND_FIXUP:
        if (bwd) hipLaunchKernelGGL((k_fixup<G, true>), grid, block, 0, s, A);
        else hipLaunchKernelGGL((k_fixup<G, false>), grid, block, 0, s, A);
        break;
    case KIND_LOOKBACK:
        if (!bwd) hipLaunchKernelGGL((k_lookback<G, false, false>), grid, block, 0, s, A);
        else if (hp_late) hipLaunchKernelGGL((k_lookback<G, true, true>), grid, block, 0, s, A);
        else hipLaunchKernelGGL((k_lookback<G, true, false>), grid, block, 0, s, A);
        break;
    }
    return hipGetLastError();
}

#define LINREC_CAT2(a, b) a##b
#define LINREC_CAT(a, b) LINREC_CAT2(a, b)
#define X(ID, VEC, R, WC, WT)                                                                        \
    template <int I> struct TileOf##ID { using type = Geo<VEC, R, WC, WT>; };
LINREC_TILES(X)
#undef X
#define LINREC_TILE_TYPE LINREC_CAT(TileOf, LINREC_TILE_ID)<0>::type

hipError_t LINREC_CAT(launch_tile_, LINREC_TILE_ID)(Kind kind, bool bwd, bool hp_late, const Args &A, hipStream_t s)
{
    return launch_for<LINREC_TILE_TYPE>(kind, bwd, hp_late, A, s);
}

}  // namespace linrec
