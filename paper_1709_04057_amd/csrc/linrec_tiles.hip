// Instantiates the tile kernels for ONE tile shape; compiled once per shape with
// -DLINREC_TILE_ID=<id> so that the shapes build in parallel.
#include "linrec_device.h"

#include <algorithm>
#include <map>
#include <mutex>
#include <utility>

#ifndef LINREC_TILE_ID
#error "compile with -DLINREC_TILE_ID=<id>"
#endif

namespace linrec {

// Persistent workgroups of `kernel` to launch on the current device: compute units x workgroups per unit.
// cap_per_cu > 0 asks for at most that many per unit, < 0 for as many as fit; 0 is the library's own
// choice, 8 wavefronts per unit (two per SIMD): one workgroup of 512 threads or two of 256.  More
// resident tiles than it takes to keep the memory system busy only lengthen a tile's life -- bytes in
// flight over bandwidth -- and with it the start and the end of a launch, when that life is spent at
// less than full bandwidth (measured on an MI355X: 2-10 % on launches of a few hundred microseconds for
// the shapes of which three or more would fit a unit, nothing lost anywhere).
static int64_t resident_capacity(const void *kernel, int threads, int cap_per_cu)
{
    static std::mutex mu;
    static std::map<std::pair<int, const void *>, int64_t> cache;
    int dev = 0;
    (void)hipGetDevice(&dev);
    std::lock_guard<std::mutex> lock(mu);
    static std::map<int, int> cu_count;
    auto it = cache.find({dev, kernel});
    if (it == cache.end()) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess || per_cu < 1) per_cu = 1;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        cu_count[dev] = cus;
        it = cache.emplace(std::make_pair(dev, kernel), (int64_t)per_cu).first;
    }
    int64_t want = it->second;
    if (cap_per_cu > 0) want = cap_per_cu;
    else if (cap_per_cu == 0) want = std::max(1, 8 / std::max(1, threads / 64));
    return std::min(want, it->second) * cu_count[dev];
}

template <class G>
static hipError_t launch_for(Kind kind, bool bwd, bool hp_late, int form, bool bf16, const Args &A, hipStream_t s)
{
    const dim3 grid((unsigned)(A.K * A.G)), block(G::THREADS);
    // Which kernels exist for this shape: those of the entry-point families the build selects it for
    // (bit LINREC_ENTRY_* of tile_families; the three-phase kernels belong to the plain fp32 family).
    constexpr unsigned kFam = tile_families(LINREC_TILE_ID);
    constexpr bool kHasF32 = kFam >> 0 & 1, kHasGated = kFam >> 1 & 1, kHasLstm = kFam >> 2 & 1, kHasBf16 = kFam >> 3 & 1,
                   kHasGated16 = kFam >> 4 & 1, kHasLstm16 = kFam >> 5 & 1;
    if (form < FORM_PLAIN || form > FORM_LSTM) return hipErrorInvalidValue;
    if ((form != FORM_PLAIN || bf16) && kind != KIND_LOOKBACK && kind != KIND_WALK) return hipErrorInvalidValue;
    void (*kern)(const Args) = nullptr;
    if constexpr (kHasF32) {
        if (form == FORM_PLAIN && !bf16) {
            switch (kind) {
            case KIND_REDUCE:
                if (bwd) hipLaunchKernelGGL((k_reduce<G, true>), grid, block, 0, s, A);
                else hipLaunchKernelGGL((k_reduce<G, false>), grid, block, 0, s, A);
                return hipGetLastError();
            case KIND_FIXUP:
                if (bwd) hipLaunchKernelGGL((k_fixup<G, true>), grid, block, 0, s, A);
                else hipLaunchKernelGGL((k_fixup<G, false>), grid, block, 0, s, A);
                return hipGetLastError();
            case KIND_WALK: kern = bwd ? k_walk<G, true> : k_walk<G, false>; break;
            case KIND_LOOKBACK:
                kern = !bwd ? k_lookback<G, false, false> : hp_late ? k_lookback<G, true, true> : k_lookback<G, true, false>;
                break;
            }
        }
    }
    const bool walk = kind == KIND_WALK;
    if constexpr (kHasBf16) {
        using GB = Geo<G::VEC, G::R, G::WC, G::WT, IO_BF16>;
        if (bf16 && form == FORM_PLAIN)
            kern = walk ? (bwd ? k_walk<GB, true> : k_walk<GB, false>)
                        : (bwd ? k_lookback<GB, true, false> : k_lookback<GB, false, false>);
    }
    if constexpr (kHasGated) {
        if (form == FORM_GATED && !bf16)
            kern = walk ? (bwd ? k_walk<G, true, FORM_GATED> : k_walk<G, false, FORM_GATED>)
                        : (bwd ? k_lookback<G, true, true, FORM_GATED> : k_lookback<G, false, false, FORM_GATED>);
    }
    if constexpr (kHasLstm) {
        if (form == FORM_LSTM && !bf16)
            kern = walk ? (bwd ? k_walk<G, true, FORM_LSTM> : k_walk<G, false, FORM_LSTM>)
                        : (bwd ? k_lookback<G, true, true, FORM_LSTM> : k_lookback<G, false, false, FORM_LSTM>);
    }
    if constexpr (kHasGated16) {
        using GW = Geo<G::VEC, G::R, G::WC, G::WT, IO_BF16W>;
        if (form == FORM_GATED && bf16)
            kern = walk ? (bwd ? k_walk<GW, true, FORM_GATED> : k_walk<GW, false, FORM_GATED>)
                        : (bwd ? k_lookback<GW, true, true, FORM_GATED> : k_lookback<GW, false, false, FORM_GATED>);
    }
    if constexpr (kHasLstm16) {
        using GW = Geo<G::VEC, G::R, G::WC, G::WT, IO_BF16W>;
        if (form == FORM_LSTM && bf16)
            kern = walk ? (bwd ? k_walk<GW, true, FORM_LSTM> : k_walk<GW, false, FORM_LSTM>)
                        : (bwd ? k_lookback<GW, true, true, FORM_LSTM> : k_lookback<GW, false, false, FORM_LSTM>);
    }
    if (!kern) return hipErrorInvalidValue;
    if (walk) {  // one workgroup per column group
        hipLaunchKernelGGL(kern, dim3((unsigned)A.G), block, 0, s, A);
        return hipGetLastError();
    }
    // persistent workgroups: as many as the device holds at once, never more than there are tiles
    const int64_t cap = resident_capacity(reinterpret_cast<const void *>(kern), G::THREADS, A.grid_cap);
    const dim3 pgrid((unsigned)(A.persistent ? std::min<int64_t>(A.K * A.G, cap) : A.K * A.G));
    // With a workgroup for every tile nobody needs to ask for a second one (and wait for the answer
    // before it can end): a few microseconds off a small problem.
    Args L = A;
    if ((int64_t)pgrid.x == A.K * A.G) L.persistent = 0;
    // Workgroups that start together load, scan and store together, and the memory system idles while
    // they all scan.  When the launch is at least two rounds long, every other workgroup of the first
    // round starts a little late (the kernel sleeps, see there).
    const int64_t first_round = std::min<int64_t>(A.K * A.G, cap);
    L.stagger_n = A.K * A.G >= 2 * first_round ? (int32_t)first_round : 0;
    hipLaunchKernelGGL(kern, pgrid, block, 0, s, L);
    return hipGetLastError();
}

#define LINREC_CAT2(a, b) a##b
#define LINREC_CAT(a, b) LINREC_CAT2(a, b)
#define X(ID, VEC, R, WC, WT)                                                                        \
    template <int I> struct TileOf##ID { using type = Geo<VEC, R, WC, WT>; };
LINREC_TILES(X)
#undef X
#define LINREC_TILE_TYPE LINREC_CAT(TileOf, LINREC_TILE_ID)<0>::type

hipError_t LINREC_CAT(launch_tile_, LINREC_TILE_ID)(Kind kind, bool bwd, bool hp_late, int form, bool bf16,
                                                    const Args &A, hipStream_t s)
{
    return launch_for<LINREC_TILE_TYPE>(kind, bwd, hp_late, form, bf16, A, s);
}

}  // namespace linrec
