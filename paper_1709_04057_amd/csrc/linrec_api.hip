// C ABI of liblinrec (see include/linrec.h): argument checks, choice of variant and tile shape,
// the cached per-(device, stream) workspace, and the kernel launches.
#include "linrec.h"
#include "linrec_launch.h"

#include <stddef.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <initializer_list>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

namespace linrec {

#define X(ID, VEC, R, WC, WT) hipError_t launch_tile_##ID(Kind, bool, bool, int, bool, const Args &, hipStream_t);
LINREC_TILES(X)
#undef X

struct TileTable {  // indexed by id; unassigned ids hold zeros
    TileDesc t[MAX_TILE_ID + 1];
    constexpr TileTable() : t{}
    {
#define X(ID, VEC, R, WC, WT) t[ID] = TileDesc{VEC, R, WC, WT};
        LINREC_TILES(X)
#undef X
    }
};
static constexpr TileTable kTable{};

struct FamilyTable {  // indexed by id: the families this build has kernels of that shape for
    unsigned m[MAX_TILE_ID + 1];
    constexpr FamilyTable() : m{}
    {
        for (int id = 0; id <= MAX_TILE_ID; ++id) m[id] = tile_families(id);
    }
};
static constexpr FamilyTable kFamilies{};

bool tile_has(int id, int family) { return id >= 1 && id <= MAX_TILE_ID && (kFamilies.m[id] >> family & 1u); }
bool tile_exists(int id) { return id >= 1 && id <= MAX_TILE_ID && kFamilies.m[id] != 0; }
const TileDesc &tile_desc(int id) { return kTable.t[id]; }

hipError_t launch_tile_kernel(int id, Kind kind, bool bwd, bool hp_late, int form, bool bf16, const Args &A, hipStream_t s)
{
    switch (id) {
#define X(ID, VEC, R, WC, WT) \
    case ID: return launch_tile_##ID(kind, bwd, hp_late, form, bf16, A, s);
        LINREC_TILES(X)
#undef X
    default: return hipErrorInvalidValue;
    }
}

namespace {

// ---- options: one set per host thread ------------------------------------------------------
// (A call reads the options of the thread that makes it, so a thread that changes them -- a sweep, the
// tuner -- cannot change the plan of a call another thread is making.)
struct Options {
    int64_t variant = LINREC_VARIANT_AUTO;
    int64_t tile = 0;
    int64_t chunk_tiles = 0;
    int64_t spin_limit = 1 << 22;
    int64_t hp_late = -1;  // -1 automatic
    int64_t taper = -1;  // -1 automatic
    int64_t grid_cap = 0;
    int64_t stagger = 3;
    int64_t persistent = -1;  // -1 automatic (persistent)
    // test aids (see linrec.h): what a fresh look-back workspace is filled with, and a stored epoch to
    // plant into the workspace of the thread's next single-pass call (-1: none)
    int64_t test_fill = 0;
    int64_t test_epoch = -1;
    Options()
    {
        if (const char *v = getenv("LINREC_VARIANT")) {
            if (!strcmp(v, "threephase")) variant = LINREC_VARIANT_THREEPHASE;
            else if (!strcmp(v, "lookback")) variant = LINREC_VARIANT_LOOKBACK;
            else if (!strcmp(v, "serial")) variant = LINREC_VARIANT_SERIAL;
            else if (!strcmp(v, "walk")) variant = LINREC_VARIANT_WALK;
        }
        if (const char *v = getenv("LINREC_TILE")) {
            const long t = strtol(v, nullptr, 10);
            if (t == 0 || tile_exists((int)t)) tile = t;
        }
    }
};
Options &opts()
{
    static thread_local Options o;
    return o;
}

// A plan handed to the calls of this thread explicitly (the tuner times its candidates this way):
// takes the place of the variant / tile / persistent / taper options while `active`.
struct ForcedPlan {
    bool active = false;
    int variant = LINREC_VARIANT_LOOKBACK, tile = 0, persistent = -1, taper = 0;
};
ForcedPlan &forced()
{
    static thread_local ForcedPlan f;
    return f;
}

thread_local char g_hip_error[256] = "";  // per host thread, like the options: the thread that got LINREC_ERR_HIP reads its own
unsigned long long *g_trace = nullptr;  // set by linrec_debug_trace (trace builds)
int hip_fail(hipError_t e, const char *what)
{
    snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", what, hipGetErrorString(e));
    return LINREC_ERR_HIP;
}

// ---- workspace -----------------------------------------------------------------------------
// One per (device, stream).  The look-back words live in their own allocation that nothing else
// ever writes, because a stale word is told from a fresh one only by its epoch.
// A block that has been handed to a launch is never freed before linrec_release_workspace(): when a
// larger problem arrives a new block is allocated and the old one is retired, so kernels still queued
// on the stream, and launches recorded in a HIP graph, keep pointing at memory that exists.
struct Workspace {
    // look-back: [LookbackHeader, padded to kLbHeader bytes][3*K*C u64 words]
    void *lb = nullptr;
    size_t lb_bytes = 0;
    unsigned long long calls_since_clear = 0;
    // three-phase: aggP, aggS, carry, each K*C fp64
    void *tp = nullptr;
    size_t tp_bytes = 0;
    std::vector<void *> retired_lb, retired_tp;
};
std::mutex g_mu;
std::map<std::pair<int, hipStream_t>, Workspace> g_ws;

constexpr size_t kLbHeader = 512;
static_assert(sizeof(LookbackHeader) <= kLbHeader, "header must fit its slot");

// Grows the block if needed: a new allocation (at least half as large again as the old one, so that
// the retired blocks of a stream whose problems keep growing add up to less than twice the live one),
// filled on the stream.  Nothing waits: the old block stays valid for whatever still uses it.  Look-back
// blocks start as zeros (header and words: the kernels' epoch convention makes that a valid start), or,
// for the reuse tests, with the words holding LINREC_OPT_TEST_FILL.
int ensure(Workspace &ws, void **buf, size_t *have, size_t need, bool lookback, hipStream_t s)
{
    if (*have >= need) return LINREC_OK;
    hipError_t e;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone) return LINREC_ERR_CAPTURE;
    need = std::max(need, *have + *have / 2);
    need = (need + ((size_t)1 << 20) - 1) & ~(((size_t)1 << 20) - 1);
    void *fresh = nullptr;
    if ((e = hipMalloc(&fresh, need)) != hipSuccess) return hip_fail(e, "hipMalloc(workspace)");
    if (lookback) {
        e = launch_fill((float *)fresh, 0.0f, (int64_t)(kLbHeader / sizeof(float)), s);
        uint32_t bits = (uint32_t)opts().test_fill;
        float pattern;
        memcpy(&pattern, &bits, sizeof pattern);
        if (e == hipSuccess)
            e = launch_fill((float *)((char *)fresh + kLbHeader), pattern, (int64_t)((need - kLbHeader) / sizeof(float)), s);
        if (e != hipSuccess) {
            (void)hipFree(fresh);
            return hip_fail(e, "launch(fill workspace)");
        }
    }
    if (*buf) (lookback ? ws.retired_lb : ws.retired_tp).push_back(*buf);
    *buf = fresh;
    *have = need;
    if (lookback) ws.calls_since_clear = 0;
    return LINREC_OK;
}

// Look-back workspace for callers that cannot allocate (linrec_forward_noalloc): one array in the
// library's device image, so every GPU the library runs on holds its own copy, zero-initialised when
// the image is loaded -- which is a valid start, as for an allocated block.  Host code never uses the
// array's name for anything but the address query below; kernels get the queried address as an argument.
constexpr size_t kScratchBytes = LINREC_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned long long g_noalloc_scratch[kScratchBytes / sizeof(unsigned long long)];
constexpr int kMaxDevices = 64;
struct ScratchOfDevice {
    void *ptr = nullptr;  // this device's address of g_noalloc_scratch
    unsigned long long calls_since_clear = 0;
};
ScratchOfDevice g_scratch[kMaxDevices];  // guarded by g_mu

// The address of the current device's scratch array (queried once per device, with that device current).
int scratch_of_current_device(int dev, ScratchOfDevice **out)
{
    if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice, "linrec_forward_noalloc: device index");
    ScratchOfDevice &sd = g_scratch[dev];
    if (!sd.ptr) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_noalloc_scratch));
        if (e != hipSuccess || !p) return hip_fail(e != hipSuccess ? e : hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
        sd.ptr = p;
    }
    *out = &sd;
    return LINREC_OK;
}

// Compute units of a device (256 on an MI355X; also what is assumed when the device cannot be asked).
int compute_units(int dev)
{
    static std::mutex mu;
    static std::map<int, int> cache;
    std::lock_guard<std::mutex> lock(mu);
    auto it = cache.find(dev);
    if (it != cache.end()) return it->second;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    return cache[dev] = cus;
}

bool aligned16(const void *p) { return p == nullptr || ((uintptr_t)p & 15u) == 0; }

// Widest per-thread access (columns) that C and the pointers' alignment allow: 4, 2 or 1.
int max_vec(int64_t C, std::initializer_list<const void *> ptrs)
{
    uintptr_t bits = (uintptr_t)(C * 4);
    for (const void *p : ptrs) bits |= (uintptr_t)p;
    return (bits & 15u) == 0 ? 4 : (bits & 7u) == 0 ? 2 : 1;
}

// The same for bf16 storage: four columns are 8 bytes, two are 4.
int max_vec_bf16(int64_t C, std::initializer_list<const void *> ptrs)
{
    uintptr_t bits = (uintptr_t)(C * 2);
    for (const void *p : ptrs) bits |= (uintptr_t)p;
    return (bits & 7u) == 0 ? 4 : (bits & 3u) == 0 ? 2 : 1;
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- static plans --------------------------------------------------------------------------
// What a first call on a shape gets: per entry-point family, pass and problem size the variant and tile
// shape that measured fastest on an MI355X, from a table written by plan_sweep.py (a grid of powers of
// two in T, half octaves in C; per cell the best shape among those whose accesses are 1, 2 or 4 columns
// wide, and the walk's shape where the walk was ahead).  A problem between grid points takes the plan of
// the nearest one (in ratio); one smaller or larger than everything measured at its width, the nearest
// measured size.  After a change of driver, compiler or clocks the table is measured again, not edited.
#include "linrec_plan_table.inc"
static_assert(sizeof kPlanCells / sizeof kPlanCells[0] == LINREC_ENTRY_LSTM_CELL_BF16 + 1, "one table per family");
static_assert(LINREC_ENTRY_PLAIN == 0 && LINREC_ENTRY_GILR == 1 && LINREC_ENTRY_LSTM_CELL == 2 && LINREC_ENTRY_BF16 == 3 &&
                  LINREC_ENTRY_GILR_BF16 == 4 && LINREC_ENTRY_LSTM_CELL_BF16 == 5,
              "the family masks of tile_families() are indexed by LINREC_ENTRY_*");

struct StaticPlan {
    int lookback;  // the single pass's tile shape (0: the family has no kernel at this access width)
    int walk;      // the walk's, where the walk is the better variant; else 0
    int taper;     // eighths of the single pass's last round cut into shorter tiles, where that measured ahead
};
StaticPlan static_plan(int family, bool bwd, int64_t T, int64_t C, int vec)
{
    const int w = vec >= 4 ? 2 : vec >= 2 ? 1 : 0;
    int ci = 0;  // nearest column count of the grid, in ratio
    for (int i = 1; i < kPlanNc; ++i)
        if ((double)C * C >= (double)kPlanC[i - 1] * kPlanC[i]) ci = i;
    int lt = kPlanLtMin;  // nearest power of two
    while (lt < kPlanLtMax && (double)T * T >= (double)((int64_t)1 << lt) * (double)((int64_t)2 << lt)) ++lt;
    const int nt = kPlanLtMax - kPlanLtMin + 1;
    for (int d = 0; d < nt; ++d) {
        for (const int l : {lt - d, lt + d}) {
            if (l < kPlanLtMin || l > kPlanLtMax) continue;
            const PlanCell &c = kPlanCells[family][bwd ? 1 : 0][l - kPlanLtMin][ci];
            // (the walk keeps one workgroup per column group busy for the whole sequence: a plan measured on a
            // much shorter or longer sequence says nothing about it)
            if (c.lookback[w] && tile_has(c.lookback[w], family))
                return StaticPlan{c.lookback[w], (d <= 1 && tile_has(c.walk[w], family)) ? c.walk[w] : 0,
                                  d <= 1 ? c.taper[w] : 0};
        }
    }
    // nothing measured at this width: any shape the family has
    for (int id = 1; id <= MAX_TILE_ID; ++id)
        if (tile_has(id, family) && kTable.t[id].vec <= vec) return StaticPlan{id, 0, 0};
    return StaticPlan{0, 0, 0};
}

int entry_family(int form, bool bf16)
{
    if (form == FORM_GATED) return bf16 ? LINREC_ENTRY_GILR_BF16 : LINREC_ENTRY_GILR;
    if (form == FORM_LSTM) return bf16 ? LINREC_ENTRY_LSTM_CELL_BF16 : LINREC_ENTRY_LSTM_CELL;
    return bf16 ? LINREC_ENTRY_BF16 : LINREC_ENTRY_PLAIN;
}
int entry_form(int entry_point)
{
    return (entry_point == LINREC_ENTRY_GILR || entry_point == LINREC_ENTRY_GILR_BF16)             ? FORM_GATED
           : (entry_point == LINREC_ENTRY_LSTM_CELL || entry_point == LINREC_ENTRY_LSTM_CELL_BF16) ? FORM_LSTM
                                                                                                   : FORM_PLAIN;
}
bool entry_bf16(int entry_point)
{
    return entry_point == LINREC_ENTRY_BF16 || entry_point == LINREC_ENTRY_GILR_BF16 ||
           entry_point == LINREC_ENTRY_LSTM_CELL_BF16;
}

struct Plan {
    int variant, tile;
    bool hp_late;
    int persistent;  // -1: not decided by the plan
    int taper;       // eighths of the last round cut into shorter tiles (LINREC_OPT_TAPER, or what tuning found)
};

// Plans found by linrec_tune, keyed by (device, T, C, pass).  Guarded by g_tuned_mu.
struct TunedKey {
    int dev;
    int64_t T, C;
    bool bwd;
    int family;  // LINREC_ENTRY_*
    bool operator<(const TunedKey &o) const
    {
        if (dev != o.dev) return dev < o.dev;
        if (T != o.T) return T < o.T;
        if (C != o.C) return C < o.C;
        if (bwd != o.bwd) return bwd < o.bwd;
        return family < o.family;
    }
};
struct TunedPlan {
    int tile, persistent, variant;
    int taper = 0;
};
std::mutex g_tuned_mu;
std::map<TunedKey, TunedPlan> g_tuned;

// Picks variant and tile, honouring the options where they apply to this problem.
Plan make_plan(int64_t T, int64_t C, int vec, bool bwd, int form = FORM_PLAIN, bool bf16 = false)
{
    const bool gated = form != FORM_PLAIN;
    Plan p;
    // what the caller asked for: the thread's options, or the plan a tuner forces on this thread's calls
    const ForcedPlan &fp = forced();
    const int want_variant = fp.active ? fp.variant : (int)opts().variant;
    p.variant = want_variant;
    if (p.variant == LINREC_VARIANT_AUTO) p.variant = LINREC_VARIANT_LOOKBACK;
    p.tile = fp.active ? fp.tile : (int)opts().tile;
    p.persistent = fp.active ? fp.persistent : (int)opts().persistent;
    p.taper = fp.active ? fp.taper : (int)opts().taper;
    if (p.tile == 0 && p.variant == LINREC_VARIANT_LOOKBACK) {  // a pinned or tuned plan, if there is one for this shape
        int dev = 0;
        if (hipGetDevice(&dev) == hipSuccess) {
            std::lock_guard<std::mutex> lock(g_tuned_mu);
            auto it = g_tuned.find(TunedKey{dev, T, C, bwd, entry_family(form, bf16)});
            if (it != g_tuned.end() && (it->second.variant == LINREC_VARIANT_LOOKBACK || want_variant == LINREC_VARIANT_AUTO)) {
                p.tile = it->second.tile;
                p.variant = it->second.variant;
                if (p.persistent < 0) p.persistent = it->second.persistent;
                if (p.taper < 0) p.taper = it->second.taper;
            }
        }
    }
    // What the options, a pinned or a tuned plan name must be a shape this family has kernels for, with
    // accesses no wider than this call's alignment allows; else the static plan decides.
    const int family = entry_family(form, bf16);
    if (p.tile && (!tile_has(p.tile, family) || kTable.t[p.tile].vec > vec)) p.tile = 0;
    if (!p.tile) {
        const StaticPlan sp = static_plan(family, bwd, T, C, vec);
        if (want_variant == LINREC_VARIANT_AUTO && sp.walk) {  // short, wide problems take the walk
            p.variant = LINREC_VARIANT_WALK;
            p.tile = sp.walk;
        } else {
            // (the walk asked for by option without a shape: the shape the table has for it, else the single pass's)
            p.tile = (p.variant == LINREC_VARIANT_WALK && sp.walk) ? sp.walk : sp.lookback;
            if (p.taper < 0 && p.tile == sp.lookback) p.taper = sp.taper;
        }
    }
    if (p.taper < 0) p.taper = 0;
    // bf16 tensors that are not even 4-byte aligned, or an odd number of columns: the serial kernel
    // (the gated forms have one-column shapes with 2-byte accesses for those)
    if ((bf16 && !gated && vec < 2) || !p.tile) {
        p.variant = LINREC_VARIANT_SERIAL;
        for (int id = 1; id <= MAX_TILE_ID && !p.tile; ++id)  // (a plan always names a shape of its family)
            if (tile_has(id, family)) p.tile = id;
    }
    const TileDesc &d = kTable.t[p.tile];
    // per-thread byte offsets inside a tile are 32-bit, tickets of a call are 31-bit
    const int64_t G = ceil_div(C, d.cols()), K = ceil_div(T, d.rows());
    // (the short tiles that end a look-back sequence can raise the tile count, by less than 4x)
    if (((int64_t)d.rows() * C + d.cols()) * 4 >= ((int64_t)1 << 32) || 4 * K * G >= ((int64_t)1 << 31))
        p.variant = LINREC_VARIANT_SERIAL;
    p.hp_late = opts().hp_late > 0;
    return p;
}

// Tiles along time of a single-pass launch: K1 of full height, then K2 of half height, the rest a quarter
// (the tapered tail; K2 = 0 and K = K1 without it).
struct TimeTiles {
    int64_t K, K1, K2;
};
TimeTiles time_tiles(int64_t T, int64_t G, const TileDesc &d, int taper, int dev)
{
    const int64_t tiles_t = ceil_div(T, d.rows());
    TimeTiles tt{tiles_t, tiles_t, 0};
    if (taper && d.r % 4 == 0 && d.r >= 8) {
        const int64_t rows = d.rows();
        const int64_t full = T / rows;                                   // complete full-height tiles
        // full tiles per chain that are in flight at once; `taper` eighths of them are cut up
        // (a launch holds eight wavefronts per compute unit)
        const int64_t resident = (int64_t)compute_units(dev) * std::max(1, 8 / std::max(1, d.threads() / 64));
        const int64_t round = ceil_div(resident, G);
        const int64_t taper_tiles = std::min(full / 2, (round * taper + 7) / 8);
        if (taper_tiles > 0) {
            tt.K1 = full - taper_tiles;
            const int64_t left = T - tt.K1 * rows;                        // rows in the tapered region
            tt.K2 = (left / 2) / (rows / 2);
            const int64_t rest = left - tt.K2 * (rows / 2);
            tt.K = tt.K1 + tt.K2 + ceil_div(rest, rows / 4);
        }
    }
    return tt;
}

size_t lookback_bytes(int64_t K, int64_t C) { return kLbHeader + 3 * (size_t)K * (size_t)C * sizeof(unsigned long long); }

// Hands a single-pass launch its look-back block: clears it when its tags are about to come round, and
// plants the stored epoch a reuse test asked for.  `calls` is the block's count of calls since it was
// last cleared.
int prepare_lookback(Args &A, void *block, size_t bytes, unsigned long long *calls, hipStream_t s)
{
    hipError_t e;
    // The 31-bit epoch wraps after 2^31 - 1 calls; long before that, forget every stale word so that a
    // slot untouched for that long cannot be mistaken for a fresh one.
    if (++*calls >= (1ull << 30)) {
        if ((e = launch_fill((float *)((char *)block + kLbHeader), 0.0f, (int64_t)((bytes - kLbHeader) / sizeof(float)), s)) != hipSuccess)
            return hip_fail(e, "launch(fill)");
        *calls = 0;
    }
    if (opts().test_epoch >= 0) {  // test aid: the next clear comes two calls from now, before the planted epoch can wrap
        if ((e = launch_set_epoch((LookbackHeader *)block, (uint32_t)opts().test_epoch, s)) != hipSuccess)
            return hip_fail(e, "launch(set_epoch)");
        *calls = (1ull << 30) - 2;
        opts().test_epoch = -1;
    }
    A.hdr = (LookbackHeader *)block;
    A.lbAgg = (unsigned long long *)((char *)block + kLbHeader);
    return LINREC_OK;
}

// gated: the form of Section 3.1 (activations applied in the kernel); it exists as the single-pass and
// walk kernels of the tile shapes with a multiple of 8 (or fewer than 8) rows per thread, and as the
// serial kernel.  noalloc: the look-back words live in the device-resident scratch array instead of a
// cached allocation, and nothing is allocated (LINREC_ERR_SCRATCH when they do not fit).
int run(Args A, bool bwd, int vec, hipStream_t s, int form = FORM_PLAIN, bool bf16 = false, bool noalloc = false)
{
    const bool gated = form != FORM_PLAIN;
    Plan plan = make_plan(A.T, A.C, vec, bwd, form, bf16);
    if ((gated || bf16 || noalloc) && plan.variant == LINREC_VARIANT_THREEPHASE) plan.variant = LINREC_VARIANT_LOOKBACK;
    hipError_t e;
    if (plan.variant == LINREC_VARIANT_SERIAL) {
        if ((e = launch_serial(A, bwd, form, bf16, s)) != hipSuccess) return hip_fail(e, "launch(serial)");
        return LINREC_OK;
    }
    const TileDesc &d = kTable.t[plan.tile];
    A.G = (int32_t)ceil_div(A.C, d.cols());
    const int64_t tiles_t = ceil_div(A.T, d.rows());

    if (plan.variant == LINREC_VARIANT_WALK) {  // one kernel, no workspace
        A.M = 1;
        A.K = tiles_t;
        if ((e = launch_tile_kernel(plan.tile, KIND_WALK, bwd, false, form, bf16, A, s)) != hipSuccess)
            return hip_fail(e, "launch(walk)");
        return LINREC_OK;
    }

    int dev = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return hip_fail(e, "hipGetDevice");

    if (plan.variant == LINREC_VARIANT_THREEPHASE) {
        // enough chunks to fill the GPU several times over, few enough that phase 2 stays small
        int64_t M = opts().chunk_tiles;
        if (M <= 0) M = ceil_div(tiles_t * A.G, 4096);
        if (M < 1) M = 1;
        if (M > (1 << 20)) M = 1 << 20;
        A.M = (int32_t)M;
        A.K = ceil_div(tiles_t, M);
        const size_t kc = (size_t)A.K * (size_t)A.C;
        {
            std::lock_guard<std::mutex> lock(g_mu);  // (the workspace table only; launches run unlocked)
            Workspace &ws = g_ws[std::make_pair(dev, s)];
            const int rc = ensure(ws, &ws.tp, &ws.tp_bytes, 3 * kc * sizeof(double), false, s);
            if (rc != LINREC_OK) return rc;
            A.aggP = (double *)ws.tp;
        }
        A.aggS = A.aggP + kc;
        A.carry = A.aggS + kc;
        if ((e = launch_tile_kernel(plan.tile, KIND_REDUCE, bwd, false, FORM_PLAIN, false, A, s)) != hipSuccess)
            return hip_fail(e, "launch(reduce)");
        if ((e = launch_scan_summaries(A.aggP, A.aggS, bwd ? nullptr : A.h0, A.carry, A.K, A.C, s)) != hipSuccess)
            return hip_fail(e, "launch(scan_summaries)");
        if ((e = launch_tile_kernel(plan.tile, KIND_FIXUP, bwd, false, FORM_PLAIN, false, A, s)) != hipSuccess)
            return hip_fail(e, "launch(fixup)");
        return LINREC_OK;
    }

    // Single pass with look-back.  The rows that the last "round" of resident workgroups would take
    // as full tiles are cut into half- and quarter-height tiles instead when the plan says so (see k_lookback).
    A.M = 1;
    const TimeTiles tt = time_tiles(A.T, A.G, d, plan.taper, dev);
    A.K = tt.K;
    A.K1 = tt.K1;
    A.K2 = tt.K2;
    const size_t need = lookback_bytes(A.K, A.C);
    {
        std::lock_guard<std::mutex> lock(g_mu);
        int rc;
        if (noalloc) {
            if (need > kScratchBytes) return LINREC_ERR_SCRATCH;
            ScratchOfDevice *sd = nullptr;
            if ((rc = scratch_of_current_device(dev, &sd)) != LINREC_OK) return rc;
            rc = prepare_lookback(A, sd->ptr, kScratchBytes, &sd->calls_since_clear, s);
        } else {
            Workspace &ws = g_ws[std::make_pair(dev, s)];
            if ((rc = ensure(ws, &ws.lb, &ws.lb_bytes, need, true, s)) != LINREC_OK) return rc;
            rc = prepare_lookback(A, ws.lb, ws.lb_bytes, &ws.calls_since_clear, s);
        }
        if (rc != LINREC_OK) return rc;
    }
    A.spin_limit = (uint32_t)opts().spin_limit;
    A.persistent = plan.persistent < 0 ? 1 : plan.persistent;
    // Workgroups per compute unit: eight wavefronts for the plain fp32 recurrence (see the launch code); the
    // other families compute activations per element or hold half the bytes per register and keep as many
    // workgroups resident as fit, which measures 5-18 % faster for them.
    A.grid_cap = opts().grid_cap != 0 ? (int32_t)opts().grid_cap : (form == FORM_PLAIN && !bf16) ? 0 : -1;
    A.stagger = (int32_t)opts().stagger;
    A.stagger_n = 0;
    A.trace = g_trace;
    if ((e = launch_tile_kernel(plan.tile, KIND_LOOKBACK, bwd, plan.hp_late, form, bf16, A, s)) != hipSuccess)
        return hip_fail(e, "launch(lookback)");
    return LINREC_OK;
}

}  // namespace
}  // namespace linrec

using namespace linrec;

extern "C" int linrec_forward(const float *lambda, const float *x, const float *h0, float *h_out, int64_t T, int64_t B,
                              int64_t n, void *stream)
{
    const int rc = linrec_validate_forward(lambda, x, h0, h_out, T, B, n);
    if (rc != LINREC_OK) return rc;
    const int64_t C = B * n;
    if (T == 0 || C == 0) return LINREC_OK;
    Args A;
    memset(&A, 0, sizeof A);
    A.a = lambda;
    A.b = x;
    A.h0 = h0;
    A.out0 = h_out;
    A.T = T;
    A.C = C;
    return run(A, false, max_vec(C, {lambda, x, h0, h_out}), (hipStream_t)stream);
}

extern "C" int linrec_forward_noalloc(const float *lambda, const float *x, const float *h0, float *h_out, int64_t T,
                                      int64_t B, int64_t n, void *stream)
{
    const int rc = linrec_validate_forward(lambda, x, h0, h_out, T, B, n);
    if (rc != LINREC_OK) return rc;
    const int64_t C = B * n;
    if (T == 0 || C == 0) return LINREC_OK;
    Args A;
    memset(&A, 0, sizeof A);
    A.a = lambda;
    A.b = x;
    A.h0 = h0;
    A.out0 = h_out;
    A.T = T;
    A.C = C;
    return run(A, false, max_vec(C, {lambda, x, h0, h_out}), (hipStream_t)stream, FORM_PLAIN, false, /*noalloc=*/true);
}

extern "C" int64_t linrec_noalloc_scratch_bytes(void) { return (int64_t)kScratchBytes; }

extern "C" int linrec_backward(const float *lambda, const float *h, const float *h0, const float *grad_h, float *grad_x,
                               float *grad_lambda, float *grad_h0, int64_t T, int64_t B, int64_t n, void *stream)
{
    const int rc = linrec_validate_backward(lambda, h, h0, grad_h, grad_x, grad_lambda, grad_h0, T, B, n);
    if (rc != LINREC_OK) return rc;
    const int64_t C = B * n;
    if (C == 0) return LINREC_OK;
    hipStream_t s = (hipStream_t)stream;
    if (T == 0) {
        if (grad_h0) {
            const hipError_t e = launch_fill(grad_h0, 0.0f, C, s);
            if (e != hipSuccess) return hip_fail(e, "launch(fill)");
        }
        return LINREC_OK;
    }
    if (!grad_x && !grad_lambda && !grad_h0) return LINREC_OK;
    Args A;
    memset(&A, 0, sizeof A);
    A.a = lambda;
    A.b = grad_h;
    A.hprev = h;
    A.h0 = h0;
    A.out0 = grad_x;
    A.out1 = grad_lambda;
    A.gh0 = grad_h0;
    A.T = T;
    A.C = C;
    return run(A, true, max_vec(C, {lambda, h, h0, grad_h, grad_x, grad_lambda, grad_h0}), s);
}

extern "C" int linrec_forward_bf16(const uint16_t *lambda, const uint16_t *x, const uint16_t *h0, uint16_t *h_out,
                                   int64_t T, int64_t B, int64_t n, void *stream)
{
    const int rc = linrec_validate_forward_bf16(lambda, x, h0, h_out, T, B, n);
    if (rc != LINREC_OK) return rc;
    const int64_t C = B * n;
    if (T == 0 || C == 0) return LINREC_OK;
    Args A;
    memset(&A, 0, sizeof A);
    // (the kernels' argument block types every tensor float*; with bf16 storage they address 2-byte elements)
    A.a = (const float *)lambda;
    A.b = (const float *)x;
    A.h0 = (const float *)h0;
    A.out0 = (float *)h_out;
    A.T = T;
    A.C = C;
    return run(A, false, max_vec_bf16(C, {lambda, x, h_out}), (hipStream_t)stream, FORM_PLAIN, true);
}

extern "C" int linrec_backward_bf16(const uint16_t *lambda, const uint16_t *h, const uint16_t *h0, const uint16_t *grad_h,
                                    uint16_t *grad_x, uint16_t *grad_lambda, uint16_t *grad_h0, int64_t T, int64_t B,
                                    int64_t n, void *stream)
{
    const int rc = linrec_validate_backward_bf16(lambda, h, h0, grad_h, grad_x, grad_lambda, grad_h0, T, B, n);
    if (rc != LINREC_OK) return rc;
    const int64_t C = B * n;
    if (C == 0) return LINREC_OK;
    hipStream_t s = (hipStream_t)stream;
    if (T == 0) {
        if (grad_h0) {
            const hipError_t e = launch_fill16(grad_h0, C, s);
            if (e != hipSuccess) return hip_fail(e, "launch(fill)");
        }
        return LINREC_OK;
    }
    if (!grad_x && !grad_lambda && !grad_h0) return LINREC_OK;
    Args A;
    memset(&A, 0, sizeof A);
    A.a = (const float *)lambda;
    A.b = (const float *)grad_h;
    A.hprev = (const float *)h;
    A.h0 = (const float *)h0;
    A.out0 = (float *)grad_x;
    A.out1 = (float *)grad_lambda;
    A.gh0 = (float *)grad_h0;
    A.T = T;
    A.C = C;
    return run(A, true, max_vec_bf16(C, {lambda, h, grad_h, grad_x, grad_lambda}), s, FORM_PLAIN, true);
}

// The gated layer and the LSTM cell in either storage type: E = float, or uint16_t holding bf16.  (The
// kernels' argument block types every tensor float*; with bf16 storage they address 2-byte elements.)
namespace {

template <class E>
constexpr bool is_bf16 = sizeof(E) == 2;
template <class E>
const float *in_ptr(const E *p) { return reinterpret_cast<const float *>(p); }
template <class E>
float *out_ptr(E *p) { return reinterpret_cast<float *>(p); }
template <class E>
int zero_state(E *p, int64_t C, hipStream_t s)
{
    const hipError_t e = is_bf16<E> ? launch_fill16(p, C, s) : launch_fill(reinterpret_cast<float *>(p), 0.0f, C, s);
    return e == hipSuccess ? LINREC_OK : hip_fail(e, "launch(fill)");
}
// widest access the [T, C] tensors allow (the [C] vectors are read element by element with bf16 storage)
template <class E>
int form_vec(int64_t C, std::initializer_list<const void *> big, std::initializer_list<const void *> small_)
{
    if (is_bf16<E>) return max_vec_bf16(C, big);
    return std::min(max_vec(C, big), max_vec(C, small_));
}

template <class E>
int gilr_forward(const E *g_pre, const E *i_pre, const E *h0, E *h_out, int tau, int64_t T, int64_t B, int64_t n,
                 hipStream_t s)
{
    const int64_t C = B * n;
    if (T == 0 || C == 0) return LINREC_OK;
    Args A;
    memset(&A, 0, sizeof A);
    A.a = in_ptr(g_pre);
    A.b = in_ptr(i_pre);
    A.h0 = in_ptr(h0);
    A.out0 = out_ptr(h_out);
    A.tau = tau;
    A.T = T;
    A.C = C;
    return run(A, false, form_vec<E>(C, {g_pre, i_pre, h_out}, {h0}), s, FORM_GATED, is_bf16<E>);
}

template <class E>
int gilr_backward(const E *g_pre, const E *i_pre, const E *h, const E *h0, const E *grad_h, E *grad_g_pre, E *grad_i_pre,
                  E *grad_h0, int tau, int64_t T, int64_t B, int64_t n, hipStream_t s)
{
    const int64_t C = B * n;
    if (C == 0) return LINREC_OK;
    if (T == 0) return grad_h0 ? zero_state(grad_h0, C, s) : LINREC_OK;
    if (!grad_g_pre && !grad_i_pre && !grad_h0) return LINREC_OK;
    Args A;
    memset(&A, 0, sizeof A);
    A.a = in_ptr(g_pre);
    A.b = in_ptr(grad_h);
    A.c = in_ptr(i_pre);
    A.hprev = in_ptr(h);
    A.h0 = in_ptr(h0);
    A.out0 = out_ptr(grad_g_pre);
    A.out1 = out_ptr(grad_i_pre);
    A.gh0 = out_ptr(grad_h0);
    A.tau = tau;
    A.T = T;
    A.C = C;
    return run(A, true, form_vec<E>(C, {g_pre, i_pre, h, grad_h, grad_g_pre, grad_i_pre}, {h0, grad_h0}), s, FORM_GATED,
               is_bf16<E>);
}

template <class E>
int lstm_cell_forward(const E *f_pre, const E *i_pre, const E *z_pre, const E *o_pre, const E *c0, E *c_out, E *h_out,
                      int64_t T, int64_t B, int64_t n, hipStream_t s)
{
    const int64_t C = B * n;
    if (T == 0 || C == 0) return LINREC_OK;
    Args A;
    memset(&A, 0, sizeof A);
    A.a = in_ptr(f_pre);
    A.b = in_ptr(i_pre);
    A.c = in_ptr(z_pre);
    A.d = in_ptr(o_pre);
    A.h0 = in_ptr(c0);
    A.out0 = out_ptr(c_out);
    A.out1 = out_ptr(h_out);
    A.T = T;
    A.C = C;
    return run(A, false, form_vec<E>(C, {f_pre, i_pre, z_pre, o_pre, c_out, h_out}, {c0}), s, FORM_LSTM, is_bf16<E>);
}

template <class E>
int lstm_cell_backward(const E *f_pre, const E *i_pre, const E *z_pre, const E *o_pre, const E *c, const E *c0,
                       const E *grad_h, E *grad_f_pre, E *grad_i_pre, E *grad_z_pre, E *grad_o_pre, E *grad_c0, int64_t T,
                       int64_t B, int64_t n, hipStream_t s)
{
    const int64_t C = B * n;
    if (C == 0) return LINREC_OK;
    if (T == 0) return grad_c0 ? zero_state(grad_c0, C, s) : LINREC_OK;
    if (!grad_f_pre && !grad_i_pre && !grad_z_pre && !grad_o_pre && !grad_c0) return LINREC_OK;
    Args A;
    memset(&A, 0, sizeof A);
    A.a = in_ptr(f_pre);
    A.b = in_ptr(grad_h);
    A.c = in_ptr(i_pre);
    A.d = in_ptr(z_pre);
    A.e = in_ptr(o_pre);
    A.hprev = in_ptr(c);
    A.h0 = in_ptr(c0);
    A.out0 = out_ptr(grad_f_pre);
    A.out1 = out_ptr(grad_i_pre);
    A.out2 = out_ptr(grad_z_pre);
    A.out3 = out_ptr(grad_o_pre);
    A.gh0 = out_ptr(grad_c0);
    A.T = T;
    A.C = C;
    return run(A, true,
               form_vec<E>(C, {f_pre, i_pre, z_pre, o_pre, c, grad_h, grad_f_pre, grad_i_pre, grad_z_pre, grad_o_pre},
                           {c0, grad_c0}),
               s, FORM_LSTM, is_bf16<E>);
}

}  // namespace

extern "C" int linrec_gilr_forward(const float *g_pre, const float *i_pre, const float *h0, float *h_out, int tau,
                                   int64_t T, int64_t B, int64_t n, void *stream)
{
    const int rc = linrec_validate_gilr_forward(g_pre, i_pre, h0, h_out, tau, T, B, n);
    return rc != LINREC_OK ? rc : gilr_forward(g_pre, i_pre, h0, h_out, tau, T, B, n, (hipStream_t)stream);
}

extern "C" int linrec_gilr_backward(const float *g_pre, const float *i_pre, const float *h, const float *h0,
                                    const float *grad_h, float *grad_g_pre, float *grad_i_pre, float *grad_h0, int tau,
                                    int64_t T, int64_t B, int64_t n, void *stream)
{
    const int rc = linrec_validate_gilr_backward(g_pre, i_pre, h, h0, grad_h, grad_g_pre, grad_i_pre, grad_h0, tau, T, B, n);
    return rc != LINREC_OK ? rc
                           : gilr_backward(g_pre, i_pre, h, h0, grad_h, grad_g_pre, grad_i_pre, grad_h0, tau, T, B, n,
                                           (hipStream_t)stream);
}

extern "C" int linrec_lstm_cell_forward(const float *f_pre, const float *i_pre, const float *z_pre, const float *o_pre,
                                        const float *c0, float *c_out, float *h_out, int64_t T, int64_t B, int64_t n,
                                        void *stream)
{
    const int rc = linrec_validate_lstm_cell_forward(f_pre, i_pre, z_pre, o_pre, c0, c_out, h_out, T, B, n);
    return rc != LINREC_OK ? rc : lstm_cell_forward(f_pre, i_pre, z_pre, o_pre, c0, c_out, h_out, T, B, n, (hipStream_t)stream);
}

extern "C" int linrec_lstm_cell_backward(const float *f_pre, const float *i_pre, const float *z_pre, const float *o_pre,
                                         const float *c, const float *c0, const float *grad_h, float *grad_f_pre,
                                         float *grad_i_pre, float *grad_z_pre, float *grad_o_pre, float *grad_c0,
                                         int64_t T, int64_t B, int64_t n, void *stream)
{
    const int rc = linrec_validate_lstm_cell_backward(f_pre, i_pre, z_pre, o_pre, c, c0, grad_h, grad_f_pre, grad_i_pre,
                                                      grad_z_pre, grad_o_pre, grad_c0, T, B, n);
    return rc != LINREC_OK ? rc
                           : lstm_cell_backward(f_pre, i_pre, z_pre, o_pre, c, c0, grad_h, grad_f_pre, grad_i_pre, grad_z_pre,
                                                grad_o_pre, grad_c0, T, B, n, (hipStream_t)stream);
}

extern "C" int linrec_gilr_forward_bf16(const uint16_t *g_pre, const uint16_t *i_pre, const uint16_t *h0, uint16_t *h_out,
                                        int tau, int64_t T, int64_t B, int64_t n, void *stream)
{
    const int rc = linrec_validate_gilr_forward_bf16(g_pre, i_pre, h0, h_out, tau, T, B, n);
    return rc != LINREC_OK ? rc : gilr_forward(g_pre, i_pre, h0, h_out, tau, T, B, n, (hipStream_t)stream);
}

extern "C" int linrec_gilr_backward_bf16(const uint16_t *g_pre, const uint16_t *i_pre, const uint16_t *h, const uint16_t *h0,
                                         const uint16_t *grad_h, uint16_t *grad_g_pre, uint16_t *grad_i_pre,
                                         uint16_t *grad_h0, int tau, int64_t T, int64_t B, int64_t n, void *stream)
{
    const int rc = linrec_validate_gilr_backward_bf16(g_pre, i_pre, h, h0, grad_h, grad_g_pre, grad_i_pre, grad_h0, tau, T, B, n);
    return rc != LINREC_OK ? rc
                           : gilr_backward(g_pre, i_pre, h, h0, grad_h, grad_g_pre, grad_i_pre, grad_h0, tau, T, B, n,
                                           (hipStream_t)stream);
}

extern "C" int linrec_lstm_cell_forward_bf16(const uint16_t *f_pre, const uint16_t *i_pre, const uint16_t *z_pre,
                                             const uint16_t *o_pre, const uint16_t *c0, uint16_t *c_out, uint16_t *h_out,
                                             int64_t T, int64_t B, int64_t n, void *stream)
{
    const int rc = linrec_validate_lstm_cell_forward_bf16(f_pre, i_pre, z_pre, o_pre, c0, c_out, h_out, T, B, n);
    return rc != LINREC_OK ? rc : lstm_cell_forward(f_pre, i_pre, z_pre, o_pre, c0, c_out, h_out, T, B, n, (hipStream_t)stream);
}

extern "C" int linrec_lstm_cell_backward_bf16(const uint16_t *f_pre, const uint16_t *i_pre, const uint16_t *z_pre,
                                              const uint16_t *o_pre, const uint16_t *c, const uint16_t *c0,
                                              const uint16_t *grad_h, uint16_t *grad_f_pre, uint16_t *grad_i_pre,
                                              uint16_t *grad_z_pre, uint16_t *grad_o_pre, uint16_t *grad_c0, int64_t T,
                                              int64_t B, int64_t n, void *stream)
{
    const int rc = linrec_validate_lstm_cell_backward_bf16(f_pre, i_pre, z_pre, o_pre, c, c0, grad_h, grad_f_pre, grad_i_pre,
                                                           grad_z_pre, grad_o_pre, grad_c0, T, B, n);
    return rc != LINREC_OK ? rc
                           : lstm_cell_backward(f_pre, i_pre, z_pre, o_pre, c, c0, grad_h, grad_f_pre, grad_i_pre, grad_z_pre,
                                                grad_o_pre, grad_c0, T, B, n, (hipStream_t)stream);
}

extern "C" int linrec_set_option(int option, int64_t value)
{
    switch (option) {
    case LINREC_OPT_VARIANT:
        if (value < LINREC_VARIANT_AUTO || value > LINREC_VARIANT_WALK) return LINREC_ERR_OPTION;
        opts().variant = value;
        return LINREC_OK;
    case LINREC_OPT_TILE:
        if (value != 0 && !tile_exists((int)value)) return LINREC_ERR_OPTION;
        opts().tile = value;
        return LINREC_OK;
    case LINREC_OPT_CHUNK_TILES:
        if (value < 0 || value > (1 << 20)) return LINREC_ERR_OPTION;
        opts().chunk_tiles = value;
        return LINREC_OK;
    case LINREC_OPT_SPIN_LIMIT:
        if (value < 1 || value > 0x7fffffff) return LINREC_ERR_OPTION;
        opts().spin_limit = value;
        return LINREC_OK;
    case LINREC_OPT_HPREV_LATE:
        if (value < -1 || value > 1) return LINREC_ERR_OPTION;
        opts().hp_late = value;
        return LINREC_OK;
    case LINREC_OPT_TAPER:
        if (value < -1 || value > 8) return LINREC_ERR_OPTION;
        opts().taper = value;
        return LINREC_OK;
    case LINREC_OPT_PERSISTENT:
        if (value < -1 || value > 1) return LINREC_ERR_OPTION;
        opts().persistent = value;
        return LINREC_OK;
    case LINREC_OPT_GRID_CAP:
        if (value < -1 || value > 64) return LINREC_ERR_OPTION;
        opts().grid_cap = value;
        return LINREC_OK;
    case LINREC_OPT_STAGGER:
        if (value < 0 || value > 16) return LINREC_ERR_OPTION;
        opts().stagger = value;
        return LINREC_OK;
    case LINREC_OPT_TEST_FILL:
        if (value < 0 || value > 0xffffffffll) return LINREC_ERR_OPTION;
        opts().test_fill = value;
        return LINREC_OK;
    case LINREC_OPT_TEST_EPOCH:
        if (value < -1 || value > 0x7ffffffdll) return LINREC_ERR_OPTION;
        opts().test_epoch = value;
        return LINREC_OK;
    default: return LINREC_ERR_OPTION;
    }
}

extern "C" int64_t linrec_get_option(int option)
{
    switch (option) {
    case LINREC_OPT_VARIANT: return opts().variant;
    case LINREC_OPT_TILE: return opts().tile;
    case LINREC_OPT_CHUNK_TILES: return opts().chunk_tiles;
    case LINREC_OPT_SPIN_LIMIT: return opts().spin_limit;
    case LINREC_OPT_HPREV_LATE: return opts().hp_late;
    case LINREC_OPT_TAPER: return opts().taper;
    case LINREC_OPT_PERSISTENT: return opts().persistent;
    case LINREC_OPT_GRID_CAP: return opts().grid_cap;
    case LINREC_OPT_STAGGER: return opts().stagger;
    case LINREC_OPT_TEST_FILL: return opts().test_fill;
    case LINREC_OPT_TEST_EPOCH: return opts().test_epoch;
    default: return LINREC_ERR_OPTION;
    }
}

extern "C" int linrec_tile_info(int tile_id, int *threads_cols, int *threads_time, int *rows_per_thread,
                                int *cols_per_thread)
{
    if (!tile_exists(tile_id)) return LINREC_ERR_OPTION;
    const TileDesc &d = tile_desc(tile_id);
    if (threads_cols) *threads_cols = d.wc;
    if (threads_time) *threads_time = d.wt;
    if (rows_per_thread) *rows_per_thread = d.r;
    if (cols_per_thread) *cols_per_thread = d.vec;
    return LINREC_OK;
}

extern "C" int linrec_tile_has(int tile_id, int entry_point)
{
    return entry_point >= LINREC_ENTRY_PLAIN && entry_point <= LINREC_ENTRY_LSTM_CELL_BF16 && tile_has(tile_id, entry_point);
}

extern "C" int linrec_plan(int64_t T, int64_t B, int64_t n, int backward, int alignment_bytes, int *variant,
                           int *tile_id)
{
    int64_t C = B * n;
    if (T <= 0 || B <= 0 || n <= 0) return LINREC_ERR_SHAPE;
    const int vec = max_vec(C, {(const void *)(uintptr_t)(alignment_bytes > 0 ? alignment_bytes : 4)});
    const Plan p = make_plan(T, C, vec, backward != 0);
    if (variant) *variant = p.variant;
    if (tile_id) *tile_id = p.tile;
    return LINREC_OK;
}

extern "C" int linrec_plan_for(int entry_point, int64_t T, int64_t B, int64_t n, int backward, int alignment_bytes,
                               int *variant, int *tile_id)
{
    int64_t C = B * n;
    if (T <= 0 || B <= 0 || n <= 0) return LINREC_ERR_SHAPE;
    if (entry_point < LINREC_ENTRY_PLAIN || entry_point > LINREC_ENTRY_LSTM_CELL_BF16) return LINREC_ERR_OPTION;
    const void *al = (const void *)(uintptr_t)(alignment_bytes > 0 ? alignment_bytes : 2);
    const bool bf16 = entry_bf16(entry_point);
    const int form = entry_form(entry_point);
    const int vec = bf16 ? max_vec_bf16(C, {al}) : max_vec(C, {al});
    Plan p = make_plan(T, C, vec, backward != 0, form, bf16);
    if ((form != FORM_PLAIN || bf16) && p.variant == LINREC_VARIANT_THREEPHASE) p.variant = LINREC_VARIANT_LOOKBACK;
    if (variant) *variant = p.variant;
    if (tile_id) *tile_id = p.tile;
    return LINREC_OK;
}

extern "C" int linrec_plan_taper(int entry_point, int64_t T, int64_t B, int64_t n, int backward, int alignment_bytes)
{
    int64_t C = B * n;
    if (T <= 0 || B <= 0 || n <= 0) return LINREC_ERR_SHAPE;
    if (entry_point < LINREC_ENTRY_PLAIN || entry_point > LINREC_ENTRY_LSTM_CELL_BF16) return LINREC_ERR_OPTION;
    const void *al = (const void *)(uintptr_t)(alignment_bytes > 0 ? alignment_bytes : 2);
    const bool bf16 = entry_bf16(entry_point);
    const int vec = bf16 ? max_vec_bf16(C, {al}) : max_vec(C, {al});
    const Plan p = make_plan(T, C, vec, backward != 0, entry_form(entry_point), bf16);
    return p.variant == LINREC_VARIANT_LOOKBACK ? p.taper : 0;
}

extern "C" int linrec_stream_probe(const float *in0, const float *in1, const float *in2, float *out0, float *out1,
                                   int64_t n, void *stream)
{
    if (n < 0 || (n & 3)) return LINREC_ERR_SHAPE;
    if (!out0 && !out1 && !in0 && !in1 && !in2) return LINREC_ERR_NULL;
    const void *ptrs[5] = {in0, in1, in2, out0, out1};
    for (const void *p : ptrs)
        if (!aligned16(p)) return LINREC_ERR_SHAPE;
    if (n == 0) return LINREC_OK;
    const hipError_t e = launch_stream_probe(in0, in1, in2, out0, out1, n, (hipStream_t)stream);
    return e == hipSuccess ? LINREC_OK : hip_fail(e, "launch(stream_probe)");
}

extern "C" int linrec_stream_probe_rows(const float *in0, const float *in1, const float *in2, float *out0, float *out1,
                                        int64_t T, int64_t C, void *stream)
{
    if (T < 0 || C < 0 || T % 32 || C % 256 || (C > 0 && T > ((int64_t)1 << 40) / C)) return LINREC_ERR_SHAPE;
    // inputs and outputs are given from the front: in1 needs in0, in2 needs in1, out1 needs out0
    if ((in1 && !in0) || (in2 && !in1) || (out1 && !out0) || (!in0 && !out0)) return LINREC_ERR_NULL;
    const void *ptrs[5] = {in0, in1, in2, out0, out1};
    for (const void *p : ptrs)
        if ((uintptr_t)p & 3u) return LINREC_ERR_SHAPE;
    if (T == 0 || C == 0) return LINREC_OK;
    const int nin = in2 ? 3 : in1 ? 2 : in0 ? 1 : 0, nout = out1 ? 2 : out0 ? 1 : 0;
    const hipError_t e = launch_rows_probe(nin, nout, in0, in1, in2, out0, out1, T, C, (hipStream_t)stream);
    return e == hipSuccess ? LINREC_OK : hip_fail(e, "launch(rows_probe)");
}

// Times the look-back kernel under every candidate plan on scratch tensors of the given shape and
// remembers the fastest for later calls with that shape on this device.
extern "C" int linrec_tune_for(int entry_point, int64_t T, int64_t B, int64_t n, int backward, void *stream)
{
    if (T <= 0 || B <= 0 || n <= 0 || B > ((int64_t)1 << 40) / n || T > ((int64_t)1 << 40) / (B * n))
        return LINREC_ERR_SHAPE;
    if (entry_point < LINREC_ENTRY_PLAIN || entry_point > LINREC_ENTRY_LSTM_CELL_BF16) return LINREC_ERR_OPTION;
    const int64_t C = B * n, E = T * C;
    hipStream_t s = (hipStream_t)stream;
    const bool bwd = backward != 0;
    int dev = 0;
    hipError_t e;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return hip_fail(e, "hipGetDevice");

    // Scratch tensors.  Tensor 0 is the multiplier (lambda, or the forget / gate pre-activation): 0.96875
    // as lambda, 3.4 as a pre-activation (sigmoid = 0.968), so that products neither overflow nor vanish
    // within a tile; the other inputs are 1, the state vectors 0.  With bf16 storage the same fills are
    // written as 16-bit patterns (both constants are exact in bf16).
    const bool bf16 = entry_bf16(entry_point);
    const int form = entry_form(entry_point);
    const int n_in = form == FORM_LSTM ? (bwd ? 6 : 4) : form == FORM_GATED ? (bwd ? 4 : 2) : (bwd ? 3 : 2);
    const int n_out = form == FORM_LSTM ? (bwd ? 4 : 2) : (bwd ? 2 : 1);
    const int n_big = n_in + n_out;
    float *big[10] = {}, *small_[2] = {nullptr, nullptr};
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    int rc = LINREC_OK;
    for (int i = 0; i < n_big && rc == LINREC_OK; ++i)
        if ((e = hipMalloc((void **)&big[i], (size_t)E * sizeof(float))) != hipSuccess) rc = hip_fail(e, "hipMalloc(tune)");
    for (int i = 0; i < 2 && rc == LINREC_OK; ++i)
        if ((e = hipMalloc((void **)&small_[i], (size_t)C * sizeof(float))) != hipSuccess) rc = hip_fail(e, "hipMalloc(tune)");
    if (rc == LINREC_OK && ((e = hipEventCreate(&ev0)) != hipSuccess || (e = hipEventCreate(&ev1)) != hipSuccess))
        rc = hip_fail(e, "hipEventCreate");
    if (rc == LINREC_OK) {
        const float first = form != FORM_PLAIN ? 3.40625f : 0.96875f;
        // a float whose two halves are the same bf16 pattern fills a bf16 tensor with that value
        auto both_halves = [](float v) {
            uint32_t b;
            memcpy(&b, &v, 4);
            b = (b & 0xffff0000u) | (b >> 16);
            float r;
            memcpy(&r, &b, 4);
            return r;
        };
        e = launch_fill(big[0], bf16 ? both_halves(first) : first, E, s);
        for (int i = 1; i < n_big && e == hipSuccess; ++i) e = launch_fill(big[i], bf16 ? both_halves(1.0f) : 1.0f, E, s);
        for (int i = 0; i < 2 && e == hipSuccess; ++i) e = launch_fill(small_[i], 0.0f, C, s);
        if (e != hipSuccess) rc = hip_fail(e, "launch(fill)");
    }
    auto call = [&]() -> int {
        typedef const uint16_t *cb;
        typedef uint16_t *mb;
        switch (entry_point) {
        case LINREC_ENTRY_GILR:
            return bwd ? linrec_gilr_backward(big[0], big[1], big[2], small_[0], big[3], big[4], big[5], small_[1],
                                              LINREC_TAU_TANH, T, B, n, s)
                       : linrec_gilr_forward(big[0], big[1], small_[0], big[2], LINREC_TAU_TANH, T, B, n, s);
        case LINREC_ENTRY_LSTM_CELL:
            return bwd ? linrec_lstm_cell_backward(big[0], big[1], big[2], big[3], big[4], small_[0], big[5], big[6], big[7],
                                                   big[8], big[9], small_[1], T, B, n, s)
                       : linrec_lstm_cell_forward(big[0], big[1], big[2], big[3], small_[0], big[4], big[5], T, B, n, s);
        case LINREC_ENTRY_GILR_BF16:
            return bwd ? linrec_gilr_backward_bf16((cb)big[0], (cb)big[1], (cb)big[2], (cb)small_[0], (cb)big[3], (mb)big[4],
                                                   (mb)big[5], (mb)small_[1], LINREC_TAU_TANH, T, B, n, s)
                       : linrec_gilr_forward_bf16((cb)big[0], (cb)big[1], (cb)small_[0], (mb)big[2], LINREC_TAU_TANH, T, B, n, s);
        case LINREC_ENTRY_LSTM_CELL_BF16:
            return bwd ? linrec_lstm_cell_backward_bf16((cb)big[0], (cb)big[1], (cb)big[2], (cb)big[3], (cb)big[4],
                                                        (cb)small_[0], (cb)big[5], (mb)big[6], (mb)big[7], (mb)big[8],
                                                        (mb)big[9], (mb)small_[1], T, B, n, s)
                       : linrec_lstm_cell_forward_bf16((cb)big[0], (cb)big[1], (cb)big[2], (cb)big[3], (cb)small_[0],
                                                       (mb)big[4], (mb)big[5], T, B, n, s);
        case LINREC_ENTRY_BF16:
            return bwd ? linrec_backward_bf16((cb)big[0], (cb)big[1], (cb)small_[0], (cb)big[2], (mb)big[3], (mb)big[4],
                                              (mb)small_[1], T, B, n, s)
                       : linrec_forward_bf16((cb)big[0], (cb)big[1], (cb)small_[0], (mb)big[2], T, B, n, s);
        default:
            return bwd ? linrec_backward(big[0], big[1], small_[0], big[2], big[3], big[4], small_[1], T, B, n, s)
                       : linrec_forward(big[0], big[1], small_[0], big[2], T, B, n, s);
        }
    };

    TunedPlan best{0, -1, LINREC_VARIANT_LOOKBACK}, second{0, -1, LINREC_VARIANT_LOOKBACK};
    float best_ms = 0.f, second_ms = 0.f;
    if (rc == LINREC_OK) {
        const int vec = bf16 ? max_vec_bf16(C, {}) : max_vec(C, {});
        // (candidates are forced on this thread's calls only; the options stay as they are)
        const int base_taper = opts().taper > 0 ? (int)opts().taper : 0;  // an explicit option holds for every candidate
        const bool try_taper = opts().taper < 0;
        ForcedPlan &fp = forced();
        // Median of five launches of the forced plan, after two warm-up launches; < 0 on failure (rc is set).
        auto time_plan = [&](int variant, int tile, int persistent, int taper) -> float {
            fp = ForcedPlan{};
            fp.active = true;
            fp.variant = variant;
            fp.tile = tile;
            fp.persistent = persistent;
            fp.taper = taper;
            float times[5];
            for (int it = -2; it < 5; ++it) {
                if ((e = hipEventRecord(ev0, s)) != hipSuccess) { rc = hip_fail(e, "hipEventRecord"); return -1.f; }
                if ((rc = call()) != LINREC_OK) return -1.f;
                float ms = 0.f;
                if ((e = hipEventRecord(ev1, s)) != hipSuccess || (e = hipEventSynchronize(ev1)) != hipSuccess ||
                    (e = hipEventElapsedTime(&ms, ev0, ev1)) != hipSuccess) {
                    rc = hip_fail(e, "tune: timing");
                    return -1.f;
                }
                if (it >= 0) times[it] = ms;
            }
            std::sort(times, times + 5);
            return times[2];
        };
        auto usable = [&](int tile) {
            const TileDesc &d = kTable.t[tile];
            return tile_has(tile, entry_point) && d.vec <= vec && ((int64_t)d.rows() * C + d.cols()) * 4 < ((int64_t)1 << 32);
        };
        // Single pass: every shape the family has, the static plan's own first so that what is remembered is
        // never slower than it, each with persistent workgroups and with one workgroup per tile.
        const StaticPlan sp = static_plan(entry_point, bwd, T, C, vec);
        std::vector<int> candidates{sp.lookback};
        for (int id = 1; id <= MAX_TILE_ID; ++id)
            if (id != sp.lookback) candidates.push_back(id);
        for (const int tile : candidates) {
            if (!usable(tile)) continue;
            if (kTable.t[tile].rows() > 2 * T && tile != sp.lookback) continue;  // far taller than the problem
            for (int persistent = 0; persistent <= 1 && rc == LINREC_OK; ++persistent) {
                const float ms = time_plan(LINREC_VARIANT_LOOKBACK, tile, persistent, base_taper);
                if (ms < 0.f) break;
                if (best.tile == 0 || ms < best_ms) {
                    if (best.tile != tile) {  // (the runner-up is a different shape)
                        second = best;
                        second_ms = best_ms;
                    }
                    best_ms = ms;
                    best = TunedPlan{tile, persistent, LINREC_VARIANT_LOOKBACK};
                } else if (tile != best.tile && (second.tile == 0 || ms < second_ms)) {
                    second_ms = ms;
                    second = TunedPlan{tile, persistent, LINREC_VARIANT_LOOKBACK};
                }
            }
            if (rc != LINREC_OK) break;
        }
        // The two best single-pass plans once more with a quarter of their last round cut into shorter
        // tiles: a launch of few rounds ends sooner that way on some shapes (kept only if it is at least
        // half a percent faster than the best so far; an explicit LINREC_OPT_TAPER, 0 included, overrides what is
        // remembered and is not second-guessed here).
        const TunedPlan untapered[2] = {best, second};
        for (int c = 0; c < 2 && rc == LINREC_OK && try_taper; ++c) {
            const TunedPlan &u = untapered[c];
            if (u.tile == 0 || kTable.t[u.tile].r % 4 != 0 || kTable.t[u.tile].r < 8) continue;
            const float ms = time_plan(LINREC_VARIANT_LOOKBACK, u.tile, u.persistent, 2);
            if (ms >= 0.f && ms < 0.995f * best_ms) {
                best_ms = ms;
                best = u;
                best.taper = 2;
            }
        }
        // The walk, where there are enough columns for it to stand a chance and the sequence is short enough (from
        // 16384 columns on, where the column groups alone fill the GPU, at any length):
        // every shape of the family that makes between one and eight workgroups per compute unit.
        if ((C >= 4096 && T <= 8192) || C >= 16384) {
            const int64_t units = compute_units(dev);
            for (int tile = 1; tile <= MAX_TILE_ID && rc == LINREC_OK; ++tile) {
                if (!usable(tile)) continue;
                const int64_t groups = ceil_div(C, kTable.t[tile].cols());
                if (2 * groups < units || groups > 8 * units || kTable.t[tile].rows() > 2 * T) continue;
                const float ms = time_plan(LINREC_VARIANT_WALK, tile, -1, 0);
                if (ms >= 0.f && (best.tile == 0 || ms < best_ms)) {
                    best_ms = ms;
                    best = TunedPlan{tile, -1, LINREC_VARIANT_WALK};
                }
            }
        }
        fp = ForcedPlan{};
    }
    if (ev0) (void)hipEventDestroy(ev0);
    if (ev1) (void)hipEventDestroy(ev1);
    (void)hipStreamSynchronize(s);
    for (float *p : big)
        if (p) (void)hipFree(p);
    for (float *p : small_)
        if (p) (void)hipFree(p);
    if (rc == LINREC_OK && best.tile != 0) {
        std::lock_guard<std::mutex> lock(g_tuned_mu);
        g_tuned[TunedKey{dev, T, C, bwd, entry_point}] = best;
    }
    return rc;
}

extern "C" int linrec_pin_plan(int entry_point, int64_t T, int64_t B, int64_t n, int backward, int variant, int tile_id,
                               int persistent, int taper)
{
    if (T <= 0 || B <= 0 || n <= 0 || B > ((int64_t)1 << 40) / n || T > ((int64_t)1 << 40) / (B * n))
        return LINREC_ERR_SHAPE;
    if (entry_point < LINREC_ENTRY_PLAIN || entry_point > LINREC_ENTRY_LSTM_CELL_BF16) return LINREC_ERR_OPTION;
    if ((tile_id != 0 && !tile_exists(tile_id)) || persistent < -1 || persistent > 1 || taper < 0 || taper > 8)
        return LINREC_ERR_OPTION;
    if (tile_id != 0 && variant != LINREC_VARIANT_LOOKBACK && variant != LINREC_VARIANT_WALK) return LINREC_ERR_OPTION;
    int dev = 0;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    const TunedKey key{dev, T, B * n, backward != 0, entry_point};
    std::lock_guard<std::mutex> lock(g_tuned_mu);
    if (tile_id == 0) {
        g_tuned.erase(key);
    } else {
        TunedPlan tp{tile_id, persistent, variant};
        tp.taper = taper;
        g_tuned[key] = tp;
    }
    return LINREC_OK;
}

extern "C" int linrec_reserve_workspace(int entry_point, int64_t T, int64_t B, int64_t n, int backward, void *stream)
{
    if (T <= 0 || B <= 0 || n <= 0 || B > ((int64_t)1 << 40) / n || T > ((int64_t)1 << 40) / (B * n))
        return LINREC_ERR_SHAPE;
    if (entry_point < LINREC_ENTRY_PLAIN || entry_point > LINREC_ENTRY_LSTM_CELL_BF16) return LINREC_ERR_OPTION;
    const int64_t C = B * n;
    hipStream_t s = (hipStream_t)stream;
    int dev = 0;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    // Room for what a call of this shape would use under the calling thread's options and the plans pinned
    // or tuned so far, whatever the alignment of its tensors turns out to be (the widest access a plan may
    // use depends on it).
    const bool bf16 = entry_bf16(entry_point), bwd = backward != 0;
    const int form = entry_form(entry_point);
    size_t need_lb = 0, need_tp = 0;
    for (int vec = 1; vec <= 4; vec *= 2) {
        if (vec > 1 && C % vec != 0) continue;
        Plan plan = make_plan(T, C, vec, bwd, form, bf16);
        if ((form != FORM_PLAIN || bf16) && plan.variant == LINREC_VARIANT_THREEPHASE) plan.variant = LINREC_VARIANT_LOOKBACK;
        if (plan.variant != LINREC_VARIANT_LOOKBACK && plan.variant != LINREC_VARIANT_THREEPHASE) continue;
        const TileDesc &d = kTable.t[plan.tile];
        const int64_t G = ceil_div(C, d.cols());
        if (plan.variant == LINREC_VARIANT_LOOKBACK) {
            need_lb = std::max(need_lb, lookback_bytes(time_tiles(T, G, d, plan.taper, dev).K, C));
        } else {
            const int64_t tiles_t = ceil_div(T, d.rows());
            int64_t M = opts().chunk_tiles;
            if (M <= 0) M = ceil_div(tiles_t * G, 4096);
            M = std::max<int64_t>(1, std::min<int64_t>(M, 1 << 20));
            need_tp = std::max(need_tp, 3 * (size_t)ceil_div(tiles_t, M) * (size_t)C * sizeof(double));
        }
    }
    std::lock_guard<std::mutex> lock(g_mu);
    Workspace &ws = g_ws[std::make_pair(dev, s)];
    int rc = LINREC_OK;
    if (need_lb) rc = ensure(ws, &ws.lb, &ws.lb_bytes, need_lb, true, s);
    if (rc == LINREC_OK && need_tp) rc = ensure(ws, &ws.tp, &ws.tp_bytes, need_tp, false, s);
    return rc;
}

extern "C" int linrec_tune(int64_t T, int64_t B, int64_t n, int backward, void *stream)
{
    return linrec_tune_for(LINREC_ENTRY_PLAIN, T, B, n, backward, stream);
}

#ifdef LINREC_TRACE
// Trace builds only: device buffer of 8 u64 per tile that look-back kernels fill with their timeline.
extern "C" void linrec_debug_trace(unsigned long long *device_buffer) { g_trace = device_buffer; }
#endif

extern "C" int linrec_check(void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    int dev = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return hip_fail(e, "hipGetDevice");
    // every block that may hold the header of a launch on this stream: the live look-back block, the
    // retired ones, and this device's no-allocation scratch
    std::vector<void *> headers;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        auto it = g_ws.find(std::make_pair(dev, s));
        if (it != g_ws.end()) {
            if (it->second.lb) headers.push_back(it->second.lb);
            headers.insert(headers.end(), it->second.retired_lb.begin(), it->second.retired_lb.end());
        }
        if (dev >= 0 && dev < kMaxDevices && g_scratch[dev].ptr) headers.push_back(g_scratch[dev].ptr);
    }
    int rc = LINREC_OK;
    for (void *h : headers) {
        uint32_t flag = 0;
        char *p = (char *)h + offsetof(LookbackHeader, err);
        if ((e = hipMemcpy(&flag, p, sizeof flag, hipMemcpyDeviceToHost)) != hipSuccess) return hip_fail(e, "hipMemcpy");
        if (!flag) continue;
        if ((e = hipMemset(p, 0, sizeof flag)) != hipSuccess) return hip_fail(e, "hipMemset");
        rc = LINREC_ERR_DEVICE;
    }
    return rc;
}

extern "C" int linrec_release_workspace(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    int rc = LINREC_OK;
    int cur = 0;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    for (auto &kv : g_ws) {
        if (hipSetDevice(kv.first.first) != hipSuccess) { rc = LINREC_ERR_HIP; continue; }
        if (kv.second.lb && hipFree(kv.second.lb) != hipSuccess) rc = LINREC_ERR_HIP;
        if (kv.second.tp && hipFree(kv.second.tp) != hipSuccess) rc = LINREC_ERR_HIP;
        for (void *p : kv.second.retired_lb)
            if (hipFree(p) != hipSuccess) rc = LINREC_ERR_HIP;
        for (void *p : kv.second.retired_tp)
            if (hipFree(p) != hipSuccess) rc = LINREC_ERR_HIP;
    }
    g_ws.clear();
    if (have_cur) (void)hipSetDevice(cur);
    return rc;
}

extern "C" const char *linrec_last_hip_error(void) { return g_hip_error; }
