// Device code of liblinrec: tile primitives and the three scan kernels built from them.
//
// The problem is a [T, C] fp32 matrix pair (lambda, x) scanned down the rows under the affine-pair
// operator (a1,b1)(+)(a2,b2) = (a1*a2, a2*b1 + b2) -- Algorithm 1 of arXiv 1709.04057 with diagonal
// Lambda (Section 2.1).  A *tile* is ROWS = WT*R consecutive time steps by COLS = WC*VEC columns,
// owned by one workgroup of WC*WT threads: thread (tt, tc) keeps R consecutive rows of VEC adjacent
// columns in registers, so every global access is a VEC*4-byte load/store that is contiguous along
// the column axis across the WC lanes of a row segment.
//
// Inside a tile Algorithm 1 is applied with p = WT "processors": each thread reduces its rows to a
// pair (P, S) (phase 1), the WT pairs of a column are combined in time order through LDS (phase 2),
// and every thread re-runs the recurrence over its registers from its carry-in (phase 3).  Across
// tiles the same three phases are either three kernels (k_reduce, k_scan_summaries, k_fixup) or one
// kernel that finds the tile's carry-in by decoupled look-back over the published tile summaries
// (k_lookback).
//
// The backward pass (Section 2.2) is the same scan on reversed time: logical step u maps to row
// t = T-1-u, the multiplier of step u is lambda[t+1] (0 for u == 0: the last row has no successor
// and row T of lambda is never read), the addend is grad_h[t], and the outputs are
// grad_x[t] = g_t, grad_lambda[t] = g_t*h[t-1] (h[-1] = h0), grad_h0 = lambda[0]*g_0.
#pragma once
#include "linrec_launch.h"

namespace linrec {

template <int VEC_, int R_, int WC_, int WT_>
struct Geo {
    static constexpr int VEC = VEC_, R = R_, WC = WC_, WT = WT_;
    static constexpr int THREADS = WC * WT, ROWS = WT * R, COLS = WC * VEC;
};

// VEC adjacent columns of one row, kept as one SSA value (never addressed through a pointer, so the
// register tile cannot end up in scratch memory).
template <int N>
using vec = float __attribute__((ext_vector_type(N)));

// Summaries are kept in fp64.  A product of many lambdas computed in fp32 drifts coherently when the
// factors repeat (constant decay along T), which no fp32 evaluation order avoids; in fp64 the drift is
// far below the fp32 resolution of the result.  Only the O(T*C/R) summary arithmetic pays for this,
// the per-element rescan stays fp32.
template <int N>
using dvec = double __attribute__((ext_vector_type(N)));

template <int N>
__device__ __forceinline__ dvec<N> widen(vec<N> v)
{
    return __builtin_convertvector(v, dvec<N>);
}
template <int N>
__device__ __forceinline__ vec<N> narrow(dvec<N> v)
{
    return __builtin_convertvector(v, vec<N>);
}
template <int N>
__device__ __forceinline__ dvec<N> dsplat(double x)
{
    return dvec<N>(x);
}
template <int N>
__device__ __forceinline__ dvec<N> dfma(dvec<N> a, dvec<N> b, dvec<N> c)
{
    return __builtin_elementwise_fma(a, b, c);
}

template <int N>
__device__ __forceinline__ vec<N> ld(const float *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const vec<N> *>(p));
}
template <int N>
__device__ __forceinline__ void st(float *p, vec<N> v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<vec<N> *>(p));
}
template <int N>
__device__ __forceinline__ vec<N> vfma(vec<N> a, vec<N> b, vec<N> c)
{
    return __builtin_elementwise_fma(a, b, c);
}
template <int N>
__device__ __forceinline__ vec<N> splat(float x)
{
    return vec<N>(x);
}

// ---------------------------------------------------------------------------------------------
// Tile addressing.  Every access of a tile is written as (workgroup-uniform 64-bit base) +
// (per-thread unsigned 32-bit byte offset), which maps onto the scalar-base + vector-offset form of
// the global load/store instructions and keeps the per-row addresses out of the vector registers.
// The host guarantees (ROWS*C + COLS)*4 < 2^32.
//
// Forward: the base is the tile's first row, thread (tt, tc) starts tt*R rows further down.
// Backward: logical step u is row t = T-1-u, so rows go DOWN with u; the base is the tile's lowest
// row t_low = T - tu0 - ROWS (negative for the last, partial tile: such rows are masked and never
// dereferenced) and thread (tt, tc) starts (WT-1-tt)*R rows above it.
// ---------------------------------------------------------------------------------------------
template <class G, bool BWD>
struct TileAddr {
    int64_t base;   // element index of the tile's reference corner (uniform)
    uint32_t toff;  // this thread's byte offset from it
    int64_t C;
    __device__ __forceinline__ TileAddr(const Args &A, int64_t tu0, int g, int tt, int tc) : C(A.C)
    {
        if constexpr (!BWD) {
            base = tu0 * A.C + (int64_t)g * G::COLS;
            toff = ((uint32_t)(tt * G::R) * (uint32_t)A.C + (uint32_t)(tc * G::VEC)) * 4u;
        } else {
            base = (A.T - tu0 - G::ROWS) * A.C + (int64_t)g * G::COLS;
            toff = ((uint32_t)((G::WT - 1 - tt) * G::R) * (uint32_t)A.C + (uint32_t)(tc * G::VEC)) * 4u;
        }
    }
    // address of the thread's row j of tensor p, shifted by `shift` rows (+1: lambda one row ahead,
    // -1: h one row behind; backward only)
    __device__ __forceinline__ const float *at(const float *p, int j, int shift = 0) const
    {
        const float *row = BWD ? p + (base + (int64_t)(G::R - 1 - j + shift) * C) : p + (base + (int64_t)(j + shift) * C);
        return reinterpret_cast<const float *>(reinterpret_cast<const char *>(row) + (size_t)toff);
    }
    __device__ __forceinline__ float *at(float *p, int j) const
    {
        return const_cast<float *>(at(static_cast<const float *>(p), j, 0));
    }
};

// The thread's R rows of the two scan operands.
template <class G>
struct Rows {
    vec<G::VEC> a[G::R], b[G::R];
};

// Loads the thread's R rows.  `interior` is workgroup-uniform: no row or column of the tile needs
// masking (and, backward, no row is one of the boundary cases u == 0, t == 0).  Masked steps are the
// identity pair (1, 0).
template <class G, bool BWD>
__device__ __forceinline__ void tile_load(const Args &A, const TileAddr<G, BWD> &ad, int64_t u0, bool col_ok,
                                          bool interior, Rows<G> &r)
{
    constexpr int R = G::R, VEC = G::VEC;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int64_t u = u0 + j;
        vec<VEC> va = splat<VEC>(1.0f), vb = splat<VEC>(0.0f);
        if (interior || (col_ok && u < A.T)) {
            vb = ld<VEC>(ad.at(A.b, j));
            if constexpr (!BWD) {
                va = ld<VEC>(ad.at(A.a, j));
            } else {
                va = splat<VEC>(0.0f);  // the last row has no successor
                if (interior || u > 0) va = ld<VEC>(ad.at(A.a, j, +1));
            }
        }
        r.a[j] = va;
        r.b[j] = vb;
    }
}

// Backward only: h one row behind each step (h[-1] = h0, zero when h0 is null).
template <class G>
__device__ __forceinline__ void tile_load_hprev(const Args &A, const TileAddr<G, true> &ad, int64_t u0, int64_t col,
                                                bool col_ok, bool interior, vec<G::VEC> (&hp)[G::R])
{
    constexpr int R = G::R, VEC = G::VEC;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int64_t u = u0 + j;
        vec<VEC> v = splat<VEC>(0.0f);
        if (interior || (col_ok && u < A.T - 1)) v = ld<VEC>(ad.at(A.hprev, j, -1));
        else if (col_ok && u == A.T - 1 && A.h0) v = ld<VEC>(A.h0 + col);
        hp[j] = v;
    }
}

// Phase 1 of Algorithm 1 for one thread: P = prod a_j (fp64),  S = recurrence over the rows from
// state 0 (fp32: at most R roundings, each relative to the running value).
template <class G>
__device__ __forceinline__ void local_reduce(const Rows<G> &r, dvec<G::VEC> &P, vec<G::VEC> &S)
{
    dvec<G::VEC> p = widen<G::VEC>(r.a[0]);
    vec<G::VEC> s = r.b[0];
#pragma unroll
    for (int j = 1; j < G::R; ++j) {
        p *= widen<G::VEC>(r.a[j]);
        s = vfma<G::VEC>(r.a[j], s, r.b[j]);
    }
    P = p;
    S = s;
}

// Phase 3 for one thread: re-run the recurrence over the registers from carry-in c; b becomes the output.
template <class G>
__device__ __forceinline__ void rescan(Rows<G> &r, vec<G::VEC> c)
{
    vec<G::VEC> s = c;
#pragma unroll
    for (int j = 0; j < G::R; ++j) {
        s = vfma<G::VEC>(r.a[j], s, r.b[j]);
        r.b[j] = s;
    }
}

template <class G, bool BWD>
__device__ __forceinline__ void tile_store(const Args &A, const TileAddr<G, BWD> &ad, int64_t u0, int64_t col,
                                           bool col_ok, bool interior, const Rows<G> &r, const vec<G::VEC> *hp)
{
    constexpr int R = G::R, VEC = G::VEC;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int64_t u = u0 + j;
        if (interior || (col_ok && u < A.T)) {
            if constexpr (!BWD) {
                st<VEC>(ad.at(A.out0, j), r.b[j]);
            } else {
                if (A.out0) st<VEC>(ad.at(A.out0, j), r.b[j]);
                if (A.out1) st<VEC>(ad.at(A.out1, j), r.b[j] * hp[j]);
                if (!interior && u == A.T - 1 && A.gh0)  // row 0: grad_h0 = lambda[0] * g_0
                    st<VEC>(A.gh0 + col, ld<VEC>(A.a + col) * r.b[j]);
            }
        }
    }
}

// `interior` test shared by the kernels: tile starts at logical step tu0, covers ROWS steps.
template <class G, bool BWD>
__device__ __forceinline__ bool tile_interior(const Args &A, int64_t tu0, int g)
{
    const bool cols_full = ((int64_t)(g + 1) * G::COLS <= A.C);
    if constexpr (!BWD) return cols_full && (tu0 + G::ROWS <= A.T);
    else return cols_full && tu0 > 0 && (tu0 + G::ROWS < A.T);
}

// Phase 2 inside a tile: thread (tt, tc) gets the composition of the summaries of the threads with
// smaller tt in its columns (identity for tt == 0).  sP/sS must have been filled and a barrier passed.
template <class G>
__device__ __forceinline__ void lds_exclusive(const dvec<G::VEC> (*sP)[G::WC], const vec<G::VEC> (*sS)[G::WC], int tt,
                                              int tc, dvec<G::VEC> &Pe, dvec<G::VEC> &Se)
{
    dvec<G::VEC> pe = dsplat<G::VEC>(1.0), se = dsplat<G::VEC>(0.0);
    for (int i = 0; i < tt; ++i) {
        const dvec<G::VEC> p = sP[i][tc];
        const dvec<G::VEC> s = widen<G::VEC>(sS[i][tc]);
        se = dfma<G::VEC>(p, se, s);
        pe *= p;
    }
    Pe = pe;
    Se = se;
}

template <int N>
__device__ __forceinline__ dvec<N> ldd(const double *p)
{
    return *reinterpret_cast<const dvec<N> *>(p);
}
template <int N>
__device__ __forceinline__ void std_(double *p, dvec<N> v)
{
    *reinterpret_cast<dvec<N> *>(p) = v;
}

// ---------------------------------------------------------------------------------------------
// Three-phase variant, kernel 1: per-chunk reduce (Algorithm 1, first parallel-for).
// grid = K*G workgroups, workgroup (k, g) walks the M tiles of chunk k in column group g.
// ---------------------------------------------------------------------------------------------
template <class G, bool BWD>
__global__ __launch_bounds__(G::THREADS) void k_reduce(const Args A)
{
    constexpr int VEC = G::VEC, R = G::R, WC = G::WC, WT = G::WT, ROWS = G::ROWS;
    __shared__ dvec<VEC> sP[WT][WC];
    __shared__ vec<VEC> sS[WT][WC];
    const int tid = threadIdx.x, tc = tid % WC, tt = tid / WC;
    const int g = (int)(blockIdx.x % (unsigned)A.G);
    const int64_t k = blockIdx.x / (unsigned)A.G;
    const int64_t col = ((int64_t)g * WC + tc) * VEC;
    const bool col_ok = col < A.C;

    dvec<VEC> Pc = dsplat<VEC>(1.0), Sc = dsplat<VEC>(0.0);  // chunk total so far (tt == WT-1 only)
    for (int m = 0; m < A.M; ++m) {
        const int64_t tu0 = (k * A.M + m) * ROWS;
        if (tu0 >= A.T) break;
        const bool interior = tile_interior<G, BWD>(A, tu0, g);
        Rows<G> r;
        dvec<VEC> P;
        vec<VEC> S;
        const TileAddr<G, BWD> ad(A, tu0, g, tt, tc);
        tile_load<G, BWD>(A, ad, tu0 + (int64_t)tt * R, col_ok, interior, r);
        local_reduce<G>(r, P, S);
        if (m > 0) __syncthreads();  // the previous tile's summaries have been consumed
        sP[tt][tc] = P;
        sS[tt][tc] = S;
        __syncthreads();
        if (tt == WT - 1) {
            dvec<VEC> Pe, Se;
            lds_exclusive<G>(sP, sS, tt, tc, Pe, Se);
            // tile total = (earlier threads) (+) (own rows); chunk total = (earlier tiles) (+) (tile total)
            const dvec<VEC> St = dfma<VEC>(P, Se, widen<VEC>(S)), Pt = Pe * P;
            Sc = dfma<VEC>(Pt, Sc, St);
            Pc *= Pt;
        }
    }
    if (tt == WT - 1 && col_ok) {
        std_<VEC>(A.aggP + k * A.C + col, Pc);
        std_<VEC>(A.aggS + k * A.C + col, Sc);
    }
}

// ---------------------------------------------------------------------------------------------
// Three-phase variant, kernel 3: per-chunk rescan from the carry (Algorithm 1, second parallel-for).
// ---------------------------------------------------------------------------------------------
template <class G, bool BWD>
__global__ __launch_bounds__(G::THREADS) void k_fixup(const Args A)
{
    constexpr int VEC = G::VEC, R = G::R, WC = G::WC, WT = G::WT, ROWS = G::ROWS;
    __shared__ dvec<VEC> sP[WT][WC];
    __shared__ vec<VEC> sS[WT][WC];
    __shared__ dvec<VEC> sTot[2][WC];
    const int tid = threadIdx.x, tc = tid % WC, tt = tid / WC;
    const int g = (int)(blockIdx.x % (unsigned)A.G);
    const int64_t k = blockIdx.x / (unsigned)A.G;
    const int64_t col = ((int64_t)g * WC + tc) * VEC;
    const bool col_ok = col < A.C;

    dvec<VEC> cc = dsplat<VEC>(0.0);  // state entering the current tile
    if (col_ok) cc = ldd<VEC>(A.carry + k * A.C + col);

    for (int m = 0; m < A.M; ++m) {
        const int64_t tu0 = (k * A.M + m) * ROWS;
        if (tu0 >= A.T) break;
        const bool interior = tile_interior<G, BWD>(A, tu0, g);
        const int64_t u0 = tu0 + (int64_t)tt * R;
        Rows<G> r;
        vec<VEC> hp[BWD ? R : 1], S;
        dvec<VEC> P;
        const TileAddr<G, BWD> ad(A, tu0, g, tt, tc);
        tile_load<G, BWD>(A, ad, u0, col_ok, interior, r);
        if constexpr (BWD) {
            if (A.out1) tile_load_hprev<G>(A, ad, u0, col, col_ok, interior, hp);
        }
        local_reduce<G>(r, P, S);
        sP[tt][tc] = P;
        sS[tt][tc] = S;
        __syncthreads();
        dvec<VEC> Pe, Se;
        lds_exclusive<G>(sP, sS, tt, tc, Pe, Se);
        if (tt == WT - 1) {
            sTot[0][tc] = Pe * P;
            sTot[1][tc] = dfma<VEC>(P, Se, widen<VEC>(S));
        }
        rescan<G>(r, narrow<VEC>(dfma<VEC>(Pe, cc, Se)));
        tile_store<G, BWD>(A, ad, u0, col, col_ok, interior, r, hp);
        __syncthreads();
        cc = dfma<VEC>(sTot[0][tc], cc, sTot[1][tc]);
    }
}

// ---------------------------------------------------------------------------------------------
// Single-pass variant.  Tiles are handed out by an atomic ticket in time-major order (column group
// fastest), so every predecessor of a tile already holds a ticket and publishes its summary without
// waiting on anybody: the waits below always end.  A tile
//   1. loads its rows, reduces them, publishes its (P, S) summary,
//   2. looks back over its predecessors in windows of WT tiles (thread (tt, tc) polls predecessor
//      k-1-w*WT-tt for its own columns) composing summaries until it meets a published inclusive
//      state, which gives its carry-in,
//   3. publishes its own inclusive state, re-runs the recurrence over its registers and stores.
// A published word carries 32 payload bits and the call's epoch in one 64-bit relaxed agent-scope
// atomic, so the flag can never be seen without its value and no fence or workspace clear is needed
// between calls; the flag is never a data value.  Per tile and column there are four words: the two
// halves of the fp64 product P, the fp32 sum S, and (later) the fp32 inclusive state.
// ---------------------------------------------------------------------------------------------
enum { ST_AGG = 1, ST_INCL = 2 };

__device__ __forceinline__ unsigned long long lb_pack(uint32_t bits, uint32_t epoch)
{
    return ((unsigned long long)epoch << 32) | (unsigned long long)bits;
}
__device__ __forceinline__ void lb_store(unsigned long long *p, unsigned long long w)
{
    __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long lb_load(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <class G, bool BWD, bool HP_LATE>
__global__ __launch_bounds__(G::THREADS) void k_lookback(const Args A)
{
    constexpr int VEC = G::VEC, R = G::R, WC = G::WC, WT = G::WT, ROWS = G::ROWS;
    __shared__ dvec<VEC> sP[WT][WC];
    __shared__ vec<VEC> sS[WT][WC];
    __shared__ int sSt[WT][WC];
    __shared__ dvec<VEC> sTot[2][WC];
    __shared__ dvec<VEC> sCarry[WC];
    __shared__ uint32_t sTicket;
    const int tid = threadIdx.x, tc = tid % WC, tt = tid / WC;
    // the host keeps K*G below 2^31, so a call's tickets fit 32 bits
    if (tid == 0) sTicket = (uint32_t)(atomicAdd(A.ticket, 1ull) - A.ticket_base);
    __syncthreads();
    const uint32_t ticket = __builtin_amdgcn_readfirstlane(sTicket);
    const int g = (int)(ticket % (uint32_t)A.G);
    const int64_t k = (int64_t)(ticket / (uint32_t)A.G);
    if (k >= A.K) return;  // cannot happen with a matching launch; keeps a mismatched one in bounds
    const int64_t col = ((int64_t)g * WC + tc) * VEC;
    const bool col_ok = col < A.C;
    const int64_t tu0 = k * ROWS;
    const int64_t u0 = tu0 + (int64_t)tt * R;
    const bool interior = tile_interior<G, BWD>(A, tu0, g);
    const uint32_t epoch = A.epoch;

    Rows<G> r;
    vec<VEC> hp[BWD ? R : 1], S;
    dvec<VEC> P;
    const TileAddr<G, BWD> ad(A, tu0, g, tt, tc);
    tile_load<G, BWD>(A, ad, u0, col_ok, interior, r);
    if constexpr (BWD && !HP_LATE) {
        if (A.out1) tile_load_hprev<G>(A, ad, u0, col, col_ok, interior, hp);
    }
    local_reduce<G>(r, P, S);
    sP[tt][tc] = P;
    sS[tt][tc] = S;
    __syncthreads();
    dvec<VEC> Pe, Se;
    lds_exclusive<G>(sP, sS, tt, tc, Pe, Se);
    const bool publish = (k + 1 < A.K) && col_ok;
    if (tt == WT - 1) {
        const dvec<VEC> Pt = Pe * P;
        // the published S is fp32; keep the same rounded value locally so that every tile composes
        // exactly what its successors read
        const vec<VEC> St = narrow<VEC>(dfma<VEC>(P, Se, widen<VEC>(S)));
        sTot[0][tc] = Pt;
        sTot[1][tc] = widen<VEC>(St);
        if (publish) {
            unsigned long long *w = A.lbAgg + (k * A.C + col) * 3;
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const unsigned long long pb = (unsigned long long)__double_as_longlong(Pt[v]);
                lb_store(w + 3 * v, lb_pack((uint32_t)pb, epoch));
                lb_store(w + 3 * v + 1, lb_pack((uint32_t)(pb >> 32), epoch));
                lb_store(w + 3 * v + 2, lb_pack(__float_as_uint(St[v]), epoch));
            }
        }
    }
    __syncthreads();  // every thread is done reading sP/sS; they now hold the look-back window

    // ---- look-back --------------------------------------------------------------------------
    // (Pr, Sr): composition of the predecessors visited so far, nearest first (tt == 0 threads only)
    dvec<VEC> Pr = dsplat<VEC>(1.0), Sr = dsplat<VEC>(0.0);
    bool done = false;
    for (int64_t base = k - 1;; base -= WT) {
        const int64_t pred = base - tt;
        int status = ST_INCL;
        dvec<VEC> vP = dsplat<VEC>(0.0);
        vec<VEC> vS = splat<VEC>(0.0f);
        if (pred < 0 || !col_ok) {
            // before the first tile: the initial state (h0 forward, zero backward)
            if (!BWD && pred == -1 && col_ok && A.h0) vS = ld<VEC>(A.h0 + col);
        } else {
            const unsigned long long *wi = A.lbIncl + (pred * A.C + col);
            const unsigned long long *wa = A.lbAgg + (pred * A.C + col) * 3;
            uint32_t spins = 0;
            for (;;) {
                bool ok = true;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const unsigned long long w = lb_load(wi + v);
                    ok = ok && ((uint32_t)(w >> 32) == epoch);
                    vS[v] = __uint_as_float((uint32_t)w);
                }
                if (ok) { status = ST_INCL; break; }
                ok = true;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const unsigned long long wl = lb_load(wa + 3 * v), wh = lb_load(wa + 3 * v + 1),
                                             ws = lb_load(wa + 3 * v + 2);
                    ok = ok && ((uint32_t)(wl >> 32) == epoch) && ((uint32_t)(wh >> 32) == epoch) &&
                         ((uint32_t)(ws >> 32) == epoch);
                    vP[v] = __longlong_as_double((long long)((wh << 32) | (wl & 0xffffffffull)));
                    vS[v] = __uint_as_float((uint32_t)ws);
                }
                if (ok) { status = ST_AGG; break; }
                if (++spins > A.spin_limit) {  // give up: flag the error, finish with a zero state
                    atomicOr(A.err, 1u);
                    vS = splat<VEC>(0.0f);
                    status = ST_INCL;
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
            }
        }
        sP[tt][tc] = vP;
        sS[tt][tc] = vS;
        sSt[tt][tc] = status;
        __syncthreads();
        if (tt == 0 && !done) {
            dvec<VEC> carry = dsplat<VEC>(0.0);
#pragma unroll
            for (int j = 0; j < WT; ++j) {
                const int stj = sSt[j][tc];
                const dvec<VEC> p = sP[j][tc];
                const dvec<VEC> s = widen<VEC>(sS[j][tc]);
                if (!done) {
                    // (p, s) is earlier in time than everything in (Pr, Sr): it goes on the left
                    const dvec<VEC> t = dfma<VEC>(Pr, s, Sr);
                    if (stj == ST_INCL) { carry = t; done = true; }
                    else { Sr = t; Pr = p * Pr; }
                }
            }
            if (done) {
                sCarry[tc] = carry;
                if (publish) {
                    const vec<VEC> incl = narrow<VEC>(dfma<VEC>(sTot[0][tc], carry, sTot[1][tc]));
#pragma unroll
                    for (int v = 0; v < VEC; ++v)
                        lb_store(A.lbIncl + (k * A.C + col + v), lb_pack(__float_as_uint(incl[v]), epoch));
                }
            }
        }
        if (!__syncthreads_or((tt == 0 && !done) ? 1 : 0)) break;
    }

    // ---- rescan from the carry and store -------------------------------------------------------
    rescan<G>(r, narrow<VEC>(dfma<VEC>(Pe, sCarry[tc], Se)));
    if constexpr (BWD && HP_LATE) {
        if (A.out1) tile_load_hprev<G>(A, ad, u0, col, col_ok, interior, hp);
    }
    tile_store<G, BWD>(A, ad, u0, col, col_ok, interior, r, hp);
}

}  // namespace linrec
