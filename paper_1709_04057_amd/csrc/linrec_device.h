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
//
// Two things vary around that core.  The FORM (template parameter of the tile functions): the plain
// recurrence, the gated layer of Section 3.1 or the LSTM cell of Section 3.2, the latter two with
// their activations applied in a prologue after the loads and their chain rule in an epilogue before
// the stores.  And the STORAGE type of the tensors (part of the tile geometry): fp32, or bf16 with
// the packed words kept in registers; the arithmetic is fp32 steps and fp64 chunk products always.
#pragma once
#include "linrec_launch.h"

namespace linrec {

// Storage type of the [T, C] tensors and of the [C] state vectors: fp32, or bf16 (the upper half of an
// fp32; widened exactly on load, rounded to nearest even on store).  Arithmetic is the same either way.
// IO_BF16 keeps the rows packed in registers between the load and the store (the plain recurrence);
// IO_BF16W widens them on load, for the gated forms, whose register tile holds computed fp32 values.
enum IoType { IO_F32 = 0, IO_BF16 = 1, IO_BF16W = 2 };

template <int VEC_, int R_, int WC_, int WT_, int IO_ = IO_F32>
struct Geo {
    static constexpr int VEC = VEC_, R = R_, WC = WC_, WT = WT_, IO = IO_;
    static constexpr int ES = IO_ == IO_F32 ? 4 : 2;  // bytes per stored element
    static constexpr int THREADS = WC * WT, ROWS = WT * R, COLS = WC * VEC;
    // minimum wavefronts per SIMD handed to __launch_bounds__ (1 = leave the choice to the compiler,
    // which lands on 2*R*VEC data registers plus 40-100 of overhead per lane)
#ifdef LINREC_OCC_OVERRIDE
    static constexpr int OCC = LINREC_OCC_OVERRIDE;
#else
    static constexpr int OCC = 1;
#endif
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

// Streaming accesses: every element is touched once, so loads and stores carry the non-temporal
// hint and do not displace the look-back words from the caches.
#ifndef LINREC_NT_LOAD
#define LINREC_NT_LOAD 1
#endif
#ifndef LINREC_NT_STORE
#define LINREC_NT_STORE 1
#endif
template <int N>
__device__ __forceinline__ vec<N> ld(const float *p)
{
#if LINREC_NT_LOAD
    return __builtin_nontemporal_load(reinterpret_cast<const vec<N> *>(p));
#else
    return *reinterpret_cast<const vec<N> *>(p);
#endif
}
template <int N>
__device__ __forceinline__ void st(float *p, vec<N> v)
{
#if LINREC_NT_STORE
    __builtin_nontemporal_store(v, reinterpret_cast<vec<N> *>(p));
#else
    *reinterpret_cast<vec<N> *>(p) = v;
#endif
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
// Forms of the recurrence.  FORM_PLAIN is h = a*h + b on the caller's lambda.  FORM_GATED serves the
// gated layers of Section 3.1 (g = sigmoid(g_pre), h_t = g_t*h_{t-1} + (1-g_t)*i_t): the register
// tile holds the gate's COMPLEMENT c = 1 - g = sigmoid(-g_pre), computed without cancellation, and a
// step is h = (h - c*h) + b.  A gate close to one is then as accurate as any other -- rounding g
// itself to fp32 would be an error of 2^-25 against a complement that may be 1e-6, i.e. a wrong
// decay rate, which adds up over the 1/c steps such a gate remembers.
// ---------------------------------------------------------------------------------------------
// FORM_LSTM is the cell of Section 3.2's GILR-LSTM, c_t = f_t*c_{t-1} + i_t*z_t, h_t = o_t*c_t, with the forget
// gate in the same complement form.  (enum Form: linrec_launch.h)

template <int FORM, int N>
__device__ __forceinline__ vec<N> step(vec<N> a, vec<N> s, vec<N> b)
{
    if constexpr (FORM == FORM_PLAIN) return vfma<N>(a, s, b);
    else return vfma<N>(-a, s, s) + b;
}
// the multiplier of a step as an fp64 factor of the chunk product
template <int FORM, int N>
__device__ __forceinline__ dvec<N> factor(vec<N> a)
{
    if constexpr (FORM == FORM_PLAIN) return widen<N>(a);
    else return dsplat<N>(1.0) - widen<N>(a);
}
// sigmoid(z) = 1 / (1 + exp(-z)) from one v_exp_f32 and one v_rcp_f32 (each good to about one ulp).
// The relative accuracy holds in BOTH tails: for z -> -inf the result is 1/exp(-z) with nothing added
// that matters, for z -> +inf it is 1/(1 + tiny); exp overflowing to +inf gives exactly 0.  So the
// gate's complement is sigmoid(-g_pre), not 1 - sigmoid(g_pre).  A NaN pre-activation gives NaN.
__device__ __forceinline__ float sigmoid_f32(float z)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z * -1.44269504088896340736f));
}
template <int N>
__device__ __forceinline__ vec<N> gate_value(vec<N> z)
{
    vec<N> r;
#pragma unroll
    for (int i = 0; i < N; ++i) r[i] = sigmoid_f32(z[i]);
    return r;
}
template <int N>
__device__ __forceinline__ vec<N> gate_complement(vec<N> z)
{
    vec<N> r;
#pragma unroll
    for (int i = 0; i < N; ++i) r[i] = sigmoid_f32(-z[i]);
    return r;
}
// sigmoid(z) and 1 - sigmoid(z) for the derivative g*(1-g), where the complement only needs its
// absolute accuracy
template <int N>
__device__ __forceinline__ void gate_both(vec<N> z, vec<N> &g, vec<N> &c)
{
    g = gate_value<N>(z);
    c = splat<N>(1.0f) - g;
}
// tanh(y) = 1 - 2 / (1 + exp(2y)): any sign, saturates to +-1 without overflow trouble (exp -> inf gives
// rcp -> 0), NaN stays NaN.  Its ABSOLUTE error is about 1e-7 everywhere (near zero the subtraction cancels,
// so small results lose relative, not absolute, accuracy).  That is what the recurrence needs: tau enters the
// state as the addend (1-g)*tau -- like one more rounding of a value of order one per step -- and the
// gradients through 1 - tau^2; both tolerances are relative to the largest value of the tensor.  (A first
// version switched to an odd series below |y| < 1/8 for relative accuracy; these kernels are bound by
// vector-ALU issue slots, and the series, compare and select were 7 of their ~37 slots per element.)
__device__ __forceinline__ float tanh_f32(float y)
{
#ifdef LINREC_TANH_SERIES
    const float big = fmaf(-2.0f, __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(y * 2.88539008177792681472f)), 1.0f);
    const float y2 = y * y;
    const float small = y * fmaf(y2, fmaf(y2, fmaf(y2, -17.0f / 315.0f, 2.0f / 15.0f), -1.0f / 3.0f), 1.0f);
    return fabsf(y) < 0.125f ? small : big;
#else
    return fmaf(-2.0f, __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(y * 2.88539008177792681472f)), 1.0f);
#endif
}
// the impulse activation tau of Section 3.1: tanh, or the identity
template <int N>
__device__ __forceinline__ vec<N> impulse(vec<N> y, int tau)
{
    if (!tau) return y;
    vec<N> r;
#pragma unroll
    for (int i = 0; i < N; ++i) r[i] = tanh_f32(y[i]);
    return r;
}

// ---------------------------------------------------------------------------------------------
// Tile addressing.  Every tensor access of a tile goes through a buffer resource whose base is a
// workgroup-uniform corner of the tile, plus a per-thread 32-bit byte offset (one vector register
// for the whole tile) plus a per-row scalar byte offset.  No 64-bit address ever lives in a vector
// register, and rows past the end of the tensor fall outside the resource's range (loads return 0,
// stores are dropped) on top of the explicit masks below.  The host guarantees
// (ROWS*C + COLS)*4 < 2^32.
//
// Forward: the corner is the tile's first row; thread (tt, tc) starts tt*rk rows further down
// (rk = rows per thread of this tile, R except in the short tiles that end the sequence).
// Backward: logical step u is row t = T-1-u, so rows go DOWN with u; the corner is the tile's lowest
// row t_low = T - tu0 - WT*rk (negative for the last, partial tile: those rows are masked and never
// touched) and thread (tt, tc) starts (WT-1-tt)*rk rows above it.
// ---------------------------------------------------------------------------------------------
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
constexpr int kBufNT = 2;  // cache-policy bit "nt": streaming data, touched once

template <int N>
__device__ __forceinline__ vec<N> buf_ld(rsrc_t rs, uint32_t voff, uint32_t soff)
{
    if constexpr (N == 4) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, LINREC_NT_LOAD ? kBufNT : 0);
        return __builtin_bit_cast(vec<4>, v);
    } else if constexpr (N == 2) {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soff, LINREC_NT_LOAD ? kBufNT : 0);
        return __builtin_bit_cast(vec<2>, v);
    } else {
        static_assert(N == 1, "one, two or four columns per thread");
        const unsigned int v = __builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff, LINREC_NT_LOAD ? kBufNT : 0);
        return vec<1>(__uint_as_float(v));
    }
}
template <int N>
__device__ __forceinline__ void buf_st(rsrc_t rs, uint32_t voff, uint32_t soff, vec<N> v)
{
    if constexpr (N == 4) {
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rs, voff, soff, LINREC_NT_STORE ? kBufNT : 0);
    } else if constexpr (N == 2) {
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, v), rs, voff, soff, LINREC_NT_STORE ? kBufNT : 0);
    } else {
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v[0]), rs, voff, soff, LINREC_NT_STORE ? kBufNT : 0);
    }
}

// bf16 <-> fp32.  Two bf16 values travel in one 32-bit word, the lower-addressed one in the low half.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned int pack_bf16(float lo, float hi)
{
    const vec<2> v = {lo, hi};
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2));  // v_cvt_pk_bf16_f32: RNE
}
__device__ __forceinline__ float bf16_lo(unsigned int w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned int w) { return __uint_as_float(w & 0xffff0000u); }

// Tile element access in the geometry's storage type: VEC adjacent columns of one row as fp32.
template <class G>
__device__ __forceinline__ vec<G::VEC> gld(rsrc_t rs, uint32_t voff, uint32_t soff)
{
    constexpr int N = G::VEC;
    if constexpr (G::IO == IO_F32) {
        return buf_ld<N>(rs, voff, soff);
    } else if constexpr (N == 4) {
        const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soff, LINREC_NT_LOAD ? kBufNT : 0);
        return vec<4>{bf16_lo(w[0]), bf16_hi(w[0]), bf16_lo(w[1]), bf16_hi(w[1])};
    } else if constexpr (N == 2) {
        const unsigned int w = __builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff, LINREC_NT_LOAD ? kBufNT : 0);
        return vec<2>{bf16_lo(w), bf16_hi(w)};
    } else {
        const unsigned short w = __builtin_amdgcn_raw_buffer_load_b16(rs, voff, soff, LINREC_NT_LOAD ? kBufNT : 0);
        return vec<1>(__uint_as_float((unsigned int)w << 16));
    }
}
template <class G>
__device__ __forceinline__ void gst(rsrc_t rs, uint32_t voff, uint32_t soff, vec<G::VEC> v)
{
    constexpr int N = G::VEC;
    if constexpr (G::IO == IO_F32) {
        buf_st<N>(rs, voff, soff, v);
        // A store of more than 64 bits still reads its data registers during the next two cycles.  The
        // epilogues of the gated forms compute the next row right behind each store, in the registers
        // the stored temporaries just left, and the compiler does not space the two apart for this
        // form of the instruction (a register as scalar offset): some lanes then stored the next
        // row's intermediate values.  Two idle cycles per store are not measurable.  (The statement
        // names the stored registers as its operand, so nothing that overwrites them can be scheduled
        // between the store and the pause.)
#ifndef LINREC_NO_STORE_PAUSE  // (defined only by the test that shows the build's assembly check finds the hazard)
        if constexpr (N == 4) asm volatile("s_nop 1" : "+v"(v));
#endif
    } else if constexpr (N == 4) {
        const u32x2 w = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        __builtin_amdgcn_raw_buffer_store_b64(w, rs, voff, soff, LINREC_NT_STORE ? kBufNT : 0);
    } else if constexpr (N == 2) {
        __builtin_amdgcn_raw_buffer_store_b32(pack_bf16(v[0], v[1]), rs, voff, soff, LINREC_NT_STORE ? kBufNT : 0);
    } else {
        __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(pack_bf16(v[0], 0.0f) & 0xffffu), rs, voff, soff,
                                              LINREC_NT_STORE ? kBufNT : 0);
    }
}
// The same for the [C] vectors (initial state and its gradient), addressed by column through a pointer.
template <class G>
__device__ __forceinline__ vec<G::VEC> pld(const float *base, int64_t col)
{
    constexpr int N = G::VEC;
    if constexpr (G::IO == IO_F32) {
        return ld<N>(base + col);
    } else {
        const unsigned short *p = reinterpret_cast<const unsigned short *>(base) + col;
        vec<N> r;
#pragma unroll
        for (int i = 0; i < N; ++i) r[i] = __uint_as_float((unsigned int)p[i] << 16);
        return r;
    }
}
template <class G>
__device__ __forceinline__ void pst(float *base, int64_t col, vec<G::VEC> v)
{
    constexpr int N = G::VEC;
    if constexpr (G::IO == IO_F32) {
        st<N>(base + col, v);
    } else {
        unsigned short *p = reinterpret_cast<unsigned short *>(base) + col;
#pragma unroll
        for (int i = 0; i < N; ++i) p[i] = (unsigned short)(pack_bf16(v[i], 0.0f) & 0xffffu);
    }
}

// How a thread keeps one row of its VEC columns between the load and the store.  fp32 storage: the
// fp32 values themselves.  bf16 storage: the packed words as loaded, two elements per register, widened
// where they are used -- a register then carries the same number of BYTES in flight as with fp32
// storage, which is what the achieved bandwidth depends on (holding widened values halved it).
template <int N>
using uvec = unsigned int __attribute__((ext_vector_type(N)));
template <int VEC, int IO>
struct RowSel {
    using type = vec<VEC>;
};
template <int VEC>
struct RowSel<VEC, IO_BF16> {
    static_assert(VEC == 2 || VEC == 4, "bf16 storage: two or four columns per thread");
    using type = uvec<VEC / 2>;
};
template <class G>
using row_t = typename RowSel<G::VEC, G::IO>::type;

template <class G>
__device__ __forceinline__ vec<G::VEC> unpack(row_t<G> w)
{
    if constexpr (G::IO != IO_BF16) {
        return w;
    } else {
        vec<G::VEC> v;
#pragma unroll
        for (int i = 0; i < G::VEC / 2; ++i) {
            v[2 * i] = bf16_lo(w[i]);
            v[2 * i + 1] = bf16_hi(w[i]);
        }
        return v;
    }
}
template <class G>
__device__ __forceinline__ row_t<G> pack(vec<G::VEC> v)
{
    if constexpr (G::IO != IO_BF16) {
        return v;
    } else {
        row_t<G> w;
#pragma unroll
        for (int i = 0; i < G::VEC / 2; ++i) w[i] = pack_bf16(v[2 * i], v[2 * i + 1]);
        return w;
    }
}
// Hides where a packed row came from.  The rescan widens the same words the reduce phase widened; left
// alone, the compiler keeps the widened copies alive from one phase to the other and the tile occupies
// twice the registers again.
template <class G>
__device__ __forceinline__ row_t<G> reread(row_t<G> w)
{
    if constexpr (G::IO == IO_BF16) {
#pragma unroll
        for (int i = 0; i < G::VEC / 2; ++i) {
            unsigned int x = w[i];
            asm volatile("" : "+v"(x));
            w[i] = x;
        }
    }
    return w;
}
// a row of copies of x (x must be a bf16 value when the storage is bf16: 0, 1, +-inf are)
template <class G>
__device__ __forceinline__ row_t<G> row_const(float x)
{
    if constexpr (G::IO != IO_BF16) {
        return splat<G::VEC>(x);
    } else {
        const unsigned int b = __float_as_uint(x);
        return row_t<G>((b >> 16) | (b & 0xffff0000u));
    }
}
template <class G>
__device__ __forceinline__ row_t<G> rld(rsrc_t rs, uint32_t voff, uint32_t soff)
{
    if constexpr (G::IO != IO_BF16) {
        return gld<G>(rs, voff, soff);
    } else if constexpr (G::VEC == 4) {
        return __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soff, LINREC_NT_LOAD ? kBufNT : 0);
    } else {
        return row_t<G>(__builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff, LINREC_NT_LOAD ? kBufNT : 0));
    }
}
template <class G>
__device__ __forceinline__ void rst(rsrc_t rs, uint32_t voff, uint32_t soff, row_t<G> w)
{
    if constexpr (G::IO == IO_F32) {
        buf_st<G::VEC>(rs, voff, soff, w);
    } else if constexpr (G::IO == IO_BF16W) {
        gst<G>(rs, voff, soff, w);
    } else if constexpr (G::VEC == 4) {
        __builtin_amdgcn_raw_buffer_store_b64(w, rs, voff, soff, LINREC_NT_STORE ? kBufNT : 0);
    } else {
        __builtin_amdgcn_raw_buffer_store_b32(w[0], rs, voff, soff, LINREC_NT_STORE ? kBufNT : 0);
    }
}

template <class G, bool BWD>
struct TileAddr {
    int64_t base;   // element index of the tile's reference corner (uniform)
    int64_t total;  // T*C
    uint32_t toff;  // this thread's byte offset from the corner
    uint32_t rowb;  // bytes per row
    int rk;         // rows per thread of this tile: R, or R/2, R/4 for the short tiles at the end of T
    __device__ __forceinline__ TileAddr(const Args &A, int64_t tu0, int g, int tt, int tc, int rk_ = G::R)
        : total(A.T * A.C), rowb((uint32_t)A.C * (uint32_t)G::ES), rk(rk_)
    {
        if constexpr (!BWD) {
            base = tu0 * A.C + (int64_t)g * G::COLS;
            toff = (uint32_t)(tt * rk) * rowb + (uint32_t)(tc * G::VEC) * (uint32_t)G::ES;
        } else {
            base = (A.T - tu0 - (int64_t)G::WT * rk) * A.C + (int64_t)g * G::COLS;
            toff = (uint32_t)((G::WT - 1 - tt) * rk) * rowb + (uint32_t)(tc * G::VEC) * (uint32_t)G::ES;
        }
    }
    // Resource for tensor p seen `shift` rows away from the tile (+1: lambda one row ahead, -1: h one
    // row behind; backward only).  Its range ends where the tensor ends.
    __device__ __forceinline__ rsrc_t rsrc(const float *p, int shift = 0) const
    {
        const int64_t first = base + (int64_t)shift * (int64_t)(rowb / (uint32_t)G::ES);
        int64_t bytes = (total - first) * G::ES;
        if (first < 0 || bytes > 0xffffffffll) bytes = 0xffffffffll;
        if (bytes < 0) bytes = 0;
        // (tensor pointers are typed float* throughout; with bf16 storage they address 2-byte elements)
        char *origin = reinterpret_cast<char *>(const_cast<float *>(p)) + first * G::ES;
        return __builtin_amdgcn_make_buffer_rsrc(origin, 0, (int)(uint32_t)bytes, 0x00020000);
    }
    // scalar byte offset of the thread's row j < rk (rows go up with j forward, down backward)
    __device__ __forceinline__ uint32_t soff(int j) const { return (uint32_t)(BWD ? rk - 1 - j : j) * rowb; }
    // the same for a row index that differs between lanes (goes into the vector offset)
    __device__ __forceinline__ uint32_t soff_rt(int j) const { return (uint32_t)(BWD ? rk - 1 - j : j) * rowb; }
};

// The thread's R rows of the two scan operands.
template <class G>
struct Rows {
    row_t<G> a[G::R], b[G::R];
};

// Which of the thread's R rows exist, as small integers computed once per tile (row j is compared
// against them with j a compile-time constant, so the masks cost no per-row registers).
//   n   rows j < n are inside the tensor (0 when the thread's columns are outside)
//   nh  backward: rows j < nh have a row t-1 inside the tensor; row j == nh < n is row t == 0
//   first_has_next  backward: row j == 0 has a successor row t+1 (false only for the very last row T-1)
template <class G, bool BWD>
struct RowMask {
    int n, nh;
    bool first_has_next;
    __device__ __forceinline__ RowMask(const Args &A, int64_t u0, bool col_ok, int rk = G::R)
    {
        int64_t left = A.T - u0;
        left = left < 0 ? 0 : (left > rk ? rk : left);
        n = col_ok ? (int)left : 0;
        int64_t lefth = A.T - 1 - u0;
        lefth = lefth < 0 ? 0 : (lefth > rk ? rk : lefth);
        nh = col_ok ? (int)lefth : 0;
        first_has_next = u0 > 0;
    }
};

// Loads the thread's R rows.  `interior` is workgroup-uniform: no row or column of the tile needs
// masking (and, backward, no row is one of the boundary cases u == 0, t == 0).  Masked steps are the
// identity pair.  FORM_GATED: A.a holds the gate pre-activations and r.a becomes the gate complement;
// forward, A.b holds the impulse pre-activations and r.b becomes (1-g)*tau(i_pre).
// FORM_LSTM backward also returns the cell state c_t of the thread's rows in `cst` (the epilogue needs
// c_{t-1}, which is the next row's entry).
// INTERIOR is the workgroup-uniform "no row or column needs masking" as a compile-time constant: with
// it the loads are unconditional straight-line code, and the compiler's wait counters let the
// arithmetic on the first rows start while the later rows are still in flight.  (With every load
// inside a run-time condition it cannot know how many loads follow a given one and waits for all of
// them before the first use.)
template <class G, bool BWD, int FORM, int NC, bool INTERIOR>
__device__ __forceinline__ void tile_load_impl(const Args &A, const TileAddr<G, BWD> &ad, const RowMask<G, BWD> &mk,
                                               Rows<G> &r, vec<G::VEC> (&cst)[NC])
{
    constexpr int R = G::R, VEC = G::VEC;
    constexpr bool interior = INTERIOR;
    static_assert(NC == ((FORM == FORM_LSTM && BWD) ? R : 1), "cst: R entries for the LSTM cell's backward pass");
    const rsrc_t ra = ad.rsrc(A.a, BWD ? +1 : 0), rb = ad.rsrc(A.b);
    // What a masked step holds BEFORE the activations are applied: the gated forms run them over every
    // row after all loads have been issued (inside the per-row conditions they would make each load
    // wait for the one before), and sigmoid(-(+inf)) = 0, sigmoid(-(-inf)) = 1 give the identity
    // and the forgetting step.
    const float raw_identity = FORM == FORM_PLAIN ? 1.0f : __builtin_inff();
    const float raw_forget = FORM == FORM_PLAIN ? 0.0f : -__builtin_inff();
    // FORM_LSTM has a third operand per row: forward the candidate's pre-activation (A.c), backward
    // the output gate's (A.e); the addend is sigmoid(i_pre)*tanh(z_pre), resp. grad_h*sigmoid(o_pre).
    // Backward, the cell state c_t comes along as a fourth: grad_o_pre = grad_h*c_t*o(1-o) does not
    // depend on the scan and is written right here, while grad_h and o are at hand.
    constexpr bool LSTM = FORM == FORM_LSTM;
    vec<VEC> third[LSTM ? R : 1];
    const rsrc_t r3 = ad.rsrc(LSTM ? (BWD ? A.e : A.c) : A.b), r4 = ad.rsrc(LSTM && BWD ? A.hprev : A.b);
    const bool want_go = LSTM && BWD && A.out3 != nullptr;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        row_t<G> va = row_const<G>(raw_identity), vb = row_const<G>(0.0f);
        vec<VEC> v3 = splat<VEC>(0.0f), v4 = splat<VEC>(0.0f);
        if (interior || j < mk.n) {
            vb = rld<G>(rb, ad.toff, ad.soff(j));
            if constexpr (LSTM) v3 = gld<G>(r3, ad.toff, ad.soff(j));
            if constexpr (LSTM && BWD) v4 = gld<G>(r4, ad.toff, ad.soff(j));
            if constexpr (!BWD) {
                va = rld<G>(ra, ad.toff, ad.soff(j));
            } else {
                va = row_const<G>(raw_forget);  // the last row has no successor
                if (interior || j > 0 || mk.first_has_next) va = rld<G>(ra, ad.toff, ad.soff(j));
            }
        }
        r.a[j] = va;
        r.b[j] = vb;
        if constexpr (LSTM) third[j] = v3;
        if constexpr (LSTM && BWD) cst[j] = v4;
    }
    // every load is issued before any arithmetic on the rows: the scheduler may not pull activation
    // math in between the loads
    if constexpr (FORM != FORM_PLAIN) __builtin_amdgcn_sched_barrier(0);
    if constexpr (FORM == FORM_GATED && !BWD && G::R * G::VEC >= 64) {
        // Shapes of 64 elements per thread: the gate complements in one in-place loop, then the impulse.
        // (Written as below, the compiler hoists the exponentials that both branches share in front of
        // the branch and keeps 64 of them alive next to the tile: 155 instead of 125 registers for a
        // 32-element thread, more for these.  The 64-element shapes run 4-20 % faster this way; the
        // smaller ones 2-6 % slower, although they gain a wavefront per SIMD, so they keep the form below.)
#pragma unroll
        for (int j = 0; j < R; ++j) r.a[j] = gate_complement<VEC>(r.a[j]);
        if (A.tau) {
#pragma unroll
            for (int j = 0; j < R; ++j) r.b[j] = r.a[j] * impulse<VEC>(r.b[j], 1);
        } else {
#pragma unroll
            for (int j = 0; j < R; ++j) r.b[j] = r.a[j] * r.b[j];
        }
    } else if constexpr (FORM == FORM_GATED) {
        // (the choice of tau stays outside the row loops: a branch per row would cut the straight line)
        if (BWD || A.tau) {
#pragma unroll
            for (int j = 0; j < R; ++j) {
                r.a[j] = gate_complement<VEC>(r.a[j]);
                if constexpr (!BWD) r.b[j] = r.a[j] * impulse<VEC>(r.b[j], 1);
            }
        } else {
#pragma unroll
            for (int j = 0; j < R; ++j) {
                r.a[j] = gate_complement<VEC>(r.a[j]);
                r.b[j] = r.a[j] * r.b[j];
            }
        }
    }
    if constexpr (LSTM) {
        const rsrc_t rgo = ad.rsrc(BWD ? A.out3 : A.out0);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            r.a[j] = gate_complement<VEC>(r.a[j]);
            // (masked rows hold b = 0, and sigmoid(0)*tanh(0) = 0, 0*sigmoid(0) = 0)
            if constexpr (!BWD) {
                r.b[j] = gate_value<VEC>(r.b[j]) * impulse<VEC>(third[j], 1);
            } else {
                vec<VEC> og, oc;
                gate_both<VEC>(third[j], og, oc);
                if (want_go && (interior || j < mk.n))
                    gst<G>(rgo, ad.toff, ad.soff(j), r.b[j] * cst[j] * (og * oc));
                r.b[j] = r.b[j] * og;
            }
        }
    }
}

template <class G, bool BWD, int FORM = FORM_PLAIN, int NC = 1>
__device__ __forceinline__ void tile_load(const Args &A, const TileAddr<G, BWD> &ad, const RowMask<G, BWD> &mk,
                                          bool interior, Rows<G> &r, vec<G::VEC> (&cst)[NC])
{
    // (The LSTM cell's forward kernel of the 64-lane-wide shapes measures 7 % slower with the separate
    // interior path -- neither the earlier start of the arithmetic nor the order of the loads explains
    // it -- so that one keeps the masked path throughout; everything else gains 1-12 %.)
    constexpr bool kSeparateInterior = !(FORM == FORM_LSTM && !BWD && G::WC >= 64);
    if (kSeparateInterior && interior) tile_load_impl<G, BWD, FORM, NC, true>(A, ad, mk, r, cst);
    else tile_load_impl<G, BWD, FORM, NC, false>(A, ad, mk, r, cst);
}
template <class G, bool BWD, int FORM = FORM_PLAIN>
__device__ __forceinline__ void tile_load(const Args &A, const TileAddr<G, BWD> &ad, const RowMask<G, BWD> &mk,
                                          bool interior, Rows<G> &r)
{
    vec<G::VEC> none[1];
    tile_load<G, BWD, FORM, 1>(A, ad, mk, interior, r, none);
}

// Backward only: h one row behind each step (h[-1] = h0, zero when h0 is null).  Two instances like
// tile_load: with unconditional loads here the reduce phase waits for lambda and grad_h only, not
// for these loads that were issued after them.
template <class G, bool INTERIOR>
__device__ __forceinline__ void tile_load_hprev_impl(const Args &A, const TileAddr<G, true> &ad,
                                                     const RowMask<G, true> &mk, int64_t col, row_t<G> (&hp)[G::R])
{
    constexpr int R = G::R;
    const rsrc_t rh = ad.rsrc(A.hprev, -1);
#pragma unroll
    for (int j = 0; j < R; ++j) {
        row_t<G> v = row_const<G>(0.0f);
        if (INTERIOR || j < mk.nh) v = rld<G>(rh, ad.toff, ad.soff(j));
        else if (j == mk.nh && j < mk.n && A.h0) v = pack<G>(pld<G>(A.h0, col));
        hp[j] = v;
    }
}
template <class G>
__device__ __forceinline__ void tile_load_hprev(const Args &A, const TileAddr<G, true> &ad,
                                                const RowMask<G, true> &mk, int64_t col, bool interior,
                                                row_t<G> (&hp)[G::R])
{
    if (interior) tile_load_hprev_impl<G, true>(A, ad, mk, col, hp);
    else tile_load_hprev_impl<G, false>(A, ad, mk, col, hp);
}

// Phase 1 of Algorithm 1 for one thread: P = prod of the multipliers (fp64),  S = recurrence over
// the rows from state 0 (fp32: at most R roundings, each relative to the running value).
template <class G, int FORM = FORM_PLAIN>
__device__ __forceinline__ void local_reduce(const Rows<G> &r, dvec<G::VEC> &P, vec<G::VEC> &S)
{
    dvec<G::VEC> p = factor<FORM, G::VEC>(unpack<G>(r.a[0]));
    vec<G::VEC> s = unpack<G>(r.b[0]);
#pragma unroll
    for (int j = 1; j < G::R; ++j) {
        const vec<G::VEC> a = unpack<G>(r.a[j]);
        // (gated forms: p*(1 - a) as one fp64 fma, p - a*p; these kernels are short of ALU slots, not of bytes)
        if constexpr (FORM == FORM_PLAIN) p *= factor<FORM, G::VEC>(a);
        else p = dfma<G::VEC>(-widen<G::VEC>(a), p, p);
        s = step<FORM, G::VEC>(a, s, unpack<G>(r.b[j]));
    }
    P = p;
    S = s;
}

// Phase 3 for one thread: re-run the recurrence over the registers from carry-in c; b becomes the output.
template <class G, int FORM = FORM_PLAIN>
__device__ __forceinline__ void rescan(Rows<G> &r, vec<G::VEC> c)
{
    vec<G::VEC> s = c;
#pragma unroll
    for (int j = 0; j < G::R; ++j) {
        s = step<FORM, G::VEC>(unpack<G>(reread<G>(r.a[j])), s, unpack<G>(reread<G>(r.b[j])));
        r.b[j] = pack<G>(s);  // (bf16 storage: the stored value is rounded, the running state is not)
    }
}

// bf16 storage, backward: the products that depend on the unrounded g_t are formed while it is at hand.
// hp[j] (h one row behind) becomes grad_lambda, and grad_h0 = lambda[0]*g_0 is written from the row t == 0.
template <class G>
__device__ __forceinline__ void rescan_bwd_packed(const Args &A, const RowMask<G, true> &mk, int64_t col, bool interior,
                                                  Rows<G> &r, row_t<G> (&hp)[G::R], vec<G::VEC> c)
{
    vec<G::VEC> s = c;
#pragma unroll
    for (int j = 0; j < G::R; ++j) {
        s = step<FORM_PLAIN, G::VEC>(unpack<G>(reread<G>(r.a[j])), s, unpack<G>(reread<G>(r.b[j])));
        r.b[j] = pack<G>(s);
        hp[j] = pack<G>(s * unpack<G>(hp[j]));
        if (!interior && j == mk.nh && j < mk.n && A.gh0) pst<G>(A.gh0, col, pld<G>(A.a, col) * s);
    }
}

// (Two instances, as for tile_load: in the interior one the stores are straight-line code instead of
// one exec-mask branch per row.)
template <class G, bool BWD, bool INTERIOR>
__device__ __forceinline__ void tile_store_impl(const Args &A, const TileAddr<G, BWD> &ad, const RowMask<G, BWD> &mk,
                                                int64_t col, const Rows<G> &r, const row_t<G> *hp)
{
    constexpr int R = G::R;
    constexpr bool interior = INTERIOR;
    const rsrc_t r0 = ad.rsrc(A.out0), r1 = ad.rsrc(BWD ? A.out1 : A.out0);
#pragma unroll
    for (int j = 0; j < R; ++j) {
        if (interior || j < mk.n) {
            if constexpr (!BWD) {
                rst<G>(r0, ad.toff, ad.soff(j), r.b[j]);
            } else if constexpr (G::IO == IO_BF16) {  // (rescan_bwd_packed has formed grad_lambda and grad_h0)
                if (A.out0) rst<G>(r0, ad.toff, ad.soff(j), r.b[j]);
                if (A.out1) rst<G>(r1, ad.toff, ad.soff(j), hp[j]);
            } else {
                if (A.out0) rst<G>(r0, ad.toff, ad.soff(j), r.b[j]);
                if (A.out1) rst<G>(r1, ad.toff, ad.soff(j), r.b[j] * hp[j]);
                if (!interior && j == mk.nh && A.gh0)  // row t == 0: grad_h0 = lambda[0] * g_0
                    pst<G>(A.gh0, col, pld<G>(A.a, col) * r.b[j]);
            }
        }
    }
}
template <class G, bool BWD>
__device__ __forceinline__ void tile_store(const Args &A, const TileAddr<G, BWD> &ad, const RowMask<G, BWD> &mk,
                                           int64_t col, bool interior, const Rows<G> &r, const row_t<G> *hp)
{
    if (interior) tile_store_impl<G, BWD, true>(A, ad, mk, col, r, hp);
    else tile_store_impl<G, BWD, false>(A, ad, mk, col, r, hp);
}

// Backward epilogue of the gated form.  After the rescan r.b[j] = d_t, the accumulated gradient of
// row t, and r.a[j] is the gate complement of row t+1; so the complement of the row itself sits in
// r.a[j+1] (the thread's next row is t-1) and only the thread's last row needs one of its own.
//   grad_g_pre = d * (h_{t-1} - i) * g * (1-g)     grad_i_pre = d * (1-g) * tau'(i_pre)
//   grad_h0    = g_0 * d_0
// h one row behind and the impulse pre-activations are loaded here, after the rescan, when the
// registers of the scan are free again.
template <class G>
__device__ __forceinline__ void tile_store_gated_bwd(const Args &A, const TileAddr<G, true> &ad,
                                                     const RowMask<G, true> &mk, int64_t col, bool interior,
                                                     const Rows<G> &r)
{
    constexpr int R = G::R, VEC = G::VEC;
    constexpr int CH = R < 8 ? R : 8;  // rows whose loads are in flight together
    static_assert(R % CH == 0, "rows per thread: a multiple of 8, or fewer than 8");
    const rsrc_t r0 = ad.rsrc(A.out0), r1 = ad.rsrc(A.out1), rh = ad.rsrc(A.hprev, -1), ri = ad.rsrc(A.c),
                 rg = ad.rsrc(A.a);
    const int nv = interior ? R : mk.n;  // the thread's rows j < nv exist
    vec<VEC> c_last = splat<VEC>(__builtin_inff());
    if (nv > 0) c_last = gld<G>(rg, ad.toff + ad.soff_rt(nv - 1), 0);
    c_last = gate_complement<VEC>(c_last);
#pragma unroll
    for (int j0 = 0; j0 < R; j0 += CH) {
        vec<VEC> hp[CH], y[CH];
#pragma unroll
        for (int q = 0; q < CH; ++q) {  // loads only: nothing in here waits for a load
            const int j = j0 + q;
            hp[q] = splat<VEC>(0.0f);
            y[q] = splat<VEC>(0.0f);
            if (interior || j < mk.n) {
                y[q] = gld<G>(ri, ad.toff, ad.soff(j));
                if (interior || j < mk.nh) hp[q] = gld<G>(rh, ad.toff, ad.soff(j));
                else if (A.h0) hp[q] = pld<G>(A.h0, col);  // row t == 0
            }
        }
#pragma unroll
        for (int q = 0; q < CH; ++q) {
            const int j = j0 + q;
            vec<VEC> c = c_last;
            if (j + 1 < R) c = (j + 1 < nv) ? r.a[j + 1] : c_last;
            const vec<VEC> g = splat<VEC>(1.0f) - c, d = r.b[j];
            const vec<VEC> i = impulse<VEC>(y[q], A.tau);
            const vec<VEC> dg = d * (hp[q] - i) * (g * c);
            vec<VEC> di = d * c;
            if (A.tau) di = di * vfma<VEC>(-i, i, splat<VEC>(1.0f));
            if (interior || j < mk.n) {
                if (A.out0) gst<G>(r0, ad.toff, ad.soff(j), dg);
                if (A.out1) gst<G>(r1, ad.toff, ad.soff(j), di);
                if (!interior && j == mk.nh && A.gh0) pst<G>(A.gh0, col, g * d);
            }
        }
    }
}

// The same epilogue in three steps for the shapes of at most 32 elements per thread, whose registers hold
// all four operand tiles at once.  Everything of it that does not depend on the carry-in is moved in front of
// the look-back: the loads of h one row behind and of the impulse pre-activations are issued with the tile's
// own (gated_bwd_early_load), the activations and the factors
//     ga = (h_{t-1} - i) * g * (1-g)        gb = (1-g) * tau'(i_pre)
// are formed after the tile's summary has been published, while its predecessors are still being waited for
// (gated_bwd_early_math), and what is left behind the rescan is two products and two stores per element
// (gated_bwd_early_store).  With the loads and the tanh behind the rescan a tile spent 60 % of its life in
// its epilogue (per-tile timeline of the bf16-storage kernel: 20 of 33 us).
template <class G>
struct GatedBwdEarly {
    vec<G::VEC> ga[G::R], gb[G::R];
    vec<G::VEC> c_last;  // gate complement of the thread's last existing row (its successor in time holds no copy)
};
#ifndef LINREC_GATED_BWD_EARLY
#define LINREC_GATED_BWD_EARLY 1
#endif
template <class G>
constexpr bool kGatedBwdEarly = LINREC_GATED_BWD_EARLY && G::R * G::VEC <= 32;
struct NoEarly {};
template <class G, bool ON>
struct EarlySel { using type = GatedBwdEarly<G>; };
template <class G>
struct EarlySel<G, false> { using type = NoEarly; };

// (Two instances, as for tile_load: in the interior one the loads are unconditional straight-line code; inside
// run-time conditions the compiler waits for every load before it issues the next.)
template <class G, bool INTERIOR>
__device__ __forceinline__ void gated_bwd_early_load_impl(const Args &A, const TileAddr<G, true> &ad,
                                                          const RowMask<G, true> &mk, int64_t col, GatedBwdEarly<G> &e)
{
    constexpr int R = G::R, VEC = G::VEC;
    const rsrc_t rh = ad.rsrc(A.hprev, -1), ri = ad.rsrc(A.c), rg = ad.rsrc(A.a);
    const int nv = INTERIOR ? R : mk.n;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        e.ga[j] = splat<VEC>(0.0f);
        e.gb[j] = splat<VEC>(0.0f);
        if (INTERIOR || j < mk.n) {
            e.gb[j] = gld<G>(ri, ad.toff, ad.soff(j));
            if (INTERIOR || j < mk.nh) e.ga[j] = gld<G>(rh, ad.toff, ad.soff(j));
            else if (A.h0) e.ga[j] = pld<G>(A.h0, col);  // row t == 0
        }
    }
    e.c_last = splat<VEC>(__builtin_inff());
    if (INTERIOR) e.c_last = gld<G>(rg, ad.toff, ad.soff(R - 1));
    else if (nv > 0) e.c_last = gld<G>(rg, ad.toff + ad.soff_rt(nv - 1), 0);
}
template <class G>
__device__ __forceinline__ void gated_bwd_early_load(const Args &A, const TileAddr<G, true> &ad, const RowMask<G, true> &mk,
                                                     int64_t col, bool interior, GatedBwdEarly<G> &e)
{
    if (interior) gated_bwd_early_load_impl<G, true>(A, ad, mk, col, e);
    else gated_bwd_early_load_impl<G, false>(A, ad, mk, col, e);
}
template <class G>
__device__ __forceinline__ vec<G::VEC> gated_own_complement(const Rows<G> &r, const GatedBwdEarly<G> &e, int j, int nv)
{
    // r.a[j] is the complement of row t+1; the row's own is the next entry (the thread's next row is t-1)
    if (j + 1 < G::R) return (j + 1 < nv) ? r.a[j + 1] : e.c_last;
    return e.c_last;
}
template <class G>
__device__ __forceinline__ void gated_bwd_early_math(const Args &A, const RowMask<G, true> &mk, bool interior,
                                                     const Rows<G> &r, GatedBwdEarly<G> &e)
{
    constexpr int R = G::R, VEC = G::VEC;
    const int nv = interior ? R : mk.n;
    e.c_last = gate_complement<VEC>(e.c_last);
    if (A.tau) {  // (the choice of tau stays outside the row loop)
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const vec<VEC> c = gated_own_complement<G>(r, e, j, nv), g = splat<VEC>(1.0f) - c;
            const vec<VEC> i = impulse<VEC>(e.gb[j], 1);
            e.ga[j] = (e.ga[j] - i) * (g * c);
            e.gb[j] = c * vfma<VEC>(-i, i, splat<VEC>(1.0f));
        }
    } else {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const vec<VEC> c = gated_own_complement<G>(r, e, j, nv), g = splat<VEC>(1.0f) - c;
            e.ga[j] = (e.ga[j] - e.gb[j]) * (g * c);
            e.gb[j] = c;
        }
    }
}
template <class G>
__device__ __forceinline__ void gated_bwd_early_store(const Args &A, const TileAddr<G, true> &ad, const RowMask<G, true> &mk,
                                                      int64_t col, bool interior, const Rows<G> &r,
                                                      const GatedBwdEarly<G> &e)
{
    constexpr int R = G::R, VEC = G::VEC;
    const rsrc_t r0 = ad.rsrc(A.out0), r1 = ad.rsrc(A.out1);
    const int nv = interior ? R : mk.n;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const vec<VEC> d = r.b[j];
        if (interior || j < mk.n) {
            if (A.out0) gst<G>(r0, ad.toff, ad.soff(j), d * e.ga[j]);
            if (A.out1) gst<G>(r1, ad.toff, ad.soff(j), d * e.gb[j]);
            if (!interior && j == mk.nh && A.gh0)
                pst<G>(A.gh0, col, (splat<VEC>(1.0f) - gated_own_complement<G>(r, e, j, nv)) * d);
        }
    }
}

// Forward epilogue of the LSTM cell: r.b[j] = c_t; the output gate's pre-activation is loaded here, in
// chunks, and c_t and h_t = sigmoid(o_pre)*c_t are stored (either output may be absent).
template <class G>
__device__ __forceinline__ void tile_store_lstm_fwd(const Args &A, const TileAddr<G, false> &ad,
                                                    const RowMask<G, false> &mk, bool interior, const Rows<G> &r)
{
    constexpr int R = G::R, VEC = G::VEC;
    constexpr int CH = R < 8 ? R : 8;
    static_assert(R % CH == 0, "rows per thread: a multiple of 8, or fewer than 8");
    const rsrc_t r0 = ad.rsrc(A.out0), r1 = ad.rsrc(A.out1), ro = ad.rsrc(A.d);
#pragma unroll
    for (int j0 = 0; j0 < R; j0 += CH) {
        vec<VEC> op[CH];
#pragma unroll
        for (int q = 0; q < CH; ++q) {
            op[q] = splat<VEC>(0.0f);
            if (A.out1 && (interior || j0 + q < mk.n)) op[q] = gld<G>(ro, ad.toff, ad.soff(j0 + q));
        }
#pragma unroll
        for (int q = 0; q < CH; ++q) {
            const int j = j0 + q;
            const vec<VEC> h = gate_value<VEC>(op[q]) * r.b[j];
            if (interior || j < mk.n) {
                if (A.out0) gst<G>(r0, ad.toff, ad.soff(j), r.b[j]);
                if (A.out1) gst<G>(r1, ad.toff, ad.soff(j), h);
            }
        }
    }
}

// The same with the output gate formed early (single-pass kernel, shapes of few elements per thread).  The
// output gate does not depend on the scan, so its pre-activation is loaded together with the tile's operands
// (lstm_fwd_early_load: the latency of a load behind the rescan is otherwise spent in full, once per chunk),
// turned into the gate after the tile's summary has been published, while its predecessors are waited for,
// and what is left behind the rescan is one product and two stores per element.  Costs R*VEC registers
// from the loads to the stores: no wavefront per SIMD at 16 elements per thread, one at 24 and 32, where it
// measured ahead all the same (2-5 % with fp32 storage, 7-18 % with bf16), so every shape of the cell has it.
#ifndef LINREC_LSTM_FWD_EARLY_MAX
#define LINREC_LSTM_FWD_EARLY_MAX 32
#endif
template <class G>
constexpr bool kLstmFwdEarly = G::R * G::VEC <= LINREC_LSTM_FWD_EARLY_MAX;

// (an interior instance of its own: inside run-time conditions the compiler waits for every load before it
// issues the next)
template <class G, bool INTERIOR>
__device__ __forceinline__ void lstm_fwd_early_load_impl(const Args &A, const TileAddr<G, false> &ad,
                                                         const RowMask<G, false> &mk, vec<G::VEC> (&og)[G::R])
{
    const rsrc_t ro = ad.rsrc(A.d);
#pragma unroll
    for (int j = 0; j < G::R; ++j) {
        og[j] = splat<G::VEC>(0.0f);
        if (INTERIOR || j < mk.n) og[j] = gld<G>(ro, ad.toff, ad.soff(j));
    }
}
template <class G>
__device__ __forceinline__ void lstm_fwd_early_load(const Args &A, const TileAddr<G, false> &ad, const RowMask<G, false> &mk,
                                                    bool interior, vec<G::VEC> (&og)[G::R])
{
    if (interior) lstm_fwd_early_load_impl<G, true>(A, ad, mk, og);
    else lstm_fwd_early_load_impl<G, false>(A, ad, mk, og);
}
template <class G>
__device__ __forceinline__ void lstm_fwd_early_gate(vec<G::VEC> (&og)[G::R])
{
#pragma unroll
    for (int j = 0; j < G::R; ++j) og[j] = gate_value<G::VEC>(og[j]);
}
template <class G>
__device__ __forceinline__ void lstm_fwd_early_store(const Args &A, const TileAddr<G, false> &ad, const RowMask<G, false> &mk,
                                                     bool interior, const Rows<G> &r, const vec<G::VEC> (&og)[G::R])
{
    const rsrc_t r0 = ad.rsrc(A.out0), r1 = ad.rsrc(A.out1);
#pragma unroll
    for (int j = 0; j < G::R; ++j) {
        if (interior || j < mk.n) {
            if (A.out0) gst<G>(r0, ad.toff, ad.soff(j), r.b[j]);
            if (A.out1) gst<G>(r1, ad.toff, ad.soff(j), og[j] * r.b[j]);
        }
    }
}

// Backward epilogue of the LSTM cell.  After the rescan r.b[j] = d_t (accumulated gradient of c_t) and
// r.a[j] is the forget gate's complement of row t+1, so the row's own is r.a[j+1] (see the gated form).
//   grad_f_pre = d * c_{t-1} * f(1-f)   (c_{-1} = c0)      grad_i_pre = d * z * i(1-i)
//   grad_z_pre = d * i * (1 - z^2)                          grad_c0    = f_0 * d_0
// (grad_o_pre was written by the prologue.)  c_{t-1} is the cell state of the thread's next row, which
// the prologue kept in `cst`; i_pre and z_pre are loaded here, in chunks of rows, after the rescan.
template <class G>
__device__ __forceinline__ void tile_store_lstm_bwd(const Args &A, const TileAddr<G, true> &ad,
                                                    const RowMask<G, true> &mk, int64_t col, bool interior,
                                                    const Rows<G> &r, const vec<G::VEC> (&cst)[G::R])
{
    constexpr int R = G::R, VEC = G::VEC;
    constexpr int CH = R < 8 ? R : 8;
    static_assert(R % CH == 0, "rows per thread: a multiple of 8, or fewer than 8");
    const rsrc_t rf = ad.rsrc(A.out0), ri = ad.rsrc(A.out1), rz = ad.rsrc(A.out2);
    const rsrc_t rcp = ad.rsrc(A.hprev, -1), rip = ad.rsrc(A.c), rzp = ad.rsrc(A.d), rg = ad.rsrc(A.a);
    const int nv = interior ? R : mk.n;
    // The thread's last existing row: its own forget-gate complement and the cell state before it
    // are not among the thread's registers (c0 when that row is t == 0).
    vec<VEC> c_last = splat<VEC>(__builtin_inff()), cp_last = splat<VEC>(0.0f);
    if (nv > 0) {
        c_last = gld<G>(rg, ad.toff + ad.soff_rt(nv - 1), 0);
        if (interior || nv - 1 < mk.nh) cp_last = gld<G>(rcp, ad.toff + ad.soff_rt(nv - 1), 0);
        else if (A.h0) cp_last = pld<G>(A.h0, col);
    }
    c_last = gate_complement<VEC>(c_last);
#pragma unroll
    for (int j0 = 0; j0 < R; j0 += CH) {
        vec<VEC> ip[CH], zp[CH];
#pragma unroll
        for (int q = 0; q < CH; ++q) {  // loads only
            const int j = j0 + q;
            ip[q] = zp[q] = splat<VEC>(0.0f);
            if (interior || j < mk.n) {
                ip[q] = gld<G>(rip, ad.toff, ad.soff(j));
                zp[q] = gld<G>(rzp, ad.toff, ad.soff(j));
            }
        }
#pragma unroll
        for (int q = 0; q < CH; ++q) {
            const int j = j0 + q;
            vec<VEC> cf = c_last, cp = cp_last;
            if (j + 1 < R) {
                cf = (j + 1 < nv) ? r.a[j + 1] : c_last;
                cp = (j + 1 < nv) ? cst[j + 1] : cp_last;
            }
            const vec<VEC> f = splat<VEC>(1.0f) - cf, d = r.b[j];
            vec<VEC> ig, ic;
            gate_both<VEC>(ip[q], ig, ic);
            const vec<VEC> z = impulse<VEC>(zp[q], 1);
            if (interior || j < mk.n) {
                if (A.out0) gst<G>(rf, ad.toff, ad.soff(j), d * cp * (f * cf));
                if (A.out1) gst<G>(ri, ad.toff, ad.soff(j), d * z * (ig * ic));
                if (A.out2) gst<G>(rz, ad.toff, ad.soff(j), d * ig * vfma<VEC>(-z, z, splat<VEC>(1.0f)));
                if (!interior && j == mk.nh && A.gh0) pst<G>(A.gh0, col, f * d);
            }
        }
    }
}

// The same with everything that does not depend on the carry-in moved in front of the look-back (single-pass
// kernel), as for the gated layer's backward pass.  i_pre and z_pre are loaded behind the prologue
// (lstm_bwd_early_load, with the two values the thread's last row needs); after the tile's summary has been
// published, while its predecessors are waited for, the three factors
//   c_{t-1} * f(1-f)        z * i(1-i)        i * (1 - z^2)
// are formed in place of c_t, i_pre and z_pre (lstm_bwd_early_math); behind the rescan three products and three
// stores per element are left (lstm_bwd_early_store).  Costs two more register tiles across the look-back
// (124 -> 154 registers at 16 elements per thread; at 32 the kernel spills), hence the limit of 24 elements per
// thread; measured 1-4 % ahead with fp32 storage and 5-22 % with bf16 on the shapes that have it.
#ifndef LINREC_LSTM_BWD_EARLY_MAX
#define LINREC_LSTM_BWD_EARLY_MAX 24
#endif
template <class G>
constexpr bool kLstmBwdEarly = G::R * G::VEC <= LINREC_LSTM_BWD_EARLY_MAX;
template <class G>
struct LstmBwdEarly {
    vec<G::VEC> ei[G::R], ez[G::R];  // i_pre, z_pre; then z * i(1-i), i * (1 - z^2)
    vec<G::VEC> c_last, cp_last;     // the thread's last existing row: its forget-gate pre-activation (then complement)
                                     // and the cell state before it (c0 when that row is t == 0)
    vec<G::VEC> f_first;             // the forget gate of row t == 0, where the thread holds it (grad_c0)
};
template <class G, bool ON>
struct LstmEarlySel { using type = LstmBwdEarly<G>; };
template <class G>
struct LstmEarlySel<G, false> { using type = NoEarly; };

template <class G, bool INTERIOR>
__device__ __forceinline__ void lstm_bwd_early_load_impl(const Args &A, const TileAddr<G, true> &ad,
                                                         const RowMask<G, true> &mk, int64_t col, LstmBwdEarly<G> &e)
{
    constexpr int R = G::R, VEC = G::VEC;
    const rsrc_t rcp = ad.rsrc(A.hprev, -1), rip = ad.rsrc(A.c), rzp = ad.rsrc(A.d), rg = ad.rsrc(A.a);
    const int nv = INTERIOR ? R : mk.n;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        e.ei[j] = e.ez[j] = splat<VEC>(0.0f);
        if (INTERIOR || j < mk.n) {
            e.ei[j] = gld<G>(rip, ad.toff, ad.soff(j));
            e.ez[j] = gld<G>(rzp, ad.toff, ad.soff(j));
        }
    }
    e.c_last = splat<VEC>(__builtin_inff());
    e.cp_last = splat<VEC>(0.0f);
    if (INTERIOR) {
        e.c_last = gld<G>(rg, ad.toff, ad.soff(R - 1));
        e.cp_last = gld<G>(rcp, ad.toff, ad.soff(R - 1));
    } else if (nv > 0) {
        e.c_last = gld<G>(rg, ad.toff + ad.soff_rt(nv - 1), 0);
        if (nv - 1 < mk.nh) e.cp_last = gld<G>(rcp, ad.toff + ad.soff_rt(nv - 1), 0);
        else if (A.h0) e.cp_last = pld<G>(A.h0, col);
    }
}
template <class G>
__device__ __forceinline__ void lstm_bwd_early_load(const Args &A, const TileAddr<G, true> &ad, const RowMask<G, true> &mk,
                                                    int64_t col, bool interior, LstmBwdEarly<G> &e)
{
    if (interior) lstm_bwd_early_load_impl<G, true>(A, ad, mk, col, e);
    else lstm_bwd_early_load_impl<G, false>(A, ad, mk, col, e);
}
// r.a[j] is the forget gate's complement of row t+1, so the row's own is r.a[j+1], and c_{t-1} is cst[j+1]
// (the thread's next row is t-1); cst[j] becomes c_{t-1} * f(1-f).
template <class G>
__device__ __forceinline__ void lstm_bwd_early_math(const RowMask<G, true> &mk, bool interior, const Rows<G> &r,
                                                    vec<G::VEC> (&cst)[G::R], LstmBwdEarly<G> &e)
{
    constexpr int R = G::R, VEC = G::VEC;
    const int nv = interior ? R : mk.n;
    e.c_last = gate_complement<VEC>(e.c_last);
    e.f_first = splat<VEC>(0.0f);
#pragma unroll
    for (int j = 0; j < R; ++j) {
        vec<VEC> cf = e.c_last, cp = e.cp_last;
        if (j + 1 < R) {
            cf = (j + 1 < nv) ? r.a[j + 1] : e.c_last;
            cp = (j + 1 < nv) ? cst[j + 1] : e.cp_last;
        }
        const vec<VEC> f = splat<VEC>(1.0f) - cf;
        if (!interior && j == mk.nh) e.f_first = f;
        vec<VEC> ig, ic;
        gate_both<VEC>(e.ei[j], ig, ic);
        const vec<VEC> z = impulse<VEC>(e.ez[j], 1);
        cst[j] = cp * (f * cf);  // (row j-1, which read cst[j], is done)
        e.ei[j] = z * (ig * ic);
        e.ez[j] = ig * vfma<VEC>(-z, z, splat<VEC>(1.0f));
    }
}
template <class G>
__device__ __forceinline__ void lstm_bwd_early_store(const Args &A, const TileAddr<G, true> &ad, const RowMask<G, true> &mk,
                                                     int64_t col, bool interior, const Rows<G> &r,
                                                     const vec<G::VEC> (&cst)[G::R], const LstmBwdEarly<G> &e)
{
    const rsrc_t rf = ad.rsrc(A.out0), ri = ad.rsrc(A.out1), rz = ad.rsrc(A.out2);
#pragma unroll
    for (int j = 0; j < G::R; ++j) {
        const vec<G::VEC> d = r.b[j];
        if (interior || j < mk.n) {
            if (A.out0) gst<G>(rf, ad.toff, ad.soff(j), d * cst[j]);
            if (A.out1) gst<G>(ri, ad.toff, ad.soff(j), d * e.ei[j]);
            if (A.out2) gst<G>(rz, ad.toff, ad.soff(j), d * e.ez[j]);
            if (!interior && j == mk.nh && A.gh0) pst<G>(A.gh0, col, e.f_first * d);
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
// Phase 2 inside a tile, in two levels.
//   1. The TPW = 64/WC time-threads that share a wavefront (lanes tc + WC*ttl) run a Kogge-Stone
//      scan over ttl with cross-lane moves (log2(TPW) steps, no LDS storage, no barrier).  (A tile wider
//      than 64 threads has one time-thread per wavefront and several wavefronts side by side: no level 1.)
//   2. The NW wavefront totals along time go through LDS; every thread composes the totals of the
//      wavefronts before its own (at most NW-1 of them) with its in-wavefront prefix.
// Every thread returns its exclusive prefix (Pe, Se) -- the composition of all threads with smaller
// tt in its columns -- and the tile total (Pt, St).  P travels in fp64; S is stored in fp32 between
// steps but every combination is evaluated in fp64.  One __syncthreads inside.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float lane_move(float v, int src_lane)
{
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(v)));
}
__device__ __forceinline__ double lane_move(double v, int src_lane)
{
    const int lo = __builtin_amdgcn_ds_bpermute(src_lane << 2, __double2loint(v));
    const int hi = __builtin_amdgcn_ds_bpermute(src_lane << 2, __double2hiint(v));
    return __hiloint2double(hi, lo);
}
template <int N>
__device__ __forceinline__ vec<N> lane_move(vec<N> v, int src_lane)
{
    vec<N> r;
#pragma unroll
    for (int i = 0; i < N; ++i) r[i] = lane_move((float)v[i], src_lane);
    return r;
}
template <int N>
__device__ __forceinline__ dvec<N> lane_move(dvec<N> v, int src_lane)
{
    dvec<N> r;
#pragma unroll
    for (int i = 0; i < N; ++i) r[i] = lane_move((double)v[i], src_lane);
    return r;
}

template <class G>
struct ScanLds {
    // Wavefronts side by side along the columns (tiles wider than 64 threads), and along time: a wavefront holds
    // 64/WC time-threads of a narrow tile, or a 64-column piece of one time-thread's row of a wide one.
    static constexpr int WPR = G::WC > 64 ? G::WC / 64 : 1;
    static constexpr int NW = G::THREADS / 64 / WPR;  // wavefronts along time
    dvec<G::VEC> wP[NW][G::WC];
    vec<G::VEC> wS[NW][G::WC];
    int wClosed[NW][G::WC];
};

// With CLOSED = true every element also carries a flag "closed": the element is a complete state, not
// a map (a published inclusive state in the look-back).  Composition then keeps the LATEST closed
// element and what follows it and drops everything earlier without touching it -- in particular a
// NaN or Inf that sits before a closed element cannot leak into the result, and a zero product is
// not mistaken for the end of the dependence (0 * NaN stays NaN, as in the sequential recurrence).
// `closed` is in/out: in, the thread's own element; out, whether the tile total is closed.
template <class G, bool CLOSED = false>
__device__ __forceinline__ void tile_scan(ScanLds<G> &lds, int tid, dvec<G::VEC> P, vec<G::VEC> S, dvec<G::VEC> &Pe,
                                          vec<G::VEC> &Se, dvec<G::VEC> &Pt, vec<G::VEC> &St, bool *closed = nullptr)
{
    constexpr int VEC = G::VEC, WC = G::WC;
    static_assert(WC <= 64 ? 64 % WC == 0 : WC % 64 == 0, "a wavefront holds whole rows of a tile, or a row whole wavefronts");
    constexpr int TPW = WC >= 64 ? 1 : ((64 / WC) < G::WT ? (64 / WC) : G::WT);  // time-threads per wavefront
    constexpr int NW = ScanLds<G>::NW;
    // (`wave` counts along time: the wavefronts that share a row of a tile wider than 64 threads have the same one)
    const int lane = tid & 63, wave = (tid >> 6) / ScanLds<G>::WPR, tc = tid % WC, ttl = lane / WC;
    int cl = 0;
    if constexpr (CLOSED) cl = *closed ? 1 : 0;

    // level 1: inclusive scan over ttl inside the wavefront
#pragma unroll
    for (int d = 1; d < TPW; d <<= 1) {
        const int src = lane - d * WC;
        const dvec<VEC> ps = lane_move<VEC>(P, src < 0 ? lane : src);
        const vec<VEC> ss = lane_move<VEC>(S, src < 0 ? lane : src);
        int cs = 0;
        if constexpr (CLOSED) cs = __builtin_amdgcn_ds_bpermute((src < 0 ? lane : src) << 2, cl);
        if (ttl >= d && !cl) {  // (ps, ss) is earlier in time: it goes on the left
            S = narrow<VEC>(dfma<VEC>(P, widen<VEC>(ss), widen<VEC>(S)));
            P = ps * P;
            cl = cs;
        }
    }
    if (ttl == TPW - 1) {
        lds.wP[wave][tc] = P;
        lds.wS[wave][tc] = S;
        if constexpr (CLOSED) lds.wClosed[wave][tc] = cl;
    }
    // exclusive prefix inside the wavefront = inclusive value of the previous time-thread
    // (not needed, and not meaningful, for the flagged form: its callers use the total only)
    dvec<VEC> Px = dsplat<VEC>(1.0);
    vec<VEC> Sx = splat<VEC>(0.0f);
    if constexpr (TPW > 1 && !CLOSED) {
        const int src = lane - WC;
        const dvec<VEC> ps = lane_move<VEC>(P, src < 0 ? lane : src);
        const vec<VEC> ss = lane_move<VEC>(S, src < 0 ? lane : src);
        if (ttl >= 1) { Px = ps; Sx = ss; }
    }
    __syncthreads();
    // level 2: compose the wavefront totals; the running value when w reaches this thread's
    // wavefront is what came before it
    dvec<VEC> pt = dsplat<VEC>(1.0);
    vec<VEC> st_ = splat<VEC>(0.0f);
    int ct = 0;
    Pe = Px;
    Se = Sx;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        if (!CLOSED && w == wave) {  // (waves before) (+) (in-wave prefix)
            Se = narrow<VEC>(dfma<VEC>(Px, widen<VEC>(st_), widen<VEC>(Sx)));
            Pe = pt * Px;
        }
        const dvec<VEC> p = lds.wP[w][tc];
        const vec<VEC> sw = lds.wS[w][tc];
        if (CLOSED && lds.wClosed[w][tc]) {  // a closed element replaces all that came before it
            pt = p;
            st_ = sw;
            ct = 1;
        } else {
            st_ = narrow<VEC>(dfma<VEC>(p, widen<VEC>(st_), widen<VEC>(sw)));
            pt *= p;
        }
    }
    Pt = pt;
    St = st_;
    if constexpr (CLOSED) *closed = ct != 0;
}

// ---------------------------------------------------------------------------------------------
// Three-phase variant, kernel 1: per-chunk reduce (Algorithm 1, first parallel-for).
// grid = K*G workgroups, workgroup (k, g) walks the M tiles of chunk k in column group g.
// ---------------------------------------------------------------------------------------------
template <class G, bool BWD>
__global__ __launch_bounds__(G::THREADS, G::OCC) void k_reduce(const Args A)
{
    constexpr int VEC = G::VEC, R = G::R, WC = G::WC, ROWS = G::ROWS;
    __shared__ ScanLds<G> lds;
    const int tid = threadIdx.x, tc = tid % WC, tt = tid / WC;
    const int g = (int)(blockIdx.x % (unsigned)A.G);
    const int64_t k = blockIdx.x / (unsigned)A.G;
    const int64_t col = ((int64_t)g * WC + tc) * VEC;
    const bool col_ok = col < A.C;

    dvec<VEC> Pc = dsplat<VEC>(1.0), Sc = dsplat<VEC>(0.0);  // chunk total so far
    for (int m = 0; m < A.M; ++m) {
        const int64_t tu0 = (k * A.M + m) * ROWS;
        if (tu0 >= A.T) break;
        const bool interior = tile_interior<G, BWD>(A, tu0, g);
        Rows<G> r;
        dvec<VEC> P, Pe, Pt;
        vec<VEC> S, Se, St;
        const TileAddr<G, BWD> ad(A, tu0, g, tt, tc);
        const RowMask<G, BWD> mk(A, tu0 + (int64_t)tt * R, col_ok);
        tile_load<G, BWD>(A, ad, mk, interior, r);
        local_reduce<G>(r, P, S);
        if (m > 0) __syncthreads();  // the previous tile's wavefront totals have been consumed
        tile_scan<G>(lds, tid, P, S, Pe, Se, Pt, St);
        Sc = dfma<VEC>(Pt, Sc, widen<VEC>(St));  // (earlier tiles) (+) (this tile)
        Pc *= Pt;
    }
    if (tt == 0 && col_ok) {
        std_<VEC>(A.aggP + k * A.C + col, Pc);
        std_<VEC>(A.aggS + k * A.C + col, Sc);
    }
}

// ---------------------------------------------------------------------------------------------
// Three-phase variant, kernel 3: per-chunk rescan from the carry (Algorithm 1, second parallel-for).
// ---------------------------------------------------------------------------------------------
template <class G, bool BWD>
__global__ __launch_bounds__(G::THREADS, G::OCC) void k_fixup(const Args A)
{
    constexpr int VEC = G::VEC, R = G::R, WC = G::WC, ROWS = G::ROWS;
    __shared__ ScanLds<G> lds;
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
        row_t<G> hp[BWD ? R : 1];
        vec<VEC> S, Se, St;
        dvec<VEC> P, Pe, Pt;
        const TileAddr<G, BWD> ad(A, tu0, g, tt, tc);
        const RowMask<G, BWD> mk(A, u0, col_ok);
        tile_load<G, BWD>(A, ad, mk, interior, r);
        if constexpr (BWD) {
            if (A.out1) tile_load_hprev<G>(A, ad, mk, col, interior, hp);
        }
        local_reduce<G>(r, P, S);
        if (m > 0) __syncthreads();
        tile_scan<G>(lds, tid, P, S, Pe, Se, Pt, St);
        rescan<G>(r, narrow<VEC>(dfma<VEC>(Pe, cc, widen<VEC>(Se))));
        tile_store<G, BWD>(A, ad, mk, col, interior, r, hp);
        cc = dfma<VEC>(Pt, cc, widen<VEC>(St));
    }
}

// ---------------------------------------------------------------------------------------------
// Walk: grid = G workgroups, each goes through ALL the tiles of its column group in time order from
// the initial state (zero for the backward pass), carrying the state in fp64.  There are no chunk
// summaries, no other kernel and nothing between workgroups; the sequence is parallel inside a tile
// only.  The choice for short, wide problems, where the columns alone fill the GPU and summaries
// between workgroups are pure overhead (the overhead Section 4.1.1 names for short sequences: several
// passes over the data, communication between processors).  Exists for every form and storage type
// the single-pass kernel exists for, with the same prologues and epilogues.
// ---------------------------------------------------------------------------------------------
template <class G, bool BWD, int FORM = FORM_PLAIN>
__global__ __launch_bounds__(G::THREADS, G::OCC) void k_walk(const Args A)
{
    constexpr int VEC = G::VEC, R = G::R, WC = G::WC, ROWS = G::ROWS;
    __shared__ ScanLds<G> lds;
    const int tid = threadIdx.x, tc = tid % WC, tt = tid / WC;
    const int g = (int)blockIdx.x;
    const int64_t col = ((int64_t)g * WC + tc) * VEC;
    const bool col_ok = col < A.C;

    dvec<VEC> cc = dsplat<VEC>(0.0);  // state entering the current tile
    if (!BWD && col_ok && A.h0) cc = widen<VEC>(pld<G>(A.h0, col));

    for (int64_t m = 0;; ++m) {
        const int64_t tu0 = m * ROWS;
        if (tu0 >= A.T) break;
        const bool interior = tile_interior<G, BWD>(A, tu0, g);
        const int64_t u0 = tu0 + (int64_t)tt * R;
        Rows<G> r;
        row_t<G> hp[(BWD && FORM == FORM_PLAIN) ? R : 1];
        const TileAddr<G, BWD> ad(A, tu0, g, tt, tc);
        const RowMask<G, BWD> mk(A, u0, col_ok);
        constexpr int NC = (BWD && FORM == FORM_LSTM) ? R : 1;
        vec<VEC> cst[NC];
        tile_load<G, BWD, FORM, NC>(A, ad, mk, interior, r, cst);
        if constexpr (BWD && FORM == FORM_PLAIN) {
            if (A.out1) tile_load_hprev<G>(A, ad, mk, col, interior, hp);
        }
        constexpr bool EARLY = BWD && FORM == FORM_GATED && kGatedBwdEarly<G>;
        typename EarlySel<G, EARLY>::type early[1];
        if constexpr (EARLY) gated_bwd_early_load<G>(A, ad, mk, col, interior, early[0]);
        vec<VEC> S, Se, St;
        dvec<VEC> P, Pe, Pt;
        local_reduce<G, FORM>(r, P, S);
        if (m > 0) __syncthreads();  // the previous tile's wavefront totals have been consumed
        tile_scan<G>(lds, tid, P, S, Pe, Se, Pt, St);
        if constexpr (EARLY) gated_bwd_early_math<G>(A, mk, interior, r, early[0]);
        const vec<VEC> carry_in = narrow<VEC>(dfma<VEC>(Pe, cc, widen<VEC>(Se)));
        if constexpr (BWD && G::IO == IO_BF16) {
            static_assert(FORM == FORM_PLAIN, "bf16 storage: the plain recurrence");
            rescan_bwd_packed<G>(A, mk, col, interior, r, hp, carry_in);
        } else {
            rescan<G, FORM>(r, carry_in);
        }
        if constexpr (EARLY) {
            gated_bwd_early_store<G>(A, ad, mk, col, interior, r, early[0]);
        } else if constexpr (BWD && FORM == FORM_GATED) {
            __builtin_amdgcn_sched_barrier(0);  // the epilogue's loads stay behind the rescan
            tile_store_gated_bwd<G>(A, ad, mk, col, interior, r);
        } else if constexpr (FORM == FORM_LSTM) {
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (BWD) tile_store_lstm_bwd<G>(A, ad, mk, col, interior, r, cst);
            else tile_store_lstm_fwd<G>(A, ad, mk, interior, r);
        } else {
            tile_store<G, BWD>(A, ad, mk, col, interior, r, hp);
        }
        cc = dfma<VEC>(Pt, cc, widen<VEC>(St));
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
// Per tile and column there are three 64-bit words, each {tag : 32 | payload : 32}, written and read
// with single relaxed agent-scope atomics, so a tag can never be seen without its payload and no
// fence or workspace clear is needed between calls; the tag is never a data value:
//   word 0, 1   low / high half of the fp64 product P            tag = epoch << 1
//   word 2      fp32 S, tag = epoch << 1;  later overwritten by the fp32 inclusive state with
//               tag = epoch << 1 | 1 (P is then irrelevant: the look-back ends at this tile)
// ---------------------------------------------------------------------------------------------
// Optional per-tile timeline (builds with -DLINREC_TRACE only): thread 0 of a tile stores the
// constant-rate wall clock at the phase boundaries into Args::trace[ticket*8 + slot].
#ifdef LINREC_TRACE
#define LINREC_TRACE_MARK(slot)                                                         \
    do {                                                                                \
        if (A.trace && threadIdx.x == 0) A.trace[(size_t)ticket * 8 + (slot)] = wall_clock64(); \
    } while (0)
#define LINREC_TRACE_VAL(slot, val)                                                     \
    do {                                                                                \
        if (A.trace && threadIdx.x == 0) A.trace[(size_t)ticket * 8 + (slot)] = (unsigned long long)(val); \
    } while (0)
#else
#define LINREC_TRACE_MARK(slot) do { } while (0)
#define LINREC_TRACE_VAL(slot, val) do { } while (0)
#endif

__device__ __forceinline__ unsigned long long lb_pack(uint32_t bits, uint32_t tag)
{
    return ((unsigned long long)tag << 32) | (unsigned long long)bits;
}
__device__ __forceinline__ void lb_store(unsigned long long *p, unsigned long long w)
{
    __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long lb_load(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Pause between polls of a predecessor's flag once the first few quick ones have failed, in units of 64 clocks.
#ifndef LINREC_POLL_SLEEP
#define LINREC_POLL_SLEEP 16
#endif
template <class G, bool BWD, bool HP_LATE, int FORM = FORM_PLAIN>
__global__ __launch_bounds__(G::THREADS, G::OCC) void k_lookback(const Args A)
{
    constexpr int VEC = G::VEC, R = G::R, WC = G::WC, WT = G::WT, ROWS = G::ROWS;
    __shared__ ScanLds<G> lds;
    __shared__ dvec<VEC> sPt[WC];   // tile total, kept for the inclusive-state publication
    __shared__ vec<VEC> sSt[WC];
    __shared__ uint32_t sTicket[2], sEpoch;  // the ticket slot alternates from tile to tile
    const int tid = threadIdx.x, tc = tid % WC, tt = tid / WC;
    // Workgroups are persistent: each takes tickets until none is left (a workgroup works through its
    // tickets in increasing order, so the owner of the lowest unfinished ticket is always free to run
    // it: no deadlock).
    // The host keeps K*G below 2^31, so a call's tickets fit 32 bits.
    const uint32_t total = (uint32_t)A.K * (uint32_t)A.G;
    // The odd workgroups of the first round start a few microseconds late: the others, which are
    // enough to saturate the memory system, are then scanning and storing while these load, instead of
    // all of them doing each thing at the same time (consecutive workgroups go to different XCDs, so
    // this is every other XCD).  Measured on an MI355X: up to 4 % on the forward pass of long sequences.
    if ((int)blockIdx.x < A.stagger_n && (blockIdx.x & 1u)) {
        for (int i = 0; i < A.stagger; ++i) __builtin_amdgcn_s_sleep(32);
    }
    if (tid == 0) {
        sTicket[0] = (uint32_t)atomicAdd(&A.hdr->ticket, 1ull);
        sEpoch = __hip_atomic_load(&A.hdr->epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    // The header stores the number of calls completed so far (modulo 2^31 - 1); the call's epoch is one
    // more, 1 .. 2^31-1, so that a zero-filled workspace -- header and words -- is a valid start: tag 0 is
    // what untouched words carry and no call ever uses it.
    const uint32_t epoch = __builtin_amdgcn_readfirstlane(sEpoch) + 1u;
    const uint32_t tag_agg = epoch << 1, tag_incl = tag_agg | 1u;
    uint32_t ticket = __builtin_amdgcn_readfirstlane(sTicket[0]);
    int slot = 0;
    unsigned long long finished = 0;  // thread 0: workgroups known to be past their last look-back read
  while (ticket < total) {
    slot ^= 1;
    const int g = (int)(ticket % (uint32_t)A.G);
    const int64_t k = (int64_t)(ticket / (uint32_t)A.G);
    const int64_t col = ((int64_t)g * WC + tc) * VEC;
    const bool col_ok = col < A.C;
    // Tiles k < K1 are full height; then come K2 tiles of half height and, to the end, tiles of a
    // quarter height (each thread then owns R/2 or R/4 rows, its other rows are masked).  They are the
    // last tickets handed out, so that the kernel does not end on a few workgroups finishing big tiles.
    int rk = R;
    int64_t tu0 = k * ROWS;
    if (k >= A.K1) {
        if (k < A.K1 + A.K2) {
            rk = R / 2;
            tu0 = A.K1 * ROWS + (k - A.K1) * (ROWS / 2);
        } else {
            rk = R / 4;
            tu0 = A.K1 * ROWS + A.K2 * (ROWS / 2) + (k - A.K1 - A.K2) * (ROWS / 4);
        }
    }
    const int64_t u0 = tu0 + (int64_t)tt * rk;
    const bool interior = rk == R && tile_interior<G, BWD>(A, tu0, g);
    LINREC_TRACE_MARK(0);

    Rows<G> r;
    row_t<G> hp[(BWD && FORM == FORM_PLAIN) ? R : 1];
    const TileAddr<G, BWD> ad(A, tu0, g, tt, tc, rk);
    const RowMask<G, BWD> mk(A, u0, col_ok, rk);
    constexpr int NC = (BWD && FORM == FORM_LSTM) ? R : 1;
    vec<VEC> cst[NC];
    tile_load<G, BWD, FORM, NC>(A, ad, mk, interior, r, cst);
    if constexpr (BWD && !HP_LATE && FORM == FORM_PLAIN) {
        if (A.out1) tile_load_hprev<G>(A, ad, mk, col, interior, hp);
    }
    constexpr bool EARLY = BWD && FORM == FORM_GATED && kGatedBwdEarly<G>;
    typename EarlySel<G, EARLY>::type early[1];
    if constexpr (EARLY) gated_bwd_early_load<G>(A, ad, mk, col, interior, early[0]);
    constexpr bool EARLY_L = BWD && FORM == FORM_LSTM && kLstmBwdEarly<G>;
    typename LstmEarlySel<G, EARLY_L>::type early_l[1];
    if constexpr (EARLY_L) lstm_bwd_early_load<G>(A, ad, mk, col, interior, early_l[0]);
    constexpr bool EARLY_O = !BWD && FORM == FORM_LSTM && kLstmFwdEarly<G>;
    vec<VEC> og[EARLY_O ? R : 1];  // the cell's output gate (pre-activations until the summary is out)
    if constexpr (EARLY_O) {
        if (A.out1) lstm_fwd_early_load<G>(A, ad, mk, interior, og);
    }
    // thread-exclusive prefix inside the tile; rounded to fp32 once (it is used once, in the
    // rescan's carry-in, and is not fed on along the chain of tiles)
    vec<VEC> Pe32, Se32;
    const bool publish = (k + 1 < A.K) && col_ok;
    unsigned long long *const my_words = A.lbAgg + (k * A.C + col) * 3;
    {
        dvec<VEC> P, Pe, Pt;
        vec<VEC> S, St32;
        local_reduce<G, FORM>(r, P, S);
#ifdef LINREC_TRACE
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the mark below means "rows have arrived"
#endif
        LINREC_TRACE_MARK(1);
        tile_scan<G>(lds, tid, P, S, Pe, Se32, Pt, St32);
        Pe32 = narrow<VEC>(Pe);
        if (tt == 0) {
            // the tile's own inclusive state below is built from the same fp32 S that is published,
            // so that the tile and its successors agree on what it contributes
            sPt[tc] = Pt;
            sSt[tc] = St32;
            if (publish) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const unsigned long long pb = (unsigned long long)__double_as_longlong(Pt[v]);
                    lb_store(my_words + 3 * v, lb_pack((uint32_t)pb, tag_agg));
                    lb_store(my_words + 3 * v + 1, lb_pack((uint32_t)(pb >> 32), tag_agg));
                    lb_store(my_words + 3 * v + 2, lb_pack(__float_as_uint(St32[v]), tag_agg));
                }
            }
        }
    }
    // (the carry-independent part of the gated backward epilogue: behind the publication, so that it does not
    // delay the tiles that wait for this one, and in front of this tile's own waits)
    if constexpr (EARLY) gated_bwd_early_math<G>(A, mk, interior, r, early[0]);
    if constexpr (EARLY_L) lstm_bwd_early_math<G>(mk, interior, r, cst, early_l[0]);
    if constexpr (EARLY_O) {
        if (A.out1) lstm_fwd_early_gate<G>(og);
    }
    LINREC_TRACE_MARK(2);
    [[maybe_unused]] int n_windows = 0;  // (read by trace builds)
    unsigned long long next_ticket = 0xffffffffull;

    // ---- look-back --------------------------------------------------------------------------
    // Window w covers predecessors k-1-w*WT down to k-(w+1)*WT; thread (tt, tc) reads the one that is
    // WT-1-tt tiles before the window's nearest, so that tt increases with time like inside a tile.
    // A predecessor that has published its inclusive state I enters as a "closed" element: composed
    // in time order, the latest closed element and what follows it are kept and everything earlier is
    // dropped unread, so the window total is either a state (closed: the walk ends, Sr becomes the
    // carry-in) or the affine map of the whole window (open: the next, earlier window is needed).
    // (Pr, Sr) composes the windows visited so far.  The initial state is a closed element too, so
    // the walk always ends at the window that contains it.
    dvec<VEC> Pr = dsplat<VEC>(1.0);
    vec<VEC> Sr = splat<VEC>(0.0f);
    bool have_state = false;
    for (int64_t base = k - 1;; base -= WT) {
        const int64_t pred = base - (WT - 1 - tt);
        dvec<VEC> vP = dsplat<VEC>(0.0);
        vec<VEC> vS = splat<VEC>(0.0f);
        bool closed = true;  // this thread's element is a complete state (inclusive state, initial state)
        if (pred < 0 || !col_ok) {
            // before the first tile: the initial state (h0 forward, zero backward)
            if (!BWD && pred == -1 && col_ok && A.h0) vS = pld<G>(A.h0, col);
        } else {
            const unsigned long long *w = A.lbAgg + (pred * A.C + col) * 3;
            // Wait on ONE word of the predecessor (the S word of the column group's first column,
            // the same address for all lanes that look at this predecessor) with a growing pause:
            // hundreds of workgroups poll at once and must not crowd out the data streams.
            const unsigned long long *flag = A.lbAgg + (pred * A.C + (int64_t)g * G::COLS) * 3 + 2;
            uint32_t spins = 0;
            bool gave_up = false;
            for (;;) {
                const uint32_t t = (uint32_t)(lb_load(flag) >> 32);
                if (t == tag_agg || t == tag_incl) break;
                if (++spins > A.spin_limit) { gave_up = true; break; }
                if (spins < 4) __builtin_amdgcn_s_sleep(2);
                else __builtin_amdgcn_s_sleep(LINREC_POLL_SLEEP);
            }
            // then read this thread's own words until they are consistent
            while (!gave_up) {
                bool all_incl = true, all_agg = true;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const unsigned long long wl = lb_load(w + 3 * v), wh = lb_load(w + 3 * v + 1),
                                             ws = lb_load(w + 3 * v + 2);
                    const uint32_t ts = (uint32_t)(ws >> 32);
                    all_incl = all_incl && (ts == tag_incl);
                    all_agg = all_agg && (ts == tag_agg) && ((uint32_t)(wl >> 32) == tag_agg) &&
                              ((uint32_t)(wh >> 32) == tag_agg);
                    vP[v] = __longlong_as_double((long long)((wh << 32) | (wl & 0xffffffffull)));
                    vS[v] = __uint_as_float((uint32_t)ws);
                }
                // (a predecessor caught between its two publications has some columns of this
                // thread tagged inclusive and some not: neither test holds and it is read again)
                if (all_incl) break;
                if (all_agg) { closed = false; break; }
                if (++spins > A.spin_limit) gave_up = true;
                else __builtin_amdgcn_s_sleep(2);
            }
            if (gave_up) {  // flag the error and finish with a zero state
                atomicOr(&A.hdr->err, 1u);
                vS = splat<VEC>(0.0f);
                closed = true;
            }
        }
        __syncthreads();  // the previous use of the scan's LDS staging is over
        dvec<VEC> Pe, Pw;
        vec<VEC> Se, Sw;
        tile_scan<G, true>(lds, tid, vP, vS, Pe, Se, Pw, Sw, &closed);
        // (window) is earlier in time than everything in (Pr, Sr): it goes on the left.  Columns that
        // met a state in an earlier window are complete and take nothing more.
        if (!have_state) {
            Sr = narrow<VEC>(dfma<VEC>(Pr, widen<VEC>(Sw), widen<VEC>(Sr)));
            Pr = Pw * Pr;
            have_state = closed;
        }
        ++n_windows;
        // every wavefront of a tile at most 64 threads wide holds every tc, so this vote is the same in all of
        // them; the wavefronts of a wider tile hold different columns and vote through the workgroup.  A window
        // that reached back to the initial state always closes (nothing precedes it).
        bool open_left;
        if constexpr (WC > 64) open_left = __syncthreads_or(!have_state) != 0;
        else open_left = __any(!have_state);
        if (!open_left || base - (WT - 1) <= -1) break;
    }
    LINREC_TRACE_MARK(3);
    LINREC_TRACE_VAL(5, n_windows);
    LINREC_TRACE_VAL(6, ((unsigned long long)k << 32) | (unsigned)g);
    if (tt == 0 && publish) {
        const vec<VEC> incl = narrow<VEC>(dfma<VEC>(sPt[tc], widen<VEC>(Sr), widen<VEC>(sSt[tc])));
#pragma unroll
        for (int v = 0; v < VEC; ++v) lb_store(my_words + 3 * v + 2, lb_pack(__float_as_uint(incl[v]), tag_incl));
    }
    // ---- rescan from the carry and store -------------------------------------------------------
    // The next ticket is requested here, so that the counter's latency hides behind the stores; taking
    // it any earlier would hold a tile that other workgroups already wait for.
    // (A workgroup that takes a single tile reports itself finished at this point instead: every
    // look-back read of the tile is over, and waiting for the counter after the stores would hold the
    // workgroup until they have all been acknowledged.)
    if (tid == 0) {
        if (A.persistent) next_ticket = atomicAdd(&A.hdr->ticket, 1ull);
        else finished = atomicAdd(&A.hdr->done, 1ull) + 1ull;
    }
    if constexpr (BWD && G::IO == IO_BF16) {
        static_assert(FORM == FORM_PLAIN && !HP_LATE, "bf16 storage: the plain recurrence, h loaded with the tile");
        rescan_bwd_packed<G>(A, mk, col, interior, r, hp, vfma<VEC>(Pe32, Sr, Se32));
    } else {
        rescan<G, FORM>(r, vfma<VEC>(Pe32, Sr, Se32));
    }
    if constexpr (EARLY) {
        gated_bwd_early_store<G>(A, ad, mk, col, interior, r, early[0]);
    } else if constexpr (BWD && FORM == FORM_GATED) {
        __builtin_amdgcn_sched_barrier(0);  // the epilogue's loads stay behind the rescan
        tile_store_gated_bwd<G>(A, ad, mk, col, interior, r);
    } else if constexpr (EARLY_L) {
        lstm_bwd_early_store<G>(A, ad, mk, col, interior, r, cst, early_l[0]);
    } else if constexpr (EARLY_O) {
        lstm_fwd_early_store<G>(A, ad, mk, interior, r, og);
    } else if constexpr (FORM == FORM_LSTM) {
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (BWD) tile_store_lstm_bwd<G>(A, ad, mk, col, interior, r, cst);
        else tile_store_lstm_fwd<G>(A, ad, mk, interior, r);
    } else {
        if constexpr (BWD && HP_LATE) {
            // keep these loads behind the rescan: they take over the registers lambda occupied until now
            __builtin_amdgcn_sched_barrier(0);
            if (A.out1) tile_load_hprev<G>(A, ad, mk, col, interior, hp);
        }
        tile_store<G, BWD>(A, ad, mk, col, interior, r, hp);
    }
    LINREC_TRACE_MARK(4);
    if (tid == 0) sTicket[slot] = (uint32_t)(next_ticket > 0xffffffffull ? 0xffffffffull : next_ticket);
    __syncthreads();  // this tile's LDS state has been consumed
    ticket = __builtin_amdgcn_readfirstlane(sTicket[slot]);
  }
    // Out of tickets.  The workgroup that finds every other one out of tickets too rewinds the counter
    // and moves to the next epoch, for the next call (which starts only after this kernel has ended).
    if (tid == 0) {
        if (A.persistent) finished = atomicAdd(&A.hdr->done, 1ull) + 1ull;
        if (finished == (unsigned long long)gridDim.x) {
            __hip_atomic_store(&A.hdr->done, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&A.hdr->ticket, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&A.hdr->epoch, epoch >= 0x7fffffffu ? 0u : epoch, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace linrec
