// Kernels that do not depend on the tile shape:
//   k_scan_summaries -- phase 2 of Algorithm 1 (arXiv 1709.04057): C_i = P_i*C_{i-1} + R_i with
//                       C_{-1} = h_0, over the K chunk summaries of every column;
//   k_serial_fwd/bwd -- the paper's comparison kernel of Section 4.1.1: serial over the sequence
//                       length, parallel over features and minibatch.
#include "linrec_device.h"

#include <algorithm>

namespace linrec {

// DPP helpers: a lane takes `src` from another lane of the wavefront, or keeps `old` when the
// source lane does not exist or the row is masked off.  fp64 values move as two 32-bit halves.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp32(int old, int src)
{
    return __builtin_amdgcn_update_dpp(old, src, CTRL, ROW_MASK, 0xF, false);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp(double old, double src)
{
    const int lo = dpp32<CTRL, ROW_MASK>(__double2loint(old), __double2loint(src));
    const int hi = dpp32<CTRL, ROW_MASK>(__double2hiint(old), __double2hiint(src));
    return __hiloint2double(hi, lo);
}

// One Kogge-Stone step of the inclusive scan of affine pairs: (pe, se) is the pair of the earlier
// lane (identity (1,0) when there is none), combined on the left of the lane's own pair.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void scan_step(double &P, double &S)
{
    const double pe = dpp<CTRL, ROW_MASK>(1.0, P);
    const double se = dpp<CTRL, ROW_MASK>(0.0, S);
    S = fma(P, se, S);
    P = pe * P;
}

// Inclusive scan over the 64 lanes of a wavefront, lane index = time order.
__device__ __forceinline__ void wave_scan_pairs(double &P, double &S)
{
    scan_step<0x111, 0xF>(P, S);  // row_shr:1
    scan_step<0x112, 0xF>(P, S);  // row_shr:2
    scan_step<0x114, 0xF>(P, S);  // row_shr:4
    scan_step<0x118, 0xF>(P, S);  // row_shr:8   -> inclusive inside each row of 16 lanes
    scan_step<0x142, 0xA>(P, S);  // row_bcast:15 into rows 1 and 3
    scan_step<0x143, 0xC>(P, S);  // row_bcast:31 into rows 2 and 3
}

constexpr int SCAN_COLS = 16;     // columns per workgroup
constexpr int SCAN_WAVES = 4;

// grid = ceil(C / SCAN_COLS).  Blocks of 64 chunks x SCAN_COLS columns are staged through LDS
// (coalesced along the columns in global memory, transposed so that lanes hold consecutive chunks),
// scanned with DPP, and the state entering each chunk is written back the same way.  The state is
// carried across the K/64 blocks in a register per (wavefront, column).  All in fp64.
__global__ __launch_bounds__(SCAN_WAVES * 64) void k_scan_summaries(const double *__restrict__ aggP,
                                                                    const double *__restrict__ aggS,
                                                                    const float *__restrict__ h0,
                                                                    double *__restrict__ carry, int64_t K, int64_t C)
{
    __shared__ double tP[64][SCAN_COLS + 1];
    __shared__ double tS[64][SCAN_COLS + 1];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t c0 = (int64_t)blockIdx.x * SCAN_COLS;
    constexpr int PER_WAVE = SCAN_COLS / SCAN_WAVES;
    double run[PER_WAVE];
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
        const int64_t c = c0 + wave + SCAN_WAVES * i;
        run[i] = (h0 && c < C) ? (double)h0[c] : 0.0;
    }
    for (int64_t k0 = 0; k0 < K; k0 += 64) {
        for (int idx = tid; idx < 64 * SCAN_COLS; idx += SCAN_WAVES * 64) {
            const int kk = idx / SCAN_COLS, cc = idx % SCAN_COLS;
            double p = 1.0, s = 0.0;
            if (k0 + kk < K && c0 + cc < C) {
                p = aggP[(k0 + kk) * C + c0 + cc];
                s = aggS[(k0 + kk) * C + c0 + cc];
            }
            tP[kk][cc] = p;
            tS[kk][cc] = s;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int cc = wave + SCAN_WAVES * i;
            double P = tP[lane][cc], S = tS[lane][cc];
            wave_scan_pairs(P, S);
            const double state = fma(P, run[i], S);              // state after chunk k0 + lane
            tS[lane][cc] = dpp<0x138, 0xF>(run[i], state);       // wave_shr:1 -> state entering the chunk
            run[i] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(state), 63),
                                      __builtin_amdgcn_readlane(__double2loint(state), 63));
        }
        __syncthreads();
        for (int idx = tid; idx < 64 * SCAN_COLS; idx += SCAN_WAVES * 64) {
            const int kk = idx / SCAN_COLS, cc = idx % SCAN_COLS;
            if (k0 + kk < K && c0 + cc < C) carry[(k0 + kk) * C + c0 + cc] = tS[kk][cc];
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void k_serial_fwd(const float *__restrict__ a, const float *b,
                                                    const float *__restrict__ h0, float *out, int64_t T, int64_t C)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float s = h0 ? h0[c] : 0.0f;
#pragma unroll 8
    for (int64_t t = 0; t < T; ++t) {
        s = fmaf(a[t * C + c], s, b[t * C + c]);
        out[t * C + c] = s;
    }
}

__global__ __launch_bounds__(256) void k_serial_bwd(const float *__restrict__ lam, const float *__restrict__ h,
                                                    const float *__restrict__ h0, const float *e, float *gx, float *gl,
                                                    float *gh0, int64_t T, int64_t C)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float g = 0.0f;
#pragma unroll 4
    for (int64_t t = T - 1; t >= 0; --t) {
        const float l = (t + 1 < T) ? lam[(t + 1) * C + c] : 0.0f;
        g = fmaf(l, g, e[t * C + c]);
        const float hp = (t > 0) ? h[(t - 1) * C + c] : (h0 ? h0[c] : 0.0f);
        if (gx) gx[t * C + c] = g;
        if (gl) gl[t * C + c] = g * hp;
    }
    if (gh0) gh0[c] = lam[c] * g;
}

// The same two kernels on bf16 storage (fp32 arithmetic, results rounded to nearest even on store).
__device__ __forceinline__ float bf16_in(const unsigned short *p, int64_t i) { return __uint_as_float((unsigned int)p[i] << 16); }
__device__ __forceinline__ void bf16_out(unsigned short *p, int64_t i, float v) { p[i] = (unsigned short)(pack_bf16(v, 0.0f) & 0xffffu); }

__global__ __launch_bounds__(256) void k_serial_fwd_bf16(const unsigned short *__restrict__ a, const unsigned short *b,
                                                         const unsigned short *__restrict__ h0, unsigned short *out,
                                                         int64_t T, int64_t C)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float s = h0 ? bf16_in(h0, c) : 0.0f;
#pragma unroll 8
    for (int64_t t = 0; t < T; ++t) {
        s = fmaf(bf16_in(a, t * C + c), s, bf16_in(b, t * C + c));
        bf16_out(out, t * C + c, s);
    }
}

__global__ __launch_bounds__(256) void k_serial_bwd_bf16(const unsigned short *__restrict__ lam,
                                                         const unsigned short *__restrict__ h,
                                                         const unsigned short *__restrict__ h0, const unsigned short *e,
                                                         unsigned short *gx, unsigned short *gl, unsigned short *gh0,
                                                         int64_t T, int64_t C)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float g = 0.0f;
#pragma unroll 4
    for (int64_t t = T - 1; t >= 0; --t) {
        const float l = (t + 1 < T) ? bf16_in(lam, (t + 1) * C + c) : 0.0f;
        g = fmaf(l, g, bf16_in(e, t * C + c));
        const float hp = (t > 0) ? bf16_in(h, (t - 1) * C + c) : (h0 ? bf16_in(h0, c) : 0.0f);
        if (gx) bf16_out(gx, t * C + c, g);
        if (gl) bf16_out(gl, t * C + c, g * hp);
    }
    if (gh0) bf16_out(gh0, c, bf16_in(lam, c) * g);
}

__global__ void k_fill16(unsigned short *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// Element access of the serial form kernels in either storage type (E = float, or unsigned short for bf16).
template <class E>
__device__ __forceinline__ float el_in(const E *p, int64_t i)
{
    if constexpr (sizeof(E) == 4) return p[i];
    else return bf16_in(p, i);
}
template <class E>
__device__ __forceinline__ void el_out(E *p, int64_t i, float v)
{
    if constexpr (sizeof(E) == 4) p[i] = v;
    else bf16_out(p, i, v);
}

// The gated form of Section 3.1 (sigmoid and tau applied here), serial over the sequence length.
template <class E>
__global__ __launch_bounds__(256) void k_serial_gated_fwd(const E *__restrict__ g_pre, const E *i_pre,
                                                          const E *__restrict__ h0, E *out, int tau, int64_t T, int64_t C)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float s = h0 ? el_in(h0, c) : 0.0f;
#pragma unroll 4
    for (int64_t t = 0; t < T; ++t) {
        const vec<1> cm = gate_complement<1>(vec<1>(el_in(g_pre, t * C + c)));
        const vec<1> i = impulse<1>(vec<1>(el_in(i_pre, t * C + c)), tau);
        s = step<FORM_GATED, 1>(cm, vec<1>(s), cm * i)[0];
        el_out(out, t * C + c, s);
    }
}

template <class E>
__global__ __launch_bounds__(256) void k_serial_gated_bwd(const E *__restrict__ g_pre, const E *__restrict__ i_pre,
                                                          const E *__restrict__ h, const E *__restrict__ h0, const E *e,
                                                          E *gg, E *gi, E *gh0, int tau, int64_t T, int64_t C)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float d = 0.0f;
    float cnext = 1.0f;  // complement of the gate one row ahead; the last row has no successor (g = 0)
    float g0 = 0.0f;
#pragma unroll 2
    for (int64_t t = T - 1; t >= 0; --t) {
        d = step<FORM_GATED, 1>(vec<1>(cnext), vec<1>(d), vec<1>(el_in(e, t * C + c)))[0];
        const float cm = gate_complement<1>(vec<1>(el_in(g_pre, t * C + c)))[0];
        const float g = 1.0f - cm;
        const float i = impulse<1>(vec<1>(el_in(i_pre, t * C + c)), tau)[0];
        const float hp = (t > 0) ? el_in(h, (t - 1) * C + c) : (h0 ? el_in(h0, c) : 0.0f);
        if (gg) el_out(gg, t * C + c, d * (hp - i) * (g * cm));
        if (gi) el_out(gi, t * C + c, tau ? d * cm * fmaf(-i, i, 1.0f) : d * cm);
        cnext = cm;
        g0 = g;
    }
    if (gh0) el_out(gh0, c, g0 * d);
}

// The LSTM cell of Section 3.2 (c_t = f_t*c_{t-1} + i_t*z_t, h_t = o_t*c_t), serial over the sequence length.
template <class E>
__global__ __launch_bounds__(256) void k_serial_lstm_fwd(const E *__restrict__ f_pre, const E *__restrict__ i_pre,
                                                         const E *__restrict__ z_pre, const E *__restrict__ o_pre,
                                                         const E *__restrict__ c0, E *c_out, E *h_out, int64_t T, int64_t C)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float s = c0 ? el_in(c0, c) : 0.0f;
#pragma unroll 2
    for (int64_t t = 0; t < T; ++t) {
        const vec<1> cf = gate_complement<1>(vec<1>(el_in(f_pre, t * C + c)));
        const vec<1> x = gate_value<1>(vec<1>(el_in(i_pre, t * C + c))) * impulse<1>(vec<1>(el_in(z_pre, t * C + c)), 1);
        s = step<FORM_LSTM, 1>(cf, vec<1>(s), x)[0];
        if (c_out) el_out(c_out, t * C + c, s);
        if (h_out) el_out(h_out, t * C + c, gate_value<1>(vec<1>(el_in(o_pre, t * C + c)))[0] * s);
    }
}

template <class E>
__global__ __launch_bounds__(256) void k_serial_lstm_bwd(const E *__restrict__ f_pre, const E *__restrict__ i_pre,
                                                         const E *__restrict__ z_pre, const E *__restrict__ o_pre,
                                                         const E *__restrict__ cst, const E *__restrict__ c0,
                                                         const E *__restrict__ e, E *gf, E *gi, E *gz, E *go, E *gc0,
                                                         int64_t T, int64_t C)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float d = 0.0f, cnext = 1.0f, f0 = 0.0f;  // cnext: complement of the forget gate one row ahead
    for (int64_t t = T - 1; t >= 0; --t) {
        vec<1> og, oc, ig, ic;
        gate_both<1>(vec<1>(el_in(o_pre, t * C + c)), og, oc);
        gate_both<1>(vec<1>(el_in(i_pre, t * C + c)), ig, ic);
        const float et = el_in(e, t * C + c);
        d = step<FORM_LSTM, 1>(vec<1>(cnext), vec<1>(d), vec<1>(et * og[0]))[0];
        const float cf = gate_complement<1>(vec<1>(el_in(f_pre, t * C + c)))[0];
        const float f = 1.0f - cf;
        const float z = tanh_f32(el_in(z_pre, t * C + c));
        const float cp = (t > 0) ? el_in(cst, (t - 1) * C + c) : (c0 ? el_in(c0, c) : 0.0f);
        if (gf) el_out(gf, t * C + c, d * cp * (f * cf));
        if (gi) el_out(gi, t * C + c, d * z * (ig[0] * ic[0]));
        if (gz) el_out(gz, t * C + c, d * ig[0] * fmaf(-z, z, 1.0f));
        if (go) el_out(go, t * C + c, et * el_in(cst, t * C + c) * (og[0] * oc[0]));
        cnext = cf;
        f0 = f;
    }
    if (gc0) el_out(gc0, c, f0 * d);
}

__global__ void k_fill(float *p, float value, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = value;
}

// Test aid: plants a stored epoch (calls completed so far) into a look-back header, so that the
// reuse paths close to the epoch's wrap can be exercised without 2^31 calls.
__global__ void k_set_epoch(LookbackHeader *hdr, uint32_t stored_epoch)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) hdr->epoch = stored_epoch;
}

// Streaming probe: the bandwidth a kernel with this library's access instructions reaches when it
// does nothing but move data.  Reads the non-null inputs, writes the non-null outputs, 16 bytes per
// lane per access, PROBE_R independent accesses per tensor in flight per thread (4 measured 3-6 % ahead
// of 8 and 10 % ahead of 16 on an MI355X).  Without an output it only reads: the sum of what it read
// decides a store that never happens, so the loads cannot be dropped.
constexpr int PROBE_R = 4;
__device__ float g_probe_sink[4];
__global__ __launch_bounds__(256) void k_stream_probe(const float *in0, const float *in1, const float *in2, float *out0,
                                                      float *out1, int64_t n4)
{
    const int64_t chunk = (int64_t)blockIdx.x * (256 * PROBE_R);
    vec<4> acc[PROBE_R];
#pragma unroll
    for (int j = 0; j < PROBE_R; ++j) {
        const int64_t i = chunk + j * 256 + threadIdx.x;
        vec<4> v = splat<4>(1.0f);
        if (i < n4) {
            if (in0) v = ld<4>(in0 + 4 * i);
            if (in1) v *= ld<4>(in1 + 4 * i);
            if (in2) v += ld<4>(in2 + 4 * i);
        }
        acc[j] = v;
    }
    if (!out0 && !out1) {  // read-only
        vec<4> sum = acc[0];
#pragma unroll
        for (int j = 1; j < PROBE_R; ++j) sum += acc[j];
        if (sum[0] == -1.0f && sum[1] == -2.0f && sum[2] == -3.0f && sum[3] == -4.0f) {
#pragma unroll
            for (int v = 0; v < 4; ++v) g_probe_sink[v] = sum[v];
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < PROBE_R; ++j) {
        const int64_t i = chunk + j * 256 + threadIdx.x;
        if (i < n4) {
            if (out0) st<4>(out0 + 4 * i, acc[j]);
            if (out1) st<4>(out1 + 4 * i, acc[j] * acc[j]);
        }
    }
}

hipError_t launch_stream_probe(const float *in0, const float *in1, const float *in2, float *out0, float *out1,
                               int64_t n, hipStream_t s)
{
    const int64_t n4 = n / 4;
    if (n4 <= 0) return hipSuccess;
    const unsigned grid = (unsigned)((n4 + 256 * PROBE_R - 1) / (256 * PROBE_R));
    hipLaunchKernelGGL(k_stream_probe, dim3(grid), dim3(256), 0, s, in0, in1, in2, out0, out1, n4);
    return hipGetLastError();
}

// The same streams in the geometry of a tile: [T, C] arrays, a workgroup of 512 threads on PROBE_ROWS rows of
// PROBE_WC adjacent columns, one column per lane, every thread PROBE_RR consecutive rows at the row stride -- 256
// lanes side by side, the widest arrangement, which streams fastest (a compute unit then touches 1 KiB of a row
// at about the same time).  NIN inputs and NOUT outputs, compile-time so that the loads are straight-line code.
constexpr int PROBE_WC = 256, PROBE_RR = 16, PROBE_ROWS = (512 / PROBE_WC) * PROBE_RR;
template <int NIN, int NOUT>
__global__ __launch_bounds__(512) void k_rows_probe(const float *in0, const float *in1, const float *in2, float *out0,
                                                    float *out1, int64_t C)
{
    const int tc = threadIdx.x % PROBE_WC, tt = threadIdx.x / PROBE_WC;
    const int64_t G = C / PROBE_WC, g = blockIdx.x % G, k = blockIdx.x / G;
    const int64_t off = (k * PROBE_ROWS + (int64_t)tt * PROBE_RR) * C + g * PROBE_WC + tc;
    float v[PROBE_RR];
#pragma unroll
    for (int j = 0; j < PROBE_RR; ++j) {
        v[j] = 1.0f + j;
        if constexpr (NIN >= 1) v[j] = __builtin_nontemporal_load(in0 + off + j * C);
        if constexpr (NIN >= 2) v[j] *= __builtin_nontemporal_load(in1 + off + j * C);
        if constexpr (NIN >= 3) v[j] += __builtin_nontemporal_load(in2 + off + j * C);
    }
    if constexpr (NOUT == 0) {  // read-only: what was read decides a store that never happens
        float sum = v[0];
#pragma unroll
        for (int j = 1; j < PROBE_RR; ++j) sum += v[j];
        if (sum == -123.25f) g_probe_sink[0] = sum;
    } else {
#pragma unroll
        for (int j = 0; j < PROBE_RR; ++j) {
            __builtin_nontemporal_store(v[j], out0 + off + j * C);
            if constexpr (NOUT >= 2) __builtin_nontemporal_store(v[j] * v[j], out1 + off + j * C);
        }
    }
}

hipError_t launch_rows_probe(int nin, int nout, const float *in0, const float *in1, const float *in2, float *out0,
                             float *out1, int64_t T, int64_t C, hipStream_t s)
{
    if (T % PROBE_ROWS || C % PROBE_WC || nin < 0 || nin > 3 || nout < 0 || nout > 2 || nin + nout == 0)
        return hipErrorInvalidValue;
    const int64_t blocks = (T / PROBE_ROWS) * (C / PROBE_WC);
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(512);
#define LINREC_ROWS_PROBE(NI, NO) \
    if (nin == NI && nout == NO) hipLaunchKernelGGL((k_rows_probe<NI, NO>), grid, block, 0, s, in0, in1, in2, out0, out1, C);
    LINREC_ROWS_PROBE(1, 0) LINREC_ROWS_PROBE(2, 0) LINREC_ROWS_PROBE(3, 0)
    LINREC_ROWS_PROBE(0, 1) LINREC_ROWS_PROBE(1, 1) LINREC_ROWS_PROBE(2, 1) LINREC_ROWS_PROBE(3, 1)
    LINREC_ROWS_PROBE(0, 2) LINREC_ROWS_PROBE(1, 2) LINREC_ROWS_PROBE(2, 2) LINREC_ROWS_PROBE(3, 2)
#undef LINREC_ROWS_PROBE
    return hipGetLastError();
}

hipError_t launch_scan_summaries(const double *aggP, const double *aggS, const float *h0, double *carry, int64_t K,
                                 int64_t C, hipStream_t s)
{
    const unsigned grid = (unsigned)((C + SCAN_COLS - 1) / SCAN_COLS);
    hipLaunchKernelGGL(k_scan_summaries, dim3(grid), dim3(SCAN_WAVES * 64), 0, s, aggP, aggS, h0, carry, K, C);
    return hipGetLastError();
}

template <class E>
static hipError_t launch_serial_form(const Args &A, bool bwd, int form, unsigned grid, hipStream_t s)
{
    typedef const E *cp;
    typedef E *mp;
    if (form == FORM_LSTM) {
        if (!bwd)
            hipLaunchKernelGGL(k_serial_lstm_fwd<E>, dim3(grid), dim3(256), 0, s, (cp)A.a, (cp)A.b, (cp)A.c, (cp)A.d,
                               (cp)A.h0, (mp)A.out0, (mp)A.out1, A.T, A.C);
        else
            hipLaunchKernelGGL(k_serial_lstm_bwd<E>, dim3(grid), dim3(256), 0, s, (cp)A.a, (cp)A.c, (cp)A.d, (cp)A.e,
                               (cp)A.hprev, (cp)A.h0, (cp)A.b, (mp)A.out0, (mp)A.out1, (mp)A.out2, (mp)A.out3, (mp)A.gh0,
                               A.T, A.C);
    } else {
        if (!bwd)
            hipLaunchKernelGGL(k_serial_gated_fwd<E>, dim3(grid), dim3(256), 0, s, (cp)A.a, (cp)A.b, (cp)A.h0, (mp)A.out0,
                               A.tau, A.T, A.C);
        else
            hipLaunchKernelGGL(k_serial_gated_bwd<E>, dim3(grid), dim3(256), 0, s, (cp)A.a, (cp)A.c, (cp)A.hprev, (cp)A.h0,
                               (cp)A.b, (mp)A.out0, (mp)A.out1, (mp)A.gh0, A.tau, A.T, A.C);
    }
    return hipGetLastError();
}

hipError_t launch_serial(const Args &A, bool bwd, int form, bool bf16, hipStream_t s)
{
    const unsigned grid = (unsigned)((A.C + 255) / 256);
    if (form != FORM_PLAIN)
        return bf16 ? launch_serial_form<unsigned short>(A, bwd, form, grid, s) : launch_serial_form<float>(A, bwd, form, grid, s);
    if (bf16) {
        typedef const unsigned short *cp;
        typedef unsigned short *mp;
        if (!bwd)
            hipLaunchKernelGGL(k_serial_fwd_bf16, dim3(grid), dim3(256), 0, s, (cp)A.a, (cp)A.b, (cp)A.h0, (mp)A.out0, A.T,
                               A.C);
        else
            hipLaunchKernelGGL(k_serial_bwd_bf16, dim3(grid), dim3(256), 0, s, (cp)A.a, (cp)A.hprev, (cp)A.h0, (cp)A.b,
                               (mp)A.out0, (mp)A.out1, (mp)A.gh0, A.T, A.C);
        return hipGetLastError();
    }
    if (!bwd) hipLaunchKernelGGL(k_serial_fwd, dim3(grid), dim3(256), 0, s, A.a, A.b, A.h0, A.out0, A.T, A.C);
    else
        hipLaunchKernelGGL(k_serial_bwd, dim3(grid), dim3(256), 0, s, A.a, A.hprev, A.h0, A.b, A.out0, A.out1, A.gh0,
                           A.T, A.C);
    return hipGetLastError();
}

hipError_t launch_fill16(void *p, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int64_t blocks = std::min<int64_t>((n + 255) / 256, 65536);
    hipLaunchKernelGGL(k_fill16, dim3((unsigned)blocks), dim3(256), 0, s, (unsigned short *)p, n);
    return hipGetLastError();
}

hipError_t launch_set_epoch(LookbackHeader *hdr, uint32_t stored_epoch, hipStream_t s)
{
    hipLaunchKernelGGL(k_set_epoch, dim3(1), dim3(64), 0, s, hdr, stored_epoch);
    return hipGetLastError();
}

hipError_t launch_fill(float *p, float value, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int64_t blocks = std::min<int64_t>((n + 255) / 256, 65536);
    hipLaunchKernelGGL(k_fill, dim3((unsigned)blocks), dim3(256), 0, s, p, value, n);
    return hipGetLastError();
}

}  // namespace linrec
