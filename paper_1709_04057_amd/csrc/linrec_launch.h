// Host-visible part of the kernel layer: the argument block every kernel takes, the table of tile
// shapes, and the launch functions the C API calls.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace linrec {

// Device-resident state of a look-back workspace.  The kernel itself hands out tickets, counts
// finished workgroups, and its last workgroup rewinds the ticket and advances the epoch, so nothing
// about a call is baked into the kernel arguments: a launch recorded in a HIP graph can be replayed.
// The three words every workgroup touches sit in different 128-byte lines: atomics on one address are
// served one at a time, and a read of the epoch must not queue behind the ticket traffic.
struct LookbackHeader {
    unsigned long long ticket;  // next tile of the running call
    unsigned long long pad0[15];
    unsigned long long done;    // workgroups of the running call that have finished their look-back
    unsigned long long pad1[15];
    uint32_t epoch;             // calls completed, 0 .. 2^31-2; the running call's epoch is this + 1, and its
                                // tags are epoch<<1 (summary) and epoch<<1|1 (inclusive state)
    uint32_t err;               // set when a look-back wait gave up
    unsigned long long pad2[15];
};

struct Args {
    const float *a;      // lambda (gated form: the gate pre-activations g_pre)      [T, C]
    const float *b;      // forward: x (gated: i_pre);  backward: grad_h            [T, C]
    const float *c;      // gated form, backward: the impulse pre-activations i_pre  [T, C]
                         // LSTM cell: forward z_pre (a = f_pre, b = i_pre), backward i_pre (a = f_pre, b = grad_h)
    const float *d;      // LSTM cell: forward o_pre, backward z_pre
    const float *e;      // LSTM cell, backward: o_pre
    const float *hprev;  // backward: h (forward output);  forward: unused
    const float *h0;     // [C] or nullptr
    float *out0;         // forward: h_out;  backward: grad_x (gated: grad_g_pre) (may be nullptr)
    float *out1;         // backward: grad_lambda (gated: grad_i_pre) (may be nullptr)
                         // LSTM cell: forward out0 = c, out1 = h; backward out0..3 = grad_f/i/z/o_pre
    float *out2, *out3;
    float *gh0;          // backward: grad_h0 [C] (may be nullptr)
    int64_t T, C;
    int64_t K;           // tiles (look-back) or chunks (three-phase) along time
    int64_t K1, K2;      // look-back: K1 full-height tiles, then K2 of half height, the rest a quarter
    int32_t G;           // column groups of COLS columns
    int32_t M;           // three-phase: tiles walked per chunk
    int32_t tau;         // gated form: impulse activation (0 identity, 1 tanh)
    // three-phase workspace, each [K, C] fp64
    double *aggP, *aggS, *carry;
    // look-back workspace: 64-bit words {tag : 32 | payload bits : 32}
    unsigned long long *lbAgg;   // [K, C, 3]  low and high half of the fp64 P; fp32 S, later the fp32 inclusive state
    struct LookbackHeader *hdr;  // device-resident call state (ticket, epoch, ...)
    uint32_t spin_limit;
    int32_t persistent;          // look-back: workgroups loop over tickets (1) or take exactly one (0)
    int32_t grid_cap;            // look-back, persistent: at most this many workgroups per compute unit (0: no cap)
    int32_t stagger;             // look-back: pause of the odd workgroups among the first stagger_n, in units of
                                 // 2048 clocks (about a microsecond); stagger_n is set at launch
    int32_t stagger_n;
    unsigned long long *trace;  // only read by builds with -DLINREC_TRACE: 8 words per tile
};

enum Kind { KIND_REDUCE = 0, KIND_FIXUP = 1, KIND_LOOKBACK = 2, KIND_WALK = 3 };
enum Form { FORM_PLAIN = 0, FORM_GATED = 1, FORM_LSTM = 2 };

struct TileDesc {
    int vec, r, wc, wt;
    int rows() const { return r * wt; }
    int cols() const { return vec * wc; }
    int threads() const { return wc * wt; }
};

// Tile shapes by id, as used by LINREC_OPT_TILE: (id, columns per thread, rows per thread, threads along
// columns, threads along time).  A shape with v columns per thread makes 4v-byte accesses and needs
// C % v == 0 and 4v-byte aligned tensors; v = 1 works for any C and alignment.  (With bf16 storage the
// accesses are 2v bytes; the plain recurrence on bf16 storage has kernels for v = 2 and 4 only.)  Shapes with
// more than 64 elements per thread exist for bf16 storage only, where two elements share a register.  This
// is the catalogue: which of these shapes a build has kernels for, and for which entry-point families, is
// in linrec_tile_set.inc, written from measurements (plan_sweep.py) -- a shape no plan takes is not built.
// Ids are stable across versions of the library.
//   one column per thread, 512 threads (one workgroup per compute unit): 44, 43, 42, 38, 41 (64 wide, 64 ..
//   24 rows per thread), 22, 35, 34, 33 (32 wide); 256 threads: 20, 21, 45 (64 wide), 17, 19, 18 (32 wide),
//   1, 2 (8 rows per thread), 23 (16 wide, for a handful of columns); 52, 53 (64 wide, 36 and 28 rows per
//   thread) for wide problems whose row length is a large power of two: the threads of a workgroup that share a
//   column start rows-per-thread rows apart, and from 16384 columns on a distance that is a multiple of 2 MiB
//   (32 or 64 rows of 16384 floats, 48 rows of 32768 ...) measured 10-15 % less bandwidth than the same shape
//   on 12288 or 24576 columns; 36 and 28 rows keep it an odd multiple of at most 1 MiB up to 65536 columns
//   one column per thread, more than 64 threads side by side (two or four wavefronts share a row of the tile,
//   so a workgroup reads and writes 512-byte or 1-KiB pieces of a row at about the same time, which the memory
//   system serves faster than the same bytes from different compute units): 56, 57, 58, 60 (128 wide, 64 .. 24
//   rows per thread), 59 (256 wide); 61, 62 the same with two columns per thread, for bf16 storage
//   two and four columns per thread (8- and 16-byte accesses; 4- and 8-byte with bf16 storage): the rest
//   (54, 55: 40 and 56 rows per thread, 64 wide, 256 threads: the same for bf16 storage)
#define LINREC_TILES(X) \
    X(1, 1, 8, 64, 4)   \
    X(2, 1, 8, 16, 16)  \
    X(3, 4, 8, 8, 32)   \
    X(4, 4, 8, 16, 16)  \
    X(5, 4, 8, 32, 8)   \
    X(6, 4, 8, 64, 4)   \
    X(7, 4, 16, 8, 32)  \
    X(8, 4, 16, 16, 16) \
    X(9, 4, 16, 32, 8)  \
    X(10, 4, 16, 64, 4) \
    X(13, 2, 32, 16, 16) \
    X(14, 2, 24, 16, 16) \
    X(15, 2, 16, 16, 16) \
    X(16, 2, 32, 32, 8)  \
    X(17, 1, 64, 32, 8)  \
    X(18, 1, 32, 32, 8)  \
    X(19, 1, 48, 32, 8)  \
    X(20, 1, 64, 64, 4)  \
    X(21, 1, 32, 64, 4)  \
    X(22, 1, 64, 32, 16) \
    X(23, 1, 64, 16, 16) \
    X(24, 2, 64, 32, 8)  \
    X(25, 2, 64, 16, 16) \
    X(26, 4, 32, 16, 16) \
    X(27, 4, 32, 32, 8)  \
    X(28, 2, 64, 64, 4)  \
    X(29, 2, 48, 32, 8)  \
    X(30, 2, 64, 32, 16) \
    X(33, 1, 16, 32, 16) \
    X(34, 1, 24, 32, 16) \
    X(35, 1, 32, 32, 16) \
    X(38, 1, 32, 64, 8)  \
    X(41, 1, 24, 64, 8)  \
    X(42, 1, 40, 64, 8)  \
    X(43, 1, 48, 64, 8)  \
    X(44, 1, 64, 64, 8)  \
    X(45, 1, 24, 64, 4)  \
    X(47, 2, 64, 64, 8)  \
    X(48, 2, 48, 64, 8)  \
    X(51, 2, 48, 32, 16) \
    X(52, 1, 36, 64, 4)  \
    X(53, 1, 28, 64, 4)  \
    X(54, 2, 40, 64, 4)  \
    X(55, 2, 56, 64, 4)  \
    X(56, 1, 64, 128, 4) \
    X(57, 1, 48, 128, 4) \
    X(58, 1, 32, 128, 4) \
    X(59, 1, 64, 256, 2) \
    X(60, 1, 24, 128, 4) \
    X(61, 2, 64, 128, 4) \
    X(62, 2, 48, 128, 4)
constexpr int MAX_TILE_ID = 62;

// Families (bit LINREC_ENTRY_*) whose kernels can exist for a shape at all:
//   plain fp32         at most 64 elements per thread and operand (one register each)
//   plain, bf16        2 or 4 columns per thread (4- and 8-byte accesses); two elements share a register
//   gated layer        at most 64 elements per thread, rows per thread a multiple of 8 or fewer than 8 (the
//                      epilogues work in chunks of 8 rows); the same on bf16 storage, whose register tile
//                      holds computed fp32 values (one-column shapes make 2-byte accesses there)
//   LSTM cell          the same with at most 32 elements per thread and operand (three operands in flight)
constexpr unsigned geometry_families(const TileDesc &d)
{
    const bool f32 = d.r * d.vec <= 64, gated = f32 && (d.r % 8 == 0 || d.r < 8), cell = gated && d.r * d.vec <= 32;
    return (f32 ? 1u << 0 : 0u) | (gated ? (1u << 1 | 1u << 4) : 0u) | (cell ? (1u << 2 | 1u << 5) : 0u) |
           (d.vec >= 2 ? 1u << 3 : 0u);
}

// Families this build has kernels of shape `id` for.  -DLINREC_ALL_SHAPES builds every kernel the geometry
// allows (what plan_sweep.py measures on); the default is the measured selection.
#ifndef LINREC_ALL_SHAPES
#include "linrec_tile_set.inc"
#endif
constexpr unsigned tile_families(int id)
{
    unsigned geometry = 0, built = 0;
    switch (id) {
#define X(ID, VEC, R, WC, WT) \
    case ID: geometry = geometry_families(TileDesc{VEC, R, WC, WT}); break;
        LINREC_TILES(X)
#undef X
    default: break;
    }
#ifdef LINREC_ALL_SHAPES
    built = ~0u;
#else
    switch (id) {
#define X(ID, MASK) \
    case ID: built = MASK; break;
        LINREC_BUILT_TILES(X)
#undef X
    default: break;
    }
#endif
    return geometry & built;
}

bool tile_has(int id, int family);  // this build has kernels of shape `id` for entry-point family LINREC_ENTRY_*
bool tile_exists(int id);           // ... for at least one family
const TileDesc &tile_desc(int id);  // the geometry of a catalogued id

// Launches kernel `kind` for tile shape `id` with grid A.K * A.G.  hp_late (look-back, backward):
// load h after the rescan instead of together with lambda and grad_h.  `form` is FORM_PLAIN, FORM_GATED
// (Section 3.1: sigmoid / tau applied in the kernel) or FORM_LSTM (Section 3.2); bf16: the tensors hold
// bf16.  hipErrorInvalidValue when this build has no such kernel (see tile_families; the three-phase
// kernels exist for the plain fp32 family only).
hipError_t launch_tile_kernel(int id, Kind kind, bool bwd, bool hp_late, int form, bool bf16, const Args &A,
                              hipStream_t s);

hipError_t launch_scan_summaries(const double *aggP, const double *aggS, const float *h0, double *carry, int64_t K,
                                 int64_t C, hipStream_t s);
hipError_t launch_serial(const Args &A, bool bwd, int form, bool bf16, hipStream_t s);
hipError_t launch_fill(float *p, float value, int64_t n, hipStream_t s);
hipError_t launch_set_epoch(LookbackHeader *hdr, uint32_t stored_epoch, hipStream_t s);  // test aid
hipError_t launch_fill16(void *p, int64_t n, hipStream_t s);  // n 16-bit zeros
hipError_t launch_stream_probe(const float *in0, const float *in1, const float *in2, float *out0, float *out1,
                               int64_t n, hipStream_t s);
// The probe in the geometry of a tile: the first `nin` inputs and `nout` outputs, [T, C] arrays, T a multiple of 32
// and C of 256 (hipErrorInvalidValue otherwise).
hipError_t launch_rows_probe(int nin, int nout, const float *in0, const float *in1, const float *in2, float *out0,
                             float *out1, int64_t T, int64_t C, hipStream_t s);

}  // namespace linrec
