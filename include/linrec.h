/*
 * linrec.h -- C ABI of liblinrec: the diagonal linear recurrence
 *
 *     h_t = lambda_t (.) h_{t-1} + x_t                     (arXiv 1709.04057, Section 2)
 *
 * evaluated in parallel over the sequence length as a scan of the affine pairs
 * (lambda_t, x_t) under  (a1,b1) (+) (a2,b2) = (a1*a2, a2*b1 + b2)  (Algorithm 1 of the
 * paper: per-chunk reduce, scan of the chunk summaries, per-chunk rescan from the carry),
 * and its backward pass, the same recurrence run in reverse over the upstream gradient
 * (Section 2.2).  AMD MI355X (gfx950) only.
 *
 * Conventions shared by every entry point
 *   - Tensors are fp32, contiguous, time-major [T, B, n]: element (t, b, i) lives at
 *     (t*B + b)*n + i.  The C = B*n columns are independent recurrences (the layout of
 *     Section 3.1.1: T vectors of B*n elements); time runs down the rows.
 *   - Row t (0-based) holds the paper's lambda_{t+1}, x_{t+1}, h_{t+1}.  h0 [B, n] is the
 *     paper's h_0: an input, never an output row (the SCAN of Section 1 returns T outputs
 *     for T inputs).
 *   - Every pointer is a DEVICE pointer owned by the caller, valid on the device the stream
 *     belongs to.  The library neither frees nor retains them.  Any 4-byte aligned pointer
 *     is accepted; 16-byte (8-byte) accesses are used only when every tensor pointer is
 *     16-byte (8-byte) aligned and C is a multiple of 4 (2).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work and return: there is no host synchronisation, device-side faults surface
 *     at the caller's next synchronisation.
 *   - The library keeps one cached device workspace (chunk summaries, carries, look-back
 *     flags) per (device, stream); it is allocated on first use and grown on demand, and
 *     linrec_reserve_workspace() sizes it ahead of time.  Growing allocates a new block
 *     (hipMalloc: the only place a call may block) and RETIRES the old one, which stays
 *     allocated until linrec_release_workspace(): kernels still queued on the stream, and
 *     launches recorded in a HIP graph, keep pointing at memory that exists.  A call that
 *     would have to grow the workspace while its stream is being captured returns
 *     LINREC_ERR_CAPTURE and enqueues nothing: reserve, or make one eager call of the largest
 *     shape, before capturing.  Calls that use the same stream from several host threads at
 *     once are not supported; calls on different streams are independent.
 *   - Return value: LINREC_OK (0) or a negative LINREC_ERR_* code.  Arguments are validated
 *     before any HIP call is made.  T == 0 or B*n == 0 is a successful no-op (for T == 0 a
 *     non-NULL grad_h0 is zero-filled).
 *   - No floating-point atomics anywhere.  The three-phase, walk and serial variants are
 *     bitwise reproducible for a fixed tile shape.  The single pass (look-back) composes a
 *     tile's carry-in from whichever predecessor summaries and states are published when
 *     it looks, so two runs may associate the same terms differently and differ in the last
 *     bit or two of a row; every such result is within the stated tolerances.  Different
 *     variants / tile shapes differ in the last bits too.
 *   - Domain: finite inputs whose partial products of lambda stay finite (|lambda| <= 1 is
 *     always safe).  NaN/Inf propagate along their own column only.
 */
#ifndef LINREC_H
#define LINREC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    LINREC_OK = 0,
    LINREC_ERR_NULL = -1,   /* a required pointer is NULL                                   */
    LINREC_ERR_SHAPE = -2,  /* negative dimension, or T*B*n overflows / exceeds 2^40        */
    LINREC_ERR_ALIAS = -3,  /* forbidden overlap between an output and another tensor       */
    LINREC_ERR_HIP = -4,    /* a HIP allocation or launch failed; see linrec_last_hip_error */
    LINREC_ERR_OPTION = -5, /* unknown option or value out of range                         */
    LINREC_ERR_DEVICE = -6, /* a kernel reported a look-back wait that exceeded its limit   */
    LINREC_ERR_CAPTURE = -7,/* the workspace would have to grow while the stream is capturing */
    LINREC_ERR_SCRATCH = -8 /* linrec_forward_noalloc: problem too large for the fixed scratch */
};

/* Which kernel family evaluates the scan (linrec_set_option(LINREC_OPT_VARIANT, ...)). */
enum {
    LINREC_VARIANT_AUTO = 0,       /* library picks: the single pass, or the walk for short,
                                      wide problems                                           */
    LINREC_VARIANT_THREEPHASE = 1, /* Algorithm 1 as three kernels: reduce, scan, rescan     */
    LINREC_VARIANT_LOOKBACK = 2,   /* one kernel; chunk carries found by decoupled look-back */
    LINREC_VARIANT_SERIAL = 3,     /* one thread per column walks T: serial over the sequence,
                                      parallel over features and minibatch (the comparison
                                      kernel of Section 4.1.1)                               */
    LINREC_VARIANT_WALK = 4        /* one workgroup per group of columns walks T tile by tile:
                                      parallel over the sequence inside a tile only, nothing is
                                      exchanged between workgroups; what the library picks for
                                      short, wide problems                                      */
};

enum {
    LINREC_OPT_VARIANT = 1,    /* LINREC_VARIANT_*                                           */
    LINREC_OPT_TILE = 2,       /* tile-shape id, 0 = automatic (see linrec_tile_info; an id the
                                  entry point has no kernel of -- linrec_tile_has -- is ignored) */
    LINREC_OPT_CHUNK_TILES = 3,/* three-phase: tiles walked per chunk, 0 = automatic         */
    LINREC_OPT_SPIN_LIMIT = 4, /* look-back: polls before a wait is declared failed          */
    LINREC_OPT_HPREV_LATE = 5, /* look-back backward: load h after the rescan (1), together
                                  with lambda and grad_h (0), or let the library decide (-1)  */
    LINREC_OPT_TAPER = 6,      /* look-back: cut this many eighths (0..8) of the last round of
                                  tiles into half- and quarter-height tiles, so that a launch
                                  of few rounds does not end on a few workgroups finishing
                                  big tiles; 0 = none; -1 (default) = what linrec_tune
                                  remembered for the shape, else what the static plan has
                                  (2 where that measured ahead, mostly long sequences on few
                                  columns; it loses on wide problems)                        */
    LINREC_OPT_PERSISTENT = 7, /* look-back: launch as many workgroups as LINREC_OPT_GRID_CAP
                                  allows and let each loop over tiles (1; also what -1, the
                                  default, means), or one workgroup per tile (0)               */
    LINREC_OPT_GRID_CAP = 8,   /* look-back, persistent: workgroups per compute unit.  0
                                  (default): eight wavefronts per unit, i.e. one workgroup of
                                  512 threads or two of 256 -- more resident tiles than the
                                  memory system needs only lengthen the start and the end of
                                  a launch; n > 0: at most n; -1: as many as fit               */
    LINREC_OPT_STAGGER = 9,    /* look-back: every other workgroup of the first round starts
                                  this many microseconds (roughly; 0..16) late, so that the
                                  workgroups do not load, scan and store in lock-step;
                                  only launches of two rounds or more; default 3, 0 = off    */
    /* Test aids for the workspace-reuse paths of the single pass (no use outside tests): */
    LINREC_OPT_TEST_FILL = 10, /* 32-bit pattern that the words of a NEWLY allocated look-back
                                  workspace are filled with instead of zeros (stale words with
                                  foreign tags); default 0                                    */
    LINREC_OPT_TEST_EPOCH = 11 /* 0 .. 2^31-3: the thread's next single-pass call first sets its
                                  workspace's stored epoch (calls completed; it wraps to 0 after
                                  2^31-2) to this value and schedules the periodic clearing of
                                  stale words for two calls later, i.e. before a small epoch can
                                  run again; consumed by that call (-1 = none)                 */
};

/*
 * Forward pass.  (Section 2; Algorithm 1.)
 *   lambda, x : [T, B, n] inputs.
 *   h0        : [B, n] initial state, or NULL for a zero state.
 *   h_out     : [T, B, n] output; h_out[t] is the state after consuming row t.
 * h_out may alias x exactly (same pointer): every tile reads its rows before it writes
 * them.  Any other overlap of h_out with an input returns LINREC_ERR_ALIAS.
 */
int linrec_forward(const float *lambda, const float *x, const float *h0, float *h_out,
                   int64_t T, int64_t B, int64_t n, void *stream);

/*
 * Backward pass.  (Section 2.2.)  With e = grad_h, the direct upstream dL/dh_t, and
 * g_t the accumulated gradient nabla_{h_t} L:
 *     g_{T-1} = e_{T-1},   g_t = lambda_{t+1} * g_{t+1} + e_t      (row T of lambda is never read)
 *     grad_x[t]      = g_t
 *     grad_lambda[t] = g_t * h[t-1]          (h[-1] = h0, zero if h0 == NULL)
 *     grad_h0        = lambda[0] * g_0
 *   lambda, h, grad_h : [T, B, n] inputs; h is the forward pass' h_out (x is not needed).
 *   h0                : [B, n] or NULL.
 *   grad_x, grad_lambda : [T, B, n] outputs; either may be NULL to skip it.
 *   grad_h0           : [B, n] output or NULL to skip it.
 * grad_x may alias grad_h exactly; any other overlap of an output with another tensor
 * returns LINREC_ERR_ALIAS.  grad_lambda is the partial derivative with x held fixed.
 */
int linrec_backward(const float *lambda, const float *h, const float *h0, const float *grad_h,
                    float *grad_x, float *grad_lambda, float *grad_h0,
                    int64_t T, int64_t B, int64_t n, void *stream);

/*
 * linrec_forward for callers that cannot allocate device memory -- code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, layout, NULL and aliasing
 * rules and results (to the tolerances above) as linrec_forward, but the single pass keeps its
 * look-back words in a fixed array of LINREC_NOALLOC_SCRATCH_BYTES inside the library's device image
 * instead of the cached workspace: the call makes no hipMalloc / hipFree and touches no allocator.
 * Every GPU the library runs on holds its own copy of the array until the process ends.
 *   - A problem whose look-back words do not fit -- 512 + 24 * K * B*n bytes, K = tiles along T of
 *     the plan in force (linrec_plan and linrec_tile_info: ceil(T / rows of the tile), a few more
 *     with a tapered tail) -- returns LINREC_ERR_SCRATCH and enqueues nothing.  All five benchmark
 *     workloads fit (the largest, [262144, 8, 512] on 512-row tiles, takes 48 MiB of the 64).
 *   - The three-phase variant is not available here (an explicit request runs the single pass).
 *   - All calls on one GPU share that GPU's array, on whatever stream: calls that may overlap in time
 *     on one GPU race on it and give wrong results.  Serialise them (one stream, or events).
 *   - The array keeps the previous call's words; they are told from the running call's by their epoch,
 *     as in the cached workspace, so nothing is cleared between calls.
 */
#define LINREC_NOALLOC_SCRATCH_BYTES (64u << 20)
int linrec_forward_noalloc(const float *lambda, const float *x, const float *h0, float *h_out,
                           int64_t T, int64_t B, int64_t n, void *stream);
/* LINREC_NOALLOC_SCRATCH_BYTES as the library was built with. */
int64_t linrec_noalloc_scratch_bytes(void);

/*
 * The same two passes on bf16 STORAGE: every tensor (and h0, grad_h0) holds bfloat16, i.e. the upper
 * 16 bits of an fp32, passed as uint16_t.  Values are widened exactly on load, all arithmetic is that
 * of linrec_forward / linrec_backward (fp32 steps, fp64 chunk products), results are rounded to
 * nearest even on store.  6 bytes per element forward, 10 backward.  The paper's kernel is fp32 only
 * (Section 2.3): this is a bandwidth option, not one of its experiments.  Same layout, NULL and
 * aliasing rules as above.  Accuracy: each stored value is within half a bf16 unit in the last place
 * (2^-8 relative at worst: bf16 keeps 8 significant bits) of what the fp32 entry points would store for the same (bf16-valued) inputs, up
 * to their own tolerance; the backward pass consumes the ROUNDED h it is given.
 * 4-byte aligned tensors with an even B*n use 4-byte accesses (8-byte ones when 8-byte aligned and
 * B*n is a multiple of 4); anything else falls back to the serial kernel.
 */
int linrec_forward_bf16(const uint16_t *lambda, const uint16_t *x, const uint16_t *h0,
                        uint16_t *h_out, int64_t T, int64_t B, int64_t n, void *stream);
int linrec_backward_bf16(const uint16_t *lambda, const uint16_t *h, const uint16_t *h0,
                         const uint16_t *grad_h, uint16_t *grad_x, uint16_t *grad_lambda,
                         uint16_t *grad_h0, int64_t T, int64_t B, int64_t n, void *stream);

/* Impulse activation tau of the gated layer (Section 3.1 leaves it open; its LSTM uses tanh). */
enum { LINREC_TAU_IDENTITY = 0, LINREC_TAU_TANH = 1 };

/*
 * Gated impulse linear recurrent layer, the part after its two matrix products, with the
 * activations applied inside the scan kernel (Section 3.1):
 *     g_t = sigmoid(g_pre[t]),   i_t = tau(i_pre[t]),   h_t = g_t * h_{t-1} + (1 - g_t) * i_t
 *   g_pre, i_pre : [T, B, n] pre-activations (U x_t + b_g and V x_t + b_z in the paper).
 *   h0           : [B, n] or NULL (zero state).      h_out : [T, B, n].
 *   tau          : LINREC_TAU_TANH or LINREC_TAU_IDENTITY (LINREC_ERR_OPTION otherwise).
 * Moves the same 12 bytes per element as linrec_forward; separate activation kernels in front
 * of it would move 16 more.  The kernel works with 1 - g_t = sigmoid(-g_pre[t]), formed without
 * cancellation, so gates arbitrarily close to one keep their decay rate (an fp32 g_t could not).
 * h_out may alias i_pre exactly; any other overlap returns LINREC_ERR_ALIAS.  Always evaluated
 * by the single-pass kernel (or the serial one when LINREC_OPT_VARIANT asks for it).
 */
int linrec_gilr_forward(const float *g_pre, const float *i_pre, const float *h0, float *h_out,
                        int tau, int64_t T, int64_t B, int64_t n, void *stream);

/*
 * Gradients of the layer above with respect to its pre-activations (Section 2.2's reverse
 * recurrence followed by the chain rule through the gate and tau).  With e = grad_h (direct
 * dL/dh_t) and d_t = g_{t+1} * d_{t+1} + e_t, d_{T-1} = e_{T-1}:
 *     grad_g_pre[t] = d_t * (h[t-1] - i_t) * g_t * (1 - g_t)          (h[-1] = h0)
 *     grad_i_pre[t] = d_t * (1 - g_t) * tau'(i_pre[t])
 *     grad_h0       = g_0 * d_0
 *   g_pre, i_pre, h, grad_h : [T, B, n] inputs; h is linrec_gilr_forward's h_out.
 *   grad_g_pre, grad_i_pre  : [T, B, n] outputs, either may be NULL; grad_h0 : [B, n] or NULL.
 * 24 bytes per element (four tensors in, two out).  No output may overlap any other tensor
 * (LINREC_ERR_ALIAS).
 */
int linrec_gilr_backward(const float *g_pre, const float *i_pre, const float *h, const float *h0,
                         const float *grad_h, float *grad_g_pre, float *grad_i_pre, float *grad_h0,
                         int tau, int64_t T, int64_t B, int64_t n, void *stream);

/*
 * Cell of the GILR-LSTM, the part after its matrix products, with the activations applied inside
 * the scan kernel (Section 3.2: the LSTM whose gates are computed from
 * the surrogate state, so that c_t depends only linearly on c_{t-1}):
 *     f, i, o = sigmoid(f_pre, i_pre, o_pre)[t],   z = tanh(z_pre[t]),
 *     c_t = f * c_{t-1} + i * z,                    h_t = o * c_t
 *   f_pre, i_pre, z_pre, o_pre : [T, B, n] pre-activations.      c0 : [B, n] or NULL (zero).
 *   c_out, h_out : [T, B, n] outputs; either may be NULL (o_pre may then be NULL too when h_out
 *   is), not both.  c_out is what linrec_lstm_cell_backward needs.
 * 24 bytes per element with both outputs.  No output may overlap any other tensor of the call
 * (LINREC_ERR_ALIAS).  The forget gate is kept as 1 - f = sigmoid(-f_pre), as in the gated layer.
 */
int linrec_lstm_cell_forward(const float *f_pre, const float *i_pre, const float *z_pre,
                             const float *o_pre, const float *c0, float *c_out, float *h_out,
                             int64_t T, int64_t B, int64_t n, void *stream);

/*
 * Gradients of the cell with respect to its pre-activations and c0 for an upstream gradient
 * e = grad_h = dL/dh_t (c_t reaches the loss through h_t and c_{t+1} only).  With
 * d_t = e_t * o_t + f_{t+1} * d_{t+1}, d_{T-1} = e_{T-1} * o_{T-1} (Section 2.2 on the cell state):
 *     grad_o_pre[t] = e_t * c[t] * o(1-o)           grad_f_pre[t] = d_t * c[t-1] * f(1-f)   (c[-1] = c0)
 *     grad_i_pre[t] = d_t * z * i(1-i)              grad_z_pre[t] = d_t * i * (1 - z^2)
 *     grad_c0       = f_0 * d_0
 *   f_pre, i_pre, z_pre, o_pre, c, grad_h : [T, B, n] inputs; c is the forward pass' c_out.
 *   grad_*_pre : [T, B, n] outputs, each may be NULL; grad_c0 : [B, n] or NULL.
 * 40 bytes per element (six tensors in, four out).  No output may overlap any other tensor.
 */
int linrec_lstm_cell_backward(const float *f_pre, const float *i_pre, const float *z_pre,
                              const float *o_pre, const float *c, const float *c0,
                              const float *grad_h, float *grad_f_pre, float *grad_i_pre,
                              float *grad_z_pre, float *grad_o_pre, float *grad_c0,
                              int64_t T, int64_t B, int64_t n, void *stream);

/*
 * The gated layer and the LSTM cell on bf16 STORAGE: every tensor holds bfloat16 (passed as uint16_t),
 * values are widened exactly on load, the arithmetic is that of the fp32 entry points above (fp32
 * activations and steps, fp64 chunk products), results are rounded to nearest even on store: 6 / 12
 * bytes per element for the layer, 12 / 20 for the cell.  Like linrec_forward_bf16 a bandwidth option,
 * not one of the paper's experiments (Section 2.3: fp32).  Same arguments, NULL and aliasing rules
 * as the fp32 entry points.  The backward passes consume the ROUNDED h (c) they are given.  Tensors
 * that are not 4-byte aligned, or an odd B*n, use the tile shapes with 2-byte accesses.
 */
int linrec_gilr_forward_bf16(const uint16_t *g_pre, const uint16_t *i_pre, const uint16_t *h0,
                             uint16_t *h_out, int tau, int64_t T, int64_t B, int64_t n, void *stream);
int linrec_gilr_backward_bf16(const uint16_t *g_pre, const uint16_t *i_pre, const uint16_t *h,
                              const uint16_t *h0, const uint16_t *grad_h, uint16_t *grad_g_pre,
                              uint16_t *grad_i_pre, uint16_t *grad_h0, int tau, int64_t T, int64_t B,
                              int64_t n, void *stream);
int linrec_lstm_cell_forward_bf16(const uint16_t *f_pre, const uint16_t *i_pre, const uint16_t *z_pre,
                                  const uint16_t *o_pre, const uint16_t *c0, uint16_t *c_out,
                                  uint16_t *h_out, int64_t T, int64_t B, int64_t n, void *stream);
int linrec_lstm_cell_backward_bf16(const uint16_t *f_pre, const uint16_t *i_pre, const uint16_t *z_pre,
                                   const uint16_t *o_pre, const uint16_t *c, const uint16_t *c0,
                                   const uint16_t *grad_h, uint16_t *grad_f_pre, uint16_t *grad_i_pre,
                                   uint16_t *grad_z_pre, uint16_t *grad_o_pre, uint16_t *grad_c0,
                                   int64_t T, int64_t B, int64_t n, void *stream);

/* Tuning knobs (LINREC_OPT_*), one set PER HOST THREAD: a call uses the options of the thread
 * that makes it, so a thread that changes them cannot disturb the calls of another.  Every
 * thread starts from the environment variables LINREC_VARIANT ("auto", "threephase",
 * "lookback", "serial", "walk") and LINREC_TILE (integer id), else the defaults.  Returns
 * LINREC_OK or LINREC_ERR_OPTION.  For a plan that holds for all threads use linrec_pin_plan. */
int linrec_set_option(int option, int64_t value);
int64_t linrec_get_option(int option);

/* Describes tile shape `tile_id`: threads along columns, threads along time, rows per thread,
 * columns per thread.  Ids are stable across versions and have gaps: the library is built for the
 * shapes that measured fastest somewhere (plan_sweep.py), and LINREC_ERR_OPTION is returned for an
 * id it has no kernel of.  Any output pointer may be NULL.  Host-only; makes no HIP call. */
int linrec_tile_info(int tile_id, int *threads_cols, int *threads_time, int *rows_per_thread,
                     int *cols_per_thread);

/* Reports the variant and tile shape the library would use for a [T, B, n] problem under the
 * current options (and the plans linrec_tune found for the current device) when every tensor
 * pointer is aligned to `alignment_bytes` (4, 8 or 16).  Launches nothing. */
int linrec_plan(int64_t T, int64_t B, int64_t n, int backward, int alignment_bytes,
                int *variant, int *tile_id);

/* The same for the other entry-point families (whose kernels exist for fewer tile shapes). */
enum {
    LINREC_ENTRY_PLAIN = 0,     /* linrec_forward / linrec_backward (what linrec_plan reports) */
    LINREC_ENTRY_GILR = 1,      /* linrec_gilr_forward / linrec_gilr_backward                  */
    LINREC_ENTRY_LSTM_CELL = 2, /* linrec_lstm_cell_forward / linrec_lstm_cell_backward        */
    LINREC_ENTRY_BF16 = 3,      /* linrec_forward_bf16 / linrec_backward_bf16                  */
    LINREC_ENTRY_GILR_BF16 = 4,      /* linrec_gilr_forward_bf16 / linrec_gilr_backward_bf16    */
    LINREC_ENTRY_LSTM_CELL_BF16 = 5  /* linrec_lstm_cell_forward_bf16 / ..._backward_bf16       */
};
int linrec_plan_for(int entry_point, int64_t T, int64_t B, int64_t n, int backward,
                    int alignment_bytes, int *variant, int *tile_id);

/* The tapered tail of that plan: eighths (0..8) of the single pass's last round of tiles that are cut
 * into shorter tiles (see LINREC_OPT_TAPER); 0 for the other variants.  Negative: LINREC_ERR_*. */
int linrec_plan_taper(int entry_point, int64_t T, int64_t B, int64_t n, int backward,
                      int alignment_bytes);

/* 1 if the library has kernels of tile shape `tile_id` for entry-point family `entry_point`
 * (LINREC_ENTRY_*), else 0: each family is built for the shapes its static plans use.  A
 * LINREC_OPT_TILE or pinned plan that names another shape falls back to the automatic choice.
 * Host-only; makes no HIP call. */
int linrec_tile_has(int tile_id, int entry_point);

/* Fixes the plan of one shape for every thread: later calls of entry-point family `entry_point`
 * (LINREC_ENTRY_*) with exactly this [T, B, n] and pass on the current device use variant
 * LINREC_VARIANT_LOOKBACK or LINREC_VARIANT_WALK with tile shape `tile_id`, `persistent` (-1, 0, 1 as
 * LINREC_OPT_PERSISTENT) and `taper` (0..8 as LINREC_OPT_TAPER) -- the table linrec_tune writes; a
 * thread's own LINREC_OPT_TILE / LINREC_OPT_VARIANT still take precedence.  A shape the family has no
 * kernel for falls back to the automatic choice.  tile_id == 0 forgets the shape's entry.  Host-only
 * apart from asking for the current device. */
int linrec_pin_plan(int entry_point, int64_t T, int64_t B, int64_t n, int backward, int variant,
                    int tile_id, int persistent, int taper);

/* Sizes the cached workspace of (current device, stream) for a later call of this family, shape and
 * pass, under the calling thread's options and the plans pinned or tuned so far and whatever the
 * alignment of its tensors, so that the call itself allocates nothing (and can be captured in a HIP
 * graph without an eager warm-up).  May allocate (blocking in hipMalloc) and enqueues a fill kernel
 * on `stream`; must not be called while `stream` is capturing (LINREC_ERR_CAPTURE). */
int linrec_reserve_workspace(int entry_point, int64_t T, int64_t B, int64_t n, int backward,
                             void *stream);

/*
 * Optional: finds the fastest plan (single-pass kernel: tile shape, persistent workgroups or not,
 * a tapered tail or not; for wide problems also the walk) for a [T, B, n] forward (backward = 0) or backward (1) pass by
 * timing the candidates on `stream`, on scratch tensors it allocates and frees, and remembers it for
 * later calls with this shape on the current device (when LINREC_OPT_TILE / LINREC_OPT_PERSISTENT /
 * LINREC_OPT_TAPER are automatic; a remembered walk only while LINREC_OPT_VARIANT is automatic too).
 * Blocking; allocates 3 (forward) or 5 (backward) tensors of T*B*n floats.  Returns LINREC_OK,
 * LINREC_ERR_SHAPE or LINREC_ERR_HIP.  The candidates are forced on the calling thread's calls only;
 * calls other threads make meanwhile keep their own plans (and disturb the timings).
 */
int linrec_tune(int64_t T, int64_t B, int64_t n, int backward, void *stream);
/* The same for one of the entry-point families LINREC_ENTRY_* (linrec_tune is LINREC_ENTRY_PLAIN);
 * allocates as many scratch tensors as the entry point has [T, B, n] arguments. */
int linrec_tune_for(int entry_point, int64_t T, int64_t B, int64_t n, int backward, void *stream);

/* Host-side argument checks only (exactly the checks linrec_forward / linrec_backward run
 * before touching the GPU); no HIP call is made, so these work on a machine without a GPU. */
int linrec_validate_forward(const float *lambda, const float *x, const float *h0,
                            const float *h_out, int64_t T, int64_t B, int64_t n);
int linrec_validate_backward(const float *lambda, const float *h, const float *h0,
                             const float *grad_h, const float *grad_x, const float *grad_lambda,
                             const float *grad_h0, int64_t T, int64_t B, int64_t n);
int linrec_validate_forward_bf16(const uint16_t *lambda, const uint16_t *x, const uint16_t *h0,
                                 const uint16_t *h_out, int64_t T, int64_t B, int64_t n);
int linrec_validate_backward_bf16(const uint16_t *lambda, const uint16_t *h, const uint16_t *h0,
                                  const uint16_t *grad_h, const uint16_t *grad_x,
                                  const uint16_t *grad_lambda, const uint16_t *grad_h0,
                                  int64_t T, int64_t B, int64_t n);
int linrec_validate_gilr_forward(const float *g_pre, const float *i_pre, const float *h0,
                                 const float *h_out, int tau, int64_t T, int64_t B, int64_t n);
int linrec_validate_gilr_backward(const float *g_pre, const float *i_pre, const float *h,
                                  const float *h0, const float *grad_h, const float *grad_g_pre,
                                  const float *grad_i_pre, const float *grad_h0, int tau,
                                  int64_t T, int64_t B, int64_t n);
int linrec_validate_lstm_cell_forward(const float *f_pre, const float *i_pre, const float *z_pre,
                                      const float *o_pre, const float *c0, const float *c_out,
                                      const float *h_out, int64_t T, int64_t B, int64_t n);
int linrec_validate_lstm_cell_backward(const float *f_pre, const float *i_pre, const float *z_pre,
                                       const float *o_pre, const float *c, const float *c0,
                                       const float *grad_h, const float *grad_f_pre,
                                       const float *grad_i_pre, const float *grad_z_pre,
                                       const float *grad_o_pre, const float *grad_c0,
                                       int64_t T, int64_t B, int64_t n);
int linrec_validate_gilr_forward_bf16(const uint16_t *g_pre, const uint16_t *i_pre, const uint16_t *h0,
                                      const uint16_t *h_out, int tau, int64_t T, int64_t B, int64_t n);
int linrec_validate_gilr_backward_bf16(const uint16_t *g_pre, const uint16_t *i_pre, const uint16_t *h,
                                       const uint16_t *h0, const uint16_t *grad_h,
                                       const uint16_t *grad_g_pre, const uint16_t *grad_i_pre,
                                       const uint16_t *grad_h0, int tau, int64_t T, int64_t B, int64_t n);
int linrec_validate_lstm_cell_forward_bf16(const uint16_t *f_pre, const uint16_t *i_pre,
                                           const uint16_t *z_pre, const uint16_t *o_pre,
                                           const uint16_t *c0, const uint16_t *c_out,
                                           const uint16_t *h_out, int64_t T, int64_t B, int64_t n);
int linrec_validate_lstm_cell_backward_bf16(const uint16_t *f_pre, const uint16_t *i_pre,
                                            const uint16_t *z_pre, const uint16_t *o_pre,
                                            const uint16_t *c, const uint16_t *c0, const uint16_t *grad_h,
                                            const uint16_t *grad_f_pre, const uint16_t *grad_i_pre,
                                            const uint16_t *grad_z_pre, const uint16_t *grad_o_pre,
                                            const uint16_t *grad_c0, int64_t T, int64_t B, int64_t n);

/*
 * Measurement aid, not part of the recurrence: a pure streaming kernel built from the same
 * 16-byte non-temporal loads and stores as the scan kernels.  Reads the n-element device arrays
 * in0, in1, in2 that are non-NULL and writes those of out0 (= in0*in1+in2, absent inputs taken
 * as 1, 1, 0) and out1 (= out0 squared) that are non-NULL.  With (in0, NULL, NULL, out0, NULL)
 * it is a plain copy of 4n bytes in and 4n bytes out, used to calibrate hardware byte
 * counters; with two inputs and one output it moves the forward pass' 12 bytes per element,
 * with three inputs and two outputs the backward pass' 20.  Without an input it only writes,
 * without an output it only reads (what it read decides a store that never happens): the two
 * rates a mix of reads and writes is bounded by.  n must be a multiple of 4 and all pointers
 * 16-byte aligned (LINREC_ERR_SHAPE otherwise); at least one array is required (LINREC_ERR_NULL).
 */
int linrec_stream_probe(const float *in0, const float *in1, const float *in2, float *out0,
                        float *out1, int64_t n, void *stream);

/*
 * The same measurement aid in the geometry of a tile: the arrays are [T, C] row-major like the
 * tensors of the recurrence, a workgroup streams 32 rows of 256 adjacent columns, one column per
 * lane, every thread 16 consecutive rows at the row stride -- the arrangement that streams
 * fastest on an MI355X (a compute unit touches 1 KiB of a row at about the same time), and so
 * the rate the scan kernels are measured against.  Arrays are given from the front (in1 needs
 * in0, in2 needs in1, out1 needs out0; LINREC_ERR_NULL otherwise, and when there is none);
 * out0 = in0*in1+in2 over the inputs present, out1 = out0 squared.  T must be a multiple of 32,
 * C of 256, pointers 4-byte aligned (LINREC_ERR_SHAPE otherwise).
 */
int linrec_stream_probe_rows(const float *in0, const float *in1, const float *in2, float *out0,
                             float *out1, int64_t T, int64_t C, void *stream);

/* Synchronises `stream` and reports whether any look-back kernel enqueued on it since the
 * last check gave up waiting (LINREC_ERR_DEVICE), LINREC_ERR_HIP if the synchronisation
 * itself failed, else LINREC_OK.  Optional: a healthy run never needs it. */
int linrec_check(void *stream);

/* Frees every cached workspace of the calling process (all devices, all streams), retired blocks
 * included.  The caller must make sure no linrec call is still running on the GPU and that no HIP
 * graph holding a recorded linrec launch is replayed afterwards. */
int linrec_release_workspace(void);

/* Never NULL.  linrec_status_string returns a static string.  linrec_last_hip_error describes the last
 * LINREC_ERR_HIP that a call made by the CALLING host thread returned (which HIP call failed, and
 * HIP's text for the error; empty if none has); the buffer belongs to that thread and is overwritten
 * by its next failure. */
const char *linrec_status_string(int status);
const char *linrec_last_hip_error(void);

/* ABI version of this header (major*100 + minor). */
int linrec_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LINREC_H */
