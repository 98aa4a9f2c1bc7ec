// Host-only argument checks of liblinrec.  No HIP call is made here, so the checks can be
// exercised (and run under host sanitizers) on a machine without a GPU.
#include "linrec.h"

#include <stddef.h>
#include <stdint.h>

namespace {

constexpr int64_t kMaxElements = (int64_t)1 << 40;

// Fills C = B*n and E = T*C; returns false when a dimension is negative or a product overflows the
// supported range.
bool shape_ok(int64_t T, int64_t B, int64_t n, int64_t *C, int64_t *E)
{
    if (T < 0 || B < 0 || n < 0) return false;
    if (B > kMaxElements || n > kMaxElements || T > kMaxElements) return false;
    if (B != 0 && n > kMaxElements / B) return false;
    const int64_t c = B * n;
    if (c != 0 && T > kMaxElements / c) return false;
    *C = c;
    *E = T * c;
    return true;
}

// Do the element ranges [p, p+np) and [q, q+nq) of arrays of es-byte elements share a byte?
bool overlaps(const void *p, int64_t np, const void *q, int64_t nq, size_t es = sizeof(float))
{
    if (!p || !q || np == 0 || nq == 0) return false;
    const uintptr_t a0 = (uintptr_t)p, a1 = a0 + (uintptr_t)np * es;
    const uintptr_t b0 = (uintptr_t)q, b1 = b0 + (uintptr_t)nq * es;
    return a0 < b1 && b0 < a1;
}

int validate_forward(const void *lambda, const void *x, const void *h0, const void *h_out, int64_t T, int64_t B,
                     int64_t n, size_t es)
{
    int64_t C, E;
    if (!shape_ok(T, B, n, &C, &E)) return LINREC_ERR_SHAPE;
    if (E == 0) return LINREC_OK;
    if (!lambda || !x || !h_out) return LINREC_ERR_NULL;
    if (overlaps(h_out, E, lambda, E, es)) return LINREC_ERR_ALIAS;
    if (h_out != x && overlaps(h_out, E, x, E, es)) return LINREC_ERR_ALIAS;
    if (overlaps(h_out, E, h0, C, es)) return LINREC_ERR_ALIAS;
    return LINREC_OK;
}

int validate_backward(const void *lambda, const void *h, const void *h0, const void *grad_h, const void *grad_x,
                      const void *grad_lambda, const void *grad_h0, int64_t T, int64_t B, int64_t n, size_t es)
{
    int64_t C, E;
    if (!shape_ok(T, B, n, &C, &E)) return LINREC_ERR_SHAPE;
    if (C == 0) return LINREC_OK;
    if (T == 0) return LINREC_OK;  // only grad_h0 (if given) is touched: zero-filled
    if (!lambda || !h || !grad_h) return LINREC_ERR_NULL;
    const void *outs[3] = {grad_x, grad_lambda, grad_h0};
    const int64_t out_len[3] = {E, E, C};
    const void *ins[4] = {lambda, h, grad_h, h0};
    const int64_t in_len[4] = {E, E, E, C};
    for (int o = 0; o < 3; ++o) {
        for (int i = 0; i < 4; ++i) {
            if (o == 0 && i == 2 && grad_x == grad_h) continue;  // exact in-place update of the gradient
            if (overlaps(outs[o], out_len[o], ins[i], in_len[i], es)) return LINREC_ERR_ALIAS;
        }
        for (int p = o + 1; p < 3; ++p)
            if (overlaps(outs[o], out_len[o], outs[p], out_len[p], es)) return LINREC_ERR_ALIAS;
    }
    return LINREC_OK;
}

}  // namespace

extern "C" int linrec_validate_forward(const float *lambda, const float *x, const float *h0, const float *h_out,
                                       int64_t T, int64_t B, int64_t n)
{
    return validate_forward(lambda, x, h0, h_out, T, B, n, sizeof(float));
}

extern "C" int linrec_validate_backward(const float *lambda, const float *h, const float *h0, const float *grad_h,
                                        const float *grad_x, const float *grad_lambda, const float *grad_h0,
                                        int64_t T, int64_t B, int64_t n)
{
    return validate_backward(lambda, h, h0, grad_h, grad_x, grad_lambda, grad_h0, T, B, n, sizeof(float));
}

extern "C" int linrec_validate_forward_bf16(const uint16_t *lambda, const uint16_t *x, const uint16_t *h0,
                                            const uint16_t *h_out, int64_t T, int64_t B, int64_t n)
{
    return validate_forward(lambda, x, h0, h_out, T, B, n, sizeof(uint16_t));
}

extern "C" int linrec_validate_backward_bf16(const uint16_t *lambda, const uint16_t *h, const uint16_t *h0,
                                             const uint16_t *grad_h, const uint16_t *grad_x,
                                             const uint16_t *grad_lambda, const uint16_t *grad_h0, int64_t T,
                                             int64_t B, int64_t n)
{
    return validate_backward(lambda, h, h0, grad_h, grad_x, grad_lambda, grad_h0, T, B, n, sizeof(uint16_t));
}

// No output of these entry points may share memory with any other tensor of the call.
static int check_disjoint(const void *const *outs, const int64_t *out_len, int n_out, const void *const *ins,
                          const int64_t *in_len, int n_in, size_t es)
{
    for (int o = 0; o < n_out; ++o) {
        for (int i = 0; i < n_in; ++i)
            if (overlaps(outs[o], out_len[o], ins[i], in_len[i], es)) return LINREC_ERR_ALIAS;
        for (int p = o + 1; p < n_out; ++p)
            if (overlaps(outs[o], out_len[o], outs[p], out_len[p], es)) return LINREC_ERR_ALIAS;
    }
    return LINREC_OK;
}

static int validate_gilr_forward(const void *g_pre, const void *i_pre, const void *h0, const void *h_out, int tau,
                                 int64_t T, int64_t B, int64_t n, size_t es)
{
    if (tau != LINREC_TAU_IDENTITY && tau != LINREC_TAU_TANH) return LINREC_ERR_OPTION;
    // same shapes, NULL rules and aliasing as the plain forward pass (h_out may be i_pre itself)
    return validate_forward(g_pre, i_pre, h0, h_out, T, B, n, es);
}

static int validate_gilr_backward(const void *g_pre, const void *i_pre, const void *h, const void *h0,
                                  const void *grad_h, const void *grad_g_pre, const void *grad_i_pre,
                                  const void *grad_h0, int tau, int64_t T, int64_t B, int64_t n, size_t es)
{
    if (tau != LINREC_TAU_IDENTITY && tau != LINREC_TAU_TANH) return LINREC_ERR_OPTION;
    int64_t C, E;
    if (!shape_ok(T, B, n, &C, &E)) return LINREC_ERR_SHAPE;
    if (C == 0 || T == 0) return LINREC_OK;
    if (!g_pre || !i_pre || !h || !grad_h) return LINREC_ERR_NULL;
    // A tile reads rows of g_pre and h that belong to its neighbours, so no output may share memory
    // with any input, nor with another output.
    const void *outs[3] = {grad_g_pre, grad_i_pre, grad_h0};
    const int64_t out_len[3] = {E, E, C};
    const void *ins[5] = {g_pre, i_pre, h, grad_h, h0};
    const int64_t in_len[5] = {E, E, E, E, C};
    return check_disjoint(outs, out_len, 3, ins, in_len, 5, es);
}

static int validate_lstm_cell_forward(const void *f_pre, const void *i_pre, const void *z_pre, const void *o_pre,
                                      const void *c0, const void *c_out, const void *h_out, int64_t T, int64_t B,
                                      int64_t n, size_t es)
{
    int64_t C, E;
    if (!shape_ok(T, B, n, &C, &E)) return LINREC_ERR_SHAPE;
    if (E == 0) return LINREC_OK;
    if (!f_pre || !i_pre || !z_pre || (h_out && !o_pre) || (!c_out && !h_out)) return LINREC_ERR_NULL;
    const void *outs[2] = {c_out, h_out};
    const int64_t out_len[2] = {E, E};
    const void *ins[5] = {f_pre, i_pre, z_pre, o_pre, c0};
    const int64_t in_len[5] = {E, E, E, E, C};
    return check_disjoint(outs, out_len, 2, ins, in_len, 5, es);
}

static int validate_lstm_cell_backward(const void *f_pre, const void *i_pre, const void *z_pre, const void *o_pre,
                                       const void *c, const void *c0, const void *grad_h, const void *grad_f_pre,
                                       const void *grad_i_pre, const void *grad_z_pre, const void *grad_o_pre,
                                       const void *grad_c0, int64_t T, int64_t B, int64_t n, size_t es)
{
    int64_t C, E;
    if (!shape_ok(T, B, n, &C, &E)) return LINREC_ERR_SHAPE;
    if (C == 0 || T == 0) return LINREC_OK;
    if (!f_pre || !i_pre || !z_pre || !o_pre || !c || !grad_h) return LINREC_ERR_NULL;
    const void *outs[5] = {grad_f_pre, grad_i_pre, grad_z_pre, grad_o_pre, grad_c0};
    const int64_t out_len[5] = {E, E, E, E, C};
    const void *ins[7] = {f_pre, i_pre, z_pre, o_pre, c, grad_h, c0};
    const int64_t in_len[7] = {E, E, E, E, E, E, C};
    return check_disjoint(outs, out_len, 5, ins, in_len, 7, es);
}

extern "C" int linrec_validate_gilr_forward(const float *g_pre, const float *i_pre, const float *h0,
                                            const float *h_out, int tau, int64_t T, int64_t B, int64_t n)
{
    return validate_gilr_forward(g_pre, i_pre, h0, h_out, tau, T, B, n, sizeof(float));
}

extern "C" int linrec_validate_gilr_backward(const float *g_pre, const float *i_pre, const float *h, const float *h0,
                                             const float *grad_h, const float *grad_g_pre, const float *grad_i_pre,
                                             const float *grad_h0, int tau, int64_t T, int64_t B, int64_t n)
{
    return validate_gilr_backward(g_pre, i_pre, h, h0, grad_h, grad_g_pre, grad_i_pre, grad_h0, tau, T, B, n, sizeof(float));
}

extern "C" int linrec_validate_lstm_cell_forward(const float *f_pre, const float *i_pre, const float *z_pre,
                                                 const float *o_pre, const float *c0, const float *c_out,
                                                 const float *h_out, int64_t T, int64_t B, int64_t n)
{
    return validate_lstm_cell_forward(f_pre, i_pre, z_pre, o_pre, c0, c_out, h_out, T, B, n, sizeof(float));
}

extern "C" int linrec_validate_lstm_cell_backward(const float *f_pre, const float *i_pre, const float *z_pre,
                                                  const float *o_pre, const float *c, const float *c0,
                                                  const float *grad_h, const float *grad_f_pre,
                                                  const float *grad_i_pre, const float *grad_z_pre,
                                                  const float *grad_o_pre, const float *grad_c0, int64_t T, int64_t B,
                                                  int64_t n)
{
    return validate_lstm_cell_backward(f_pre, i_pre, z_pre, o_pre, c, c0, grad_h, grad_f_pre, grad_i_pre, grad_z_pre,
                                       grad_o_pre, grad_c0, T, B, n, sizeof(float));
}

extern "C" int linrec_validate_gilr_forward_bf16(const uint16_t *g_pre, const uint16_t *i_pre, const uint16_t *h0,
                                                 const uint16_t *h_out, int tau, int64_t T, int64_t B, int64_t n)
{
    return validate_gilr_forward(g_pre, i_pre, h0, h_out, tau, T, B, n, sizeof(uint16_t));
}

extern "C" int linrec_validate_gilr_backward_bf16(const uint16_t *g_pre, const uint16_t *i_pre, const uint16_t *h,
                                                  const uint16_t *h0, const uint16_t *grad_h,
                                                  const uint16_t *grad_g_pre, const uint16_t *grad_i_pre,
                                                  const uint16_t *grad_h0, int tau, int64_t T, int64_t B, int64_t n)
{
    return validate_gilr_backward(g_pre, i_pre, h, h0, grad_h, grad_g_pre, grad_i_pre, grad_h0, tau, T, B, n,
                                  sizeof(uint16_t));
}

extern "C" int linrec_validate_lstm_cell_forward_bf16(const uint16_t *f_pre, const uint16_t *i_pre,
                                                      const uint16_t *z_pre, const uint16_t *o_pre, const uint16_t *c0,
                                                      const uint16_t *c_out, const uint16_t *h_out, int64_t T,
                                                      int64_t B, int64_t n)
{
    return validate_lstm_cell_forward(f_pre, i_pre, z_pre, o_pre, c0, c_out, h_out, T, B, n, sizeof(uint16_t));
}

extern "C" int linrec_validate_lstm_cell_backward_bf16(const uint16_t *f_pre, const uint16_t *i_pre,
                                                       const uint16_t *z_pre, const uint16_t *o_pre, const uint16_t *c,
                                                       const uint16_t *c0, const uint16_t *grad_h,
                                                       const uint16_t *grad_f_pre, const uint16_t *grad_i_pre,
                                                       const uint16_t *grad_z_pre, const uint16_t *grad_o_pre,
                                                       const uint16_t *grad_c0, int64_t T, int64_t B, int64_t n)
{
    return validate_lstm_cell_backward(f_pre, i_pre, z_pre, o_pre, c, c0, grad_h, grad_f_pre, grad_i_pre, grad_z_pre,
                                       grad_o_pre, grad_c0, T, B, n, sizeof(uint16_t));
}

extern "C" const char *linrec_status_string(int status)
{
    switch (status) {
    case LINREC_OK: return "ok";
    case LINREC_ERR_NULL: return "a required pointer is NULL";
    case LINREC_ERR_SHAPE: return "negative dimension or T*B*n out of range";
    case LINREC_ERR_ALIAS: return "an output overlaps another tensor";
    case LINREC_ERR_HIP: return "HIP allocation or launch failed";
    case LINREC_ERR_OPTION: return "unknown option or value out of range";
    case LINREC_ERR_DEVICE: return "a look-back wait exceeded its spin limit";
    case LINREC_ERR_CAPTURE: return "the workspace would have to grow while the stream is capturing";
    case LINREC_ERR_SCRATCH: return "problem too large for the fixed scratch of linrec_forward_noalloc";
    default: return "unknown status";
    }
}

extern "C" int linrec_version(void) { return 105; }
