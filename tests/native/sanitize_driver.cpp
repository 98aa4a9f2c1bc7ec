// Host-sanitizer driver: runs the fp64 oracle's C loops and the library's argument validation (both pure
// host code) inside a program that is built with -fsanitize=address,undefined, on exactly sized heap
// buffers, so that a read one row before or after a tensor, an index overflow or a signed overflow in
// the shape checks stops it.  Reads one case file, writes one result file; tests/test_sanitizers.py
// compares the results with what the ordinary builds return for the same inputs.
//
// Case file: int64 header {T, C, tau, has_h0, n_validate}; float32 arrays a, b, z, o, e [T*C] and h0 [C];
// then n_validate records of 17 int64 {kind, 12 pointer values, tau, T, B, n}.
// Result file: doubles -- every oracle output in a fixed order -- then one int64 status per record.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "linrec.h"

extern "C" {
void linrec_oracle_forward(const float *, const float *, double *, double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t);
void linrec_oracle_backward(const float *, const float *, const float *, const float *, double *, double *, double *, double *,
                            int64_t, int64_t, int64_t, int64_t, int64_t, int64_t);
void linrec_oracle_gilr_forward(const float *, const float *, int, double *, double *, int64_t, int64_t, int64_t, int64_t, int64_t,
                                int64_t);
void linrec_oracle_gilr_backward(const float *, const float *, int, const float *, const float *, const float *, double *, double *,
                                 double *, double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t);
void linrec_oracle_lstm_forward(const float *, const float *, const float *, const float *, double *, double *, double *, int64_t,
                                int64_t, int64_t, int64_t, int64_t, int64_t);
void linrec_oracle_lstm_backward(const float *, const float *, const float *, const float *, const float *, const float *,
                                 const float *, double *, double *, double *, double *, double *, double *, int64_t, int64_t,
                                 int64_t, int64_t, int64_t, int64_t);
}

// exactly sized heap arrays: one element past either end is a sanitizer report
template <class E>
struct Buf {
    E *p;
    size_t n;
    explicit Buf(size_t n_) : p(n_ ? new E[n_] : nullptr), n(n_) {}
    ~Buf() { delete[] p; }
    Buf(const Buf &) = delete;
    Buf &operator=(const Buf &) = delete;
};

static void die(const char *what)
{
    fprintf(stderr, "sanitize_driver: %s\n", what);
    exit(3);
}
static void rd(FILE *f, void *p, size_t bytes)
{
    if (bytes && fread(p, 1, bytes, f) != bytes) die("short read");
}
static void wr(FILE *f, const void *p, size_t bytes)
{
    if (bytes && fwrite(p, 1, bytes, f) != bytes) die("short write");
}
static void to_f32(const Buf<double> &src, Buf<float> &dst)
{
    for (size_t i = 0; i < src.n; ++i) dst.p[i] = (float)src.p[i];
}
static void same(const Buf<double> &a, const Buf<double> &b, const char *what)
{
    if (a.n != b.n || (a.n && memcmp(a.p, b.p, a.n * sizeof(double)) != 0)) die(what);
}

int main(int argc, char **argv)
{
    if (argc != 3) die("usage: sanitize_driver <case file> <result file>");
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) die("cannot open files");
    int64_t hdr[5];
    rd(in, hdr, sizeof hdr);
    const int64_t T = hdr[0], C = hdr[1], nval = hdr[4];
    const int tau = (int)hdr[2];
    const bool has_h0 = hdr[3] != 0;
    const size_t E = (size_t)(T * C);
    Buf<float> a(E), b(E), z(E), o(E), e(E), h0(C);
    for (Buf<float> *t : {&a, &b, &z, &o, &e}) rd(in, t->p, E * sizeof(float));
    rd(in, h0.p, (size_t)C * sizeof(float));
    const float *h0p = has_h0 ? h0.p : nullptr;
    // slab and column splits of the same problem (ragged on purpose)
    const int64_t tm = T / 3, cm = (C + 1) / 2;
    auto init_state = [&](Buf<double> &s) {
        for (int64_t c = 0; c < C; ++c) s.p[c] = has_h0 ? (double)h0.p[c] : 0.0;
    };
    auto zero = [&](Buf<double> &s) {
        for (size_t i = 0; i < s.n; ++i) s.p[i] = 0.0;
    };

    // ---- plain recurrence -------------------------------------------------------------------------
    Buf<double> href(E), href2(E), st(C), st2(C);
    init_state(st);
    linrec_oracle_forward(a.p, b.p, st.p, href.p, T, C, 0, T, 0, C);
    init_state(st2);
    for (int part = 0; part < 2; ++part) {
        const int64_t c0 = part ? cm : 0, c1 = part ? C : cm;
        linrec_oracle_forward(a.p, b.p, st2.p, href2.p, T, C, 0, tm, c0, c1);
        linrec_oracle_forward(a.p, b.p, st2.p, href2.p, T, C, tm, T, c0, c1);
    }
    same(href, href2, "forward: slab/column split differs from one shot");
    wr(out, href.p, E * sizeof(double));
    Buf<float> h32(E);
    to_f32(href, h32);
    Buf<double> gx(E), gl(E), gh0(C), g(C), gx2(E), gl2(E), gh02(C), g2(C);
    zero(g); zero(gh0); zero(g2); zero(gh02);
    linrec_oracle_backward(a.p, h32.p, h0p, e.p, g.p, gx.p, gl.p, gh0.p, T, C, 0, T, 0, C);
    for (int part = 0; part < 2; ++part) {
        const int64_t c0 = part ? cm : 0, c1 = part ? C : cm;
        linrec_oracle_backward(a.p, h32.p, h0p, e.p, g2.p, gx2.p, gl2.p, gh02.p, T, C, tm, T, c0, c1);
        linrec_oracle_backward(a.p, h32.p, h0p, e.p, g2.p, gx2.p, gl2.p, gh02.p, T, C, 0, tm, c0, c1);
    }
    same(gx, gx2, "backward grad_x: split differs");
    same(gl, gl2, "backward grad_lambda: split differs");
    if (T > 0) same(gh0, gh02, "backward grad_h0: split differs");
    wr(out, gx.p, E * sizeof(double));
    wr(out, gl.p, E * sizeof(double));
    wr(out, gh0.p, (size_t)C * sizeof(double));

    // ---- gated layer (a = g_pre, b = i_pre) ----------------------------------------------------------
    init_state(st);
    linrec_oracle_gilr_forward(a.p, b.p, tau, st.p, href.p, T, C, 0, T, 0, C);
    init_state(st2);
    linrec_oracle_gilr_forward(a.p, b.p, tau, st2.p, href2.p, T, C, 0, tm, 0, C);
    linrec_oracle_gilr_forward(a.p, b.p, tau, st2.p, href2.p, T, C, tm, T, 0, C);
    same(href, href2, "gilr forward: slab split differs");
    wr(out, href.p, E * sizeof(double));
    to_f32(href, h32);
    zero(g); zero(gh0);
    linrec_oracle_gilr_backward(a.p, b.p, tau, h32.p, h0p, e.p, g.p, gx.p, gl.p, gh0.p, T, C, 0, T, 0, C);
    wr(out, gx.p, E * sizeof(double));
    wr(out, gl.p, E * sizeof(double));
    wr(out, gh0.p, (size_t)C * sizeof(double));

    // ---- LSTM cell (a = f_pre, b = i_pre, z, o) --------------------------------------------------------
    Buf<double> cref(E);
    init_state(st);
    linrec_oracle_lstm_forward(a.p, b.p, z.p, o.p, st.p, cref.p, href.p, T, C, 0, T, 0, C);
    wr(out, cref.p, E * sizeof(double));
    wr(out, href.p, E * sizeof(double));
    to_f32(cref, h32);
    Buf<double> gf(E), gi(E), gz(E), go(E), gc0(C);
    zero(g); zero(gc0);
    linrec_oracle_lstm_backward(a.p, b.p, z.p, o.p, h32.p, h0p, e.p, g.p, gf.p, gi.p, gz.p, go.p, gc0.p, T, C, 0, T, 0, C);
    for (Buf<double> *t : {&gf, &gi, &gz, &go}) wr(out, t->p, E * sizeof(double));
    wr(out, gc0.p, (size_t)C * sizeof(double));

    // ---- argument validation (pointer VALUES only; nothing is dereferenced) -------------------------------
    for (int64_t i = 0; i < nval; ++i) {
        int64_t r[17];
        rd(in, r, sizeof r);
        const void *p[12];
        for (int k = 0; k < 12; ++k) p[k] = (const void *)(uintptr_t)r[1 + k];
        typedef const float *F;
        typedef const uint16_t *H;
        const int vt = (int)r[13];
        const int64_t vT = r[14], vB = r[15], vn = r[16];
        int64_t rc = 0;
        switch (r[0]) {
        case 0: rc = linrec_validate_forward((F)p[0], (F)p[1], (F)p[2], (F)p[3], vT, vB, vn); break;
        case 1: rc = linrec_validate_backward((F)p[0], (F)p[1], (F)p[2], (F)p[3], (F)p[4], (F)p[5], (F)p[6], vT, vB, vn); break;
        case 2: rc = linrec_validate_forward_bf16((H)p[0], (H)p[1], (H)p[2], (H)p[3], vT, vB, vn); break;
        case 3: rc = linrec_validate_backward_bf16((H)p[0], (H)p[1], (H)p[2], (H)p[3], (H)p[4], (H)p[5], (H)p[6], vT, vB, vn); break;
        case 4: rc = linrec_validate_gilr_forward((F)p[0], (F)p[1], (F)p[2], (F)p[3], vt, vT, vB, vn); break;
        case 5:
            rc = linrec_validate_gilr_backward((F)p[0], (F)p[1], (F)p[2], (F)p[3], (F)p[4], (F)p[5], (F)p[6], (F)p[7], vt, vT, vB, vn);
            break;
        case 6: rc = linrec_validate_lstm_cell_forward((F)p[0], (F)p[1], (F)p[2], (F)p[3], (F)p[4], (F)p[5], (F)p[6], vT, vB, vn); break;
        case 7:
            rc = linrec_validate_lstm_cell_backward((F)p[0], (F)p[1], (F)p[2], (F)p[3], (F)p[4], (F)p[5], (F)p[6], (F)p[7], (F)p[8],
                                                    (F)p[9], (F)p[10], (F)p[11], vT, vB, vn);
            break;
        case 8: rc = linrec_validate_gilr_forward_bf16((H)p[0], (H)p[1], (H)p[2], (H)p[3], vt, vT, vB, vn); break;
        case 9:
            rc = linrec_validate_lstm_cell_backward_bf16((H)p[0], (H)p[1], (H)p[2], (H)p[3], (H)p[4], (H)p[5], (H)p[6], (H)p[7],
                                                         (H)p[8], (H)p[9], (H)p[10], (H)p[11], vT, vB, vn);
            break;
        default: die("unknown validation kind");
        }
        wr(out, &rc, sizeof rc);
    }
    // the status strings are static storage and never NULL
    for (int s = 1; s >= -12; --s)
        if (!linrec_status_string(s) || !linrec_status_string(s)[0]) die("empty status string");
    fclose(in);
    if (fclose(out) != 0) die("close failed");
    return 0;
}
