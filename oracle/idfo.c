/*
 * CPU oracle for the incremental depth-first CNN update.  TEST INFRASTRUCTURE
 * ONLY: see idfo.h.  Plain C, no blocking, no vectorisation tricks; the
 * arithmetic is in idfo_body.inc, compiled here once for double and once for
 * int64_t.
 */
#include "idfo.h"
#include <math.h>
#include <stdlib.h>
#include <string.h>

int idfo_out_size(int n_in, int k, int s, int p)
{
    int t = n_in + 2 * p - k;
    return t < 0 ? 0 : t / s + 1;
}

/* bf16 keeps the top 16 bits of an IEEE binary32: 8 exponent bits, 7 explicit
 * mantissa bits.  Round to nearest, ties to even, computed from the value
 * itself (no detour through float, which would round twice). */
double idfo_round_bf16(double v)
{
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e;
    double m = frexp(fabs(v), &e);                /* |v| = m * 2^e, 0.5 <= m < 1 */
    /* bf16 normal numbers have 8 significant bits; the smallest normal exponent
     * of binary32 is 2^-126, below which the spacing stays 2^-133. */
    int lsb_exp = e - 8;
    if (lsb_exp < -133) lsb_exp = -133;
    double q = ldexp(fabs(v), -lsb_exp);          /* in units of the last place */
    double r = nearbyint(q);                      /* default mode: ties to even */
    double out = ldexp(r, lsb_exp);
    (void)m;
    if (out > 3.3895313892515355e38) out = INFINITY;      /* above the largest bf16 */
    return v < 0 ? -out : out;
}

static int check_layers(const idfo_layer *layers, int n_layers, int H, int W, int C0)
{
    if (n_layers <= 0 || W <= 0 || C0 <= 0 || H < 0) return -1;
    int h = H, w = W, c = C0;
    for (int n = 0; n < n_layers; ++n) {
        const idfo_layer *L = &layers[n];
        if (L->c_in != c || L->c_out <= 0) return -1;
        if (L->k_h <= 0 || L->k_w <= 0 || L->s_h <= 0 || L->s_w <= 0 || L->p_h < 0 || L->p_w < 0) return -1;
        if (L->kind == IDFO_MAXPOOL) {
            if (L->c_out != L->c_in || L->k_h != 2 || L->s_h != 2 || L->p_h != 0 || L->p_w != 0) return -1;
            if (!((L->k_w == 2 && L->s_w == 2) || (L->k_w == 1 && L->s_w == 1))) return -1;
        } else if (L->kind != IDFO_CONV) return -1;
        if (H == 0 && L->p_h != 0) return -1;
        if (H) { h = idfo_out_size(h, L->k_h, L->s_h, L->p_h); if (h <= 0) return -1; }
        w = idfo_out_size(w, L->k_w, L->s_w, L->p_w);
        if (w <= 0) return -1;
        c = L->c_out;
    }
    return 0;
}

#define CAT2(a, b) a##b
#define CAT(a, b) CAT2(a, b)

#define T double
#define FN(name) CAT(name, _f64)
#define STREAM idfo_stream_f64
#define IS_INT 0
#include "idfo_body.inc"
#undef T
#undef FN
#undef STREAM
#undef IS_INT

#define T int64_t
#define FN(name) CAT(name, _i64)
#define STREAM idfo_stream_i64
#define IS_INT 1
#include "idfo_body.inc"
