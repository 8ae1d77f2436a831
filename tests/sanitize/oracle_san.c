/*
 * Sanitizer run of the fp64 oracle (test infrastructure): this file pulls in oracle/cawn_oracle.c as it stands,
 * is built with -fsanitize=address,undefined -fno-sanitize-recover=all, and calls every entry point of the oracle
 * on small ragged cases covering each mode.  Inputs and results go to the file named by argv[1]; the CPU test
 * that built this program feeds the same inputs to the ordinary build of the oracle and compares.  An
 * out-of-bounds access, a use of uninitialised heap through an index slip, a signed overflow or a misaligned
 * access ends the run with a non-zero status.
 */
#include "../../oracle/cawn_oracle.c"

#include <stdio.h>

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static double unit(void) /* uniform in [-0.5, 0.5), 24 bits */
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(g_state >> 40) / 16777216.0 - 0.5;
}
static float *rand_f32(size_t n, double scale, double shift)
{
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = (float)(scale * unit() + shift);
    return p;
}
static double *rand_f64(size_t n, double scale)
{
    double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = scale * unit();
    return p;
}
static FILE *g_out;
static void put(const char *name, const char *ty, const void *p, size_t n, size_t esz)
{
    fprintf(g_out, "arr %s %s %zu\n", name, ty, n);
    if (n) fwrite(p, esz, n, g_out);
    fputc('\n', g_out);
}
#define PUT32(name, p, n) put(name, "f4", p, n, 4)
#define PUT64(name, p, n) put(name, "f8", p, n, 8)

typedef struct { int B, L, H, F, Kc, amp, gate_mode, ret_mode, dz64; float tau; } case_t;

static int run_case(const case_t *k)
{
    const size_t B = k->B, L = k->L, H = k->H, F = k->F, J = H * F, Kc = k->Kc, n = B * L * J;
    const size_t nt = Kc > 1 ? B * (Kc - 1) * 2 * J : 0, nv = B * L * H;
    oracle_cfg c;
    memset(&c, 0, sizeof c);
    c.B = k->B; c.L = k->L; c.H = k->H; c.F = k->F; c.conv_k = k->Kc; c.amp_mode = k->amp;
    c.nthreads = 2; c.gate_mode = k->gate_mode; c.gate_tau = k->tau; c.valve_eps = 0.3f; c.ret_mode = k->ret_mode;
    c.dz_f64 = k->dz64; c.conv_clamp = 50.0; c.out_clamp = 2.0; c.grad_clamp = 3.0;
    fprintf(g_out, "case %d %d %d %d %d %d %d %d %d %.9g\n", k->B, k->L, k->H, k->F, k->Kc, k->amp, k->gate_mode,
            k->ret_mode, k->dz64, (double)k->tau);
    float *mag = rand_f32(n, 4.0, 0.0), *ang = rand_f32(n, 6.0, 0.0);
    float *gamma = rand_f32(J, 0.1, 0.94), *theta = rand_f32(J, 3.0, 1.5);
    float *cw = rand_f32(2 * J * (Kc ? Kc : 1), 2.0, 0.0), *cb = rand_f32(2 * J, 0.4, 0.0);
    float *valve = rand_f32(B * L * H, 6.0, 3.0), *ret = rand_f32(B * L * H, 4.0, 0.0), *rbias = rand_f32(F, 3.0, 1.5);
    double *scan_in = rand_f64(B * 2 * J, 2.0);
    float *tail_in = rand_f32(nt, 2.0, 0.0);
    float *dz32[2] = {rand_f32(n, 2.0, 0.0), rand_f32(n, 2.0, 0.0)};
    double *dz64[2] = {rand_f64(n, 2.0), rand_f64(n, 2.0)};
    double *dscan = rand_f64(B * 2 * J, 2.0), *dtail = rand_f64(nt, 2.0);
    PUT32("mag", mag, n); PUT32("ang", ang, n); PUT32("gamma", gamma, J); PUT32("theta", theta, J);
    PUT32("conv_w", cw, 2 * J * (Kc ? Kc : 1)); PUT32("conv_b", cb, 2 * J); PUT32("valve", valve, B * L * H);
    PUT32("ret", ret, B * L * H); PUT32("ret_bias", rbias, F); PUT64("scan_in", scan_in, B * 2 * J);
    PUT32("tail_in", tail_in, nt); PUT64("dscan_out", dscan, B * 2 * J); PUT64("dtail_out", dtail, nt);
    if (k->dz64) { PUT64("dz_re", dz64[0], n); PUT64("dz_im", dz64[1], n); }
    else { PUT32("dz_re", dz32[0], n); PUT32("dz_im", dz32[1], n); }
    /* exactly sized outputs: one element too many written anywhere is a heap overflow */
    double *z_re = (double *)malloc(8 * (n ? n : 1)), *z_im = (double *)malloc(8 * (n ? n : 1));
    double *scan_out = (double *)malloc(8 * B * 2 * J);
    float *tail_out = (float *)malloc(4 * (nt ? nt : 1));
    uint8_t *gate = (uint8_t *)malloc(n ? n : 1);
    int rc = oracle_phase_fwd(&c, mag, ang, k->gate_mode ? valve : NULL, k->ret_mode ? ret : NULL,
                              k->ret_mode ? rbias : NULL, k->ret_mode ? NULL : gamma, theta, Kc ? cw : NULL,
                              Kc ? cb : NULL, scan_in, Kc > 1 ? tail_in : NULL, z_re, z_im, scan_out,
                              Kc > 1 ? tail_out : NULL, gate);
    if (rc) return 10 + rc;
    PUT64("z_re", z_re, n); PUT64("z_im", z_im, n); PUT64("scan_out", scan_out, B * 2 * J);
    PUT32("tail_out", tail_out, nt); put("gate", "u1", gate, n, 1);
    double *dmag = (double *)calloc(n ? n : 1, 8), *dang = (double *)calloc(n ? n : 1, 8);
    double *dgamma = (double *)calloc(J, 8), *dtheta = (double *)calloc(J, 8);
    double *dcw = (double *)calloc(2 * J * (Kc ? Kc : 1), 8), *dcb = (double *)calloc(2 * J, 8);
    double *dscan_in = (double *)calloc(B * 2 * J, 8), *dtail_in = (double *)calloc(nt ? nt : 1, 8);
    double *dvalve = (double *)calloc(nv ? nv : 1, 8), *vterm = (double *)calloc(n ? n : 1, 8);
    double *dret = (double *)calloc(nv ? nv : 1, 8), *rterm = (double *)calloc(n ? n : 1, 8);
    rc = oracle_phase_bwd(&c, mag, ang, k->gate_mode ? valve : NULL, k->ret_mode ? ret : NULL,
                          k->ret_mode ? rbias : NULL, k->ret_mode ? NULL : gamma, theta, Kc ? cw : NULL, Kc ? cb : NULL,
                          scan_in, Kc > 1 ? tail_in : NULL, k->dz64 ? (const void *)dz64[0] : (const void *)dz32[0],
                          k->dz64 ? (const void *)dz64[1] : (const void *)dz32[1], dscan, Kc > 1 ? dtail : NULL, dmag,
                          dang, k->ret_mode ? NULL : dgamma, dtheta, Kc ? dcw : NULL, Kc ? dcb : NULL, dscan_in,
                          Kc > 1 ? dtail_in : NULL, k->gate_mode ? dvalve : NULL, k->gate_mode ? vterm : NULL,
                          k->ret_mode ? dret : NULL, k->ret_mode ? rterm : NULL);
    if (rc) return 20 + rc;
    PUT64("dmag", dmag, n); PUT64("dang", dang, n); PUT64("dgamma", dgamma, J); PUT64("dtheta", dtheta, J);
    PUT64("dconv_w", dcw, 2 * J * (Kc ? Kc : 1)); PUT64("dconv_b", dcb, 2 * J); PUT64("dscan_in", dscan_in, B * 2 * J);
    PUT64("dtail_in", dtail_in, nt); PUT64("dvalve", dvalve, B * L * H); PUT64("dret", dret, B * L * H);
    fprintf(g_out, "end\n");
    free(mag); free(ang); free(gamma); free(theta); free(cw); free(cb); free(valve); free(ret); free(rbias);
    free(scan_in); free(tail_in); free(dz32[0]); free(dz32[1]); free(dz64[0]); free(dz64[1]); free(dscan); free(dtail);
    free(z_re); free(z_im); free(scan_out); free(tail_out); free(gate); free(dmag); free(dang); free(dgamma);
    free(dtheta); free(dcw); free(dcb); free(dscan_in); free(dtail_in); free(dvalve); free(vterm); free(dret); free(rterm);
    return 0;
}

static int run_convs(void)
{
    /* stand-alone Temporal Syntax Cache with history, and the harmonic convolution with its adjoint */
    const int B = 2, L = 5, Cc = 7, Kc = 4, H = 3, F = 5, Kh = 5;
    float *x = rand_f32((size_t)B * L * Cc, 4.0, 0.0), *w = rand_f32((size_t)Cc * Kc, 2.0, 0.0), *b = rand_f32(Cc, 1.0, 0.0);
    float *hin = rand_f32((size_t)B * (Kc - 1) * Cc, 2.0, 0.0);
    double *y = (double *)malloc(8 * (size_t)B * L * Cc);
    float *hout = (float *)malloc(4 * (size_t)B * (Kc - 1) * Cc);
    fprintf(g_out, "conv %d %d %d %d\n", B, L, Cc, Kc);
    PUT32("x", x, (size_t)B * L * Cc); PUT32("w", w, (size_t)Cc * Kc); PUT32("b", b, Cc); PUT32("hin", hin, (size_t)B * (Kc - 1) * Cc);
    int rc = oracle_syntax_conv(B, L, Cc, Kc, 50.0, x, w, b, hin, y, hout);
    if (rc) return 30 + rc;
    PUT64("y", y, (size_t)B * L * Cc); PUT32("hout", hout, (size_t)B * (Kc - 1) * Cc);
    fprintf(g_out, "end\n");
    const size_t n = (size_t)B * L * H * F;
    double *zr = rand_f64(n, 2.0), *zi = rand_f64(n, 2.0), *ur = rand_f64(n, 2.0), *ui = rand_f64(n, 2.0);
    float *hw = rand_f32((size_t)2 * H * Kh, 2.0, 0.0), *hb = rand_f32((size_t)2 * H, 1.0, 0.0);
    double *orr = (double *)malloc(8 * n), *oi = (double *)malloc(8 * n), *dzr = (double *)malloc(8 * n), *dzi = (double *)malloc(8 * n);
    double *dw = (double *)malloc(8 * (size_t)2 * H * Kh), *db = (double *)malloc(8 * (size_t)2 * H);
    fprintf(g_out, "hconv %d %d %d %d %d\n", B, L, H, F, Kh);
    PUT64("z_re", zr, n); PUT64("z_im", zi, n); PUT64("up_re", ur, n); PUT64("up_im", ui, n);
    PUT32("w", hw, (size_t)2 * H * Kh); PUT32("b", hb, (size_t)2 * H);
    rc = oracle_harmonic_conv(B, L, H, F, Kh, zr, zi, hw, hb, orr, oi);
    if (rc) return 40 + rc;
    rc = oracle_harmonic_conv_bwd(B, L, H, F, Kh, zr, zi, hw, ur, ui, dzr, dzi, dw, db);
    if (rc) return 50 + rc;
    PUT64("o_re", orr, n); PUT64("o_im", oi, n); PUT64("dz_re", dzr, n); PUT64("dz_im", dzi, n);
    PUT64("dw", dw, (size_t)2 * H * Kh); PUT64("dbias", db, (size_t)2 * H);
    fprintf(g_out, "end\n");
    free(x); free(w); free(b); free(hin); free(y); free(hout); free(zr); free(zi); free(ur); free(ui); free(hw);
    free(hb); free(orr); free(oi); free(dzr); free(dzi); free(dw); free(db);
    return 0;
}

int main(int argc, char **argv)
{
    if (argc < 2) return 2;
    g_out = fopen(argv[1], "wb");
    if (!g_out) return 3;
    static const case_t cases[] = {
        /* B  L  H  F Kc amp gm rm dz64 tau */
        {2, 19, 2, 3, 0, 0, 0, 0, 0, 0.0f},  {2, 19, 2, 3, 4, 0, 0, 0, 0, 0.3f},  {1, 1, 1, 1, 4, 1, 0, 0, 0, 0.8f},
        {2, 7, 2, 3, 1, 1, 0, 0, 0, 0.0f},   {2, 13, 2, 3, 3, 1, 1, 1, 0, 0.0f},  {1, 2, 3, 2, 2, 0, 1, 0, 1, 0.0f},
        {3, 11, 1, 5, 0, 0, 0, 1, 1, 0.5f},  {2, 3, 2, 2, 4, 0, 0, 0, 0, 0.1f},   {1, 0, 2, 2, 3, 0, 0, 0, 0, 0.1f},
    };
    for (size_t i = 0; i < sizeof cases / sizeof cases[0]; ++i) {
        int rc = run_case(&cases[i]);
        if (rc) { fprintf(stderr, "case %zu failed: %d\n", i, rc); return rc; }
    }
    int rc = run_convs();
    if (rc) { fprintf(stderr, "convs failed: %d\n", rc); return rc; }
    fclose(g_out);
    puts("oracle sanitizer run: done");
    return 0;
}
