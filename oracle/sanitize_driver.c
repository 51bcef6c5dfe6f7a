/*
 * Sanitizer leg of the CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * Compiled together with aet_oracle.c under -fsanitize=address,undefined (see
 * tests/test_oracle_sanitizers.py) and run as a program of its own: it drives every entry
 * point of the oracle on small synthetic inputs -- server form with stragglers, compute
 * factors, the delay checkpoint and the kink analysis on a conv / pool / dense model,
 * the peer-to-peer form on a ring, Setup's coin flips, an empty round -- so that any
 * out-of-bounds access, use after free, leak or undefined operation in the oracle ends the
 * run with a non-zero status.  It checks nothing about the values (the pins do that).
 */
#include "aet_oracle.c"

static uint64_t lcg = 88172645463325252ULL;
static float rnd(void) {
    lcg = lcg * 6364136223846793005ULL + 1442695040888963407ULL;
    return (float)((lcg >> 40) & 0xFFFF) / 65536.0f - 0.5f;
}

static int drive(const orc_model *m, int n, int per, int rounds, int64_t a, int64_t b, int p2p, int setup,
                 int d_max, double kink_eps) {
    const int64_t P = orc_n_params(m);
    if (P < 0) return 1;
    const int64_t D = (int64_t)m->in_c * m->in_h * m->in_w;
    const int classes = m->layers[m->n_layers - 1].cout;
    float **X = (float **)malloc(sizeof(float *) * n);
    int32_t **y = (int32_t **)malloc(sizeof(int32_t *) * n);
    int64_t *N = (int64_t *)malloc(sizeof(int64_t) * n);
    for (int c = 0; c < n; ++c) {
        N[c] = per + c;
        X[c] = (float *)malloc(sizeof(float) * N[c] * D);
        y[c] = (int32_t *)malloc(sizeof(int32_t) * N[c]);
        for (int64_t i = 0; i < N[c] * D; ++i) X[c][i] = rnd();
        for (int64_t i = 0; i < N[c]; ++i) y[c][i] = (int32_t)(((unsigned)(rnd() * 1000.f + 500.f)) % classes);
    }
    float *w0 = (float *)malloc(sizeof(float) * P);
    for (int64_t p = 0; p < P; ++p) w0[p] = 0.3f * rnd();
    orc_ctx *C = orc_create(m, n, (const float *const *)X, (const int32_t *const *)y, N, w0, 12345);
    if (!C) return 2;
    int rc = 0;
    int32_t *off = (int32_t *)malloc(sizeof(int32_t) * (n + 1));
    int32_t *nbr = (int32_t *)malloc(sizeof(int32_t) * 2 * n);
    uint32_t *wts = (uint32_t *)malloc(sizeof(uint32_t) * n);
    if (p2p) {   /* ring */
        int e = 0;
        for (int c = 0; c < n; ++c) {
            off[c] = e;
            int l = (c + n - 1) % n, r = (c + 1) % n;
            if (l > r) { int t = l; l = r; r = t; }
            nbr[e++] = l;
            if (r != l) nbr[e++] = r;
        }
        off[n] = e;
        rc |= orc_set_topology(C, off, nbr);
    }
    if (setup) {
        for (int c = 0; c < n; ++c) wts[c] = (uint32_t)(c + 1);
        rc |= orc_set_setup(C, wts, 77);
    }
    orc_set_kink_eps(C, kink_eps);
    int32_t *cf = (int32_t *)malloc(sizeof(int32_t) * n);
    uint8_t *st = (uint8_t *)malloc(n);
    for (int c = 0; c < n; ++c) { cf[c] = 1 + c % 3; st[c] = (uint8_t)(c % 2); }
    int32_t *fc = (int32_t *)malloc(sizeof(int32_t) * n), *fr = (int32_t *)malloc(sizeof(int32_t) * n);
    int32_t *ac = (int32_t *)malloc(sizeof(int32_t) * n * 8), *ar = (int32_t *)malloc(sizeof(int32_t) * n * 8);
    real *buf = (real *)malloc(sizeof(real) * P);
    double *allow = (double *)malloc(sizeof(double) * (orc_n_tensors(C) + 1));
    int ticks = 0;
    while (!orc_all_done(C, rounds) && ticks < 1000) {
        int32_t nf = 0, na = 0;
        rc |= orc_run_round(C, a, b, rounds, 0.05, 0.01, 0.5, cf, st, 1, 3, 999, d_max, &nf, fc, fr);
        for (int j = 0; j < nf; ++j) {
            int64_t ints[6], ev = 0; double dbl[2];
            rc |= orc_get_U(C, fc[j], fr[j], buf);
            rc |= orc_get_round_info(C, fc[j], fr[j], ints, dbl);
            if (kink_eps > 0) rc |= orc_get_round_kinks(C, fc[j], fr[j], &ev, allow);
        }
        rc |= p2p ? orc_receive(C, 0.5, &na, ac, ar) : orc_server_aggregate(C, 1.0 / n, &na, ac, ar);
        rc |= orc_get_weights(C, -1, buf);
        rc |= orc_set_weights(C, 0, buf);
        ++ticks;
    }
    if (!orc_all_done(C, rounds)) rc |= 4;
    {
        const int64_t ne = orc_event_count(C);
        int64_t *et = (int64_t *)malloc(sizeof(int64_t) * (ne + 1));
        int32_t *ec = (int32_t *)malloc(sizeof(int32_t) * (ne + 1)), *ek = (int32_t *)malloc(sizeof(int32_t) * (ne + 1));
        orc_get_events(C, et, ec, ek);
        free(et); free(ec); free(ek);
    }
    /* the stand-alone entry points */
    {
        real *w = (real *)malloc(sizeof(real) * P), *g = (real *)malloc(sizeof(real) * P);
        for (int64_t p = 0; p < P; ++p) w[p] = (real)w0[p];
        if (orc_batch_loss_grad(m, w, X[0], y[0], m->batch, g) < 0) rc |= 8;
        int32_t el[4]; int64_t eu[4];
        real *ej = (real *)malloc(sizeof(real) * 4 * P);
        if (orc_sample_kinks(m, w, X[0], y[0][0], 0.2, 4, el, eu, ej, allow) < 0) rc |= 16;
        free(w); free(g); free(ej);
    }
    orc_destroy(C);
    for (int c = 0; c < n; ++c) { free(X[c]); free(y[c]); }
    free(X); free(y); free(N); free(w0); free(off); free(nbr); free(wts); free(cf); free(st);
    free(fc); free(fr); free(ac); free(ar); free(buf); free(allow);
    return rc;
}

int main(void) {
    orc_model conv = {1, 12, 12, 5, 3, {{ORC_CONV, 3, 5, 0, 1}, {ORC_POOL, 0, 0, 0, 0}, {ORC_CONV, 4, 3, 1, 1},
                                         {ORC_DENSE, 6, 0, 0, 1}, {ORC_DENSE, 3, 0, 0, 0}}};
    orc_model mlp = {1, 1, 9, 2, 2, {{ORC_DENSE, 5, 0, 0, 1}, {ORC_DENSE, 4, 0, 0, 0}}};
    orc_model soft = {1, 1, 7, 1, 1, {{ORC_DENSE, 3, 0, 0, 0}}};
    int rc = 0;
    rc |= drive(&conv, 4, 9, 3, 3, 3, 0, 0, -1, 0.05);    /* server form, kink analysis on */
    rc |= drive(&conv, 3, 9, 3, 3, 3, 1, 0, 1, 0.0);      /* ring, delay checkpoint */
    rc |= drive(&mlp, 5, 7, 4, 2, 0, 0, 0, 2, 0.1);       /* empty first round, checkpoint */
    rc |= drive(&mlp, 4, 7, 3, 4, 8, 1, 1, -1, 0.0);      /* Setup's coin flips on a ring */
    rc |= drive(&soft, 3, 5, 4, 1, 1, 0, 0, -1, 0.3);     /* no decisions to book */
    printf("sanitizer drive: status %d\n", rc);
    return rc;
}
