/* Drives every function of oracle/vs_oracle.c on small inputs whose buffers are heap blocks of exactly
 * the documented sizes, for a build with AddressSanitizer and UndefinedBehaviorSanitizer (host only):
 * an access past any of them, or undefined arithmetic, ends the program with a report.  Values are
 * checked elsewhere (tests/pins.py); here only return codes and finiteness are. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int vs_oracle_attention(const double *, int64_t, int32_t, int32_t, int32_t, const double *, const double *, int64_t,
                        const int64_t *, double, double *, double *);
int vs_oracle_frame_prefill(const double *, const double *, const double *, int64_t, const double *, const double *,
                            int64_t, int32_t, int32_t, int32_t, double, double *, double *);
int vs_oracle_compact_append(double *, double *, int64_t, int64_t *, const double *, const double *, int64_t, int64_t,
                             int32_t, int32_t, int64_t *);
int vs_oracle_decode(const double *, double *, double *, int64_t, int64_t *, const double *, const double *, int32_t,
                     int32_t, int32_t, double, double *);
int vs_oracle_mean_pool(const double *, int64_t, int64_t, double *);
int vs_oracle_bank_victim(const double *, int64_t, int64_t, const double *, int32_t, double *, int64_t *);
int vs_oracle_bank_apply(double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, const double *, int64_t *);
int vs_oracle_frames_prefill(const double *, const double *, const double *, int64_t, const double *, const double *,
                             int64_t, int64_t, int32_t, int32_t, int32_t, double, double *);
int vs_oracle_query_prefill(const double *, double *, double *, int64_t, int64_t *, const double *, const double *,
                            int64_t, int32_t, int32_t, int32_t, double, double *);
int vs_oracle_frame_qkv(const double *, int64_t, int64_t, const double *, int64_t, double *);
int vs_oracle_rmsnorm(const double *, int64_t, int64_t, const double *, double, double *);
int vs_oracle_linear(const double *, int64_t, int64_t, const double *, int64_t, double *);
int vs_oracle_gated_unit(const double *, const double *, int64_t, int64_t, double *);
int vs_oracle_decoder_layer(const double *, int64_t, int64_t, int32_t, int32_t, int32_t, int64_t, const double *,
                            const double *, const double *, const double *, const double *, const double *,
                            const double *, const double *, const double *, double, const double *, const double *,
                            int64_t, double, double *, double *, double *);

static unsigned long long state = 88172645463325252ULL;
static double rnd(void) {  /* xorshift, in [-1, 1) */
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 4503599627370496.0 - 1.0;
}
static double *block(int64_t n) {
    double *p = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    if (!p) { fprintf(stderr, "out of memory\n"); exit(3); }
    for (int64_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
static void finite(const double *p, int64_t n, const char *what) {
    for (int64_t i = 0; i < n; ++i)
        if (!isfinite(p[i])) { fprintf(stderr, "%s: element %lld is not finite\n", what, (long long)i); exit(2); }
}
#define OK(call) do { int rc_ = (call); if (rc_ != 0) { fprintf(stderr, "%s -> %d\n", #call, rc_); exit(2); } } while (0)
#define FAILS(call) do { if ((call) == 0) { fprintf(stderr, "%s was accepted\n", #call); exit(2); } } while (0)

int main(void) {
    const int32_t Hq = 6, Hkv = 2, D = 5;
    const int64_t L = 7, T = 4, cap = L + T, d = 9, F = 11, N = 3;
    const double scale = 0.4;
    double *Q = block(T * Hq * D), *Kc = block(cap * Hkv * D), *Vc = block(cap * Hkv * D);
    double *Kf = block(T * Hkv * D), *Vf = block(T * Hkv * D), *O = block(T * Hq * D);

    {   /* attention with ragged visible prefixes, probabilities returned */
        int64_t vis[4] = {1, 7, 3, 7};
        double *P = block(Hq * T * L);
        OK(vs_oracle_attention(Q, T, Hq, Hkv, D, Kc, Vc, L, vis, scale, O, P));
        finite(O, T * Hq * D, "attention"); finite(P, Hq * T * L, "probabilities");
        vis[2] = 8;
        FAILS(vs_oracle_attention(Q, T, Hq, Hkv, D, Kc, Vc, L, vis, scale, O, P));
        free(P);
    }
    {   /* frame prefill over L rows and over none */
        double *P = block(Hq * T * (L + T));
        OK(vs_oracle_frame_prefill(Q, Kc, Vc, L, Kf, Vf, T, Hq, Hkv, D, scale, O, P));
        finite(O, T * Hq * D, "frame prefill");
        OK(vs_oracle_frame_prefill(Q, NULL, NULL, 0, Kf, Vf, T, Hq, Hkv, D, scale, O, NULL));
        finite(O, T * Hq * D, "frame prefill, empty cache");
        free(P);
    }
    {   /* compaction up to a full cache, then refused */
        int64_t len = L, row = -1;
        for (int64_t i = 0; i < T; ++i) OK(vs_oracle_compact_append(Kc, Vc, cap, &len, Kf, Vf, T, T - 1, Hkv, D, &row));
        if (len != cap || row != cap - 1) { fprintf(stderr, "compaction bookkeeping\n"); return 2; }
        FAILS(vs_oracle_compact_append(Kc, Vc, cap, &len, Kf, Vf, T, T - 1, Hkv, D, &row));
        FAILS(vs_oracle_compact_append(Kc, Vc, cap, &len, Kf, Vf, T, T, Hkv, D, &row));
    }
    {   /* decode: append then attend, and attend only */
        int64_t len = L;
        double *q = block(Hq * D), *kn = block(Hkv * D), *vn = block(Hkv * D), *o = block(Hq * D);
        OK(vs_oracle_decode(q, Kc, Vc, cap, &len, kn, vn, Hq, Hkv, D, scale, o));
        OK(vs_oracle_decode(q, Kc, Vc, cap, &len, NULL, NULL, Hq, Hkv, D, scale, o));
        finite(o, Hq * D, "decode");
        if (len != L + 1) { fprintf(stderr, "decode bookkeeping\n"); return 2; }
        len = cap;
        FAILS(vs_oracle_decode(q, Kc, Vc, cap, &len, kn, vn, Hq, Hkv, D, scale, o));
        free(q); free(kn); free(vn); free(o);
    }
    {   /* mean pool */
        double *E = block(N * d), *c = block(d);
        OK(vs_oracle_mean_pool(E, N, d, c)); finite(c, d, "mean pool");
        free(E); free(c);
    }
    {   /* memory bank: victim by both readings, then every kind of update */
        const int64_t M = 4, first = 2, width = 6, capacity = first + M;
        double *E = block(M * d), *e = block(d), *cs = block(M), *rows = block(capacity * width), *rn = block(width);
        int64_t victim = -1, n = 0;
        OK(vs_oracle_bank_victim(E, M, d, e, 0, cs, &victim));
        OK(vs_oracle_bank_victim(E, M, d, e, 1, NULL, &victim));
        FAILS(vs_oracle_bank_victim(E, M, d, e, 2, cs, &victim));
        for (int i = 0; i < 7; ++i) OK(vs_oracle_bank_apply(rows, capacity, width, first, M, n, n < M ? -1 : i % M, rn, &n));
        if (n != M) { fprintf(stderr, "bank bookkeeping\n"); return 2; }
        FAILS(vs_oracle_bank_apply(rows, capacity - 1, width, first, M, n, 0, rn, &n));
        free(E); free(e); free(cs); free(rows); free(rn);
    }
    {   /* run of frames, with and without retained rows */
        const int64_t Fr = 3;
        double *Qr = block(Fr * T * Hq * D), *Kr = block(Fr * T * Hkv * D), *Vr = block(Fr * T * Hkv * D);
        double *Or = block(Fr * T * Hq * D);
        OK(vs_oracle_frames_prefill(Qr, Kc, Vc, L, Kr, Vr, Fr, T, Hq, Hkv, D, scale, Or));
        OK(vs_oracle_frames_prefill(Qr, NULL, NULL, 0, Kr, Vr, Fr, T, Hq, Hkv, D, scale, Or));
        finite(Or, Fr * T * Hq * D, "frames prefill");
        free(Qr); free(Kr); free(Vr); free(Or);
    }
    {   /* the question: fills the cache exactly, one more token is refused */
        int64_t len = L;
        OK(vs_oracle_query_prefill(Q, Kc, Vc, cap, &len, Kf, Vf, T, Hq, Hkv, D, scale, O));
        finite(O, T * Hq * D, "question");
        if (len != cap) { fprintf(stderr, "question bookkeeping\n"); return 2; }
        FAILS(vs_oracle_query_prefill(Q, Kc, Vc, cap, &len, Kf, Vf, 1, Hq, Hkv, D, scale, O));
    }
    {   /* frame rows and projections */
        const int64_t n_out = (Hq + 2 * Hkv) * D;
        double *E = block(N * d), *W = block(n_out * d), *Y = block((N + 1) * n_out);
        OK(vs_oracle_frame_qkv(E, N, d, W, n_out, Y)); finite(Y, (N + 1) * n_out, "frame qkv");
        free(E); free(W); free(Y);
    }
    {   /* the decoder layer and its stages */
        double *H = block(T * d), *g1 = block(d), *g2 = block(d), *Wq = block(Hq * D * d), *Wk = block(Hkv * D * d);
        double *Wv = block(Hkv * D * d), *Wo = block(d * Hq * D), *Wg = block(F * d), *Wu = block(F * d), *Wd = block(d * F);
        double *Kl = block(T * Hkv * D), *Vl = block(T * Hkv * D), *Ho = block(T * d), *Y = block(T * F), *Z = block(T * F);
        OK(vs_oracle_rmsnorm(H, T, d, g1, 1e-6, Ho)); finite(Ho, T * d, "rmsnorm");
        OK(vs_oracle_linear(H, T, d, Wg, F, Y)); OK(vs_oracle_linear(H, T, d, Wu, F, Z));
        OK(vs_oracle_gated_unit(Y, Z, T, F, Y)); finite(Y, T * F, "gated unit");
        OK(vs_oracle_decoder_layer(H, T, d, Hq, Hkv, D, F, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, 1e-6, Kc, Vc, L, scale, Kl, Vl, Ho));
        finite(Ho, T * d, "decoder layer");
        OK(vs_oracle_decoder_layer(H, 1, d, Hq, Hkv, D, F, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, 0.0, NULL, NULL, 0, scale, Kl, Vl, Ho));
        FAILS(vs_oracle_decoder_layer(H, T, d, Hq, 4, D, F, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, 1e-6, Kc, Vc, L, scale, Kl, Vl, Ho));
        free(H); free(g1); free(g2); free(Wq); free(Wk); free(Wv); free(Wo); free(Wg); free(Wu); free(Wd);
        free(Kl); free(Vl); free(Ho); free(Y); free(Z);
    }
    free(Q); free(Kc); free(Vc); free(Kf); free(Vf); free(O);
    puts("oracle under sanitizers: ok");
    return 0;
}
