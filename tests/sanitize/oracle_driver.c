/* Driver for running the fp64 oracle under AddressSanitizer / UBSan (host only): calls every entry
 * point on small pseudo-random inputs, including ragged and empty cases, and exits 0.  The sanitizers
 * abort on any out-of-bounds access, leak or undefined operation inside the oracle. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../oracle/climber_oracle.c"

static double rnd(uint64_t *s)
{
    *s = *s * 6364136223846793005ULL + 1442695040888963407ULL;
    return ((double)((*s >> 11) & 0xFFFFF) / 1048576.0 - 0.5) * 2.0;
}

int main(void)
{
    uint64_t s = 12345;
    enum { B = 3, H = 2, DH = 4, D = 8, F = 12, NS = 3, NB = 2, NL = 2 };
    const int32_t tok_off[B + 1] = {0, 8, 12, 20}, hist_len[B] = {7, 0, 8}, cand_off[B + 1] = {0, 3, 3, 5};
    const int T = 20, M = 5;
    double *q = malloc(sizeof(double) * T * D), *k = malloc(sizeof(double) * T * D), *v = malloc(sizeof(double) * T * D);
    double *qc = malloc(sizeof(double) * M * D), *kc = malloc(sizeof(double) * M * D), *vc = malloc(sizeof(double) * M * D);
    double *o = malloc(sizeof(double) * T * D), *oc = malloc(sizeof(double) * M * D);
    int32_t scen[20], beh[20], cs[5], cb[5], pos[20], ts[20], cpos[5], cts[5];
    double tau[NL * NS * NB], ptab[NS * NB * H * 5], ttab[NS * NB * H * 4];
    for (int i = 0; i < T * D; ++i) q[i] = rnd(&s), k[i] = rnd(&s), v[i] = rnd(&s);
    for (int i = 0; i < M * D; ++i) qc[i] = rnd(&s), kc[i] = rnd(&s), vc[i] = rnd(&s);
    for (int i = 0; i < T; ++i) scen[i] = i % NS, beh[i] = i % NB, pos[i] = i, ts[i] = 1000 + 37 * i * i;
    for (int i = 0; i < M; ++i) cs[i] = (i + 1) % NS, cb[i] = i % NB, cpos[i] = 8, cts[i] = 2000000000 - i;
    for (int i = 0; i < NL * NS * NB; ++i) tau[i] = 0.5 + (i % 4) * 0.5;
    for (int i = 0; i < NS * NB * H * 5; ++i) ptab[i] = rnd(&s);
    for (int i = 0; i < NS * NB * H * 4; ++i) ttab[i] = rnd(&s);
    int rc = 0;
    for (int causal = 0; causal < 2; ++causal)
        for (int sub = 0; sub <= 4; sub += 4) {
            rc |= oracle_attn_history(B, tok_off, hist_len, H, DH, sub, causal, q, k, v, scen, beh, tau, NS, NB, 0.5, o);
            rc |= oracle_attn_history_bias(B, tok_off, hist_len, H, DH, sub, causal, q, k, v, scen, beh, tau, NS, NB,
                                           0.5, pos, ts, ptab, ttab, 5, 4, o);
        }
    rc |= oracle_attn_sumi(B, tok_off, hist_len, cand_off, H, DH, k, v, qc, kc, vc, cs, cb, tau, NS, NB, 0.5, oc);
    rc |= oracle_attn_sumi_bias(B, tok_off, hist_len, cand_off, H, DH, k, v, qc, kc, vc, cs, cb, tau, NS, NB, 0.5, pos,
                                ts, cpos, cts, ptab, ttab, 5, 4, oc);
    /* layer stack: encode, score, brute force, packed forward, fusion */
    oracle_layer_w w[NL];
    double *wbuf = malloc(sizeof(double) * NL * (2 * D + 3 * D * D + D * D + 2 * D * F));
    double *p = wbuf;
    for (int l = 0; l < NL; ++l) {
        w[l].g1 = p; p += D; w[l].Wqkv = p; p += 3 * D * D; w[l].Wo = p; p += D * D;
        w[l].g2 = p; p += D; w[l].W1 = p; p += D * F; w[l].W2 = p; p += D * F;
    }
    for (double *x = wbuf; x < p; ++x) *x = 0.3 * rnd(&s);
    const oracle_cfg c = {NL, D, H, DH, F, NS, NB, 4, 0, 0.5, 1e-6};
    double *kcache = malloc(sizeof(double) * NL * T * D), *vcache = malloc(sizeof(double) * NL * T * D);
    double *yh = malloc(sizeof(double) * T * D), *yc = malloc(sizeof(double) * M * D), yb[D];
    rc |= oracle_stack_encode(&c, w, tau, B, tok_off, hist_len, q, scen, beh, kcache, vcache, yh);
    rc |= oracle_stack_score(&c, w, tau, B, tok_off, hist_len, kcache, vcache, cand_off, qc, cs, cb, yc);
    rc |= oracle_stack_bruteforce(&c, w, tau, 7, q, scen, beh, qc, cs[0], cb[0], yb);
    rc |= oracle_stack_packed(&c, w, tau, 7, q, scen, beh, 3, qc, cs, cb, yh, yc);
    rc |= oracle_stack_packed(&c, w, tau, 0, q, scen, beh, 2, qc, cs, cb, NULL, yc);
    {
        enum { NBK = 3, DG = 5 };
        double tau_s[NS] = {0.5, 1.0, 2.0}, wd[NBK * D * DG], wu[DG * NBK * D], wh[NBK * D], e[M * NBK * D], g[M * NBK * D],
               y[M * NBK * D], sc[M];
        for (int i = 0; i < NBK * D * DG; ++i) wd[i] = rnd(&s), wu[i] = rnd(&s);
        for (int i = 0; i < NBK * D; ++i) wh[i] = rnd(&s);
        for (int i = 0; i < M * NBK * D; ++i) e[i] = rnd(&s);
        rc |= oracle_bgf(&c, &w[0], tau_s, NS, NBK, DG, wd, wu, wh, 0.25, M, e, cs, g, y, sc);
        rc |= oracle_bgf(&c, &w[0], tau_s, NS, 1, DG, wd, wu, wh, 0.25, M, e, cs, NULL, NULL, sc);
    }
    /* error paths: bad id, bad temperature */
    scen[0] = NS;
    if (oracle_attn_history(B, tok_off, hist_len, H, DH, 0, 0, q, k, v, scen, beh, tau, NS, NB, 0.5, o) == 0) rc |= 64;
    scen[0] = 0;
    tau[0] = 0.0;
    if (oracle_attn_sumi(B, tok_off, hist_len, cand_off, H, DH, k, v, qc, kc, vc, cs, cb, tau, NS, NB, 0.5, oc) == 0)
        rc |= 128;
    free(q); free(k); free(v); free(qc); free(kc); free(vc); free(o); free(oc); free(wbuf);
    free(kcache); free(vcache); free(yh); free(yc);
    printf("oracle under sanitizers: rc=%d\n", rc);
    return rc;
}
