/* Drives the CPU oracle (one translation unit with it) under AddressSanitizer / UndefinedBehaviorSanitizer:
 * packing, a whole forward with per-student terms and pooled states, the taps of one (student, sequence), the
 * elementary pieces, and the argument-error paths.  Prints a checksum; any sanitizer report aborts the run. */
#include "../../oracle/sp_oracle.c"

#include <stdio.h>

static unsigned long long lcg = 88172645463325252ULL;
static float rnd(void)
{
    lcg = lcg * 6364136223846793005ULL + 1442695040888963407ULL;
    return (float)((double)(lcg >> 11) / 9007199254740992.0 - 0.5);
}

int main(void)
{
    spo_config c = {3, 2, 32, 4, 64, 50, 24, 3, 1e-12};
    const size_t n = spo_blob_floats(&c);
    float* blob = (float*)malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) blob[i] = 0.6f * rnd();
    const int32_t lengths[5] = {5, 1, 24, 9, 2};
    int32_t cu[6];
    if (spo_pack(lengths, 5, cu) != 0) return 2;
    const int T = cu[5];
    int32_t* ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)T);
    for (int i = 0; i < T; ++i) ids[i] = (int32_t)((rnd() + 0.5f) * 49.99f);
    double logits[5 * 3], z[3 * 5 * 3], pooled[3 * 5 * 32];
    double sum = 0;
    for (int k = 1; k <= 3; ++k) {
        if (spo_forward(&c, blob, ids, cu, 5, k, logits, z, pooled) != 0) return 3;
        for (int i = 0; i < 15; ++i) sum += logits[i];
    }
    {
        const int L = 24;
        double *x0 = malloc(sizeof(double) * L * 32), *qkv = malloc(sizeof(double) * 2 * L * 96),
               *att = malloc(sizeof(double) * 2 * L * 32), *x1 = malloc(sizeof(double) * 2 * L * 32),
               *g = malloc(sizeof(double) * 2 * L * 64), *x2 = malloc(sizeof(double) * 2 * L * 32), zz[3];
        if (spo_forward_taps(&c, blob, ids, cu, 5, 2, 2, x0, qkv, att, x1, g, x2, zz) != 0) return 4;
        sum += zz[0] + x2[2 * L * 32 - 1] + g[2 * L * 64 - 1] + qkv[2 * L * 96 - 1];
        free(x0); free(qkv); free(att); free(x1); free(g); free(x2);
    }
    {
        double u[7] = {1, 2, 3, 4, 5, 6, 7}, o[7], s[5] = {1000, 999, -1000, 0, 3};
        float gm[7] = {1, 1, 1, 1, 1, 1, 1}, bt[7] = {0};
        spo_layernorm(u, gm, bt, 7, 1e-12, o);
        spo_softmax(s, 5);
        sum += o[6] + s[0] + spo_gelu(1.0);
        double q[3 * 8], kk[3 * 8], v[3 * 8], oo[3 * 8], pr[2 * 3 * 3];
        for (int i = 0; i < 24; ++i) { q[i] = rnd(); kk[i] = rnd(); v[i] = rnd(); }
        spo_attention(q, kk, v, 3, 2, 4, oo, pr);
        spo_attention(q, kk, v, 1, 2, 4, oo, NULL);
        sum += oo[0] + pr[17];
    }
    /* argument errors must be refused, not executed */
    const int32_t bad_len[2] = {3, 0};
    int32_t cu2[3];
    if (spo_pack(bad_len, 2, cu2) == 0) return 5;
    if (spo_forward(&c, blob, ids, cu, 5, 0, logits, NULL, NULL) == 0) return 6;
    if (spo_forward(&c, blob, ids, cu, 5, 4, logits, NULL, NULL) == 0) return 7;
    ids[3] = 50;
    if (spo_forward(&c, blob, ids, cu, 5, 1, logits, NULL, NULL) == 0) return 8;
    free(ids);
    free(blob);
    printf("oracle driver checksum %.9f\n", sum);
    return 0;
}
