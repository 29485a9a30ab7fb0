/* Drives every routine of the C oracle (oracle/ape_oracle.c, included as source) over small ragged
 * inputs -- empty contexts, no prefix, one-token contexts, selected (row, head) pairs, trees of
 * several shapes -- for a build with -fsanitize=address,undefined: an out-of-bounds index or an
 * undefined operation anywhere in the oracle aborts the program.  Outputs are only checked for
 * being finite and for rows of weights summing to one (values all ones). */
#include <stdio.h>
#include "../oracle/ape_oracle.c"

static unsigned long long lcg = 0x9E3779B97F4A7C15ull;
static float rnd(void)
{
    lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((double)(lcg >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
static float *fill(long n, int ones)
{
    float *p = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    for (long i = 0; i < n; ++i) p[i] = ones ? 1.0f : rnd();
    return p;
}
static int finite_all(const double *x, long n)
{
    for (long i = 0; i < n; ++i) if (!(x[i] == x[i]) || x[i] > 1e300 || x[i] < -1e300) return 0;
    return 1;
}

int main(void)
{
    const int configs[][5] = { /* hq, hkv, d, prefix, q_len */ {4, 2, 8, 3, 5}, {2, 2, 16, 0, 1}, {8, 1, 8, 7, 4} };
    const int chunk_sets[][5] = { {5, 0, 1, 9, 0}, {0, 0, 0, 0, 0}, {1, 1, 1, 1, 1}, {12, 3, 0, 0, 7} };
    int failures = 0;
    for (int ci = 0; ci < 3; ++ci)
        for (int si = 0; si < 4; ++si) {
            const int hq = configs[ci][0], hkv = configs[ci][1], d = configs[ci][2], lp = configs[ci][3], ql = configs[ci][4];
            const int n_chunks = 5, self_len = ql + 2;
            int cu[6] = {0};
            for (int i = 0; i < n_chunks; ++i) cu[i + 1] = cu[i] + chunk_sets[si][i];
            const long M = cu[n_chunks];
            float *kp = fill((long)lp * hkv * d, 0), *vp = fill((long)lp * hkv * d, 1);
            float *kc = fill(M * hkv * d, 0), *vc = fill(M * hkv * d, 1), *qc = fill(M * hq * d, 0);
            float *ks = fill((long)self_len * hkv * d, 0), *vs = fill((long)self_len * hkv * d, 1);
            float *q = fill((long)ql * hq * d, 0);
            const long n_all = (long)ql * hq;
            double *out = (double *)malloc(sizeof(double) * (size_t)(n_all > M * hq ? n_all : M * hq + 1) * d);
            double *lse = (double *)malloc(sizeof(double) * (size_t)(n_all > M * hq ? n_all : M * hq + 1));
            double *mass = (double *)malloc(sizeof(double) * (size_t)n_all);
            int rc = ape_oracle_attention(hq, hkv, d, kp, vp, lp, kc, vc, cu, n_chunks, ks, vs, self_len, q, ql, 0.7, 0.8,
                                          NULL, NULL, 0, out, lse, mass);
            if (rc || !finite_all(out, n_all * d) || !finite_all(lse, n_all)) { printf("attention failed cfg %d set %d\n", ci, si); ++failures; }
            for (long i = 0; i < n_all * d; ++i) if (fabs(out[i] - 1.0) > 1e-12) { printf("weights do not sum to one\n"); ++failures; break; }
            for (int per = 0; per < 2; ++per) {
                rc = ape_oracle_attention_hier(hq, hkv, d, kp, vp, lp, kc, vc, cu, n_chunks, ks, vs, self_len, q, ql, 0.7, 0.8, per,
                                               NULL, NULL, 0, out, lse);
                if (rc || !finite_all(out, n_all * d)) { printf("hier failed\n"); ++failures; }
            }
            /* selected pairs: last row / last head, first row / first head */
            const int pr[2] = {ql - 1, 0}, ph[2] = {hq - 1, 0};
            rc = ape_oracle_attention(hq, hkv, d, kp, vp, lp, kc, vc, cu, n_chunks, ks, vs, self_len, q, ql, 1.0, 1.0, pr, ph, 2, out, lse, NULL);
            if (rc || !finite_all(out, 2L * d)) { printf("pairs failed\n"); ++failures; }
            /* trees: one node; one node per context under a root; two levels */
            {
                const double s1[1] = {0.9}; const int f1[1] = {0}, c1[1] = {5}, l1[1] = {1};
                rc = ape_oracle_attention_tree(hq, hkv, d, kp, vp, lp, kc, vc, cu, n_chunks, ks, vs, self_len, q, ql, 0.7,
                                               s1, f1, c1, l1, 1, NULL, NULL, 0, out, lse);
                if (rc || !finite_all(out, n_all * d)) { printf("tree 1 failed\n"); ++failures; }
                const double s6[6] = {1.0, 0.9, 0.8, 0.7, 0.6, 0.5}; const int f6[6] = {1, 0, 1, 2, 3, 4}, c6[6] = {5, 1, 1, 1, 1, 1}, l6[6] = {0, 1, 1, 1, 1, 1};
                rc = ape_oracle_attention_tree(hq, hkv, d, kp, vp, lp, kc, vc, cu, n_chunks, ks, vs, self_len, q, ql, 0.7,
                                               s6, f6, c6, l6, 6, pr, ph, 2, out, lse);
                if (rc || !finite_all(out, 2L * d)) { printf("tree 6 failed\n"); ++failures; }
                const double s4[4] = {0.9, 0.8, 1.0, 0.7}; const int f4[4] = {1, 0, 3, 2}, c4[4] = {2, 2, 1, 3}, l4[4] = {0, 1, 0, 1};
                rc = ape_oracle_attention_tree(hq, hkv, d, kp, vp, lp, kc, vc, cu, n_chunks, ks, vs, self_len, q, ql, 0.7,
                                               s4, f4, c4, l4, 4, NULL, NULL, 0, out, lse);
                if (rc || !finite_all(out, n_all * d)) { printf("tree 4 failed\n"); ++failures; }
                /* a malformed tree must be refused, not followed out of bounds */
                const int fbad[1] = {3};
                if (ape_oracle_attention_tree(hq, hkv, d, kp, vp, lp, kc, vc, cu, n_chunks, ks, vs, self_len, q, ql, 0.7,
                                              s1, fbad, c1, l1, 1, NULL, NULL, 0, out, lse) == 0) { printf("bad tree accepted\n"); ++failures; }
            }
            if (M > 0) {
                rc = ape_oracle_encode(hq, hkv, d, kp, vp, lp, qc, kc, vc, cu, n_chunks, NULL, NULL, 0, out, lse);
                if (rc || !finite_all(out, M * hq * d)) { printf("encode failed\n"); ++failures; }
                double *y = (double *)malloc(sizeof(double) * (size_t)(M * hkv * d));
                rc = ape_oracle_rope(kc, hkv, d, cu, n_chunks, lp, 500000.0, y);
                if (rc || !finite_all(y, M * hkv * d)) { printf("rope failed\n"); ++failures; }
                free(y);
            }
            free(kp); free(vp); free(kc); free(vc); free(qc); free(ks); free(vs); free(q); free(out); free(lse); free(mass);
        }
    printf("%d failures\n", failures);
    return failures != 0;
}
