/* Runs every oracle function on a ragged problem with exactly-sized heap buffers, meant to
 * be built with -fsanitize=address,undefined: any out-of-bounds index in the oracle shows. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int32_t oracle_plan(const int64_t *, int32_t, int32_t, int64_t, int32_t, int32_t *, int64_t *, int32_t *,
                    int32_t *, int64_t *, int64_t *, int64_t *);
void oracle_reduce_scatter(const int64_t *, int32_t, int32_t, int32_t, const int64_t *, int32_t, int32_t,
                           int64_t, int64_t, int64_t, const void *const *, float *, int64_t, int32_t, int32_t);
void oracle_shard_update(int32_t, int64_t, int64_t, int64_t, const float *, float *, float *, float, float,
                         int32_t, int32_t);
void oracle_all_gather(const int64_t *, int32_t, int32_t, const int64_t *, int32_t, int32_t, int64_t, int64_t,
                       const float *, int64_t, float *const *, int32_t, int32_t);
void oracle_scatter_params(const int64_t *, int32_t, int32_t, const int64_t *, int32_t, int32_t, int64_t,
                           int64_t, int64_t, float *const *, int32_t, float *, int64_t);

#define L 7
int main(void)
{
    const int64_t n[L] = {13, 1, 70, 33, 5, 64, 2};
    for (int g = 2; g <= 4; g += 2)
        for (int P = 1; P <= 5; ++P) {
            int32_t lb[L], bf[L], bn[L];
            int64_t lo[L], bl[L], bs[L], bb[L];
            const int32_t B = oracle_plan(n, L, P, 80 * g, g, lb, lo, bf, bn, bl, bs, bb);
            if (B < 1) return 1;
            int64_t row = 0;
            for (int b = 0; b < B; ++b) row += bs[b];
            void **grad = malloc(sizeof(void *) * P * L);
            float **param = malloc(sizeof(float *) * P * L);
            for (int p = 0; p < P; ++p)
                for (int l = 0; l < L; ++l) {
                    grad[p * L + l] = calloc((size_t)n[l], (size_t)g);
                    param[p * L + l] = calloc((size_t)n[l], sizeof(float));
                }
            float *sg = malloc(sizeof(float) * P * row), *sp = malloc(sizeof(float) * P * row),
                  *sm = calloc((size_t)(P * row), sizeof(float));
            for (int b = 0; b < B; ++b)
                oracle_scatter_params(n, L, P, lo, bf[b], bn[b], bl[b], bs[b], bb[b], param, P - 1, sp, row);
            for (int b = 0; b < B; ++b) {
                oracle_reduce_scatter(n, L, P, g, lo, bf[b], bn[b], bl[b], bs[b], bb[b],
                                      (const void *const *)grad, sg, row, 0, P);
                oracle_shard_update(P, bs[b], bb[b], row, sg, sp, sm, 0.1f, 0.9f, 0, P);
            }
            for (int b = B - 1; b >= 0; --b)
                oracle_all_gather(n, L, P, lo, bf[b], bn[b], bs[b], bb[b], sp, row, param, 0, P);
            for (int i = 0; i < P * L; ++i) {
                free(grad[i]);
                free(param[i]);
            }
            free(grad); free(param); free(sg); free(sp); free(sm);
        }
    printf("oracle_sanitize: ok\n");
    return 0;
}
