/* Drives the float64 oracle (oracle/linattn_oracle.c, linked in) over small shapes with exactly sized heap
 * buffers, for a build with -fsanitize=address,undefined: an index that leaves a tensor, the rotation table
 * or the state anywhere in the oracle's loops ends the run.  Prints "OK" and returns 0 otherwise.
 * Test infrastructure like the oracle itself; computes nothing of its own. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void orc_state(const float *K, const float *V, const float *rope, int64_t B, int64_t H, int64_t N, int64_t d,
               int64_t t0, int64_t t1, int accumulate, double *S, double *z);
void orc_apply(const float *Q, const float *rope, int64_t B, int64_t H, int64_t N, int64_t d, int64_t t0, int64_t t1,
               const double *S, const double *z, double eps, double *O);
void orc_bidirectional(const float *Q, const float *K, const float *V, const float *rope, int64_t B, int64_t H,
                       int64_t N, int64_t d, double eps, double *O, double *S, double *z);
void orc_block_step(const float *Qb, const float *Kb, const float *Vb, const float *rope, int64_t B, int64_t H,
                    int64_t Nb, int64_t d, double eps, double *S, double *z, int commit, double *S_tmp, double *z_tmp,
                    double *Ob);

static uint32_t lcg = 12345u;
static float draw(void)
{
    lcg = lcg * 1664525u + 1013904223u;
    return (float)((int32_t)(lcg >> 8) % 2001 - 1000) / 1000.0f;
}
static float *tokens(int64_t n)
{
    float *p = malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) p[i] = draw();
    return p;
}

static int run(int64_t B, int64_t H, int64_t N, int64_t d, int with_rope)
{
    const int64_t tok = B * H * N * d;
    float *Q = tokens(tok), *K = tokens(tok), *V = tokens(tok), *rope = with_rope ? tokens(N * d) : 0;
    double *S = malloc(sizeof(double) * (size_t)(B * H * d * d)), *z = malloc(sizeof(double) * (size_t)(B * H * d));
    double *St = malloc(sizeof(double) * (size_t)(B * H * d * d)), *zt = malloc(sizeof(double) * (size_t)(B * H * d));
    double *O = malloc(sizeof(double) * (size_t)tok);
    int bad = 0;
    orc_bidirectional(Q, K, V, rope, B, H, N, d, 1e-6, O, S, z);
    for (int64_t i = 0; i < tok; ++i) bad |= !(O[i] == O[i]);
    orc_state(K, V, rope, B, H, N, d, 0, 0, 0, S, z);                /* empty range: zero fill */
    for (int64_t i = 0; i < B * H * d * d; ++i) bad |= S[i] != 0.0;
    orc_state(K, V, rope, B, H, N, d, 0, N / 2, 1, S, z);            /* two halves, accumulated */
    orc_state(K, V, rope, B, H, N, d, N / 2, N, 1, S, z);
    orc_apply(Q, rope, B, H, N, d, N - 1, N, S, z, 0.0, O);          /* last row only, eps = 0 */
    orc_apply(Q, rope, B, H, N, d, N, N, S, z, 1e-6, O);             /* empty range */
    orc_block_step(Q, K, V, rope, B, H, N, d, 1e-6, S, z, 0, St, zt, O);
    orc_block_step(Q, K, V, rope, B, H, N, d, 1e-6, S, z, 1, St, zt, O);
    for (int64_t i = 0; i < tok; ++i) bad |= !(O[i] == O[i]);
    free(Q); free(K); free(V); free(rope); free(S); free(z); free(St); free(zt); free(O);
    return bad;
}

int main(void)
{
    static const int64_t shapes[][4] = {{1, 1, 1, 2}, {2, 3, 7, 32}, {1, 2, 33, 112}, {1, 1, 5, 256}, {3, 1, 64, 64}};
    int bad = 0;
    for (unsigned i = 0; i < sizeof shapes / sizeof shapes[0]; ++i)
        for (int r = 0; r < 2; ++r) bad |= run(shapes[i][0], shapes[i][1], shapes[i][2], shapes[i][3], r);
    if (bad) {
        printf("FAILED\n");
        return 1;
    }
    printf("OK\n");
    return 0;
}
