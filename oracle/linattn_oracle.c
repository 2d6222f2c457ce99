/*
 * CPU oracle for ReLU-feature-map linear attention (test infrastructure only).
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  It is NOT part of the product: only tests, the smoke check and the
 * benchmark's CPU-baseline leg may build or call it, and it shares no code with
 * the HIP sources.
 *
 * What it computes, per (batch, head) pair independently, in float64:
 *
 *   phi(x)   = max(x, 0)                                   (ReLU feature map, Sec. 3.2)
 *   S[k][v]  = sum_j phi(K[j][k]) * V[j][v]                (numerator bracket of the
 *   z[k]     = sum_j phi(K[j][k])                           linear-attention equation of
 *   O[i][v]  = (sum_k phi(Q[i][k]) S[k][v])                 Sec. 3.2, without RoPE, as in the
 *              / (sum_k phi(Q[i][k]) z[k] + eps)            causal re-formulation of Sec. 3.3.1)
 *
 * and the block-causal form of Sec. 3.3.1: the sums run over all tokens of the
 * current block and of every earlier block, which enter only through the
 * carried S and z (the constant-memory cache of Alg. 1).
 *
 * Readings taken where the paper is silent: eps is added to the denominator
 * after the dot product (the paper's equations have no eps); the current block
 * is included in its own sums (the causal equation sums to j = i and attention
 * is full inside a block); there is no 1/sqrt(d) factor; S is indexed
 * [key feature][value feature].
 *
 * Inputs are float arrays holding the stored values exactly (bf16 widened to
 * fp32 is exact); every product and sum is in double.  Summation inside one
 * head is sequential in token order, so results do not depend on the thread
 * count.  Layout: tokens [B][H][N][d] with d contiguous; S [B][H][d][d];
 * z [B][H][d].
 *
 * Parity pins (tests/test_oracle_pins.py): O(N^2) kernel-score brute force, a
 * hand-computed 2-token example, matrix-product form via a library routine,
 * chunk additivity, single block == bidirectional, convexity and scale
 * invariances, degenerate rows, closed-form statistics.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAX_D 256

/* The two hot loops are compiled for several x86 vector widths and picked at
 * load time, so one shared object runs on any host.  Vectorising the loop over
 * v reorders nothing (each v is its own sum) and -ffp-contract=off keeps every
 * variant's rounding identical. */
#if defined(__x86_64__) && defined(__GNUC__) && !defined(__clang__)
#define ORC_CLONES __attribute__((target_clones("avx512f", "avx2", "default")))
#else
#define ORC_CLONES
#endif

static double relu(double x) { return x > 0.0 ? x : 0.0; }

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* S,z over tokens [t0,t1) of each head.  accumulate=0: S,z are overwritten;
 * accumulate=1: the sums are added to the S,z passed in (carried state). */
ORC_CLONES
void orc_state(const float *K, const float *V, int64_t B, int64_t H, int64_t N, int64_t d,
               int64_t t0, int64_t t1, int accumulate, double *S, double *z)
{
    const int64_t BH = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < BH; ++bh) {
        const float *Kh = K + bh * N * d;
        const float *Vh = V + bh * N * d;
        double *Sh = S + bh * d * d;
        double *zh = z + bh * d;
        if (!accumulate) {
            memset(Sh, 0, sizeof(double) * (size_t)(d * d));
            memset(zh, 0, sizeof(double) * (size_t)d);
        }
        for (int64_t j = t0; j < t1; ++j) {
            for (int64_t k = 0; k < d; ++k) {
                const double pk = relu((double)Kh[j * d + k]);
                zh[k] += pk;
                for (int64_t v = 0; v < d; ++v)
                    Sh[k * d + v] += pk * (double)Vh[j * d + v];
            }
        }
    }
}

/* O[i] for tokens i in [t0,t1) from a given state; rows outside the range are
 * left untouched. */
ORC_CLONES
void orc_apply(const float *Q, int64_t B, int64_t H, int64_t N, int64_t d,
               int64_t t0, int64_t t1, const double *S, const double *z, double eps, double *O)
{
    const int64_t BH = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < BH; ++bh) {
        const float *Qh = Q + bh * N * d;
        const double *Sh = S + bh * d * d;
        const double *zh = z + bh * d;
        double *Oh = O + bh * N * d;
        double num[ORC_MAX_D];
        for (int64_t i = t0; i < t1; ++i) {
            double den = 0.0;
            for (int64_t v = 0; v < d; ++v) num[v] = 0.0;
            for (int64_t k = 0; k < d; ++k) {
                const double pq = relu((double)Qh[i * d + k]);
                den += pq * zh[k];
                for (int64_t v = 0; v < d; ++v)
                    num[v] += pq * Sh[k * d + v];
            }
            for (int64_t v = 0; v < d; ++v)
                Oh[i * d + v] = num[v] / (den + eps);
        }
    }
}

/* Bidirectional layer: every token attends to all N tokens. Also returns S, z. */
void orc_bidirectional(const float *Q, const float *K, const float *V,
                       int64_t B, int64_t H, int64_t N, int64_t d, double eps,
                       double *O, double *S, double *z)
{
    orc_state(K, V, B, H, N, d, 0, N, 0, S, z);
    orc_apply(Q, B, H, N, d, 0, N, S, z, eps, O);
}

/* One block of the block-causal stream: fold the block's keys and values into
 * the carried state, then emit the block's outputs from the updated state.
 * commit=0 leaves the caller's S,z unchanged (the noisy denoising passes of
 * Alg. 1 read the cache without updating it); S_tmp/z_tmp must then point to
 * scratch of the same size as S/z. */
void orc_block_step(const float *Qb, const float *Kb, const float *Vb,
                    int64_t B, int64_t H, int64_t Nb, int64_t d, double eps,
                    double *S, double *z, int commit, double *S_tmp, double *z_tmp, double *Ob)
{
    double *Su = S, *zu = z;
    if (!commit) {
        memcpy(S_tmp, S, sizeof(double) * (size_t)(B * H * d * d));
        memcpy(z_tmp, z, sizeof(double) * (size_t)(B * H * d));
        Su = S_tmp;
        zu = z_tmp;
    }
    orc_state(Kb, Vb, B, H, Nb, d, 0, Nb, 1, Su, zu);
    orc_apply(Qb, B, H, Nb, d, 0, Nb, Su, zu, eps, Ob);
}
