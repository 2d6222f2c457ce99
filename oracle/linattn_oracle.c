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
 * RoPE variant (the full equation of Sec. 3.2): when a rotation table is
 * given, the NUMERATOR uses rotated features, RoPE applied after the ReLU, and
 * the denominator stays un-rotated (the paper removes RoPE there to keep it
 * positive):
 *
 *   S[k][v]  = sum_j rot_j(phi(K[j]))[k] * V[j][v]
 *   z[k]     = sum_j phi(K[j][k])
 *   O[i][v]  = (sum_k rot_i(phi(Q[i]))[k] S[k][v]) / (sum_k phi(Q[i][k]) z[k] + eps)
 *
 * rot_t rotates each adjacent feature pair (2p, 2p+1) of token t by the angle
 * whose cosine and sine are table[t][p][0] and table[t][p][1]:
 *   y[2p] = x[2p] cos - x[2p+1] sin,   y[2p+1] = x[2p] sin + x[2p+1] cos.
 * The table is shared by all batches and heads.  How the d/2 angles of a token
 * derive from its (frame, row, column) position is the caller's business (the
 * paper says "3D RoPE" and gives no frequencies); pairing adjacent features is
 * a reading taken here.
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
 * Parity pins (tests/test_oracle_pins.py, tests/test_oracle_rope_pins.py): O(N^2) kernel-score brute force, a
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

/* y = rot_t(phi(x)) for one token: `row` points at table[t] (d/2 pairs of
 * cos, sin); a null row means no rotation. */
static void phi_rot(const float *x, const float *row, int64_t d, double *y)
{
    for (int64_t p = 0; p < d / 2; ++p) {
        const double a = relu((double)x[2 * p]), b = relu((double)x[2 * p + 1]);
        if (row) {
            const double c = (double)row[2 * p], s = (double)row[2 * p + 1];
            y[2 * p] = a * c - b * s;
            y[2 * p + 1] = a * s + b * c;
        } else {
            y[2 * p] = a;
            y[2 * p + 1] = b;
        }
    }
}

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
void orc_state(const float *K, const float *V, const float *rope, int64_t B, int64_t H, int64_t N, int64_t d,
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
        double rk[ORC_MAX_D];
        for (int64_t j = t0; j < t1; ++j) {
            phi_rot(Kh + j * d, rope ? rope + j * d : 0, d, rk);   /* table row j: d/2 (cos, sin) pairs = d floats */
            for (int64_t k = 0; k < d; ++k) {
                zh[k] += relu((double)Kh[j * d + k]);               /* key sum: never rotated */
                for (int64_t v = 0; v < d; ++v)
                    Sh[k * d + v] += rk[k] * (double)Vh[j * d + v];
            }
        }
    }
}

/* O[i] for tokens i in [t0,t1) from a given state; rows outside the range are
 * left untouched. */
ORC_CLONES
void orc_apply(const float *Q, const float *rope, int64_t B, int64_t H, int64_t N, int64_t d,
               int64_t t0, int64_t t1, const double *S, const double *z, double eps, double *O)
{
    const int64_t BH = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < BH; ++bh) {
        const float *Qh = Q + bh * N * d;
        const double *Sh = S + bh * d * d;
        const double *zh = z + bh * d;
        double *Oh = O + bh * N * d;
        double num[ORC_MAX_D], rq[ORC_MAX_D];
        for (int64_t i = t0; i < t1; ++i) {
            double den = 0.0;
            for (int64_t v = 0; v < d; ++v) num[v] = 0.0;
            phi_rot(Qh + i * d, rope ? rope + i * d : 0, d, rq);
            for (int64_t k = 0; k < d; ++k) {
                den += relu((double)Qh[i * d + k]) * zh[k];          /* denominator: never rotated */
                for (int64_t v = 0; v < d; ++v)
                    num[v] += rq[k] * Sh[k * d + v];
            }
            for (int64_t v = 0; v < d; ++v)
                Oh[i * d + v] = num[v] / (den + eps);
        }
    }
}

/* Bidirectional layer: every token attends to all N tokens. Also returns S, z. */
void orc_bidirectional(const float *Q, const float *K, const float *V, const float *rope,
                       int64_t B, int64_t H, int64_t N, int64_t d, double eps,
                       double *O, double *S, double *z)
{
    orc_state(K, V, rope, B, H, N, d, 0, N, 0, S, z);
    orc_apply(Q, rope, B, H, N, d, 0, N, S, z, eps, O);
}

/* One block of the block-causal stream: fold the block's keys and values into
 * the carried state, then emit the block's outputs from the updated state.
 * commit=0 leaves the caller's S,z unchanged (the noisy denoising passes of
 * Alg. 1 read the cache without updating it); S_tmp/z_tmp must then point to
 * scratch of the same size as S/z.  `rope` is the table of the block's own
 * tokens (row i = token i of the block), or null. */
void orc_block_step(const float *Qb, const float *Kb, const float *Vb, const float *rope,
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
    orc_state(Kb, Vb, rope, B, H, Nb, d, 0, Nb, 1, Su, zu);
    orc_apply(Qb, rope, B, H, Nb, d, 0, Nb, Su, zu, eps, Ob);
}
