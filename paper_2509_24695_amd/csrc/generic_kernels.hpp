// Plain fp32-arithmetic kernels for every supported (dtype, d) pair, and the
// fixed-order partial-state reduction used by all paths.
//
// These serve the fp32 validation mode (results within 1e-5 of a float64
// evaluation) and the bf16 shapes that have no MFMA kernel.  D is the head
// dimension: 32, 64, 112 or 128.  Products are fp32
// FMAs in token order inside a chunk; chunks are combined by state_reduce.
#pragma once

#include "common.hpp"
#include "rope.hpp"

namespace sv {

// Partial state of one token chunk of one head:
//   ws[(bh*C + c)][k*D + v] = sum_{j in chunk c} phi(K[j][k]) V[j][v]     (Sec. 3.2, numerator bracket)
//   ws[(bh*C + c)][D*D + k] = sum_{j in chunk c} phi(K[j][k])             (denominator bracket)
// grid = (C, B*H), block = 256.  Tiles hold TT tokens; chunk c owns tiles
// [c*T/C, (c+1)*T/C) of the T tiles that cover [t0, t1).  Row k of S is shared
// by TPR threads (the largest power of two with D*TPR <= 256); threads past
// D*TPR only help with the loads.
// rope_mode (kRopeNone/Table/3D): the keys that meet V are rotated after the ReLU; the key sum
// uses the plain ones.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void state_partial_generic(
    const T *__restrict__ K, const T *__restrict__ V, RopeArg rope, int rope_mode, TokStrides st, int H, int t0,
    int t1, int C, float *__restrict__ ws)
{
    constexpr int TT = 32;
    constexpr int TPR = D <= 32 ? 8 : (D <= 64 ? 4 : 2);   // threads per S row
    constexpr int EPT = D / TPR;                           // S elements per thread (one row segment)
    static_assert(D % TPR == 0 && D * TPR <= kThreads, "row segments tile the state");
    __shared__ float sK[TT][D];             // keys as they enter S (rotated when rope is given)
    __shared__ float sP[TT][D];             // phi(K) as it enters the key sum
    __shared__ float sV[TT][D];

    const int tid = threadIdx.x;
    const int c = blockIdx.x, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const T *Kh = K + b * st.b + h * st.h;
    const T *Vh = V + b * st.b + h * st.h;

    const int n_tiles = (t1 - t0 + TT - 1) / TT;
    const int tile_lo = chunk_tile_begin(c, C, n_tiles);
    const int tile_hi = chunk_tile_begin(c + 1, C, n_tiles);

    const bool owner = tid < D * TPR;
    const int k = owner ? tid / TPR : 0, v0 = (tid % TPR) * EPT;
    float acc[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) acc[e] = 0.f;
    float zacc = 0.f;

    for (int tile = tile_lo; tile < tile_hi; ++tile) {
        const int tok0 = t0 + tile * TT;
        for (int idx = tid; idx < TT * D / 2; idx += kThreads) {       // one feature pair per step
            const int j = idx / (D / 2), p = idx % (D / 2);
            const int tok = tok0 + j;
            float a = 0.f, b = 0.f, va = 0.f, vb = 0.f, c = 1.f, s = 0.f;
            if (tok < t1) {
                a = fmaxf(Elem<T>::load(Kh + (int64_t)tok * st.n + 2 * p), 0.f);       // phi = ReLU
                b = fmaxf(Elem<T>::load(Kh + (int64_t)tok * st.n + 2 * p + 1), 0.f);
                va = Elem<T>::load(Vh + (int64_t)tok * st.n + 2 * p);
                vb = Elem<T>::load(Vh + (int64_t)tok * st.n + 2 * p + 1);
                if (rope_mode == kRopeTable) {
                    c = rope.table[(int64_t)tok * D + 2 * p];
                    s = rope.table[(int64_t)tok * D + 2 * p + 1];
                } else if (rope_mode == kRope3D) {
                    const f32x2 e = rope3d_entry_global(rope.r3, tok, p);
                    c = e.x;
                    s = e.y;
                }
            }
            sP[j][2 * p] = a;
            sP[j][2 * p + 1] = b;
            sK[j][2 * p] = a * c - b * s;
            sK[j][2 * p + 1] = a * s + b * c;
            sV[j][2 * p] = va;
            sV[j][2 * p + 1] = vb;
        }
        wg_barrier();
        if (owner) {
#pragma unroll 4
            for (int j = 0; j < TT; ++j) {
                const float a = sK[j][k];
                zacc += sP[j][k];
#pragma unroll
                for (int e = 0; e < EPT; ++e) acc[e] = fmaf(a, sV[j][v0 + e], acc[e]);
            }
        }
        wg_barrier();
    }

    if (!owner) return;
    float *out = ws + ((int64_t)bh * C + c) * (D * D + D);
#pragma unroll
    for (int e = 0; e < EPT; ++e) out[k * D + v0 + e] = acc[e];
    if (tid % TPR == 0) out[D * D + k] = zacc;
}

// S_out, z_out = (S_in, z_in or 0) + sum over chunks of the partial states, in chunk order:
//   x = S_in ? S_in[e] : 0;  for c = 0..C-1: x += ws[bh][c][e]
// S_in may be null or equal to S_out (in place).
// The fixed order makes the result bit-reproducible (no float atomics).
// grid = (ceil((D*D+D)/256), B*H).  C == 0 zero-fills or leaves the state as is.
// Partial c of head bh starts at ws + (bh*chunk_stride + c) * (D*D+D).
template <int D>
__global__ __launch_bounds__(kThreads) void state_reduce(
    const float *__restrict__ ws, int C, int chunk_stride, const float *S_in, const float *z_in, float *S_out,
    float *z_out)
{
    constexpr int E = D * D + D;
    const int e = blockIdx.x * kThreads + threadIdx.x;
    const int bh = blockIdx.y;
    if (e >= E) return;
    const int64_t off = e < D * D ? (int64_t)bh * D * D + e : (int64_t)bh * D + (e - D * D);
    float *dst = (e < D * D ? S_out : z_out) + off;
    float x = S_in ? (e < D * D ? S_in : z_in)[off] : 0.f;
    const float *p = ws + (int64_t)bh * chunk_stride * E + e;
    for (int c = 0; c < C; ++c) x += p[(int64_t)c * E];
    *dst = x;
}

// O[i][v] = (sum_k phi(Q[i][k]) S[k][v]) / (sum_k phi(Q[i][k]) z[k] + eps)   (Sec. 3.2, right-hand form)
// grid = (C, B*H), block = 256, dynamic LDS = apply_generic_lds_bytes<D>().  The head's
// S and z stay in LDS for the whole token range of the workgroup; D/4 threads
// serve one token, 256/(D/4) tokens (rounded down) make a tile.
// rope_mode (kRopeNone/Table/3D): the numerator uses queries rotated after the ReLU, the denominator
// the plain ones.
template <int D> __host__ __device__ constexpr int apply_generic_tile() { return kThreads / (D / 4); }
template <int D> __host__ __device__ constexpr int apply_generic_lds_bytes() {
    return (D * D + D + 2 * apply_generic_tile<D>() * D) * (int)sizeof(float);
}
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void apply_generic(
    const T *__restrict__ Q, T *__restrict__ O, RopeArg rope, int rope_mode, TokStrides st, int H, int t0, int t1,
    int C, const float *__restrict__ S, const float *__restrict__ z, float eps)
{
    constexpr int VPT = 4;                   // outputs per thread
    constexpr int TPT = D / VPT;             // threads per token
    constexpr int TT = apply_generic_tile<D>();   // tokens per tile
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    float (*sS)[D] = reinterpret_cast<float (*)[D]>(lds_raw);
    float *sz = reinterpret_cast<float *>(lds_raw) + D * D;
    float (*sQ)[D] = reinterpret_cast<float (*)[D]>(sz + D);        // queries of the numerator (rotated with rope)
    float (*sP)[D] = reinterpret_cast<float (*)[D]>(sz + D + TT * D);   // phi(Q) of the denominator

    const int tid = threadIdx.x;
    const int c = blockIdx.x, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const T *Qh = Q + b * st.b + h * st.h;
    T *Oh = O + b * st.b + h * st.h;

    for (int idx = tid; idx < D * D; idx += kThreads) sS[idx / D][idx % D] = S[(int64_t)bh * D * D + idx];
    if (tid < D) sz[tid] = z[(int64_t)bh * D + tid];

    const int n_tiles = (t1 - t0 + TT - 1) / TT;
    const int tile_lo = chunk_tile_begin(c, C, n_tiles);
    const int tile_hi = chunk_tile_begin(c + 1, C, n_tiles);
    const int j = tid / TPT, v0 = (tid % TPT) * VPT;
    const bool worker = j < TT;              // 256 is not a multiple of D/4 for every D

    for (int tile = tile_lo; tile < tile_hi; ++tile) {
        const int tok0 = t0 + tile * TT;
        wg_barrier();
        for (int idx = tid; idx < TT * D / 2; idx += kThreads) {
            const int jj = idx / (D / 2), p = idx % (D / 2);
            const int tok = tok0 + jj;
            float a = 0.f, b = 0.f, c = 1.f, s = 0.f;
            if (tok < t1) {
                a = fmaxf(Elem<T>::load(Qh + (int64_t)tok * st.n + 2 * p), 0.f);
                b = fmaxf(Elem<T>::load(Qh + (int64_t)tok * st.n + 2 * p + 1), 0.f);
                if (rope_mode == kRopeTable) {
                    c = rope.table[(int64_t)tok * D + 2 * p];
                    s = rope.table[(int64_t)tok * D + 2 * p + 1];
                } else if (rope_mode == kRope3D) {
                    const f32x2 e = rope3d_entry_global(rope.r3, tok, p);
                    c = e.x;
                    s = e.y;
                }
            }
            sP[jj][2 * p] = a;
            sP[jj][2 * p + 1] = b;
            sQ[jj][2 * p] = a * c - b * s;
            sQ[jj][2 * p + 1] = a * s + b * c;
        }
        wg_barrier();
        float num[VPT] = {0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
        if (worker) {
#pragma unroll 8
            for (int k = 0; k < D; ++k) {
                const float q = sQ[j][k];
                den = fmaf(sP[j][k], sz[k], den);
#pragma unroll
                for (int e = 0; e < VPT; ++e) num[e] = fmaf(q, sS[k][v0 + e], num[e]);
            }
        }
        const int tok = tok0 + j;
        if (worker && tok < t1) {
            const float dd = den + eps;
#pragma unroll
            for (int e = 0; e < VPT; ++e) Elem<T>::store(Oh + (int64_t)tok * st.n + v0 + e, num[e] / dd);
        }
    }
}

}  // namespace sv
