// C ABI of the gfx950 linear-attention library: argument checks, launch plans,
// kernel dispatch.  See include/sv_linattn.h for the contract of each call.
#include "../../include/sv_linattn.h"

#include <hip/hip_runtime.h>
#include <math.h>

#include "apply_mfma.hpp"
#include "common.hpp"
#include "generic_kernels.hpp"
#include "state_mfma.hpp"

namespace {

using namespace sv;

constexpr int kVersion = 100;   // 0.1.0
constexpr int kNumCUs = 256;    // MI355X

struct Shape {
    int B, H, N, d, BH;
    TokStrides st;
    bool bf16;
    int elem_bytes;
};

// Launch plan shared by the state and apply kernels: the token range is cut
// into tiles of `tile` tokens and the tiles are dealt to `chunks` workgroups per
// head.  The chunk count aims at `wgs_per_cu` workgroups per compute unit over
// the whole grid and never exceeds kMaxChunks (which sizes the workspace).
struct Plan {
    int tile, chunks;
};

Plan make_plan(int BH, int n_tokens, int tile, int wgs_per_cu, int max_chunks)
{
    Plan p{tile, 0};
    if (n_tokens <= 0) return p;
    const int n_tiles = (n_tokens + tile - 1) / tile;
    int chunks = (kNumCUs * wgs_per_cu + BH - 1) / BH;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks > n_tiles) chunks = n_tiles;
    if (chunks < 1) chunks = 1;
    p.chunks = chunks;
    return p;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

sv_status check_desc(const sv_tensor_desc *t, Shape *s)
{
    if (!t) return SV_ERR_NULL;
    if (t->dtype != SV_BF16 && t->dtype != SV_F32) return SV_ERR_UNSUPPORTED;
    if (t->d != 32 && t->d != 64) return SV_ERR_UNSUPPORTED;
    if (t->B <= 0 || t->H <= 0 || t->N <= 0) return SV_ERR_SHAPE;
    if ((int64_t)t->B * t->H > 65535) return SV_ERR_SHAPE;           // grid.y limit
    if (t->stride_n < t->d || t->stride_b < 0 || t->stride_h < 0) return SV_ERR_SHAPE;
    if (t->B > 1 && t->stride_b == 0) return SV_ERR_SHAPE;
    if (t->H > 1 && t->stride_h == 0) return SV_ERR_SHAPE;
    s->B = t->B; s->H = t->H; s->N = t->N; s->d = t->d; s->BH = t->B * t->H;
    s->st = TokStrides{t->stride_b, t->stride_h, t->stride_n};
    s->bf16 = t->dtype == SV_BF16;
    s->elem_bytes = s->bf16 ? 2 : 4;
    const int64_t per16 = 16 / s->elem_bytes;
    if (t->stride_n % per16 || t->stride_b % per16 || t->stride_h % per16) return SV_ERR_ALIGN;
    return SV_OK;
}

sv_status check_range(const Shape &s, int32_t t0, int32_t t1)
{
    return (t0 < 0 || t1 < t0 || t1 > s.N) ? SV_ERR_RANGE : SV_OK;
}

size_t workspace_bytes(int BH, int d) { return (size_t)BH * kMaxChunks * ((size_t)d * d + d) * sizeof(float); }

sv_status launch_status() { return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_LAUNCH; }

// Partial states of [t0,t1) into the workspace, then the fixed-order reduction
// into S, z.  All arguments are already validated.
sv_status enqueue_state(const void *K, const void *V, const Shape &s, int t0, int t1, int accumulate, float *S,
                        float *z, float *ws, hipStream_t stream)
{
    const int n = t1 - t0;
    const bool mfma = s.bf16 && s.d == 64;
    const Plan plan = mfma ? make_plan(s.BH, n, n >= 8192 ? 32 : 16, 2, kMaxChunks)
                           : make_plan(s.BH, n, 32, 2, kMaxChunks);
    if (n == 0 && accumulate) return SV_OK;
    if (n > 0) {
        const dim3 grid(plan.chunks, s.BH), block(kThreads);
        if (mfma) {
            auto *k = static_cast<const uint16_t *>(K);
            auto *v = static_cast<const uint16_t *>(V);
            if (plan.tile == 32)
                state_partial_mfma_d64<32><<<grid, block, 0, stream>>>(k, v, s.st, s.H, t0, t1, plan.chunks, ws);
            else
                state_partial_mfma_d64<16><<<grid, block, 0, stream>>>(k, v, s.st, s.H, t0, t1, plan.chunks, ws);
        } else if (s.bf16) {
            auto *k = static_cast<const uint16_t *>(K);
            auto *v = static_cast<const uint16_t *>(V);
            state_partial_generic<uint16_t, 32><<<grid, block, 0, stream>>>(k, v, s.st, s.H, t0, t1, plan.chunks, ws);
        } else {
            auto *k = static_cast<const float *>(K);
            auto *v = static_cast<const float *>(V);
            if (s.d == 64)
                state_partial_generic<float, 64><<<grid, block, 0, stream>>>(k, v, s.st, s.H, t0, t1, plan.chunks, ws);
            else
                state_partial_generic<float, 32><<<grid, block, 0, stream>>>(k, v, s.st, s.H, t0, t1, plan.chunks, ws);
        }
    }
    const int E = s.d * s.d + s.d;
    const dim3 rgrid((E + kThreads - 1) / kThreads, s.BH), rblock(kThreads);
    if (s.d == 64)
        state_reduce<64><<<rgrid, rblock, 0, stream>>>(ws, plan.chunks, accumulate, S, z);
    else
        state_reduce<32><<<rgrid, rblock, 0, stream>>>(ws, plan.chunks, accumulate, S, z);
    return launch_status();
}

sv_status enqueue_apply(const void *Q, const Shape &s, int t0, int t1, const float *S, const float *z, float eps,
                        void *O, hipStream_t stream)
{
    const int n = t1 - t0;
    if (n == 0) return SV_OK;
    const bool mfma = s.bf16 && s.d == 64;
    // generic tiles: 256 threads / (d/4 threads per token)
    const Plan plan = mfma ? make_plan(s.BH, n, 32, 4, 1 << 20) : make_plan(s.BH, n, kThreads / (s.d / 4), 4, 1 << 20);
    const dim3 grid(plan.chunks, s.BH), block(kThreads);
    if (mfma) {
        apply_mfma_d64<true><<<grid, block, 0, stream>>>(static_cast<const uint16_t *>(Q), static_cast<uint16_t *>(O),
                                                        s.st, s.H, t0, t1, plan.chunks, S, z, eps);
    } else if (s.bf16) {
        apply_generic<uint16_t, 32><<<grid, block, 0, stream>>>(static_cast<const uint16_t *>(Q),
                                                               static_cast<uint16_t *>(O), s.st, s.H, t0, t1,
                                                               plan.chunks, S, z, eps);
    } else if (s.d == 64) {
        apply_generic<float, 64><<<grid, block, 0, stream>>>(static_cast<const float *>(Q), static_cast<float *>(O),
                                                            s.st, s.H, t0, t1, plan.chunks, S, z, eps);
    } else {
        apply_generic<float, 32><<<grid, block, 0, stream>>>(static_cast<const float *>(Q), static_cast<float *>(O),
                                                            s.st, s.H, t0, t1, plan.chunks, S, z, eps);
    }
    return launch_status();
}

bool eps_ok(float eps) { return isfinite(eps) && eps >= 0.f; }

}  // namespace

extern "C" {

size_t sv_linattn_workspace_bytes(int32_t B, int32_t H, int32_t n_tokens, int32_t d)
{
    if (B <= 0 || H <= 0 || n_tokens < 0 || (d != 32 && d != 64)) return 0;
    if ((int64_t)B * H > 65535) return 0;
    return workspace_bytes(B * H, d);
}

sv_status sv_linattn_state(const void *K, const void *V, const sv_tensor_desc *kv, int32_t tok_begin,
                           int32_t tok_end, int accumulate, float *S, float *z, void *workspace,
                           size_t workspace_bytes_given, void *stream)
{
    if (!K || !V || !S || !z || !workspace) return SV_ERR_NULL;
    Shape s;
    sv_status rc = check_desc(kv, &s);
    if (rc != SV_OK) return rc;
    if ((rc = check_range(s, tok_begin, tok_end)) != SV_OK) return rc;
    if (!aligned16(K) || !aligned16(V) || !aligned16(S) || !aligned16(z) || !aligned16(workspace))
        return SV_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(s.BH, s.d)) return SV_ERR_WORKSPACE;
    return enqueue_state(K, V, s, tok_begin, tok_end, accumulate != 0, S, z, static_cast<float *>(workspace),
                         static_cast<hipStream_t>(stream));
}

sv_status sv_linattn_apply(const void *Q, const sv_tensor_desc *q, int32_t tok_begin, int32_t tok_end,
                           const float *S, const float *z, float eps, void *O, void *stream)
{
    if (!Q || !S || !z || !O) return SV_ERR_NULL;
    Shape s;
    sv_status rc = check_desc(q, &s);
    if (rc != SV_OK) return rc;
    if ((rc = check_range(s, tok_begin, tok_end)) != SV_OK) return rc;
    if (!eps_ok(eps)) return SV_ERR_RANGE;
    if (!aligned16(Q) || !aligned16(O) || !aligned16(S) || !aligned16(z)) return SV_ERR_ALIGN;
    return enqueue_apply(Q, s, tok_begin, tok_end, S, z, eps, O, static_cast<hipStream_t>(stream));
}

sv_status sv_block_linattn_step(const void *Qb, const void *Kb, const void *Vb, const sv_tensor_desc *blk, float *S,
                                float *z, float eps, void *Ob, void *workspace, size_t workspace_bytes_given,
                                void *stream)
{
    if (!Qb || !Kb || !Vb || !S || !z || !Ob || !workspace) return SV_ERR_NULL;
    Shape s;
    sv_status rc = check_desc(blk, &s);
    if (rc != SV_OK) return rc;
    if (!eps_ok(eps)) return SV_ERR_RANGE;
    if (!aligned16(Qb) || !aligned16(Kb) || !aligned16(Vb) || !aligned16(Ob) || !aligned16(S) || !aligned16(z) ||
        !aligned16(workspace))
        return SV_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(s.BH, s.d)) return SV_ERR_WORKSPACE;
    auto hs = static_cast<hipStream_t>(stream);
    rc = enqueue_state(Kb, Vb, s, 0, s.N, 1, S, z, static_cast<float *>(workspace), hs);
    if (rc != SV_OK) return rc;
    return enqueue_apply(Qb, s, 0, s.N, S, z, eps, Ob, hs);
}

const char *sv_status_string(int status)
{
    switch (status) {
    case SV_OK: return "ok";
    case SV_ERR_NULL: return "null pointer";
    case SV_ERR_SHAPE: return "bad shape or strides";
    case SV_ERR_UNSUPPORTED: return "unsupported head dim or dtype";
    case SV_ERR_ALIGN: return "pointer or stride not 16-byte aligned";
    case SV_ERR_RANGE: return "token range or eps out of range";
    case SV_ERR_WORKSPACE: return "workspace too small";
    case SV_ERR_LAUNCH: return "HIP launch error";
    default: return "unknown status";
    }
}

int sv_version(void) { return kVersion; }

}  // extern "C"
