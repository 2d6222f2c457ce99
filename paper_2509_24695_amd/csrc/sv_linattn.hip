// C ABI of the gfx950 linear-attention library: argument checks, launch plans,
// kernel dispatch.  See include/sv_linattn.h for the contract of each call.
#include "../../include/sv_linattn.h"
#include "../../include/sv_measure.h"

#include <hip/hip_runtime.h>
#include <math.h>

#include <atomic>
#include <chrono>
#include <mutex>
#include <type_traits>

#include "apply_mfma.hpp"
#include "block_step_fused.hpp"
#include "coop128.hpp"
#include "common.hpp"
#include "generic_kernels.hpp"
#include "state_mfma.hpp"
#include "wide_state.hpp"

namespace {

using namespace sv;

constexpr int kVersion = 500;   // 0.5.0

// Tuned launch shapes of the bf16 MFMA kernels (one workgroup per compute unit).
// DP = 64 serves d = 64; DP = 128 serves d = 112 and 128.  Depths are tiles in
// flight per wave (by RoPE mode: none, table, 3-D, where they differ).
constexpr int kStateTile = 32, kStateWaves = 4, kApplyWaves = 4;
constexpr int kCoopApplyWaves = 4, kCoopApplyNB = 1;   // d = 112/128 apply: one 128 x 32 panel of S per wave, two workgroups per compute unit
constexpr int kStateDepth = 2, kApplyDepth = 2;
// 16-token tiles in flight per wave of the wave-private d = 112/128 state kernel: three, or two with the
// factored rotation tables (that form is bound by its arithmetic and needs the registers)
constexpr int kWideStateDepth = 3, kWideStateDepth3D = 2;
constexpr int kCoopStateDepth = 4;            // 32-token tiles of the shared-tile d = 112/128 state kernel (full-table RoPE)
constexpr int kFusedStateDepth[3] = {2, 2, 2};   // one-launch block step (d = 64), by RoPE mode
constexpr int kFusedApplyDepth[3] = {6, 2, 6};   // Q tiles held in registers across the in-kernel waits
constexpr bool kApplyHiLo = true;
// d = 64: the denominators phi(Q_i).z ride through the matrix core as two more operand rows (false) or are taken on
// the vector ALU with a wavefront-level reduction (true).  Measured level (within 1 % either way at 32 760 and
// 75 600 tokens; the one-launch block step 0.5-1 us per block slower with the vector ALU form), so they stay on
// the matrix core; sv_measure_apply_variant runs both forms side by side.
constexpr bool kDenValu = false;
constexpr int kDies = 8, kCusPerDie = 32;      // MI355X: 8 accelerator dies (XCDs) of 32 compute units, one L2 each
constexpr uint32_t kSpinLimit = 1u << 24;      // polls of ~100 ns: far beyond any real wait
std::atomic<uint32_t> g_spin_limit{kSpinLimit};  // sv_linattn_set_wait_limit
uint32_t spin_limit() { return g_spin_limit.load(std::memory_order_relaxed); }
std::atomic<int> g_assumed_dies{kDies};          // sv_measure_assume_dies

struct Shape {
    int B, H, N, d, BH;
    TokStrides st;
    bool bf16;
    int elem_bytes;
    bool host_epochs_only = false;   // the workspace is the library's own static array (see next_epoch)
};

struct Device {
    int num_cu = 0;
    // how many workgroups fit on the device at once, [DP = 128][RoPE mode]
    int state_resident_wgs[2][3] = {{0, 0, 0}, {0, 0, 0}};   // state kernel with in-kernel finalize
    int fused_resident_wgs[3] = {0, 0, 0};                   // one-launch block step (d = 64), by RoPE mode
    bool ok = false;
};

// The kernels in use, by padded head dimension and RoPE mode.  LDS sizes include the room for the
// factored tables where the mode needs it.
template <int DP, int ROPE> struct Kernels;
template <int ROPE> struct Kernels<64, ROPE> {
    static constexpr int kTab = ROPE == kRope3D ? kRope3dLdsBytes : 0;
    static constexpr int W = 0;
    static constexpr auto state = state_mfma_d64<kStateTile, kStateWaves, kStateDepth, true, ROPE>;
    static constexpr auto state_partial = state_mfma_d64<kStateTile, kStateWaves, kStateDepth, false, ROPE>;
    static constexpr auto apply = apply_mfma_d64<kApplyHiLo, kApplyWaves, kApplyDepth, ROPE, false, kDenValu>;
    static constexpr auto fused = block_step_mfma<kStateTile, kStateWaves, kFusedStateDepth[ROPE], kApplyHiLo,
                                                  kFusedApplyDepth[ROPE], ROPE, false, kDenValu>;
    static constexpr auto fused_local = block_step_mfma<kStateTile, kStateWaves, kFusedStateDepth[ROPE], kApplyHiLo,
                                                        kFusedApplyDepth[ROPE], ROPE, true, kDenValu>;
    static constexpr int state_lds = state_lds_bytes<kStateTile, kStateWaves>() + kTab;
    static constexpr int apply_lds = apply_lds_bytes<kApplyWaves, ROPE>() + kTab;
    static constexpr int fused_lds = block_step_lds_bytes<kStateTile, kStateWaves, ROPE>() + kTab;
    // tokens one workgroup covers per round of its tile walk
    static constexpr int state_wg_tokens = kStateTile * kStateWaves;
    static constexpr int fused_wg_tokens = state_wg_tokens;
    static constexpr int apply_wg_tokens = kApplyTile * kApplyWaves;
    static constexpr int apply_threads = 64 * kApplyWaves;
    // workgroups launched per compute unit: the plain kernel's are short-lived and queue up (see apply_mfma_d64);
    // the RoPE kernels hold more registers and, with factored tables, fill their tables per workgroup
    static constexpr int apply_wgs_per_cu = ROPE == kRopeNone ? 8 : 1;
    static constexpr int apply_wgs_per_cu_short = apply_wgs_per_cu, apply_short_steps = 0;   // no other form for short ranges
};
template <int ROPE> struct Kernels<128, ROPE> {
    static constexpr int W = 1;
    static constexpr int kTab = ROPE == kRope3D ? kRope3dLdsBytes : 0;
    // State: wave-private tiles, except with a full rotation table, whose rows need the registers
    // the wave-private kernel spends on the whole 128 x 128 state (then: one tile shared by the four waves).
    static constexpr bool kWideState = ROPE != kRopeTable;
    template <bool FINALIZE> static constexpr auto pick_state() {
        if constexpr (kWideState) return &state_mfma_wide<(ROPE == kRope3D ? kWideStateDepth3D : kWideStateDepth), FINALIZE, ROPE>;
        else return &state_mfma_d128<kCoopStateDepth, FINALIZE, ROPE>;
    }
    static constexpr auto state = pick_state<true>();
    static constexpr auto state_partial = pick_state<false>();
    static constexpr auto apply = apply_mfma_d128<kApplyHiLo, kApplyDepth, ROPE, kCoopApplyWaves, kCoopApplyNB>;
    static constexpr int state_lds = kWideState ? kWideLdsBytes : state_d128_lds_bytes<ROPE>() + kTab;
    static constexpr int apply_lds = coop_apply_lds_bytes<kCoopApplyWaves, kCoopApplyNB>() + kTab;
    static constexpr int state_wg_tokens = kWideState ? 4 * kWideTile : 32;   // four private tiles, or one shared
    static constexpr int apply_wg_tokens = 8 * kCoopApplyWaves * kCoopApplyNB;   // the waves of a workgroup share its tiles
    static constexpr int apply_threads = 64 * kCoopApplyWaves;
    // workgroups per compute unit: with one 128 x 32 panel per wave (136-164 registers, 17-50 KB of LDS) three are
    // resident; with a full rotation table two (three measured 98 against 89 us: its rows crowd the caches)
    static constexpr int apply_wgs_per_cu = kCoopApplyNB != 1 ? 8 / (kCoopApplyWaves * kCoopApplyNB) : ROPE == kRopeTable ? 2 : 3;
    // ranges of fewer than apply_short_steps steps per workgroup: two per compute unit (see enqueue_apply)
    static constexpr int apply_wgs_per_cu_short = apply_wgs_per_cu < 2 ? apply_wgs_per_cu : 2, apply_short_steps = 6;
};

template <int DP, int ROPE> void init_kernels(Device &d)
{
    using KN = Kernels<DP, ROPE>;
    const auto attr = hipFuncAttributeMaxDynamicSharedMemorySize;
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(KN::state), attr, KN::state_lds);
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(KN::state_partial), attr, KN::state_lds);
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(KN::apply), attr, KN::apply_lds);
    int per_cu = 0;
    if constexpr (DP == 64) {                      // the one-launch block step exists for d = 64 only
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(KN::fused), attr, KN::fused_lds);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(KN::fused_local), attr, KN::fused_lds);
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(KN::fused),
                                                         64 * kStateWaves, KN::fused_lds) != hipSuccess)
            per_cu = 0;
        d.fused_resident_wgs[ROPE] = per_cu * d.num_cu;
        per_cu = 0;
    }
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(KN::state),
                                                     64 * kStateWaves, KN::state_lds) != hipSuccess)
        per_cu = 0;
    d.state_resident_wgs[KN::W][ROPE] = per_cu * d.num_cu;
}

// Calls f(Kernels<DP, ROPE>{}) for the MFMA kernel family that serves head dimension d and RoPE mode.
template <typename F> void with_mfma_kernels(int d, int rope_mode, F &&f)
{
    if (d == 64) {
        if (rope_mode == kRope3D) f(Kernels<64, kRope3D>{});
        else if (rope_mode == kRopeTable) f(Kernels<64, kRopeTable>{});
        else f(Kernels<64, kRopeNone>{});
    } else {
        if (rope_mode == kRope3D) f(Kernels<128, kRope3D>{});
        else if (rope_mode == kRopeTable) f(Kernels<128, kRopeTable>{});
        else f(Kernels<128, kRopeNone>{});
    }
}

// The rotation a call asks for, validated.
struct Rope {
    int mode = kRopeNone;
    RopeArg arg{};
};

// Switches a workspace to device-side epochs and clears its error word.  The ticket counters restart at
// zero, so the epochs drawn from them repeat those of an earlier life of the same memory: every flag word
// is cleared too (no device epoch is ever 0), or a flag left behind by that earlier life could pass for
// one of the first launch after this.
__global__ void workspace_header_init(unsigned long long *flags, size_t n_flags, unsigned long long *error,
                                      unsigned long long *magic, unsigned long long *tickets, int BH)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x, first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (size_t i = first; i < n_flags; i += stride) flags[i] = 0ull;
    for (size_t i = first; i < (size_t)BH; i += stride) tickets[i] = 0ull;
    if (first == 0) {
        *error = 0ull;
        *magic = kWsMagic;
    }
}

bool head_dim_ok(int d) { return d == 32 || d == 64 || d == 112 || d == 128; }

// Calls f(std::integral_constant<int, D>) for the supported head dimension d.
template <typename F> void with_head_dim(int d, F &&f)
{
    switch (d) {
    case 32: f(std::integral_constant<int, 32>{}); break;
    case 64: f(std::integral_constant<int, 64>{}); break;
    case 112: f(std::integral_constant<int, 112>{}); break;
    default: f(std::integral_constant<int, 128>{}); break;
    }
}

// Per-device facts, queried once (no device memory is touched).
const Device &device_info()
{
    static Device devs[64];
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        static Device bad;
        return bad;
    }
    std::lock_guard<std::mutex> lock(mu);
    Device &d = devs[dev];
    if (!d.ok) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return d;
        d.num_cu = prop.multiProcessorCount;
        init_kernels<64, kRopeNone>(d);
        init_kernels<64, kRopeTable>(d);
        init_kernels<64, kRope3D>(d);
        init_kernels<128, kRopeNone>(d);
        init_kernels<128, kRopeTable>(d);
        init_kernels<128, kRope3D>(d);
        for (int hd : {32, 64, 112, 128})          // the larger generic apply kernels need more than 64 KB of LDS
            with_head_dim(hd, [&](auto D) {
                const auto attr = hipFuncAttributeMaxDynamicSharedMemorySize;
                (void)hipFuncSetAttribute(reinterpret_cast<const void *>(apply_generic<uint16_t, D()>), attr,
                                          apply_generic_lds_bytes<D()>());
                (void)hipFuncSetAttribute(reinterpret_cast<const void *>(apply_generic<float, D()>), attr,
                                          apply_generic_lds_bytes<D()>());
            });
        (void)hipGetLastError();
        d.ok = d.num_cu > 0;
    }
    return d;
}

// Fresh 64-bit tag for the workspace's flags; unique per call within the process
// and seeded from the clock so that stale workspace contents of an earlier
// process do not look current.
unsigned long long next_epoch(bool host_epochs_only = false)
{
    static std::atomic<unsigned long long> ctr{
        (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count() * 0x9E3779B97F4A7C15ull};
    // odd, never zero, never repeated (2^62 calls apart); the top bit is the kernels' kHostEpochsOnly
    const unsigned long long e = ((ctr.fetch_add(1, std::memory_order_relaxed) << 1) | 1ull) & ~kHostEpochsOnly;
    return host_epochs_only ? e | kHostEpochsOnly : e;
}

// Token chunks (workgroups) per head: about one workgroup per compute unit over
// the whole grid, never more than kMaxChunks (which sizes the workspace) or
// than there are tiles.
int plan_chunks(int BH, int n_tokens, int tokens_per_wg_step, int num_cu)
{
    if (n_tokens <= 0) return 0;
    const int steps = (n_tokens + tokens_per_wg_step - 1) / tokens_per_wg_step;
    int chunks = num_cu / BH;
    if (chunks > kMaxChunks) chunks = kMaxChunks;
    if (chunks > steps) chunks = steps;
    if (chunks < 1) chunks = 1;
    return chunks;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

sv_status check_desc(const sv_tensor_desc *t, Shape *s)
{
    if (!t) return SV_ERR_NULL;
    if (t->dtype != SV_BF16 && t->dtype != SV_F32) return SV_ERR_UNSUPPORTED;
    if (!head_dim_ok(t->d)) return SV_ERR_UNSUPPORTED;
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
    // No two (b, h, n) rows may share memory (O rows would overwrite each other): taken in order of
    // ascending stride, every axis with more than one index must step over all that the axes below it span.
    struct Axis { int64_t stride, extent; } ax[3] = {{t->stride_b, t->B}, {t->stride_h, t->H}, {t->stride_n, t->N}};
    for (int i = 0; i < 3; ++i)
        for (int j = i + 1; j < 3; ++j)
            if (ax[j].stride < ax[i].stride) { const Axis x = ax[i]; ax[i] = ax[j]; ax[j] = x; }
    int64_t span = t->d;                             // elements covered by the axes handled so far
    for (const Axis &a : ax) {
        if (a.extent <= 1) continue;
        if (a.stride < span) return SV_ERR_SHAPE;
        if (a.stride > INT64_MAX / a.extent) return SV_ERR_SHAPE;
        span = a.stride * a.extent;
    }
    return SV_OK;
}

// The MFMA kernels address a head's tokens (and the rotation table) with 32-bit byte offsets.
bool mfma_path(const Shape &s, const Rope &rope)
{
    constexpr int64_t kLimit = int64_t(1) << 31;
    if (!s.bf16 || s.d < 64 || (int64_t)s.N * s.st.n * 2 >= kLimit) return false;
    if (rope.mode == kRopeTable && (int64_t)s.N * s.d * 4 >= kLimit) return false;
    if (rope.mode == kRope3D) {            // the three tables must fit the LDS set aside for them
        const Rope3D &r = rope.arg.r3;
        if ((int64_t)rope3d_entries(r.frames, r.rows, r.cols, r.n_t, r.n_h, r.n_w) * 8 > kRope3dLdsBytes) return false;
        // positions are carried in 24-bit multiplies and fp32 reciprocals there
        if (r.frames >= (1 << 20) || r.rows >= (1 << 20) || r.cols >= (1 << 20)) return false;
    }
    return true;
}

sv_status check_range(const Shape &s, int32_t t0, int32_t t1)
{
    return (t0 < 0 || t1 < t0 || t1 > s.N) ? SV_ERR_RANGE : SV_OK;
}

size_t workspace_bytes(int BH, int d) { return ws_total_bytes(BH, d * d + d); }

sv_status launch_status() { return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_LAUNCH; }

bool eps_ok(float eps) { return isfinite(eps) && eps >= 0.f; }

// S_out, z_out = (S_in, z_in, or 0 when S_in is null) + state of tokens [t0,t1).  S_in may equal S_out.
// rope: rotation table or null.  All arguments are already validated.
void launch_state_mfma(const uint16_t *k, const uint16_t *v, const Rope &rope, const Shape &s, int t0, int t1,
                       const float *S_in, const float *z_in, float *S_out, float *z_out, void *ws, const Device &dev,
                       dim3 rgrid, hipStream_t stream)
{
    with_mfma_kernels(s.d, rope.mode, [&](auto kn) {
        using KN = decltype(kn);
        const int C = plan_chunks(s.BH, t1 - t0, KN::state_wg_tokens, dev.num_cu);
        if ((int64_t)C * s.BH <= dev.state_resident_wgs[KN::W][rope.mode]) {
            // the head's workgroups wait for each other inside the kernel: all must be resident
            KN::state<<<dim3(C, s.BH), 64 * kStateWaves, KN::state_lds, stream>>>(
                k, v, rope.arg, s.st, s.H, s.d, t0, t1, C, S_in, z_in, S_out, z_out, ws, next_epoch(s.host_epochs_only),
                spin_limit());
        } else {
            KN::state_partial<<<dim3(C, s.BH), 64 * kStateWaves, KN::state_lds, stream>>>(
                k, v, rope.arg, s.st, s.H, s.d, t0, t1, C, S_in, z_in, S_out, z_out, ws, 0ull, 0u);
            with_head_dim(s.d, [&](auto D) {
                state_reduce<D()><<<rgrid, kThreads, 0, stream>>>(static_cast<float *>(ws), C, kMaxChunks, S_in, z_in,
                                                                 S_out, z_out);
            });
        }
    });
}

sv_status enqueue_state(const void *K, const void *V, const Rope &rope, const Shape &s, int t0, int t1,
                        const float *S_in, const float *z_in, float *S_out, float *z_out, void *ws,
                        hipStream_t stream)
{
    const int n = t1 - t0;
    if (n == 0 && S_in == S_out) return SV_OK;
    const Device &dev = device_info();
    if (!dev.ok) return SV_ERR_LAUNCH;
    const int E = s.d * s.d + s.d;
    const dim3 rgrid((E + kThreads - 1) / kThreads, s.BH);
    float *wsf = static_cast<float *>(ws);
    if (n == 0) {                                   // the empty sum: zero fill, or a copy of the carried state
        with_head_dim(s.d, [&](auto D) {
            state_reduce<D()><<<rgrid, kThreads, 0, stream>>>(wsf, 0, 0, S_in, z_in, S_out, z_out);
        });
        return launch_status();
    }
    if (mfma_path(s, rope)) {
        launch_state_mfma(static_cast<const uint16_t *>(K), static_cast<const uint16_t *>(V), rope, s, t0, t1, S_in,
                          z_in, S_out, z_out, ws, dev, rgrid, stream);
        return launch_status();
    }
    // fp32 validation mode, bf16 d = 32 and oversized heads: plain-FMA partials, then the fixed-order reduction
    const int C = plan_chunks(s.BH, n, 32, 2 * dev.num_cu);
    const dim3 grid(C, s.BH);
    with_head_dim(s.d, [&](auto D) {
        if (s.bf16)
            state_partial_generic<uint16_t, D()><<<grid, kThreads, 0, stream>>>(
                static_cast<const uint16_t *>(K), static_cast<const uint16_t *>(V), rope.arg, rope.mode, s.st, s.H, t0, t1,
                C, wsf);
        else
            state_partial_generic<float, D()><<<grid, kThreads, 0, stream>>>(
                static_cast<const float *>(K), static_cast<const float *>(V), rope.arg, rope.mode, s.st, s.H, t0, t1, C,
                wsf);
        state_reduce<D()><<<rgrid, kThreads, 0, stream>>>(wsf, C, C, S_in, z_in, S_out, z_out);
    });
    return launch_status();
}

sv_status enqueue_apply(const void *Q, const Rope &rope, const Shape &s, int t0, int t1, const float *S,
                        const float *z, float eps, void *O, hipStream_t stream)
{
    const int n = t1 - t0;
    if (n == 0) return SV_OK;
    const Device &dev = device_info();
    if (!dev.ok) return SV_ERR_LAUNCH;
    if (mfma_path(s, rope)) {
        with_mfma_kernels(s.d, rope.mode, [&](auto kn) {
            using KN = decltype(kn);
            int C = KN::apply_wgs_per_cu * dev.num_cu / s.BH;
            const int steps = (n + KN::apply_wg_tokens - 1) / KN::apply_wg_tokens;
            // Short ranges: every workgroup starts by fetching its panels of S, so with only a few steps each,
            // fewer and longer ones win (d = 112, 20 heads, 4 680 tokens: two per compute unit 15.1 against
            // 15.8-16.2 us with three; level at 10 800 tokens, three ahead from there on).
            if (KN::apply_wgs_per_cu_short < KN::apply_wgs_per_cu && steps < KN::apply_short_steps * C)
                C = KN::apply_wgs_per_cu_short * dev.num_cu / s.BH;
            if (C > steps) C = steps;
            // Full rotation table: consecutive workgroup ids go round the dies, so with a multiple of the die
            // count per head, workgroup c of every head runs on die c mod 8 and the table rows of its tiles
            // reach that die's L2 only (d = 112, 20 heads: 25 chunks per head put every row into all eight,
            // 24 measured 81 against 88 us).  Taken when it costs at most a tenth of the workgroups.
            if (rope.mode == kRopeTable && (C - C % kDies) * 10 >= C * 9) C -= C % kDies;
            if (C < 1) C = 1;
            KN::apply<<<dim3(C, s.BH), KN::apply_threads, KN::apply_lds, stream>>>(
                static_cast<const uint16_t *>(Q), static_cast<uint16_t *>(O), rope.arg, s.st, s.H, s.d, t0, t1, C, S,
                z, eps);
        });
        return launch_status();
    }
    const int tile = kThreads / (s.d / 4);          // generic tiles: 256 threads / (d/4 threads per token)
    int C = (4 * dev.num_cu + s.BH - 1) / s.BH;
    const int n_tiles = (n + tile - 1) / tile;
    if (C > n_tiles) C = n_tiles;
    const dim3 grid(C, s.BH);
    with_head_dim(s.d, [&](auto D) {
        constexpr int lds = apply_generic_lds_bytes<D()>();
        if (s.bf16)
            apply_generic<uint16_t, D()><<<grid, kThreads, lds, stream>>>(
                static_cast<const uint16_t *>(Q), static_cast<uint16_t *>(O), rope.arg, rope.mode, s.st, s.H, t0, t1, C,
                S, z, eps);
        else
            apply_generic<float, D()><<<grid, kThreads, lds, stream>>>(
                static_cast<const float *>(Q), static_cast<float *>(O), rope.arg, rope.mode, s.st, s.H, t0, t1, C, S, z,
                eps);
    });
    return launch_status();
}

// ---- bodies shared by the plain and the RoPE entry points ------------------------------------------------------

// What an entry point was given: nothing, a full table, or factored 3-D tables.
struct RopeSpec {
    int mode;
    const float *table;
    const sv_rope3d *r3;
};
constexpr RopeSpec kNoRope{kRopeNone, nullptr, nullptr};

// Checks the rotation arguments against the descriptor and fills `out`.
sv_status resolve_rope(const RopeSpec &spec, const Shape &s, Rope *out)
{
    out->mode = spec.mode;
    if (spec.mode == kRopeTable) {
        if (!spec.table) return SV_ERR_NULL;
        if (!aligned16(spec.table)) return SV_ERR_ALIGN;
        out->arg.table = spec.table;
    } else if (spec.mode == kRope3D) {
        const sv_rope3d *r = spec.r3;
        if (!r) return SV_ERR_NULL;
        if (r->frames <= 0 || r->rows <= 0 || r->cols <= 0 || r->n_t < 0 || r->n_h < 0 || r->n_w < 0)
            return SV_ERR_SHAPE;
        if ((int64_t)r->frames * r->rows * r->cols != s.N || r->n_t + r->n_h + r->n_w != s.d / 2) return SV_ERR_SHAPE;
        if ((r->n_t > 0 && !r->cs_t) || (r->n_h > 0 && !r->cs_h) || (r->n_w > 0 && !r->cs_w)) return SV_ERR_NULL;
        if ((reinterpret_cast<uintptr_t>(r->cs_t) | reinterpret_cast<uintptr_t>(r->cs_h) |
             reinterpret_cast<uintptr_t>(r->cs_w)) & 7u)
            return SV_ERR_ALIGN;
        out->arg.r3 = Rope3D{r->cs_t, r->cs_h, r->cs_w, r->frames, r->rows, r->cols, r->n_t, r->n_h, r->n_w};
    }
    return SV_OK;
}

sv_status do_state(const void *K, const void *V, const sv_tensor_desc *kv, const RopeSpec &spec, int32_t tok_begin,
                   int32_t tok_end, int accumulate, float *S, float *z, void *workspace,
                   size_t workspace_bytes_given, void *stream)
{
    if (!K || !V || !S || !z || !workspace) return SV_ERR_NULL;
    Shape s;
    sv_status rc = check_desc(kv, &s);
    if (rc != SV_OK) return rc;
    if ((rc = check_range(s, tok_begin, tok_end)) != SV_OK) return rc;
    Rope rope;
    if ((rc = resolve_rope(spec, s, &rope)) != SV_OK) return rc;
    if (!aligned16(K) || !aligned16(V) || !aligned16(S) || !aligned16(z) || !aligned16(workspace)) return SV_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(s.BH, s.d)) return SV_ERR_WORKSPACE;
    return enqueue_state(K, V, rope, s, tok_begin, tok_end, accumulate ? S : nullptr, z, S, z, workspace,
                         static_cast<hipStream_t>(stream));
}

sv_status do_apply(const void *Q, const sv_tensor_desc *q, const RopeSpec &spec, int32_t tok_begin, int32_t tok_end,
                   const float *S, const float *z, float eps, void *O, void *stream)
{
    if (!Q || !S || !z || !O) return SV_ERR_NULL;
    Shape s;
    sv_status rc = check_desc(q, &s);
    if (rc != SV_OK) return rc;
    if ((rc = check_range(s, tok_begin, tok_end)) != SV_OK) return rc;
    if (!eps_ok(eps)) return SV_ERR_RANGE;
    Rope rope;
    if ((rc = resolve_rope(spec, s, &rope)) != SV_OK) return rc;
    if (!aligned16(Q) || !aligned16(O) || !aligned16(S) || !aligned16(z)) return SV_ERR_ALIGN;
    return enqueue_apply(Q, rope, s, tok_begin, tok_end, S, z, eps, O, static_cast<hipStream_t>(stream));
}

// The committing and the look-ahead block step: the updated state goes to S_out, z_out.
sv_status do_block_step(const void *Qb, const void *Kb, const void *Vb, const sv_tensor_desc *blk,
                        const RopeSpec &spec, const float *S_in, const float *z_in, float *S_out, float *z_out,
                        bool lookahead, float eps, void *Ob, void *workspace, size_t workspace_bytes_given,
                        void *stream, bool static_workspace = false)
{
    if (!Qb || !Kb || !Vb || !S_in || !z_in || !Ob || !workspace) return SV_ERR_NULL;
    Shape s;
    sv_status rc = check_desc(blk, &s);
    if (rc != SV_OK) return rc;
    s.host_epochs_only = static_workspace;
    if (!eps_ok(eps)) return SV_ERR_RANGE;
    Rope rope;
    if ((rc = resolve_rope(spec, s, &rope)) != SV_OK) return rc;
    if (!aligned16(Qb) || !aligned16(Kb) || !aligned16(Vb) || !aligned16(Ob) || !aligned16(S_in) ||
        !aligned16(z_in) || !aligned16(workspace))
        return SV_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(s.BH, s.d)) return SV_ERR_WORKSPACE;
    if (lookahead) {                                 // the updated state lives in the workspace only
        S_out = ws_lookahead(workspace, s.BH, s.d * s.d + s.d);
        z_out = S_out + (size_t)s.BH * s.d * s.d;
    }
    auto hs = static_cast<hipStream_t>(stream);
    if (mfma_path(s, rope) && s.d == 64) {             // one launch; d = 112, 128 are faster as two (measured)
        const Device &dev = device_info();
        if (!dev.ok) return SV_ERR_LAUNCH;
        bool launched = false;
        auto launch = [&](auto kn) {
            using KN = decltype(kn);
            // One launch when the whole grid can be resident at once (needed by the in-kernel waits).
            const int C = plan_chunks(s.BH, s.N, KN::fused_wg_tokens, dev.num_cu);
            if ((int64_t)C * s.BH > dev.fused_resident_wgs[rope.mode]) return;
            // Die-local form: consecutive workgroup ids go round the device's dies, so with B*H a multiple of the
            // die count every head can have all its workgroups on one die and agree on its state through that
            // die's L2 (23.2 against 24.4 us per 4 680-token block, 38.8 against 40.1 us per 10 800-token block).
            // The kernels check the placement themselves (a head spread over two dies gives up, like a wait
            // that ran out); devices other than the 8 x 32 compute-unit part keep the general form.
            // A full rotation table stays with the general form: there die c reads chunk c of every head, so each
            // table row reaches one L2 only; with whole heads on a die all eight would fetch every row.
            const int dies = g_assumed_dies.load(std::memory_order_relaxed);
            if (dev.num_cu == kDies * kCusPerDie && s.BH % dies == 0 && rope.mode != kRopeTable)
                KN::fused_local<<<dim3(C * s.BH), 64 * kStateWaves, KN::fused_lds, hs>>>(
                    static_cast<const uint16_t *>(Qb), static_cast<const uint16_t *>(Kb),
                    static_cast<const uint16_t *>(Vb), static_cast<uint16_t *>(Ob), rope.arg, s.st, s.H, s.N, C, S_in,
                    z_in, S_out, z_out, eps, workspace, next_epoch(s.host_epochs_only), spin_limit(), s.BH, dies);
            else
                KN::fused<<<dim3(C, s.BH), 64 * kStateWaves, KN::fused_lds, hs>>>(
                    static_cast<const uint16_t *>(Qb), static_cast<const uint16_t *>(Kb),
                    static_cast<const uint16_t *>(Vb), static_cast<uint16_t *>(Ob), rope.arg, s.st, s.H, s.N, C, S_in,
                    z_in, S_out, z_out, eps, workspace, next_epoch(s.host_epochs_only), spin_limit(), s.BH, 0);
            launched = true;
        };
        if (rope.mode == kRope3D) launch(Kernels<64, kRope3D>{});
        else if (rope.mode == kRopeTable) launch(Kernels<64, kRopeTable>{});
        else launch(Kernels<64, kRopeNone>{});
        if (launched) return launch_status();
    }
    rc = enqueue_state(Kb, Vb, rope, s, 0, s.N, S_in, z_in, S_out, z_out, workspace, hs);
    if (rc != SV_OK) return rc;
    return enqueue_apply(Qb, rope, s, 0, s.N, S_out, z_out, eps, Ob, hs);
}

// ---- the workspace of sv_block_linattn_step_static: a file-scope device array ----------------------------------
// Every GPU that loads the library holds its own copy until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress; the address that kernels and other HIP calls get is the
// one that call returns, looked up once per device with that device current.
constexpr size_t kStaticScratchBytes = SV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

void *static_scratch()
{
    static void *ptrs[64] = {};
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptrs[dev] = p;
    }
    return ptrs[dev];
}

}  // namespace

extern "C" {

size_t sv_linattn_workspace_bytes(int32_t B, int32_t H, int32_t n_tokens, int32_t d)
{
    if (B <= 0 || H <= 0 || n_tokens < 0 || !head_dim_ok(d)) return 0;
    if ((int64_t)B * H > 65535) return 0;
    return workspace_bytes(B * H, d);
}

sv_status sv_linattn_workspace_init(void *workspace, size_t workspace_bytes_given, int32_t B, int32_t H, int32_t d,
                                    void *stream)
{
    if (!workspace) return SV_ERR_NULL;
    if (B <= 0 || H <= 0 || (int64_t)B * H > 65535) return SV_ERR_SHAPE;
    if (!head_dim_ok(d)) return SV_ERR_UNSUPPORTED;
    if (!aligned16(workspace)) return SV_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(B * H, d)) return SV_ERR_WORKSPACE;
    const int BH = B * H, elems = d * d + d;
    const size_t n_flags = (size_t)BH * 2 * kMaxChunks;
    const size_t wgs = (n_flags + kThreads - 1) / kThreads;
    workspace_header_init<<<(unsigned)(wgs < 1024 ? wgs : 1024), kThreads, 0, static_cast<hipStream_t>(stream)>>>(
        ws_flag_base(workspace, BH, elems), n_flags, ws_error(workspace, BH, elems), ws_magic(workspace, BH, elems),
        ws_tickets(workspace, BH, elems), BH);
    return launch_status();
}

void sv_linattn_set_wait_limit(int64_t polls)
{
    g_spin_limit.store(polls < 0 ? kSpinLimit : polls > 0xffffffffll ? 0xffffffffu : (uint32_t)polls,
                       std::memory_order_relaxed);
}

size_t sv_linattn_workspace_status_offset(int32_t B, int32_t H, int32_t d)
{
    if (B <= 0 || H <= 0 || (int64_t)B * H > 65535 || !head_dim_ok(d)) return 0;
    return ws_error_offset(B * H, d * d + d);
}

sv_status sv_linattn_workspace_status(const void *workspace, size_t workspace_bytes_given, int32_t B, int32_t H,
                                      int32_t d, void *stream, int32_t *timed_out)
{
    if (!workspace || !timed_out) return SV_ERR_NULL;
    if (B <= 0 || H <= 0 || (int64_t)B * H > 65535) return SV_ERR_SHAPE;
    if (!head_dim_ok(d)) return SV_ERR_UNSUPPORTED;
    if (!aligned16(workspace)) return SV_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(B * H, d)) return SV_ERR_WORKSPACE;
    unsigned long long word = 0;
    auto hs = static_cast<hipStream_t>(stream);
    const unsigned char *src = static_cast<const unsigned char *>(workspace) + sv_linattn_workspace_status_offset(B, H, d);
    if (hipMemcpyAsync(&word, src, sizeof word, hipMemcpyDeviceToHost, hs) != hipSuccess ||
        hipStreamSynchronize(hs) != hipSuccess) {
        (void)hipGetLastError();
        return SV_ERR_LAUNCH;
    }
    *timed_out = word == kWsTimeoutMark ? 1 : 0;
    return SV_OK;
}

sv_status sv_linattn_state(const void *K, const void *V, const sv_tensor_desc *kv, int32_t tok_begin,
                           int32_t tok_end, int accumulate, float *S, float *z, void *workspace,
                           size_t workspace_bytes_given, void *stream)
{
    return do_state(K, V, kv, kNoRope, tok_begin, tok_end, accumulate, S, z, workspace,
                    workspace_bytes_given, stream);
}

sv_status sv_linattn_apply(const void *Q, const sv_tensor_desc *q, int32_t tok_begin, int32_t tok_end,
                           const float *S, const float *z, float eps, void *O, void *stream)
{
    return do_apply(Q, q, kNoRope, tok_begin, tok_end, S, z, eps, O, stream);
}

sv_status sv_block_linattn_step(const void *Qb, const void *Kb, const void *Vb, const sv_tensor_desc *blk, float *S,
                                float *z, float eps, void *Ob, void *workspace, size_t workspace_bytes_given,
                                void *stream)
{
    return do_block_step(Qb, Kb, Vb, blk, kNoRope, S, z, S, z, false, eps, Ob, workspace,
                         workspace_bytes_given, stream);
}

sv_status sv_block_linattn_step_static(const void *Qb, const void *Kb, const void *Vb, const sv_tensor_desc *blk,
                                       float *S, float *z, float eps, void *Ob, void *stream)
{
    // the size check needs the descriptor only and comes before the first HIP call
    Shape s;
    const sv_status rc = check_desc(blk, &s);
    if (rc != SV_OK) return rc;
    if (workspace_bytes(s.BH, s.d) > kStaticScratchBytes) return SV_ERR_WORKSPACE;
    if (!Qb || !Kb || !Vb || !S || !z || !Ob) return SV_ERR_NULL;
    void *ws = static_scratch();
    if (!ws) return SV_ERR_LAUNCH;
    return do_block_step(Qb, Kb, Vb, blk, kNoRope, S, z, S, z, false, eps, Ob, ws, kStaticScratchBytes, stream, true);
}

sv_status sv_block_linattn_lookahead(const void *Qb, const void *Kb, const void *Vb, const sv_tensor_desc *blk,
                                     const float *S, const float *z, float eps, void *Ob, void *workspace,
                                     size_t workspace_bytes_given, void *stream)
{
    return do_block_step(Qb, Kb, Vb, blk, kNoRope, S, z, nullptr, nullptr, true, eps, Ob, workspace,
                         workspace_bytes_given, stream);
}

sv_status sv_linattn_state_rope(const void *K, const void *V, const sv_tensor_desc *kv, const float *rope,
                                int32_t tok_begin, int32_t tok_end, int accumulate, float *S, float *z,
                                void *workspace, size_t workspace_bytes_given, void *stream)
{
    return do_state(K, V, kv, RopeSpec{kRopeTable, rope, nullptr}, tok_begin, tok_end, accumulate, S, z, workspace, workspace_bytes_given,
                    stream);
}

sv_status sv_linattn_apply_rope(const void *Q, const sv_tensor_desc *q, const float *rope, int32_t tok_begin,
                                int32_t tok_end, const float *S, const float *z, float eps, void *O, void *stream)
{
    return do_apply(Q, q, RopeSpec{kRopeTable, rope, nullptr}, tok_begin, tok_end, S, z, eps, O, stream);
}

sv_status sv_block_linattn_step_rope(const void *Qb, const void *Kb, const void *Vb, const sv_tensor_desc *blk,
                                     const float *rope, float *S, float *z, float eps, void *Ob, void *workspace,
                                     size_t workspace_bytes_given, void *stream)
{
    return do_block_step(Qb, Kb, Vb, blk, RopeSpec{kRopeTable, rope, nullptr}, S, z, S, z, false, eps, Ob, workspace, workspace_bytes_given,
                         stream);
}

sv_status sv_block_linattn_lookahead_rope(const void *Qb, const void *Kb, const void *Vb, const sv_tensor_desc *blk,
                                          const float *rope, const float *S, const float *z, float eps, void *Ob,
                                          void *workspace, size_t workspace_bytes_given, void *stream)
{
    return do_block_step(Qb, Kb, Vb, blk, RopeSpec{kRopeTable, rope, nullptr}, S, z, nullptr, nullptr, true, eps, Ob, workspace,
                         workspace_bytes_given, stream);
}

sv_status sv_linattn_state_rope3d(const void *K, const void *V, const sv_tensor_desc *kv, const sv_rope3d *rope,
                                  int32_t tok_begin, int32_t tok_end, int accumulate, float *S, float *z,
                                  void *workspace, size_t workspace_bytes_given, void *stream)
{
    return do_state(K, V, kv, RopeSpec{kRope3D, nullptr, rope}, tok_begin, tok_end, accumulate, S, z, workspace,
                    workspace_bytes_given, stream);
}

sv_status sv_linattn_apply_rope3d(const void *Q, const sv_tensor_desc *q, const sv_rope3d *rope, int32_t tok_begin,
                                  int32_t tok_end, const float *S, const float *z, float eps, void *O, void *stream)
{
    return do_apply(Q, q, RopeSpec{kRope3D, nullptr, rope}, tok_begin, tok_end, S, z, eps, O, stream);
}

sv_status sv_block_linattn_step_rope3d(const void *Qb, const void *Kb, const void *Vb, const sv_tensor_desc *blk,
                                       const sv_rope3d *rope, float *S, float *z, float eps, void *Ob, void *workspace,
                                       size_t workspace_bytes_given, void *stream)
{
    return do_block_step(Qb, Kb, Vb, blk, RopeSpec{kRope3D, nullptr, rope}, S, z, S, z, false, eps, Ob, workspace,
                         workspace_bytes_given, stream);
}

sv_status sv_block_linattn_lookahead_rope3d(const void *Qb, const void *Kb, const void *Vb,
                                            const sv_tensor_desc *blk, const sv_rope3d *rope, const float *S,
                                            const float *z, float eps, void *Ob, void *workspace,
                                            size_t workspace_bytes_given, void *stream)
{
    return do_block_step(Qb, Kb, Vb, blk, RopeSpec{kRope3D, nullptr, rope}, S, z, nullptr, nullptr, true, eps, Ob,
                         workspace, workspace_bytes_given, stream);
}

void sv_measure_assume_dies(int32_t dies)
{
    g_assumed_dies.store(dies == 1 || dies == 2 || dies == 4 ? dies : kDies, std::memory_order_relaxed);
}

sv_status sv_measure_apply_variant(int32_t variant, const void *Q, const sv_tensor_desc *q, int32_t tok_begin,
                                   int32_t tok_end, const float *S, const float *z, float eps, void *O, void *stream)
{
    if (!Q || !S || !z || !O) return SV_ERR_NULL;
    if (variant < 0 || variant > 3) return SV_ERR_RANGE;
    Shape s;
    sv_status rc = check_desc(q, &s);
    if (rc != SV_OK) return rc;
    if ((rc = check_range(s, tok_begin, tok_end)) != SV_OK) return rc;
    if (!eps_ok(eps)) return SV_ERR_RANGE;
    if (!aligned16(Q) || !aligned16(O) || !aligned16(S) || !aligned16(z)) return SV_ERR_ALIGN;
    Rope none;
    if (s.d != 64 || !mfma_path(s, none)) return SV_ERR_UNSUPPORTED;
    const int n = tok_end - tok_begin;
    if (n == 0) return SV_OK;
    const Device &dev = device_info();
    if (!dev.ok) return SV_ERR_LAUNCH;
    using KN = Kernels<64, kRopeNone>;
    int C = KN::apply_wgs_per_cu * dev.num_cu / s.BH;          // the launch shape of sv_linattn_apply
    const int steps = (n + KN::apply_wg_tokens - 1) / KN::apply_wg_tokens;
    if (C > steps) C = steps;
    if (C < 1) C = 1;
    auto launch = [&](auto kernel, int lds) {
        static_cast<void>(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        kernel<<<dim3(C, s.BH), KN::apply_threads, lds, static_cast<hipStream_t>(stream)>>>(
            static_cast<const uint16_t *>(Q), static_cast<uint16_t *>(O), none.arg, s.st, s.H, s.d, tok_begin, tok_end, C, S, z, eps);
    };
    constexpr int lds0 = KN::apply_lds, lds1 = KN::apply_lds + kApplyStateLdsBytes;
    switch (variant) {
    case 0: launch(apply_mfma_d64<kApplyHiLo, kApplyWaves, kApplyDepth, kRopeNone, false, false>, lds0); break;
    case 1: launch(apply_mfma_d64<kApplyHiLo, kApplyWaves, kApplyDepth, kRopeNone, true, false>, lds1); break;
    case 2: launch(apply_mfma_d64<kApplyHiLo, kApplyWaves, kApplyDepth, kRopeNone, false, true>, lds0); break;
    default: launch(apply_mfma_d64<kApplyHiLo, kApplyWaves, kApplyDepth, kRopeNone, true, true>, lds1); break;
    }
    return launch_status();
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
