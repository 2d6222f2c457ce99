/*
 * sv_linattn.h - C ABI of the MI355X (gfx950) ReLU linear-attention library.
 *
 * The library computes, per (batch, head) pair independently,
 *
 *     phi(x) = max(x, 0)
 *     S[k][v] = sum_j phi(K[j][k]) * V[j][v]        (d x d attention state)
 *     z[k]    = sum_j phi(K[j][k])                  (key sum)
 *     O[i][v] = (sum_k phi(Q[i][k]) S[k][v]) / (sum_k phi(Q[i][k]) z[k] + eps)
 *
 * which is the right-hand form of the linear-attention equation of Sec. 3.2 of
 * the SANA-Video paper (arXiv 2509.24695) without RoPE, and its block-causal
 * re-formulation of Sec. 3.3.1 in which earlier blocks enter only through the
 * carried S and z (the constant-memory cache of Alg. 1).  eps is not in the
 * paper's equations; it is added to the denominator after the dot product.
 *
 * Conventions common to every entry point
 *  - All data pointers (Q, K, V, O, S, z, workspace) are DEVICE pointers on the
 *    current HIP device.  Descriptors are HOST pointers and are read before the
 *    call returns.  The library never allocates, frees or keeps a pointer.
 *  - Token tensors are [B][H][N][d] with d contiguous; the other three strides
 *    are given in elements.  Pointers must be 16-byte aligned and the strides
 *    multiples of 16 bytes.  d must be 32, 64, 112 or 128 (112 is the head
 *    dimension of the paper's 2B model, Appendix model-configuration table).
 *  - S is [B][H][d][d] fp32, row = key feature k, column = value feature v, so
 *    that out = phi(Q) * S.  z is [B][H][d] fp32.  Both dense.
 *  - SV_BF16 tokens: bf16 storage, bf16 MFMA products with fp32 accumulation,
 *    outputs rounded to bf16 (nearest even).  SV_F32: fp32 validation mode,
 *    plain fp32 arithmetic.
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream); nothing synchronises with the host.
 *  - Every argument is checked on the host before anything is launched: a call
 *    that returns an error other than SV_ERR_LAUNCH has not touched S, z or O.
 *  - For fixed arguments the results are bit-reproducible: partial sums over
 *    token chunks are combined in a fixed order, never with float atomics.
 *  - Inputs must be finite; O must not alias Q, K or V.
 *  - Workgroups that wait for each other.  sv_linattn_state and the block steps
 *    split a head's tokens over several workgroups which, when the whole grid fits
 *    the device at once (about one workgroup per compute unit; the library checks
 *    this against the device's capacity and otherwise takes a path of two
 *    launches without waits), exchange their partial sums INSIDE the kernel: each
 *    publishes a flag in the workspace and polls for the others'.  That is only
 *    live if all of a launch's workgroups get to run together, so such a call
 *    needs the device's compute units to itself: do not run it concurrently with
 *    kernels of other streams or processes that may hold compute units for long
 *    (two of these calls on two streams, each with its own workspace, can starve
 *    each other).  Every wait is bounded (2^24 polls, several seconds): no kernel
 *    hangs.  A wait that runs out stores a mark in the workspace
 *    (sv_linattn_workspace_status) and the workgroup stores nothing further - its
 *    part of S, z keeps its old contents, its rows of O are not written - so S, z
 *    and O of that call are then INVALID as a whole (other workgroups may have
 *    stored their parts) and a carried state must be rebuilt or restored by the
 *    caller.  Callers that cannot rule out contention check the status at their
 *    synchronisation points.
 *  - The first call on a device queries it and raises kernel LDS limits (function
 *    attributes).  Make one call (sv_linattn_workspace_init will do) before
 *    capturing a stream into a HIP graph; later calls only enqueue kernels.
 */
#ifndef SV_LINATTN_H
#define SV_LINATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SV_OK = 0,
    SV_ERR_NULL = 1,        /* a required pointer is NULL                           */
    SV_ERR_SHAPE = 2,       /* B, H, N <= 0, stride_n < d, or strides under which two
                               (batch, head, token) rows share memory: taken in
                               ascending order, each stride of an axis longer than 1
                               must be >= stride * extent of the axis below it     */
    SV_ERR_UNSUPPORTED = 3, /* d not in {32, 64, 112, 128} or unknown dtype          */
    SV_ERR_ALIGN = 4,       /* pointer or stride not a multiple of 16 bytes          */
    SV_ERR_RANGE = 5,       /* token range outside [0, N], or eps negative/non-finite */
    SV_ERR_WORKSPACE = 6,   /* workspace smaller than sv_linattn_workspace_bytes()   */
    SV_ERR_LAUNCH = 7       /* HIP reported an error while enqueuing                  */
} sv_status;

typedef enum { SV_BF16 = 0, SV_F32 = 1 } sv_dtype;

/* Describes one token tensor (Q, K, V and O of a call share one descriptor). */
typedef struct {
    int32_t B, H, N, d;     /* N = tokens addressable through the pointer            */
    int64_t stride_b;       /* elements between batches                               */
    int64_t stride_h;       /* elements between heads                                 */
    int64_t stride_n;       /* elements between tokens (>= d)                         */
    int32_t dtype;          /* sv_dtype                                               */
} sv_tensor_desc;

/* Bytes of device workspace that sv_linattn_state / sv_block_linattn_step need
 * for a call over n_tokens tokens per head.  Pure host function.  The value
 * depends on B*H and d only (it is an upper bound over n_tokens), so a stream
 * of blocks of any length reuses one allocation: the library-attributable
 * memory of block-causal generation is this plus S and z, independent of the
 * video length (Sec. 3.3.1, cost table).  Returns 0 for unsupported arguments. */
size_t sv_linattn_workspace_bytes(int32_t B, int32_t H, int32_t n_tokens, int32_t d);

/* Optional: prepares a workspace for calls that are recorded into a HIP graph.
 * (For callers that replay captured launches; no passage of the paper.)
 * sv_linattn_state and the block steps tag their cross-workgroup flags with an
 * epoch that the host draws afresh for every call and passes as a kernel
 * argument; a captured launch replays with the SAME argument, and a replay would
 * mistake the flags of the previous replay for its own.  After this call (one
 * tiny kernel on `stream`; it must have completed, in stream order, before the
 * workspace is used) the kernels draw their epochs from a counter inside the
 * workspace instead, so the same launches may be captured once and replayed any
 * number of times.  The call also clears every flag and the timeout mark of the
 * workspace, so it may be repeated, and a workspace may be re-initialised after
 * its memory served something else.  B, H, d as given to
 * sv_linattn_workspace_bytes.  The
 * workspace must then serve one stream at a time (as always), and a graph must be
 * replayed with the workspace it was captured with.  Eager calls work with or
 * without initialisation. */
sv_status sv_linattn_workspace_init(void *workspace, size_t workspace_bytes,
                                    int32_t B, int32_t H, int32_t d, void *stream);

/* Where the workspace records that an in-kernel wait ran out (see "Workgroups
 * that wait for each other" above; for callers that monitor the library, no
 * passage of the paper): byte offset of an 8-byte word inside a workspace for
 * B, H, d.  Pure host function; 0 for unsupported arguments.  The word holds
 * 0x54494d454f555421 after a timeout and anything else otherwise (the contents of
 * a fresh workspace are undefined and need not be cleared for this);
 * sv_linattn_workspace_init resets it. */
size_t sv_linattn_workspace_status_offset(int32_t B, int32_t H, int32_t d);

/* Reads that word: *timed_out (HOST pointer) = 1 if a wait of any call that used
 * this workspace has run out since the workspace was allocated or last
 * initialised, else 0.  Unlike every other call this one SYNCHRONISES: it copies
 * the word on `stream` and waits for the stream, so it sees all earlier work of
 * that stream.  Errors: SV_ERR_NULL, SV_ERR_SHAPE, SV_ERR_UNSUPPORTED,
 * SV_ERR_ALIGN, SV_ERR_WORKSPACE as for sv_linattn_workspace_init; SV_ERR_LAUNCH if
 * the copy failed. */
sv_status sv_linattn_workspace_status(const void *workspace, size_t workspace_bytes,
                                      int32_t B, int32_t H, int32_t d, void *stream,
                                      int32_t *timed_out);

/* Bound of the in-kernel waits, in polls (roughly 100 ns each), for all later
 * calls of this process: a negative value restores the default (2^24).  0 makes
 * every wait fail at once, which is how the tests exercise the timeout path
 * without a kernel that hangs: the kernels still run to their end, store the
 * timeout mark and leave S, z and O alone.  (For tests and for callers that want
 * a tighter bound; no passage of the paper.) */
void sv_linattn_set_wait_limit(int64_t polls);

/* State reduction (numerator and denominator brackets of the Sec. 3.2 equation;
 * S_j and the key sum of Sec. 3.3.1) over tokens [tok_begin, tok_end):
 *     accumulate == 0:  S, z  = sums            (overwritten)
 *     accumulate != 0:  S, z += sums            (carried state updated in place)
 * An empty range zero-fills (accumulate == 0) or leaves S, z unchanged.
 * The token range is split over workgroups; their fp32 partial sums go through
 * `workspace` and are combined in chunk order. */
sv_status sv_linattn_state(const void *K, const void *V, const sv_tensor_desc *kv,
                           int32_t tok_begin, int32_t tok_end, int accumulate,
                           float *S, float *z,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Apply (Sec. 3.2 equation, right-hand form; Sec. 3.3.1 first equality):
 *     O[b][h][i][:] = phi(Q[b][h][i][:]) S[b][h] / (phi(Q[b][h][i][:]) . z[b][h] + eps)
 * for i in [tok_begin, tok_end); other rows of O are not written.  O has the
 * descriptor's shape, strides and dtype.  A row whose phi(Q) is all zero gives
 * exactly 0 (0 / eps), never NaN, for eps > 0. */
sv_status sv_linattn_apply(const void *Q, const sv_tensor_desc *q,
                           int32_t tok_begin, int32_t tok_end,
                           const float *S, const float *z, float eps,
                           void *O, void *stream);

/* One block of block-causal generation (Sec. 3.3.1; the cache update and use of
 * Alg. 1): fold the block's keys and values into the carried state,
 *     S += phi(K_b)^T V_b,   z += sum phi(K_b),
 * then emit O_b from the UPDATED state, so that attention is full inside the
 * block and causal towards earlier blocks.  `blk` describes Q_b, K_b, V_b and
 * O_b (all N tokens of the descriptor form the block).  S and z are read and
 * written in place; starting from all-zero S, z gives the first block. */
sv_status sv_block_linattn_step(const void *Qb, const void *Kb, const void *Vb,
                                const sv_tensor_desc *blk,
                                float *S, float *z, float eps, void *Ob,
                                void *workspace, size_t workspace_bytes, void *stream);

/* sv_block_linattn_step for callers that cannot allocate device memory at all -
 * code inside a HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc - and so cannot bring a workspace: the same step, same kernels and
 * same results (bit for bit), with the workspace taken from an array of
 * SV_STATIC_SCRATCH_BYTES that is part of the library's device code.  Each GPU
 * the library runs on holds that array from the moment the library is loaded on
 * it until the process ends.  The call allocates and frees nothing; its first
 * use on a device looks the array's address up (no allocation either).
 *  - Limit: sv_linattn_workspace_bytes(B, H, N, d) must not exceed
 *    SV_STATIC_SCRATCH_BYTES, else SV_ERR_WORKSPACE (checked before anything is
 *    launched): B*H <= 91 at d = 64, <= 30 at d = 112, <= 23 at d = 128.
 *  - All calls on one GPU share the one array, whichever stream they use: two
 *    calls whose kernels overlap in time (different streams, or one stream and a
 *    replaying graph) race on it and give wrong results.  Calls on one stream
 *    are ordered and safe.  The array keeps what the last call left; nothing in it
 *    has to start out as zero (flags are told apart by a fresh tag per call).
 *  - A captured call replays with the tag of the capture, so a graph that holds
 *    this call may be replayed only if no other use of the array, this entry
 *    point included, ran in between.  Callers that replay graphs freely take
 *    sv_block_linattn_step with a workspace prepared by sv_linattn_workspace_init.
 *  - The timeout mark of the in-kernel waits cannot be read for this array; use
 *    sv_block_linattn_step where that matters.
 * Other arguments, checks and errors as sv_block_linattn_step; SV_ERR_LAUNCH also
 * if the array's address cannot be obtained. */
#define SV_STATIC_SCRATCH_BYTES (48u << 20)
sv_status sv_block_linattn_step_static(const void *Qb, const void *Kb, const void *Vb,
                                       const sv_tensor_desc *blk,
                                       float *S, float *z, float eps, void *Ob, void *stream);

/* The same block WITHOUT committing it (the noisy denoising passes of Alg. 1:
 * G(x; t_j, KV) attends to the cache plus the block itself, and only the final
 * pass at t = 0 updates the cache):
 *     O_b = phi(Q_b) (S + phi(K_b)^T V_b) / (phi(Q_b) (z + sum phi(K_b)) + eps)
 * S and z are read only; the updated state exists only inside `workspace`
 * during the call.  Same arguments, checks and errors as sv_block_linattn_step. */
sv_status sv_block_linattn_lookahead(const void *Qb, const void *Kb, const void *Vb,
                                     const sv_tensor_desc *blk,
                                     const float *S, const float *z, float eps, void *Ob,
                                     void *workspace, size_t workspace_bytes, void *stream);

/* ---- RoPE variants: the full linear-attention equation of Sec. 3.2 ----------------
 *
 *     O_i = RoPE(phi(Q_i)) (sum_j RoPE(phi(K_j))^T V_j) / (phi(Q_i) (sum_j phi(K_j)^T) + eps)
 *
 * RoPE is applied AFTER the ReLU and only in the numerator; the denominator keeps
 * the un-rotated features so that it stays positive.  `rope` is a DEVICE pointer
 * to fp32 [N][d/2][2]: row t belongs to token t of the descriptor (for a block
 * step: token t of the block) and holds, per feature pair p = (2p, 2p+1), the
 * cosine and sine of that pair's angle:
 *     y[2p] = x[2p] cos - x[2p+1] sin,    y[2p+1] = x[2p] sin + x[2p+1] cos.
 * One table serves all batches and heads.  How angles derive from a token's
 * (frame, row, column) position is up to the caller (the paper names "3D RoPE"
 * without frequencies).  The table must be 16-byte aligned and not NULL.  S then
 * holds the state of ROTATED keys; z, the key sum, is never rotated.  In SV_BF16
 * mode rotated features are rounded to bf16 before the MFMA.  Everything else
 * (arguments, checks, errors, determinism) is as in the call without _rope. */
sv_status sv_linattn_state_rope(const void *K, const void *V, const sv_tensor_desc *kv,
                                const float *rope, int32_t tok_begin, int32_t tok_end,
                                int accumulate, float *S, float *z,
                                void *workspace, size_t workspace_bytes, void *stream);

sv_status sv_linattn_apply_rope(const void *Q, const sv_tensor_desc *q, const float *rope,
                                int32_t tok_begin, int32_t tok_end,
                                const float *S, const float *z, float eps,
                                void *O, void *stream);

sv_status sv_block_linattn_step_rope(const void *Qb, const void *Kb, const void *Vb,
                                     const sv_tensor_desc *blk, const float *rope,
                                     float *S, float *z, float eps, void *Ob,
                                     void *workspace, size_t workspace_bytes, void *stream);

sv_status sv_block_linattn_lookahead_rope(const void *Qb, const void *Kb, const void *Vb,
                                          const sv_tensor_desc *blk, const float *rope,
                                          const float *S, const float *z, float eps, void *Ob,
                                          void *workspace, size_t workspace_bytes, void *stream);

/* ---- RoPE variants with factored 3-D tables ------------------------------------------
 *
 * The same equation as the _rope calls, for the usual 3-D rotary embedding in
 * which feature pair p is turned by ONE coordinate of the token: its frame, its
 * row or its column.  Token t of the descriptor (of the block, for a step) sits at
 *     frame t / (rows*cols),  row (t / cols) % rows,  column t % cols,
 * so frames*rows*cols must equal the descriptor's N.  Pairs [0, n_t) follow the
 * frame, pairs [n_t, n_t + n_h) the row, pairs [n_t + n_h, d/2) the column
 * (n_t + n_h + n_w = d/2); cs_t, cs_h, cs_w are DEVICE pointers to fp32
 * [frames][n_t][2], [rows][n_h][2], [cols][n_w][2] = (cos, sin), 8-byte
 * aligned, NULL allowed for an axis with no pairs.  For a block stream the
 * caller passes, per block, the frame table of that block's frames (the time
 * axis continues across blocks) and the same row and column tables.
 * The three tables are a few KB and stay on chip during the call: unlike a full
 * [N][d/2][2] table they add nothing to the token streams.  The descriptor is a
 * HOST pointer, read before the call returns.  Results equal those of the _rope
 * calls on the expanded table. */
typedef struct {
    int32_t frames, rows, cols;
    int32_t n_t, n_h, n_w;
    const float *cs_t, *cs_h, *cs_w;
} sv_rope3d;

sv_status sv_linattn_state_rope3d(const void *K, const void *V, const sv_tensor_desc *kv,
                                  const sv_rope3d *rope, int32_t tok_begin, int32_t tok_end,
                                  int accumulate, float *S, float *z,
                                  void *workspace, size_t workspace_bytes, void *stream);

sv_status sv_linattn_apply_rope3d(const void *Q, const sv_tensor_desc *q, const sv_rope3d *rope,
                                  int32_t tok_begin, int32_t tok_end,
                                  const float *S, const float *z, float eps,
                                  void *O, void *stream);

sv_status sv_block_linattn_step_rope3d(const void *Qb, const void *Kb, const void *Vb,
                                       const sv_tensor_desc *blk, const sv_rope3d *rope,
                                       float *S, float *z, float eps, void *Ob,
                                       void *workspace, size_t workspace_bytes, void *stream);

sv_status sv_block_linattn_lookahead_rope3d(const void *Qb, const void *Kb, const void *Vb,
                                            const sv_tensor_desc *blk, const sv_rope3d *rope,
                                            const float *S, const float *z, float eps, void *Ob,
                                            void *workspace, size_t workspace_bytes, void *stream);

/* Human-readable name of a status code (static storage). */
const char *sv_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int sv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SV_LINATTN_H */
