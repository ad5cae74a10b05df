/*
 * fdd.h -- C ABI of the MI355X (gfx950) block-diffusion denoise-step library.
 *
 * One denoising step of a section-aligned block, as the paper describes it:
 *   - block-causal attention (Preliminaries, "Block-Causal Diffusion"): a
 *     block attends bidirectionally to itself and causally to the prompt and
 *     all earlier blocks, whose KV cache is reused without recomputation
 *     ("Section Diffusion (SD)");
 *   - N rollouts forked from one shared KV cache (test-time scaling section,
 *     "Shared prefix"): every rollout owns a private block and they all read
 *     the single prefix, which is never copied per rollout;
 *   - confidence-threshold unmasking of still-masked value positions, with
 *     the structural scaffold frozen (Eq. 2 and the scaffold construction
 *     paragraph; "iteratively unmasks value positions").
 *
 * Conventions common to every call
 *   - Every data pointer is a DEVICE pointer owned by the caller (HBM of the
 *     current HIP device); the parameter structs themselves live on the host.
 *     The library allocates no device memory, never copies the prefix and
 *     never synchronises.  Work is enqueued on `stream` (a hipStream_t passed
 *     as void*; NULL = the default stream) and the call returns at once.
 *   - Arrays are dense, row-major, in the index order written next to them.
 *   - The return code covers what the host can see: NULL pointers, shapes,
 *     element type, workspace size, launch failure.  On error nothing is
 *     launched and fdd_last_error() holds a message (thread-local).
 *   - Inputs are never modified, except arrays documented as in/out.
 *   - Scratch (`workspace`) must be at least what the matching
 *     *_workspace() call returns for the same params, 256-byte aligned;
 *     its contents before and after a call are unspecified.  Calls that
 *     share a workspace must be ordered on one stream.
 */
#ifndef FDD_H
#define FDD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FDD_OK = 0,
    FDD_ERR_NULL = 1,        /* a required pointer is NULL */
    FDD_ERR_SHAPE = 2,       /* non-positive size, Hq % Hkv != 0, ... */
    FDD_ERR_DTYPE = 3,       /* element type not FDD_F32 / FDD_BF16 */
    FDD_ERR_UNSUPPORTED = 4, /* head size or option outside the supported set */
    FDD_ERR_WORKSPACE = 5,   /* workspace missing, misaligned or too small */
    FDD_ERR_LAUNCH = 6       /* the HIP runtime refused a launch */
} fdd_status;

typedef enum { FDD_F32 = 0, FDD_BF16 = 1 } fdd_dtype;

/* ------------------------------------------------------------------------
 * fdd_block_attn: shared-prefix block-causal attention for N rollouts.
 *
 * For rollout n, block position b, query head h (KV head kh = h / (Hq/Hkv)):
 *   keys   = prefix_k[0..L) ++ block_k[n, 0..B)      (head kh)
 *   values = prefix_v[0..L) ++ block_v[n, 0..B)
 *   out[n,b,h,:] = softmax(scale * q[n,b,h,:] . keys^T) values
 * Every one of the L+B keys is visible (bidirectional inside the block,
 * causal to the prefix); other rollouts' blocks are not.  This is the
 * attention rule of "Block-Causal Diffusion" applied to rollouts that were
 * forked from one cache ("Shared prefix").  Position encoding is outside
 * this call: q and k arrive already rotated.
 *
 * scaffold_mask does not enter the arithmetic: scaffold tokens are ordinary
 * visible tokens of the block (pre-filled, never masked), both as keys and
 * as queries.  It is accepted so the signature matches the step's problem
 * statement, may be NULL, and the output is the same for any value.
 *
 * dtype FDD_BF16: q/k/v/out are bfloat16, products on the matrix cores with
 * fp32 accumulation, softmax in fp32.  dtype FDD_F32: fp32 storage and
 * arithmetic.  D must be 64 or 128.  L may be 0.  `out` must not alias an
 * input.  splits: number of pieces the prefix is cut into along L
 * (0 = chosen by the library); the result does not depend on it beyond
 * fp32 rounding.
 */
/* In-block attention is causal instead of bidirectional: block position b sees
 * the prefix and block positions <= b of its own rollout.  This is the verify
 * pass of Scaffold Speculative Decoding (paper, "Scaffold Speculative Decoding
 * (SS)", step 3: "a causal forward pass over the entire block"); the draft pass
 * of step 2 is the default bidirectional form. */
#define FDD_ATTN_CAUSAL_BLOCK 1

typedef struct fdd_attn_params {
    int32_t N, B, L, Hq, Hkv, D;
    int32_t dtype;                 /* fdd_dtype of q, k, v and out */
    float scale;                   /* softmax scale; <= 0 selects 1/sqrt(D) */
    const void *q;                 /* [N,B,Hq,D] */
    const void *prefix_k;          /* [L,Hkv,D]  one copy for all rollouts; may be NULL iff L == 0 */
    const void *prefix_v;          /* [L,Hkv,D] */
    const void *block_k;           /* [N,B,Hkv,D] */
    const void *block_v;           /* [N,B,Hkv,D] */
    const uint8_t *scaffold_mask;  /* [N,B] 1 = frozen scaffold token; may be NULL */
    void *out;                     /* [N,B,Hq,D] */
    void *workspace;               /* >= fdd_block_attn_workspace() bytes */
    size_t workspace_bytes;
    void *stream;                  /* hipStream_t */
    int32_t splits;                /* 0 = automatic */
    int32_t flags;                 /* FDD_ATTN_* bits; unknown bits are rejected */
    const void *prefix_v_packed;   /* optional: output of fdd_prefix_pack for this prefix_v, or NULL */
    /* Per-rollout extension: the blocks rollout n has finished since the fork ("Shared prefix": the
     * trajectory section is continued N times and spans several blocks; "Block-Causal Diffusion": a block
     * attends causally to all earlier blocks).  Rows ext[n, 0..E) are keys of rollout n only, between
     * the shared prefix and the live block; they are fully visible, also with FDD_ATTN_CAUSAL_BLOCK.
     * E = 0 (pointers may then be NULL) is the plain two-run form. */
    const void *ext_k;             /* [N, ext_capacity, Hkv, D] */
    const void *ext_v;             /* [N, ext_capacity, Hkv, D] */
    int32_t E;                     /* valid extension rows per rollout, 0 <= E <= ext_capacity */
    int32_t ext_capacity;          /* rows allocated per rollout */
    /* Batch of independent problems of one shape in a single launch (for callers whose problems are each
     * too small to fill the chip: several requests, each with its own prefix).  Problem i uses the arrays
     * at q + i*q_batch_stride, prefix_k/prefix_v + i*prefix_batch_stride, block_k/block_v +
     * i*block_batch_stride, ext_k/ext_v + i*ext_batch_stride, out + i*out_batch_stride (strides in
     * elements, multiples of 8, at least the size of one problem's array) and prefix_v_packed +
     * i*packed_batch_stride (bytes, a multiple of 256).  batch <= 1 is the single problem and the strides
     * are ignored.  Nothing is shared between the problems of a batch. */
    int32_t batch;
    int32_t n_q_positions;         /* 0: every position is computed; see q_positions */
    int64_t q_batch_stride, prefix_batch_stride, block_batch_stride, ext_batch_stride, out_batch_stride;
    size_t packed_batch_stride;
    /* Only some block positions as queries ("Scaffold": scaffold tokens are given, never predicted, so
     * where nothing but the logits of a layer's output is read - the last layer - their rows are not
     * needed).  q_positions is a DEVICE array of n_q_positions flat positions n*B + b in strictly ascending
     * order, each in [0, N*B); the rows out[n, b, :, :] of these positions are computed exactly as without
     * the list, every other row of `out` is left as it was.  Keys are not affected: block_k / block_v
     * still hold all B positions of every rollout.  With `batch`, the one list serves every problem.
     * The library cannot read the list on the host: entries out of range are clamped into it by the
     * kernels (no access out of bounds), an order other than ascending gives undefined values in `out`. */
    const int32_t *q_positions;
} fdd_attn_params;

/* Bytes of scratch fdd_block_attn needs for these params (host-only
 * arithmetic, no device is touched).  Returns 0 if the params are invalid.
 * The figure is smaller when prefix_v_packed is set. */
size_t fdd_block_attn_workspace(const fdd_attn_params *p);
fdd_status fdd_block_attn(const fdd_attn_params *p);

/* ------------------------------------------------------------------------
 * fdd_prefix_pack: one-time relayout of the prefix V for the bf16 kernel.
 *
 * The prefix KV cache does not change while a block is denoised and is shared
 * by all rollouts (paper: KV caches of the prompt and of earlier blocks are
 * reused without recomputation).  The bf16 attention kernel reads the full
 * 64-key tiles of prefix V in an order that has the key index contiguous;
 * when several workgroups stream the same V, fdd_block_attn repacks V into
 * its workspace on every call.  A caller that runs many steps on one prefix
 * can do that once: fdd_prefix_pack writes the repacked copy (a few percent
 * of a step's time) and every later fdd_block_attn on the same prefix takes
 * it through prefix_v_packed.  prefix_v itself must still be passed (the
 * ragged last tile is read from it).  The packed copy belongs to exactly the
 * (prefix_v contents, L, Hkv, D) it was made from.
 *
 * fdd_prefix_pack_bytes: size of the packed copy, 256-byte granular; 0 when
 * nothing would be packed (fp32, or L < 64).  Host-only arithmetic.
 */
size_t fdd_prefix_pack_bytes(int32_t L, int32_t Hkv, int32_t D, int32_t dtype);
fdd_status fdd_prefix_pack(const void *prefix_v, int32_t L, int32_t Hkv, int32_t D, int32_t dtype,
                           void *packed, size_t packed_bytes, void *stream);

/* ------------------------------------------------------------------------
 * fdd_unmask_step: one confidence-threshold unmask iteration over N blocks.
 *
 * A position (n,b) is eligible when mask[n,b] == 1 and scaffold_mask[n,b]
 * == 0: diffusion acts on the editable set only and visible tokens stay
 * fixed (paper, Eq. 2; "Masked Diffusion Language Models").  For every
 * eligible position
 *     cand = lowest id attaining max_v logits[n,b,v]
 *     conf = 1 / sum_v exp(logits[n,b,v] - max)      (largest softmax prob.)
 * Block n commits every eligible position with conf >= tau; if none reaches
 * tau and the block has an eligible position, it commits the eligible
 * position of highest conf (lowest b on ties), so each call makes progress.
 * Committing writes tokens[n,b] = cand and clears mask[n,b].  All other
 * positions of tokens and mask are left as they were; a mask bit set on a
 * scaffold position is ignored (the scaffold wins).
 *
 * Only the logits rows of eligible positions are read.  The arg max is taken
 * on the stored logits (exact); exp and the sum run in fp32.
 *
 * Logits: finite values, and -inf for entries that can never be chosen (their
 * probability is exactly 0; a row needs at least one finite entry).  NaN and
 * +inf are not supported: the outputs of a row that holds one are undefined
 * (nothing is read or written out of bounds).  The same holds for the logits
 * of fdd_verify_step.
 */
typedef struct fdd_unmask_params {
    int32_t N, B;
    int64_t V;
    int32_t dtype;                 /* fdd_dtype of logits */
    float tau;
    const void *logits;            /* [N,B,V] */
    const uint8_t *scaffold_mask;  /* [N,B]; may be NULL (= no scaffold) */
    uint8_t *mask;                 /* [N,B] in/out, 1 = still masked */
    int32_t *tokens;               /* [N,B] in/out */
    float *confidences;            /* [N,B] out: conf of eligible positions, -inf elsewhere */
    int32_t *n_unmasked;           /* [N] out, commits per block; may be NULL */
    uint8_t *committed;            /* [N,B] out, 1 = committed by this call; may be NULL */
    void *workspace;               /* >= fdd_unmask_workspace() bytes */
    size_t workspace_bytes;
    void *stream;
    /* Optional K/V refresh of the positions this call commits, done by the same kernel that takes the
     * commit decisions: exactly what fdd_block_kv_update would do right afterwards with this call's
     * `tokens` and `committed` (one launch less per denoise step).  All four pointers NULL (and the
     * sizes 0): no refresh.  Otherwise all four must be given, 16-byte aligned, with a row of
     * refresh_Hkv * refresh_D elements of refresh_dtype being a multiple of 16 bytes. */
    const void *refresh_table_k;   /* [refresh_T, refresh_Hkv, refresh_D] */
    const void *refresh_table_v;
    void *refresh_block_k;         /* [N, B, refresh_Hkv, refresh_D] in/out */
    void *refresh_block_v;
    int32_t refresh_Hkv, refresh_D, refresh_T;
    int32_t refresh_dtype;         /* fdd_dtype of the tables and the block K/V */
} fdd_unmask_params;

size_t fdd_unmask_workspace(const fdd_unmask_params *p);
fdd_status fdd_unmask_step(const fdd_unmask_params *p);

/* fdd_unmask_step_static: fdd_unmask_step for callers that cannot allocate
 * device memory and carry no workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * results bit for bit; `workspace` and `workspace_bytes` are ignored.  The
 * per-piece partial results of the vocabulary reduction go to a fixed array of
 * FDD_STATIC_SCRATCH_BYTES inside the library's device image instead (every GPU
 * the library runs on holds one copy until the process ends).  The call
 * allocates nothing and frees nothing.  Shapes whose partials do not fit
 * (N*B*pieces > FDD_STATIC_SCRATCH_BYTES / 16, i.e. fdd_unmask_workspace() above
 * that size; 1024 positions over V = 152064 need 64 KiB) are rejected with
 * FDD_ERR_WORKSPACE and nothing is launched.  All calls on one GPU share that
 * GPU's array: two calls that overlap in time on one GPU (different streams,
 * different threads) race and give wrong results; calls ordered on one stream
 * are safe.  Nothing in the array has to be cleared between calls: every
 * record a call reads was written by that call.  The current device must be
 * the one `stream` belongs to.
 */
#define FDD_STATIC_SCRATCH_BYTES ((size_t)1 << 20)
fdd_status fdd_unmask_step_static(const fdd_unmask_params *p);

/* ------------------------------------------------------------------------
 * fdd_verify_step: accept scan of Scaffold Speculative Decoding over N blocks
 * (paper, "Scaffold Speculative Decoding (SS)", steps 1 and 3).
 *
 * Draft positions are those with mask[n,b] == 1 and scaffold_mask[n,b] == 0;
 * scaffold positions are auto-accepted and take no part.  ar_logits[n,b,:] is
 * the AR head's distribution for the token AT position b (the caller applies
 * the usual one-position shift).  Draft positions are visited left to right:
 * while the lowest id attaining max_v ar_logits[n,b,v] equals draft[n,b], the
 * draft is accepted (tokens[n,b] = draft[n,b], mask cleared).  At the first
 * mismatch the AR token replaces the draft (tokens[n,b] = arg max, mask
 * cleared: the one bonus token) and every later draft position of the block
 * is discarded: its mask bit stays 1 and its tokens entry is not touched.
 * n_accepted[n] counts the positions unmasked by this call; accepted[n,b] is
 * 1 for an accepted draft, 2 for the replaced position, 0 otherwise.
 * Only the logits rows of draft positions are read.
 *
 * Sampled verifier (paper, "Trajectory-only stochasticity": in the trajectory
 * section the verifier samples from its softmax, which is what makes forked
 * rollouts differ).  With temperature > 0 the verifier's token at a draft
 * position is a sample of softmax(ar_logits[n,b,:] / temperature) instead of
 * the arg max, drawn by the Gumbel-max rule
 *     token = lowest id attaining max_v key(v),
 *     key(v) = fma(x_v, c, -flog2(-flog2(u_v)))          (binary32 throughout)
 *     c   = (float)(log2(e) / (double)temperature)
 *     u_v = ((r_v >> 9) + 0.5) * 2^-23
 *     r_v = word (v mod 4) of Philox-4x32-10(counter = (v div 4, n*B + b, 0, 0),
 *                                            key = (seed low word, seed high word))
 *     flog2(y) = e + f P(f) for y = m 2^e, m in [1/sqrt 2, sqrt 2), f = m - 1, with
 *                the degree-8 polynomial P listed in csrc/unmask.hip, evaluated
 *                by Horner's rule in fused multiply-adds.
 * Every step is an exactly rounded binary32 operation, so a (seed, row, logits)
 * triple names one token on any conforming implementation.  The same seed
 * gives the same tokens; rollouts differ because their rows n*B + b differ.
 * temperature == 0 selects the greedy verifier; negative or non-finite values
 * are rejected with FDD_ERR_UNSUPPORTED.
 */
typedef struct fdd_verify_params {
    int32_t N, B;
    int64_t V;
    int32_t dtype;                 /* fdd_dtype of ar_logits */
    float temperature;             /* 0 = greedy verifier, > 0 = sampled verifier */
    const void *ar_logits;         /* [N,B,V] */
    const uint8_t *scaffold_mask;  /* [N,B]; may be NULL */
    const int32_t *draft;          /* [N,B] draft tokens (used at draft positions only) */
    uint8_t *mask;                 /* [N,B] in/out */
    int32_t *tokens;               /* [N,B] in/out */
    int32_t *n_accepted;           /* [N] out; may be NULL */
    uint8_t *accepted;             /* [N,B] out; may be NULL */
    void *workspace;               /* >= fdd_verify_workspace() bytes */
    size_t workspace_bytes;
    void *stream;
    uint64_t seed;                 /* sampled verifier: key of the random stream */
} fdd_verify_params;

/* Bytes of scratch for these params (host-only arithmetic; 0 if they are invalid).  The figure depends on
 * `temperature`: the greedy verifier cuts a row into more pieces than the sampled one. */
size_t fdd_verify_workspace(const fdd_verify_params *p);
fdd_status fdd_verify_step(const fdd_verify_params *p);

/* ------------------------------------------------------------------------
 * Rollout-fork bookkeeping ("fork the KV cache N times").
 *
 * fdd_fork_block: dst[n] = src for n in [0,N), `bytes` bytes each: the
 * private per-rollout state (block K/V, tokens, mask) of the forked
 * rollouts.  The prefix is shared by pointer and is not an argument.
 * bytes must be a multiple of 4; src and dst must not overlap.
 */
fdd_status fdd_fork_block(int32_t N, size_t bytes, const void *src, void *dst, void *stream);

/* fdd_block_commit: a finished block joins its rollout's extension,
 * ext_k[n, E..E+B) = block_k[n], ext_v likewise; the caller then passes E + B as
 * the extension length of the next block's attention calls.  E + B must not
 * exceed ext_capacity; pointers 16-byte aligned; the arrays must not overlap. */
typedef struct fdd_commit_params {
    int32_t N, B, Hkv, D;
    int32_t dtype;
    int32_t E;                     /* rows already in the extension */
    int32_t ext_capacity;
    int32_t reserved;              /* must be 0 */
    const void *block_k;           /* [N,B,Hkv,D] */
    const void *block_v;
    void *ext_k;                   /* [N,ext_capacity,Hkv,D] in/out */
    void *ext_v;
    void *stream;
} fdd_commit_params;

fdd_status fdd_block_commit(const fdd_commit_params *p);

/* fdd_traj_mean: trajectory averaging (paper, "Trajectory averaging", the merge
 * equation): out[p] = (1/N) sum_n traj[n,p], p in [0,P), P = waypoints x
 * coordinates.  fp32 in and out; the sum runs over n in ascending order in
 * fp32, so the result is reproducible and within N * 2^-24 relative of the
 * exact mean of the absolute values.  (The jerk-minimizing fit that produces
 * the waypoints of a rollout is not specified by the paper and is not here.) */
fdd_status fdd_traj_mean(int32_t N, int32_t P, const float *traj, float *out, void *stream);

/* fdd_block_kv_update: refresh the K/V rows of positions committed by the
 * last unmask step.  No model is inside this library, so the new row of a
 * position holding token t is row (t mod T) of caller-provided tables: a
 * stand-in for embedding + projection.  Rows of other positions are not
 * touched. */
typedef struct fdd_kv_update_params {
    int32_t N, B, Hkv, D, T;
    int32_t dtype;                 /* fdd_dtype of the tables and the block K/V */
    const int32_t *tokens;         /* [N,B] */
    const uint8_t *committed;      /* [N,B] as written by fdd_unmask_step */
    const void *table_k;           /* [T,Hkv,D] */
    const void *table_v;           /* [T,Hkv,D] */
    void *block_k;                 /* [N,B,Hkv,D] in/out */
    void *block_v;                 /* [N,B,Hkv,D] in/out */
    void *stream;
} fdd_kv_update_params;

fdd_status fdd_block_kv_update(const fdd_kv_update_params *p);

/* ------------------------------------------------------------------------
 * Timing hook for benchmarks.  While set (both non-NULL), every
 * fdd_block_attn call made by this host thread records `start` on the call's
 * stream right before the main attention kernel (after the pre-pass that
 * repacks V, when there is one) and `stop` right after it (before the small
 * merge kernel), so hipEventElapsedTime(start, stop) is that kernel's
 * duration.  Both are hipEvent_t passed as void*, owned by the
 * caller.  Pass NULL, NULL to clear.  Not meant for production loops.
 */
fdd_status fdd_profile_attn_events(void *start, void *stop);

/* Message of the last failing call on this thread ("" if none). */
const char *fdd_last_error(void);
/* major*10000 + minor*100 + patch */
int fdd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FDD_H */
