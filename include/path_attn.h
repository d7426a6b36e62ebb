/*
 * path_attn.h -- C ABI of the PaTH attention hot path for AMD MI355X (gfx950).
 *
 * PaTH attention (paper Sec. 2.2) is causal softmax attention whose logit is
 *
 *     s_ij = scale * q_i^T H_i H_{i-1} ... H_{j+1} k_j ,   H_t = I - beta_t w_t w_t^T ,
 *
 * (j <= i; empty product for j = i), with o_i = sum_j softmax_j(s_ij) v_j and
 * lse_i = log sum_j exp(s_ij).  The library evaluates it with the paper's
 * blockwise algorithm (Sec. 3.2-3.3): per chunk of 64 tokens a UT transform
 * (triangular solve) gives boundary-adjusted queries/keys and the chunk's
 * transition product; a FlashAttention-style right-to-left sweep over key
 * chunks then applies that product to the resident query tile after each
 * chunk.  All arithmetic runs in hand-written gfx950 kernels.
 *
 * Conventions common to every entry point
 *  - Every data pointer is DEVICE memory owned by the caller.  The library
 *    never allocates, frees or synchronises; all kernels are enqueued on
 *    `stream` (a hipStream_t passed as void*, NULL = the null stream).
 *  - Layout: q, k, v, w, o, d_o, dq, dk, dv, dw are contiguous [B, H, L, d];
 *    beta, dbeta, lse are contiguous [B, H, L] (the *_layout and *_varlen entry
 *    points also take [B, L, H, d] and packed sequences).  w and beta are per
 *    token and per head.  No grouped-query sharing.
 *  - dtype `dt` is the storage type of q,k,v,w,beta,o and of all gradients
 *    (PATH_F32: float, PATH_BF16: bfloat16).  lse is always float.
 *  - Arithmetic.  PATH_F32 contracts on fp32 MFMA throughout.  PATH_BF16 accumulates
 *    in fp32 and contracts on 16-bit MFMA with TWO operand types: the softmax
 *    probabilities, the values and d_o are bf16 operands; everything the method
 *    TRANSPORTS -- the query state, the boundary-adjusted keys, the chunk products
 *    I - P, the matrices inside the chunk transform, and in the backward the
 *    gradients of the query state and of the chunk products -- are fp16 operands
 *    (11-bit significand: bf16's 8 bits there put the log-sum-exp 1e-3 .. 3e-3
 *    off; same MFMA rate).
 *  - Range rule for PATH_BF16 (a consequence of the fp16 operands; fp16 ends at
 *    65504, no status code reports a violation): the transitions are contractions
 *    for beta in [0,2], |w| <= 1, so every transported quantity is bounded by the
 *    Euclidean norms of the rows of q and k -- those norms must stay below 65504;
 *    in the backward the state gradients are bounded by
 *    scale * L * max|d_o| * max|v| * max_row|k| and must stay below it too.  Beyond
 *    the bound (or for beta, w outside those ranges, where products can grow with
 *    L) results are UNDEFINED: infinities or NaNs may appear in any output, never
 *    a fault.  Magnitudes below 6e-8 (fp16's smallest subnormal) flush to zero in
 *    the transported operands.  PATH_F32 has fp32's range throughout.
 *  - d must be 64 or 128; any L >= 1 (a ragged last chunk is handled inside).
 *  - `scale` multiplies the finished bilinear form (the paper's logits are
 *    unscaled: pass 1.0f for those); it must be > 0 (else PATH_ERR_UNSUPPORTED).
 *    lse uses the natural logarithm.
 *  - w is used as given (no normalisation), beta as given (no clipping).
 *  - Only causal attention is defined by the method (the transition product
 *    runs along the path j -> i): causal == 0 returns PATH_ERR_UNSUPPORTED.
 *  - `workspace` is caller-owned device scratch of at least
 *    path_attn_workspace_bytes(...) bytes, 256-byte aligned; its contents are
 *    undefined afterwards.  Calls that share a workspace must be ordered on
 *    one stream.
 *  - Errors are reported by return code before anything is launched (bad
 *    arguments) or after a failed launch (PATH_ERR_HIP); the library never
 *    aborts or throws.  Outputs are fully overwritten on PATH_OK.
 *  - Threads: entry points may be called from several host threads at once as
 *    long as the calls use different workspaces (and streams as the caller sees
 *    fit).  The first launch of each kernel instantiation in a process sets a
 *    launch attribute once; that is guarded (std::call_once), so concurrent first
 *    calls are safe.  path_attn_last_error is per thread.
 *  - Determinism: every result except PaTH-FoX's dlog_f is bit-reproducible run
 *    to run (no atomics, fixed summation order).  dlog_f sums its column and row
 *    sums in shared memory in no fixed order: reproducible up to fp32 rounding of
 *    those sums.
 */
#ifndef PATH_ATTN_H
#define PATH_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { PATH_F32 = 0, PATH_BF16 = 1 } path_dtype_t;

/* Layout of the caller's tensors, for the entry points that take one (the others use PATH_LAYOUT_BHLD):
 *   PATH_LAYOUT_BHLD: q, k, v, w, o and gradients [B,H,L,d]; beta, lse, log_f and gradients [B,H,L]
 *   PATH_LAYOUT_BLHD: ...                          [B,L,H,d]; ...                             [B,L,H]
 * (both contiguous, d innermost). */
typedef enum { PATH_LAYOUT_BHLD = 0, PATH_LAYOUT_BLHD = 1 } path_layout_t;

typedef enum {
    PATH_OK = 0,
    PATH_ERR_NULL = 1,        /* a required pointer is NULL                         */
    PATH_ERR_SHAPE = 2,       /* B,H,L < 1, d not in {64,128}, or sizes overflow     */
    PATH_ERR_DTYPE = 3,       /* dt is not PATH_F32 / PATH_BF16                      */
    PATH_ERR_UNSUPPORTED = 4, /* causal == 0, or scale <= 0                          */
    PATH_ERR_WORKSPACE = 5,   /* workspace too small or misaligned                   */
    PATH_ERR_HIP = 6,         /* a kernel launch failed                              */
    PATH_ERR_ALIGN = 7        /* q,k,v,w,o (or a gradient) not 16-byte aligned       */
} path_status_t;

/* Human-readable name of a status code (static storage, never NULL). */
const char* path_status_str(path_status_t status);

/* After an entry point returned PATH_ERR_HIP on this thread: which step failed
 * and the runtime's name for the error, e.g. "forward sweep: hipErrorInvalidValue (1)".
 * The entry points clear, on entry, a runtime error state left behind by other code in
 * the process and note it here ("inherited and cleared on entry: ...") without failing.
 * Thread-local storage owned by the library, never NULL; empty before any such event. */
const char* path_attn_last_error(void);

/* Bytes of device workspace needed by path_attn_fwd (for_backward == 0) or
 * path_attn_bwd (for_backward != 0) for this problem.  Returns 0 for
 * arguments the entry points would reject. */
size_t path_attn_workspace_bytes(int B, int H, int L, int d, path_dtype_t dt, int for_backward);

/* A memory-bounded backward.  path_attn_bwd (and path_attn_fox_bwd, path_attn_bwd_layout, path_attn_varlen_bwd)
 * accept ANY workspace that holds at least one head: every (batch, head) is an independent problem, so with less
 * than path_attn_workspace_bytes(..., 1) the backward passes over the heads in groups of as many as fit -- the
 * same kernels on smaller grids, the same arithmetic, bit-identical gradients; the price is more launches and,
 * for small groups, a GPU that is not filled.  The query states that dominate the workspace (one per (query
 * chunk, key block) pair) are stored only for the group in flight.
 *   path_attn_bwd_workspace_bytes_for_heads: bytes that let `heads` (clamped to B*H) heads pass together;
 *     heads = 1 is the minimum any backward accepts.  0 for arguments the entry points reject.
 *   path_attn_bwd_heads_per_pass: heads per pass a workspace of that size gives (0: too small even for one).
 * The training pair (path_attn_train_*) keeps the states of ALL heads between its two calls and needs the full size. */
size_t path_attn_bwd_workspace_bytes_for_heads(int B, int H, int L, int d, path_dtype_t dt, int heads);
int path_attn_bwd_heads_per_pass(int B, int H, int L, int d, path_dtype_t dt, size_t workspace_bytes);

/* Introspection for tests and profiling: byte offsets, inside the forward
 * workspace, of the five intermediates the chunk-preprocessing kernel (paper
 * Sec. 3.2) hands to the sweep kernel, in this order: boundary-adjusted key
 * tiles, V^T tiles, negated chunk-product tiles (I - P), boundary-adjusted
 * queries (fp32), diagonal-block logits (fp32); offsets[5] = end of the last of them
 * (further regions follow, up to path_attn_workspace_bytes).
 * Returns PATH_ERR_SHAPE / PATH_ERR_DTYPE for arguments the forward rejects. */
path_status_t path_attn_fwd_workspace_layout(int B, int H, int L, int d, path_dtype_t dt,
                                             size_t offsets[6]);

/*
 * Forward (paper Sec. 2.2 definition; Sec. 3.2-3.3 blockwise algorithm).
 *   in : q, k, v, w [B,H,L,d] (dt), beta [B,H,L] (dt)       -- device, read-only
 *   out: o [B,H,L,d] (dt), lse [B,H,L] (float)              -- device
 */
path_status_t path_attn_fwd(const void* q, const void* k, const void* v, const void* w,
                            const void* beta, void* o, float* lse,
                            int B, int H, int L, int d, int causal, float scale,
                            path_dtype_t dt, void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * The two stages of the forward as separate launches, for callers that want
 * to time or overlap them; path_attn_fwd is exactly path_attn_fwd_prep
 * followed by path_attn_fwd_sweep on the same stream and workspace.
 *   prep  (Sec. 3.2): chunk UT transform -> workspace (reads q,k,v,w,beta)
 *   sweep (Sec. 3.3): right-to-left scan over key chunks -> o, lse (reads workspace only)
 * Same argument rules and error codes as path_attn_fwd.
 */
path_status_t path_attn_fwd_prep(const void* q, const void* k, const void* v, const void* w,
                                 const void* beta, int B, int H, int L, int d, path_dtype_t dt,
                                 void* workspace, size_t workspace_bytes, void* stream);
path_status_t path_attn_fwd_sweep(void* o, float* lse, int B, int H, int L, int d, float scale,
                                  path_dtype_t dt, void* workspace, size_t workspace_bytes,
                                  void* stream);

/*
 * Backward of loss = sum(d_o * o) (the paper states no backward; this is the
 * reverse-mode derivative of the forward above, through the chunk transform).
 *   in : q, k, v, w, beta as in the forward; o, lse as the forward wrote them;
 *        d_o [B,H,L,d] (dt)                                  -- device, read-only
 *   out: dq, dk, dv, dw [B,H,L,d] (dt), dbeta [B,H,L] (dt)   -- device
 * dw is the gradient with respect to the w passed in (no projection onto the
 * unit sphere).  Results are bit-reproducible: every sum is taken in a fixed order.
 */
path_status_t path_attn_bwd(const void* q, const void* k, const void* v, const void* w,
                            const void* beta, const void* o, const float* lse, const void* d_o,
                            void* dq, void* dk, void* dv, void* dw, void* dbeta,
                            int B, int H, int L, int d, int causal, float scale,
                            path_dtype_t dt, void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * PaTH-FoX (paper Sec. 2.2, "Extension: PaTH-FoX"): the attention weight of key j for query i
 * gets the extra factor prod_{s=j+1..i} f_s of data-dependent forget gates f_s in (0,1), i.e.
 * the logit becomes  scale * q_i^T H_i ... H_{j+1} k_j + sum_{s=j+1..i} log f_s.
 * log_f [B,H,L] (dt, device, read-only) holds the LOG of the gates (<= 0); everything else as
 * in path_attn_fwd, same workspace size.  lse is the log-sum-exp of the full logits.
 */
path_status_t path_attn_fox_fwd(const void* q, const void* k, const void* v, const void* w,
                                const void* beta, const void* log_f, void* o, float* lse,
                                int B, int H, int L, int d, int causal, float scale,
                                path_dtype_t dt, void* workspace, size_t workspace_bytes,
                                void* stream);

/* Backward of path_attn_fox_fwd: as path_attn_bwd, plus dlog_f [B,H,L] (dt), the gradient with
 * respect to log_f (entry 0 of every head is exactly 0: the first gate lies on no path).
 * Same workspace size as path_attn_bwd. */
path_status_t path_attn_fox_bwd(const void* q, const void* k, const void* v, const void* w,
                                const void* beta, const void* log_f, const void* o, const float* lse,
                                const void* d_o, void* dq, void* dk, void* dv, void* dw, void* dbeta,
                                void* dlog_f, int B, int H, int L, int d, int causal, float scale,
                                path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Training pair: forward and backward of one step that share a workspace, so that the chunk
 * transform (paper Sec. 3.2) and the recurrence of the query states (Sec. 3.3) run once per step
 * instead of once in each: the forward's sweep also writes the states the backward starts from.
 * path_attn_train_fwd
 * computes o and lse exactly as path_attn_fwd (log_f == NULL) or path_attn_fox_fwd (log_f given)
 * do, but in a workspace of the BACKWARD's size (path_attn_workspace_bytes(..., for_backward = 1)),
 * where it leaves the transformed operands and the query states; path_attn_train_bwd then computes the gradients exactly
 * as path_attn_bwd / path_attn_fox_bwd do (dlog_f given iff log_f is), provided that the workspace
 * has not been written since path_attn_train_fwd returned and that q, k, v, w, beta, log_f are the
 * same tensors with the same contents.  The price is that the workspace stays alive between the
 * two calls.  Arguments, layouts and error codes as for the calls they stand in for.
 */
path_status_t path_attn_train_fwd(const void* q, const void* k, const void* v, const void* w,
                                  const void* beta, const void* log_f, void* o, float* lse,
                                  int B, int H, int L, int d, int causal, float scale,
                                  path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);
/* path_attn_train_fwd as two launches, for callers that time or overlap the stages: it is exactly
 * path_attn_train_fwd_prep followed by path_attn_train_fwd_sweep on the same stream and workspace
 * (with_gates != 0 iff log_f was given to the first). */
path_status_t path_attn_train_fwd_prep(const void* q, const void* k, const void* v, const void* w,
                                       const void* beta, const void* log_f, int B, int H, int L, int d,
                                       path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);
path_status_t path_attn_train_fwd_sweep(void* o, float* lse, int with_gates, int B, int H, int L, int d, float scale,
                                        path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);
path_status_t path_attn_train_bwd(const void* q, const void* k, const void* v, const void* w,
                                  const void* beta, const void* log_f, const void* o, const float* lse,
                                  const void* d_o, void* dq, void* dk, void* dv, void* dw, void* dbeta,
                                  void* dlog_f, int B, int H, int L, int d, int causal, float scale,
                                  path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);

/* path_attn_train_bwd in stages, for callers that time them (bench.py brackets each with events): `stages` is a
 * set of PATH_BWD_STAGE_* bits; the selected stages are enqueued in the order of their values.  Calling it with
 * one stage after the other, in that order, is exactly path_attn_train_bwd (which is `stages` = PATH_BWD_STAGE_ALL);
 * a later stage reads what the earlier ones left in the workspace.  Unknown or no bits: PATH_ERR_UNSUPPORTED. */
enum {
    PATH_BWD_STAGE_SCAN = 1,       /* dO tiles and delta; adjoint scan over the key blocks (dQ-side)          */
    PATH_BWD_STAGE_KEYS_NEAR = 2,  /* key-side sums over the query chunks of the key's own super-block       */
    PATH_BWD_STAGE_KEYS_FAR = 4,   /* key-side sums over all queries right of the key's super-block          */
    PATH_BWD_STAGE_DDP = 8,        /* gradients of the super-block products                                  */
    PATH_BWD_STAGE_CHUNK = 16,     /* adjoint of the second level and of the chunk transform: the gradients  */
    PATH_BWD_STAGE_ALL = 31
};
path_status_t path_attn_train_bwd_stages(int stages, const void* q, const void* k, const void* v, const void* w,
                                         const void* beta, const void* log_f, const void* o, const float* lse,
                                         const void* d_o, void* dq, void* dk, void* dv, void* dw, void* dbeta,
                                         void* dlog_f, int B, int H, int L, int d, int causal, float scale,
                                         path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The forward and backward on either layout.  log_f == NULL: plain PaTH (as path_attn_fwd / path_attn_bwd);
 * log_f given: PaTH-FoX (as path_attn_fox_fwd / path_attn_fox_bwd; dlog_f is required iff log_f is).
 * Same workspace sizes, argument rules and error codes; an unknown layout returns PATH_ERR_UNSUPPORTED.
 * The kernels read and write the caller's tensors in place through their strides: nothing is transposed
 * or copied.
 */
path_status_t path_attn_fwd_layout(const void* q, const void* k, const void* v, const void* w,
                                   const void* beta, const void* log_f, void* o, float* lse,
                                   int B, int H, int L, int d, path_layout_t layout, int causal, float scale,
                                   path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);
path_status_t path_attn_bwd_layout(const void* q, const void* k, const void* v, const void* w,
                                   const void* beta, const void* log_f, const void* o, const float* lse,
                                   const void* d_o, void* dq, void* dk, void* dv, void* dw, void* dbeta,
                                   void* dlog_f, int B, int H, int L, int d, path_layout_t layout, int causal,
                                   float scale, path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Variable-length batches: nseq sequences packed along the token axis, q, k, v, w, o and gradients
 * [T,H,d], beta, lse, log_f and gradients [T,H] (T = cu_seqlens[nseq]); sequence s owns the tokens
 * cu_seqlens[s] .. cu_seqlens[s+1]-1 and attends only to itself.  cu_seqlens is a HOST array of nseq+1
 * ints (cu_seqlens[0] = 0, strictly increasing; else PATH_ERR_SHAPE); it is read before the call returns
 * (copied to the head of the workspace on `stream`).
 * The whole batch is ONE set of kernel launches: sequence s is batch entry s of a problem whose workspace
 * arrays are sized for the longest sequence, every kernel takes its bounds from the entry's own length, and
 * workgroups beyond a shorter sequence's end exit at once -- results are bit-identical to calling the
 * fixed-length entry points sequence by sequence on [1,L_s,H,d] tensors.  The workspace must hold
 * path_attn_varlen_workspace_bytes(...) bytes: the sequence table plus path_attn_workspace_bytes(nseq, H,
 * longest length, ...); the backward also accepts less, down to the table plus one head's worth (see the
 * memory-bounded backward above).  log_f / dlog_f as above.
 */
size_t path_attn_varlen_workspace_bytes(const int* cu_seqlens, int nseq, int H, int d, path_dtype_t dt,
                                        int for_backward);
path_status_t path_attn_varlen_fwd(const void* q, const void* k, const void* v, const void* w,
                                   const void* beta, const void* log_f, void* o, float* lse,
                                   const int* cu_seqlens, int nseq, int H, int d, int causal, float scale,
                                   path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);
path_status_t path_attn_varlen_bwd(const void* q, const void* k, const void* v, const void* w,
                                   const void* beta, const void* log_f, const void* o, const float* lse,
                                   const void* d_o, void* dq, void* dk, void* dv, void* dw, void* dbeta,
                                   void* dlog_f, const int* cu_seqlens, int nseq, int H, int d, int causal,
                                   float scale, path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Decode path (paper Sec. 3.4 "Efficient Inference").  Caches are caller-owned device memory,
 * kcache and vcache [B,H,Lmax,d] contiguous in the I/O type dt; position i of a head holds
 * token i.  The key cache holds REFRESHED keys: after t tokens, k_i^(t) = H_t ... H_{i+1} k_i
 * (the section's first equation applied at every arrival), so that attention of q_t over the
 * cache is ordinary softmax attention.  With dt = PATH_BF16 every refresh rounds the stored
 * keys to bf16 again; that rounding is part of the method as the paper runs it.
 *
 * path_key_prefill: fills positions [0, L) of both caches after a prompt of L tokens (the
 * section's key-prefill formula, with suffix products: linear in L).  It reads the forward
 * workspace of the SAME prompt, i.e. call it after path_attn_fwd / path_attn_fwd_prep on
 * (q, k, v, w, beta) with that workspace (device, read-only here); v [B,H,L,d] is copied.
 * Errors: PATH_ERR_SHAPE also for L > Lmax.
 *
 * path_decode_step: one arriving token per (batch, head): q, k, v, w [B,H,d], beta [B,H] (dt,
 * device, read-only).  n = tokens already cached (0 <= n < Lmax).  Refreshes the n cached
 * keys in place, appends k and v at position n, writes o [B,H,d] (dt) and lse [B,H] (fp32,
 * natural log) of the attention of q over the n+1 keys.  workspace: device scratch of
 * path_decode_workspace_bytes(B, H, d) bytes, 256-byte aligned, contents undefined afterwards.
 * Nothing is allocated; all work is enqueued on `stream`.
 */
size_t path_decode_workspace_bytes(int B, int H, int d);
path_status_t path_key_prefill(const void* v, int B, int H, int L, int d, path_dtype_t dt,
                               const void* fwd_workspace, size_t fwd_workspace_bytes,
                               void* kcache, void* vcache, int Lmax, void* stream);
path_status_t path_decode_step(const void* q, const void* k, const void* v, const void* w,
                               const void* beta, void* kcache, void* vcache, int n, int Lmax,
                               void* o, float* lse, int B, int H, int d, float scale,
                               path_dtype_t dt, void* workspace, size_t workspace_bytes,
                               void* stream);

/*
 * PaTH-FoX at decode time (paper Sec. 2.2 "Extension: PaTH-FoX" applied to the decoding step of Sec. 3.4): key i's
 * logit gets sum_{s=i+1..t} log f_s.  The running sums c_i = sum_{s<=i} log f_s of the cached tokens are a third
 * cache, `ccache` [B,H,Lmax] fp32 (natural logarithm, caller-owned device memory like the other two).
 *   path_gate_prefill     fills ccache[.., 0..L) from the prompt's gates log_f [B,H,L] (I/O type).
 *   path_decode_step_fox  path_decode_step with the arriving token's log gate log_f [B,H] (I/O type): uses
 *                         c_n = c_{n-1} + log f_n (c_{-1} = 0), adds c_n - c_i to key i's logit (nothing to the
 *                         token's own) and appends c_n to ccache.  Everything else -- caches, workspace, errors --
 *                         as for path_decode_step.
 */
path_status_t path_gate_prefill(const void* log_f, int B, int H, int L, path_dtype_t dt, float* ccache, int Lmax,
                                void* stream);
path_status_t path_decode_step_fox(const void* q, const void* k, const void* v, const void* w, const void* beta,
                                   const void* log_f, void* kcache, void* vcache, float* ccache, int n, int Lmax,
                                   void* o, float* lse, int B, int H, int d, float scale, path_dtype_t dt,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sequence-parallel forward: ONE device's share of the ring of paper Sec. 3.5 ("context parallelism": the
 * sequence is split into contiguous segments, one per device; a device attends its own segment, then the
 * segments to its left one hop at a time, applying one d x d product per super-block it has passed).  The three
 * calls below are what a device runs; moving the earlier segments' tiles between devices is the caller's
 * business (on one GPU a test walks the segments in turn).  [B,H,L,d] layout, forward only; plain PaTH, or
 * PaTH-FoX with the gates of each segment given to its own path_attn_ring_local (log_f [B,H,L], NULL = plain).
 *
 *   path_attn_ring_local   the device's own segment (L tokens, causal inside it): chunk transform, second level
 *                          and sweep.  Leaves in `state` (path_attn_ring_state_bytes(B,H,L,d) bytes, 16-byte
 *                          aligned, caller-owned device memory) what the sweep holds per query -- the query state,
 *                          now carried to the segment's left edge, the unnormalised output, the running maximum
 *                          and row sum, all fp32 -- and in `workspace` (path_attn_workspace_bytes(B,H,L,d,dt,0))
 *                          the segment's tiles, which devices to the RIGHT need for their hops: the regions of
 *                          the second-level keys, the values and the super-block products (2 L d + ceil(L/1024) d^2
 *                          elements per head).
 *   path_attn_ring_hop     attends the Lq queries of `state` to every key of an EARLIER segment of Lk tokens,
 *                          given as the workspace path_attn_ring_local filled on that segment (same B, H, d, dt),
 *                          and carries the state across that segment.  Hops are made nearest segment first.  Lk
 *                          must be a multiple of 64 (PATH_ERR_SHAPE): only the last segment of a sequence may be
 *                          ragged, and it is nobody's earlier segment.  with_gates != 0: PaTH-FoX (the earlier
 *                          segment's gate sums are in its workspace; every segment of a sequence uses gates or none).
 *   path_attn_ring_finish  o = O / l, lse = m + log l from `state` (after the last hop; for the first segment
 *                          right after path_attn_ring_local).  PaTH-FoX: gates_workspace = the workspace of the
 *                          device's OWN path_attn_ring_local (it holds the segment's gate sums); NULL = plain.
 *
 * With segment lengths that are multiples of 1024 (the second blocking level) the result is bit-identical to
 * path_attn_fwd on the whole sequence: the same tiles, the same products in the same order, the state kept in
 * fp32 between the calls.  Other lengths differ from it by rounding only.  Errors as for path_attn_fwd.
 */
size_t path_attn_ring_state_bytes(int B, int H, int L, int d);
/* Byte offsets and lengths, inside a segment's workspace, of the four regions a hop reads (host arrays of 4):
 * [0] second-level keys, [1] values, [2] super-block products, [3] gate sums (PaTH-FoX only).  A device that
 * receives an earlier segment needs a buffer of path_attn_workspace_bytes(B,H,L,d,dt,0) bytes with these regions
 * filled; the rest of it is never read by path_attn_ring_hop. */
path_status_t path_attn_ring_regions(int B, int H, int L, int d, path_dtype_t dt, size_t offsets[4], size_t bytes[4]);
path_status_t path_attn_ring_local(const void* q, const void* k, const void* v, const void* w, const void* beta,
                                   const void* log_f, void* state, int B, int H, int L, int d, float scale,
                                   path_dtype_t dt, void* workspace, size_t workspace_bytes, void* stream);
path_status_t path_attn_ring_hop(void* state, int B, int H, int Lq, const void* remote_workspace,
                                 size_t remote_workspace_bytes, int Lk, int d, int with_gates, float scale,
                                 path_dtype_t dt, void* stream);
path_status_t path_attn_ring_finish(const void* state, void* o, float* lse, int B, int H, int L, int d,
                                    path_dtype_t dt, const void* gates_workspace, size_t gates_workspace_bytes,
                                    void* stream);

/*
 * Measurement aid, not part of the method: a register-resident chain of 32x32x16 fp16 MFMA products (four
 * independent accumulators per wave, `waves_per_simd` waves on each of the 1024 SIMDs, `iters` x 16 products
 * per wave, no memory traffic inside the loop) for calibrating "percent of peak" against what the matrix pipes
 * deliver at the clock they actually hold.  It enqueues one kernel on `stream`; the caller times it.  The work is
 * path_probe_mfma_flops(waves_per_simd, iters) floating-point operations.  `sink` is device memory of at least
 * 1024 * 4 * 64 * 4 bytes (one float per lane), written with values nobody needs.  waves_per_simd must be 1, 2
 * or 4 and iters >= 1 (else PATH_ERR_SHAPE).
 */
double path_probe_mfma_flops(int waves_per_simd, int iters);
path_status_t path_probe_mfma(void* sink, int waves_per_simd, int iters, void* stream);
/*
 * The same chain with a choice of operands.  random_operands = 0: smooth, slowly varying values (what
 * path_probe_mfma runs); != 0: fp16 values of random sign, random significand and magnitudes 0.25 .. 4, the kind
 * of operands the method's kernels multiply.  The products draw more power on those, the chip holds a lower
 * clock, and the rate drops from about 2.1 to about 1.6 PFLOP/s: the second figure is the practical ceiling of an
 * MFMA-bound kernel on real data.
 */
path_status_t path_probe_mfma_operands(void* sink, int waves_per_simd, int iters, int random_operands, void* stream);

/*
 * path_decode_step for callers that cannot allocate or pass scratch memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results (bit for bit) and error
 * codes as path_decode_step, minus the workspace: the per-split partial results go to a device array of
 * PATH_DECODE_STATIC_BYTES (8 MiB) that is part of the library's image -- every GPU the library runs on
 * holds one copy until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating
 * library routine); on its first use on a device it looks the array's address up once.
 *   Limit: path_decode_workspace_bytes(B, H, d) <= PATH_DECODE_STATIC_BYTES, i.e. B*H <= 252 at d = 128 and
 *   B*H <= 496 at d = 64; beyond it PATH_ERR_WORKSPACE (the reason is in path_attn_last_error()).
 *   All calls on one GPU share the one array, which keeps the previous call's contents (nothing in it has to
 *   start at zero: every record is written before it is read).  Calls that may overlap on one GPU -- different
 *   streams without an ordering between them, or several host threads -- RACE on it: order them.
 * path_decode_static_scratch_bytes returns PATH_DECODE_STATIC_BYTES.
 */
#define PATH_DECODE_STATIC_BYTES (8u * 1024u * 1024u)
size_t path_decode_static_scratch_bytes(void);
path_status_t path_decode_step_static(const void* q, const void* k, const void* v, const void* w,
                                      const void* beta, void* kcache, void* vcache, int n, int Lmax,
                                      void* o, float* lse, int B, int H, int d, float scale,
                                      path_dtype_t dt, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PATH_ATTN_H */
