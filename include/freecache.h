/*
 * freecache.h - C ABI of the FreeCache cached denoising layer-step for MI355X (gfx950).
 *
 * FreeCache (paper section 3.2.1) keeps, per transformer layer, the K/V projections of the
 * prompt and of the already committed blocks, re-projects only the rows of the active window at
 * each denoising step, overwrites exactly those rows of the cache, and lets the window's queries
 * attend bidirectionally over the whole cached sequence.  One such step per layer is what this
 * library computes; Table 1 of the paper gives its cost rows (projection O(A d^2), QK^T and
 * score x V O(A L d/h), with A the window size instead of the full length L).
 *
 * Conventions
 *  - "device" pointers are HIP device memory of the current device; "host" pointers are ordinary
 *    host memory.  Unless a function says otherwise, every pointer argument is borrowed: the
 *    library keeps no reference after the enqueued work has run.
 *  - Element type of all tensors is fc_config.dtype (float or bfloat16, the latter as raw 16-bit
 *    words), except pos (int32) and the workspace (opaque bytes).
 *  - Compute entry points only enqueue work on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream).  They never synchronise, never allocate and clear no memory with a memset
 *    node, so a caller may record them into a HIP graph on a capturing stream and replay it; what
 *    a replay reads (x, pos, the cache, tokens) is read anew, the scalar arguments (win_start, A,
 *    kv_len) are fixed at capture.  Two calls on one stream execute in order; the attention of a
 *    step relies on this to see the step's fresh K/V rows.
 *  - All argument checks happen on the host before any HIP call.  On failure a nonzero fc_status is
 *    returned, nothing has been enqueued, and fc_last_error() describes the problem.  No entry
 *    point aborts or throws across the ABI.
 *  - Calls on distinct caches are independent.  One cache must not be used from two streams at
 *    the same time.
 */
#ifndef FREECACHE_H
#define FREECACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FC_OK = 0,
    FC_ERR_INVALID_ARG = 1, /* NULL where a pointer is required, non-positive size, bad enum */
    FC_ERR_BOUNDS = 2,      /* layer, window or kv_len outside the cache */
    FC_ERR_UNSUPPORTED = 3, /* shape the kernels do not cover (see fc_config) */
    FC_ERR_OOM = 4,         /* the library could not allocate cache storage */
    FC_ERR_WORKSPACE = 5,   /* workspace missing or smaller than fc_workspace_bytes() */
    FC_ERR_HIP = 6          /* a HIP call or kernel launch failed */
} fc_status;

typedef enum { FC_F32 = 0, FC_BF16 = 1 } fc_dtype;

/* Geometry of one model's attention layers.
 * Supported: head_dim 64 or 128; n_q_heads a multiple of n_kv_heads (query head h reads KV head
 * h / (n_q_heads / n_kv_heads)); hidden a multiple of 8; max_seq up to 2^24 rows. */
typedef struct {
    int32_t n_layers;
    int32_t batch;        /* B: sequences held by the cache */
    int32_t hidden;       /* d: width of the layer input */
    int32_t n_q_heads;    /* Hq */
    int32_t n_kv_heads;   /* Hkv */
    int32_t head_dim;     /* Dh */
    int32_t max_seq;      /* Smax: cache capacity in rows per sequence */
    int32_t dtype;        /* fc_dtype */
    float rope_base;      /* rotary base, e.g. 10000 */
    float softmax_scale;  /* 0 selects 1/sqrt(head_dim) */
} fc_config;

typedef struct fc_cache fc_cache; /* opaque */

/* Thread-local description of the last failure on the calling thread ("" if none). */
const char *fc_last_error(void);

/* Tuning knobs, for A/B measurements and for tests that force a code path; the defaults are the
 * measured best and no caller needs this.  Each knob starts from the environment variable of the same
 * name (read once, at the library's first planning call) and is changed afterwards only here:
 * value NULL restores the default.  Names: FC_ATTN_TILES ("R,W": row tiles and waves per attention
 * workgroup), FC_ATTN_WGS, FC_LIN_WGS, FC_ACCEPT_WGS (target workgroup counts), FC_LIN_NO_ROWS,
 * FC_GEMM_NO_SPLIT, FC_PROJ_NO_HEADSPLIT (any value switches the named path off), FC_LIN_WIDE_SHAPE,
 * FC_PROJ_GEMM_SHAPE (one GEMM tile shape for everything), FC_LIN_KSPLIT (parts of the hidden
 * dimension).  Host only; not thread-safe against concurrent calls into the library; workspace sizes
 * depend on the knobs, so query them after setting.
 * Errors: INVALID_ARG (NULL or unknown name). */
fc_status fc_tuning_set(const char *name, const char *value);

/* ---------------------------------------------------------------------------------------------
 * Persistent per-layer KV cache (section 3.2.1, "Initialization and Partitioning": the K/V
 * projections of prompt + all blocks are saved once and then reused).
 *
 * Storage layout (private to the library, documented for snapshotting): with Spad = max_seq
 * rounded up to a multiple of 64,
 *   K: [layer][B][Hkv][Spad][Dh]            row-major rows,
 *   V: [layer][B][Hkv][Spad/64][Dh][64]     64-row tiles stored transposed (key index fastest),
 * so that both stream as 16-byte coalesced loads in the order the matrix cores consume them.
 * Use fc_cache_write_rows / fc_cache_read_rows to move rows in the plain [B][Hkv][rows][Dh] layout.
 */

/* Bytes needed for EACH of the K and the V storage of a cache with this config; 0 on bad config. */
size_t fc_cache_storage_bytes(const fc_config *cfg);

/* Create a cache handle.  k_storage / v_storage: device buffers of fc_cache_storage_bytes() bytes
 * each, borrowed for the life of the handle (e.g. torch tensors), or both NULL to let the library
 * allocate zero-filled storage it then owns.  *out receives the handle (host object).  The handle
 * also owns 32 MB of device scratch (partial sums of the short-window projection), allocated here
 * and released by fc_cache_free; this is the only allocation the library makes besides the
 * optional K/V storage, and it is why one cache must not be used from two streams at once.
 * Errors: INVALID_ARG, UNSUPPORTED (geometry), OOM. */
fc_status fc_cache_alloc(const fc_config *cfg, void *k_storage, void *v_storage, fc_cache **out);

/* Destroy the handle and free library-owned storage.  The caller must have synchronised every
 * stream that used the cache.  NULL is accepted. */
fc_status fc_cache_free(fc_cache *cache);

/* Device base pointers of one layer's K and V storage (layout above). */
fc_status fc_cache_ptrs(const fc_cache *cache, int32_t layer, void **k, void **v);

/* Copy rows [start, start+rows) of every (sequence, kv head) between the cache and plain device
 * arrays k_rows, v_rows of shape [B][Hkv][rows][Dh].  Pure bit copies (prefill, snapshot, tests).
 * Errors: INVALID_ARG, BOUNDS (start < 0 or start + rows > max_seq), HIP. */
fc_status fc_cache_write_rows(fc_cache *cache, int32_t layer, const void *k_rows, const void *v_rows,
                              int32_t start, int32_t rows, void *stream);
fc_status fc_cache_read_rows(const fc_cache *cache, int32_t layer, void *k_rows, void *v_rows,
                             int32_t start, int32_t rows, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Window schedule (section 3.2.1: the generation region [P, P+G) is cut into fixed-size blocks
 * B_1..B_N; block i is decoded over steps_per_block steps; finished blocks are frozen).
 * Host-only, pure integer function.  Step `step` works on block i = step / steps_per_block.
 *   mode 0: window = block i alone                      (rows = min(Bk, rest of the region))
 *   mode 1: window = block i and all later blocks       (the paper's reducing window)
 * *refresh_after = 1 when refresh_every > 0 and (step + 1) % refresh_every == 0: the caller is
 * expected to fc_refresh the generation region before the next step.
 * Errors: INVALID_ARG; BOUNDS when step lies past the last block. */
fc_status fc_window(int32_t step, int32_t P, int32_t G, int32_t Bk, int32_t steps_per_block,
                    int32_t refresh_every, int32_t mode, int32_t *win_start, int32_t *rows,
                    int32_t *refresh_after);

/* ---------------------------------------------------------------------------------------------
 * The cached layer-step (section 3.2.1, "Windowed Re-computation" and "Progressive Caching").
 */

/* Project the A window rows of every sequence to q, k, v (Table 1, projection row, with L -> A),
 * apply rotary embedding to q and k at each row's absolute position (half-split pairing
 * (i, i + Dh/2), angle pos * rope_base^(-2i/Dh)), write q to q_out and overwrite the cache rows
 * at those positions with k and v.  No other cache row is modified.
 *   x      device [B][A][hidden]
 *   w_qkv  device [N][hidden], N = (Hq + 2 Hkv) Dh, rows ordered q heads | k heads | v heads
 *   b_qkv  device [N] or NULL
 *   pos    device int32 [B][A] absolute positions, or NULL meaning win_start + a.  A negative
 *          entry marks a padded row: nothing is stored for it and its q is zero.  Entries
 *          >= max_seq are treated the same way (the kernel never writes out of bounds).
 *          Duplicate positions within one sequence are undefined.
 *   q_out  device [B][Hq][A][Dh]
 * Errors: INVALID_ARG (NULL cache/x/w_qkv/q_out, A < 1), BOUNDS (layer; with pos == NULL:
 * win_start < 0 or win_start + A > max_seq), HIP. */
fc_status fc_qkv_project_scatter(fc_cache *cache, int32_t layer, const void *x, const void *w_qkv,
                                 const void *b_qkv, int32_t win_start, int32_t A,
                                 const int32_t *pos, void *q_out, void *stream);

/* Workspace bytes fc_active_attention / fc_refresh need for windows of up to max_rows rows
 * (split-KV partial results).  0 on bad arguments. */
size_t fc_workspace_bytes(const fc_config *cfg, int32_t max_rows);

/* The launch plan fc_active_attention would use for a window of A rows over kv_len cached rows
 * (host, pure function of the shape and the tuning knobs; for reports and for tying a measured HBM
 * traffic figure to the plan it was measured with):
 *   plan[0] kind (0 plain kernel, 1 matrix-core split-KV kernel)   plan[1] key ranges (splits)
 *   plan[2] keys per split   plan[3] 32-row tiles per (sequence, kv head)
 *   plan[4] row tiles per workgroup   plan[5] waves per workgroup
 * Errors: INVALID_ARG, UNSUPPORTED (config), BOUNDS (kv_len). */
fc_status fc_attention_plan(const fc_config *cfg, int32_t A, int32_t kv_len, int32_t plan[6]);

/* Bidirectional attention of the window's queries over cache rows [0, kv_len) (Table 1, rows
 * "QK^T" and "score x V", L x L -> A x L): out[b][a][h*Dh + i] = sum_t softmax_t(scale q.k_t) v_t[i]
 * with the KV head h / (Hq/Hkv); no mask of any kind.
 *   q      device [B][Hq][A][Dh] (as written by fc_qkv_project_scatter)
 *   pos    device int32 [B][A] or NULL; rows with a negative entry produce zeros
 *   out    device [B][A][Hq*Dh]
 *   workspace  device, >= fc_workspace_bytes(cfg, A) bytes, contents irrelevant; may be NULL only
 *          if that size is 0.  Two calls that overlap in time must not share a workspace.
 * Errors: INVALID_ARG, BOUNDS (layer; kv_len < 1 or > max_seq), WORKSPACE, HIP. */
fc_status fc_active_attention(fc_cache *cache, int32_t layer, const void *q, int32_t A,
                              int32_t kv_len, const int32_t *pos, void *out, void *workspace,
                              size_t workspace_bytes, void *stream);

/* fc_active_attention for callers that cannot allocate or bring a workspace: code recorded under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result
 * and errors as fc_active_attention, except that the split-KV partial results go to a static device
 * array inside the library (16 MiB per GPU, held until the process ends; its address on the current
 * device is looked up on the first call there, with that device current).  The call allocates
 * nothing.  A shape whose partial results exceed fc_active_attention_static_max_bytes() (compare
 * fc_workspace_bytes) is rejected with FC_ERR_WORKSPACE.  All calls on one GPU share the one array:
 * calls that overlap in time on the same GPU (two streams, two threads) race; calls on one stream
 * are ordered and safe.  Nothing in the array has to be cleared between calls. */
size_t fc_active_attention_static_max_bytes(void);
fc_status fc_active_attention_static(fc_cache *cache, int32_t layer, const void *q, int32_t A,
                                     int32_t kv_len, const int32_t *pos, void *out, void *stream);

/* Full refresh of rows [start, start+R) (section 3.2.1: the initial pass that fills the cache for
 * prompt + all blocks, and any later re-projection of a region): fc_qkv_project_scatter with
 * pos = start + r followed, if out != NULL, by fc_active_attention over [0, kv_len).
 *   x          device [B][R][hidden]
 *   q_scratch  device [B][Hq][R][Dh], receives the rotated queries
 *   out        device [B][R][Hq*Dh], or NULL to refresh K/V only (then workspace may be NULL)
 * Errors: as the two calls above, plus BOUNDS when start + R > kv_len and out != NULL. */
fc_status fc_refresh(fc_cache *cache, int32_t layer, const void *x, const void *w_qkv,
                     const void *b_qkv, int32_t start, int32_t R, int32_t kv_len, void *q_scratch,
                     void *out, void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * The rest of the transformer layer on the window rows (Table 1, rows "Output projection (W_out)",
 * "FFN W_1" and "FFN W_2": with FreeCache each is evaluated for the A window rows only, so its cost
 * drops from O(L ...) to O(A ...) exactly like the projections above).  The paper names these
 * modules without fixing their inner form; the library implements the pre-normalised layer of the
 * checkpoints the paper evaluates (Dream, LLaDA): RMS normalisation, output projection with
 * residual, SiLU-gated W_1 (a "gate" and an "up" matrix), W_2 with residual.
 *
 * These four calls do not touch a cache; dtype is an fc_dtype and applies to every tensor.  They
 * enqueue on `stream` like the calls above and validate on the host first.
 */

/* out[r][k] = x[r][k] / sqrt(mean_k x[r][k]^2 + eps) * weight[k].
 *   x, out  device [rows][hidden] (out may be x);  weight  device [hidden]
 * Errors: INVALID_ARG (NULL pointer, rows or hidden < 1, eps < 0, bad dtype), HIP. */
fc_status fc_rmsnorm(int32_t dtype, const void *x, const void *weight, float eps, int32_t rows,
                     int32_t hidden, void *out, void *stream);

/* Workspace bytes of fc_linear_residual for this shape (cross-workgroup partial sums); for
 * fc_ffn_gate_up pass N = 2 F.  0 on bad arguments or when none is needed. */
size_t fc_linear_workspace_bytes(int32_t dtype, int32_t M, int32_t K, int32_t N);

/* out[m][n] = residual[m][n] + sum_k x[m][k] w[n][k], rounded once (W_out and W_2 of Table 1, each
 * with the residual connection folded in).
 *   x  device [M][K];  w  device [N][K];  residual  device [M][N] or NULL;  out  device [M][N]
 *   (out may be residual);  workspace  device, >= fc_linear_workspace_bytes(dtype, M, K, N) bytes.
 * Errors: INVALID_ARG, UNSUPPORTED (K not a multiple of 8), WORKSPACE, HIP. */
fc_status fc_linear_residual(int32_t dtype, const void *x, const void *w, const void *residual,
                             int32_t M, int32_t K, int32_t N, void *out, void *workspace,
                             size_t workspace_bytes, void *stream);

/* out[m][f] = silu(sum_k x[m][k] w_gate[f][k]) * (sum_k x[m][k] w_up[f][k]), silu(t) = t / (1 + e^-t)
 * (the gated form of W_1 of Table 1); the two products stay in fp32, one rounding.
 *   x  device [M][K];  w_gate, w_up  device [F][K];  out  device [M][F];
 *   workspace  device, >= fc_linear_workspace_bytes(dtype, M, K, 2 F) bytes.
 * Errors: as fc_linear_residual. */
fc_status fc_ffn_gate_up(int32_t dtype, const void *x, const void *w_gate, const void *w_up, int32_t M,
                         int32_t K, int32_t F, void *out, void *workspace, size_t workspace_bytes,
                         void *stream);

/* Weights of one layer (all device pointers, element type fc_config.dtype, borrowed). */
typedef struct {
    const void *norm1;   /* [hidden]            RMSNorm weight in front of the attention */
    const void *w_qkv;   /* [N][hidden]         as for fc_qkv_project_scatter */
    const void *b_qkv;   /* [N] or NULL */
    const void *w_out;   /* [hidden][Hq*Dh] */
    const void *norm2;   /* [hidden]            RMSNorm weight in front of the FFN */
    const void *w_gate;  /* [d_ff][hidden] */
    const void *w_up;    /* [d_ff][hidden] */
    const void *w_down;  /* [hidden][d_ff] */
    int32_t d_ff;
    float eps;           /* RMSNorm epsilon */
} fc_layer_weights;

/* Workspace bytes of fc_full_layer_step for windows of up to max_rows rows per sequence
 * (intermediate activations of B * max_rows rows, the attention workspace, partial sums). */
size_t fc_full_layer_workspace_bytes(const fc_config *cfg, int32_t d_ff, int32_t max_rows);

/* One cached step of the whole layer on the window rows (section 3.2.1 applied to every module of
 * Table 1):
 *   h1 = rmsnorm(x; norm1);   q, cache rows <- fc_qkv_project_scatter(h1);   o = fc_active_attention(q)
 *   x2 = x + o w_out^T;       h2 = rmsnorm(x2; norm2)
 *   y  = x2 + (silu(h2 w_gate^T) * (h2 w_up^T)) w_down^T
 * Every named tensor is rounded to the cache dtype.  Rows with a negative pos entry have o = 0
 * (nothing cached for them) and are otherwise processed like any other row.
 *   x, y  device [B][A][hidden] (y may be x);  pos  device int32 [B][A] or NULL = win_start + a
 *   workspace  device, >= fc_full_layer_workspace_bytes(cfg, d_ff, A) bytes
 * Errors: those of the calls it is made of; all checks precede the first launch. */
fc_status fc_full_layer_step(fc_cache *cache, int32_t layer, const fc_layer_weights *weights,
                             const void *x, int32_t win_start, int32_t A, const int32_t *pos,
                             int32_t kv_len, void *y, void *workspace, size_t workspace_bytes,
                             void *stream);

/* ---------------------------------------------------------------------------------------------
 * Unmasking step on the window rows (section 3.1: the masked set M_t = {i : x_t[i] = MASK}, the
 * logits z_t of the masked positions, and the fill x_{t-1}[i] = argmax_v softmax(z_t[i]) of a subset
 * U_t of M_t "selected e.g. by confidence"; with FreeCache only the rows of the active window are
 * evaluated).  The library's reading: confidence = the softmax probability of the arg-max token;
 * U_t = the n most confident masked window positions of each sequence.
 */

/* Workspace bytes of fc_lm_head_argmax for this shape; 0 on bad arguments. */
size_t fc_lm_head_workspace_bytes(int32_t dtype, int32_t M, int32_t K, int32_t V);

/* Vocabulary projection of M rows without materialising the logits:
 *   z[m][v] = sum_k x[m][k] w_vocab[v][k] (fp32),  tok[m] = argmax_v z[m][v] (smallest v on ties),
 *   conf[m] = softmax(z[m])[tok[m]] = 1 / sum_v exp(z[m][v] - z[m][tok[m]]).
 *   x  device [M][K];  w_vocab  device [V][K] (element type dtype);  tok  device int32 [M];
 *   conf  device float [M];  workspace  device, >= fc_lm_head_workspace_bytes(dtype, M, K, V) bytes.
 * Errors: INVALID_ARG, UNSUPPORTED (K not a multiple of 8), WORKSPACE, HIP. */
fc_status fc_lm_head_argmax(int32_t dtype, const void *x, const void *w_vocab, int32_t M, int32_t K,
                            int32_t V, int32_t *tok, float *conf, void *workspace, size_t workspace_bytes,
                            void *stream);

/* One confidence-ranked unmasking step.  For every sequence b the candidates are the window rows a
 * whose position p = pos[b][a] (or win_start + a when pos is NULL) satisfies 0 <= p < L and
 * tokens[b][p] == mask_id.  The n_unmask candidates with the largest conf (ties: smaller a first; all
 * of them if fewer remain) get tokens[b][p] = tok[b][a].  pos_next[b][.] receives the positions of the
 * candidates that stay masked, in row order, padded with -1 (it is a valid `pos` argument of the
 * next step's calls), count_next[b] their number.
 *   tok  device int32 [B][A];  conf  device float [B][A], values >= 0;  pos  device int32 [B][A] or NULL;
 *   tokens  device int32 [B][L], updated in place;  pos_next  device int32 [B][A] (not pos itself);
 *   count_next  device int32 [B].  A is limited to 8192 rows.  Duplicate positions are undefined.
 * Integer work: bit-exact.  Errors: INVALID_ARG, UNSUPPORTED (A too large), BOUNDS (pos NULL and
 * win_start < 0 or win_start + A > L), HIP. */
fc_status fc_unmask_select(const int32_t *tok, const float *conf, const int32_t *pos, int32_t win_start,
                           int32_t B, int32_t A, int32_t n_unmask, int32_t mask_id, int32_t *tokens,
                           int32_t L, int32_t *pos_next, int32_t *count_next, void *stream);

/* Row gather: out[i][:] = table[idx[i]][:], zeros where idx[i] is negative (or >= rows: the kernel
 * never reads out of bounds).  With table = the embedding matrix and idx = the token ids of the
 * window rows it forms the layer input of a step (x_t restricted to the window, section 3.1); with
 * table = the hidden states it compacts the rows of a block.  Pure bit copies.
 *   table  device [rows][width] (element type dtype);  idx  device int32 [n];  out  device [n][width]
 *   width * element size must be a multiple of 16 bytes.
 * Errors: INVALID_ARG, UNSUPPORTED (row size not a multiple of 16 bytes), HIP. */
fc_status fc_gather_rows(int32_t dtype, const void *table, int32_t rows, int32_t width, const int32_t *idx,
                         int32_t n, void *out, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Guided Diffusion acceptance (section 3.2.2 and Algorithm 1: the diffusion model proposes a token
 * for every masked position, an auto-regressive guide scores the proposal, and the longest prefix of
 * masked positions on which both agree is unmasked; if they disagree at the first one, only that one
 * is unmasked, with the diffusion model's token.  "Top-K match" and the guidance threshold tau are
 * from the paper's implementation details).
 * For every sequence b, over its still masked window rows i_1 < i_2 < ... (position valid and
 * tokens[b][p] == mask_id):  t_j = argmax_v dlm[b][i_j][v] (smallest v on ties);  row j matches when
 * t_j is among the topk largest entries of ar[b][i_j][.] (ties: smaller id first) and, if tau > 0,
 * max_v dlm[b][i_j][v] > tau * max_v ar[b][i_j][v] (float product).  With k = the longest prefix of
 * matching rows, the first max(k, 1) masked rows get tokens[b][p] = t_j.
 *   dlm, ar  device float [B][A][V] logits;  pos  device int32 [B][A] or NULL = win_start + a;
 *   tokens  device int32 [B][L], updated in place;  n_accept  device int32 [B] (0 if nothing was masked);
 *   pos_next  device int32 [B][A], count_next  device int32 [B]: the rows that stay masked (as for
 *   fc_unmask_select);  workspace  device, >= fc_guided_accept_workspace_bytes(B, A, V) bytes.
 * topk is limited to 8.  Integer work on given floats: bit-exact.
 * Errors: INVALID_ARG, UNSUPPORTED (topk > 8), BOUNDS (pos NULL and window outside [0, L)), WORKSPACE, HIP. */
size_t fc_guided_accept_workspace_bytes(int32_t B, int32_t A, int32_t V);
fc_status fc_guided_accept(const float *dlm, const float *ar, const int32_t *pos, int32_t win_start, int32_t B,
                           int32_t A, int32_t V, int32_t topk, float tau, int32_t mask_id, int32_t *tokens,
                           int32_t L, int32_t *n_accept, int32_t *pos_next, int32_t *count_next, void *workspace,
                           size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * KV drift diagnostic (section 3.2.1: the figure that motivates FreeCache shows, per token position
 * and denoising step, the similarity of the token's K / V projection to its projection one step
 * earlier; clean tokens stay near 1).  Compares rows [start, start+rows) of a layer's cache with a
 * snapshot of the same rows taken earlier with fc_cache_read_rows (before the step that re-projected
 * them):  sim[b][j][r] = <now, prev> / (|now| |prev|) over the head dimension, 0 if either is zero.
 * A runtime signal for choosing the refresh period; not part of the step itself.
 *   k_prev, v_prev  device [B][Hkv][rows][Dh] (cache dtype);  sim_k, sim_v  device float [B][Hkv][rows]
 * Errors: INVALID_ARG, BOUNDS (layer; rows outside the cache), HIP. */
fc_status fc_kv_similarity(const fc_cache *cache, int32_t layer, const void *k_prev, const void *v_prev,
                           int32_t start, int32_t rows, float *sim_k, float *sim_v, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FREECACHE_H */
