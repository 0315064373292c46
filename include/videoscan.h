/*
 * videoscan.h -- C ABI of the MI355X (gfx950) streaming attention path of VideoScan.
 *
 * The library computes, for one decoder layer at a time, the three steps the
 * method performs on every incoming video frame and on every decoded token
 * (VideoScan, Sections 3.2 and 3.3):
 *   1. frame prefill attention  -- Eq. 1 (Section 3.1) for the frame's N visual
 *      tokens followed by its semantic carrier token, over the rows retained so
 *      far plus the frame's own tokens (causal inside the frame);
 *   2. carrier compaction       -- keep the carrier token's K/V row only, append it
 *      to the per-layer cache, drop the visual tokens' K/V;
 *   3. decode attention         -- Eq. 1 for one text query per stream over the
 *      retained rows.
 * plus the mean pool that forms the carrier's input embedding (Section 3.3).
 *
 * General rules (all entry points):
 *   - Pointers named q, k_f, v_f, out, k, v, k_slab, v_slab, k_new, v_new, e,
 *     c_out and workspace are DEVICE pointers (HIP global memory of the current
 *     device), 16-byte aligned, owned by the caller.  vs_shape, vs_cache, `lens`,
 *     `row_written` are HOST memory.
 *   - The library never allocates, frees or keeps device memory.  Temporary
 *     storage comes from the caller's `workspace` (size from vs_workspace_bytes,
 *     prepared once with vs_workspace_init).
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the null stream) and return without waiting.  Buffers must stay valid until
 *     that work has finished.  Two calls that share a workspace must be ordered
 *     on one stream.
 *   - Host-side lengths (vs_cache.len, lens[]) are the truth about how many rows
 *     are valid; they are updated at enqueue time, only when VS_OK is returned.
 *   - Errors are return codes.  Argument errors are found before anything is
 *     launched and leave all lengths untouched.
 *   - Tensors are dense row-major.  Storage type is vs_shape.dtype: fp32 or
 *     bf16 (bit pattern = upper 16 bits of an fp32).  Scores, softmax and
 *     accumulation are fp32 in both cases; outputs are rounded to nearest even.
 *   - Grouped-query attention: query head h reads KV head h / (n_q_heads /
 *     n_kv_heads).
 *   - Supported: head_dim 64 or 128 for fp32; head_dim 128 for bf16;
 *     n_q_heads a multiple of n_kv_heads with a ratio of at most 8.
 */
#ifndef VIDEOSCAN_H
#define VIDEOSCAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VS_OK = 0,
    VS_ERR_NULL = 1,        /* a required pointer is NULL */
    VS_ERR_SHAPE = 2,       /* sizes out of range or inconsistent */
    VS_ERR_UNSUPPORTED = 3, /* head_dim / dtype / head ratio not implemented */
    VS_ERR_CAPACITY = 4,    /* append into a full cache, or len > capacity */
    VS_ERR_WORKSPACE = 5,   /* workspace missing or too small */
    VS_ERR_ALIGN = 6,       /* a device pointer is not 16-byte aligned */
    VS_ERR_HIP = 7,         /* the HIP runtime reported a launch failure */
    VS_ERR_PLACEMENT = 8    /* see vs_workspace_init: results of earlier prefill calls are in doubt */
} vs_status;

typedef enum { VS_F32 = 0, VS_BF16 = 1 } vs_dtype;

typedef struct {
    int32_t n_q_heads;   /* Hq */
    int32_t n_kv_heads;  /* Hkv, divides Hq */
    int32_t head_dim;    /* D */
    int32_t dtype;       /* vs_dtype of q/k/v/out */
    float softmax_scale; /* multiplies q.k; 1/sqrt(head_dim) in Eq. 1 */
} vs_shape;

/* Retained K/V rows of one layer of one stream: [text prefix | one carrier row per
 * frame seen], append-only (Section 3.3: the retained carriers and their KV pairs). */
typedef struct {
    void *k;          /* device, [capacity][n_kv_heads][head_dim] */
    void *v;          /* device, same layout */
    int32_t capacity; /* rows allocated */
    int32_t len;      /* rows valid, host-side truth */
} vs_cache;

/* Human-readable name of a status code (static string, never NULL). */
const char *vs_status_string(vs_status s);

/*
 * Bytes of device workspace that any call needs for up to `max_q_tokens` tokens
 * per frame run, `max_cache_rows` retained rows (per stream) and `n_streams`
 * decode streams.  Returns 0 if the shape is unsupported.
 */
size_t vs_workspace_bytes(const vs_shape *shape, int32_t max_q_tokens, int32_t max_cache_rows,
                          int32_t n_streams);

/*
 * Prepares a freshly allocated (or overwritten) workspace: clears the control
 * block at its start, which holds arrival counters that the kernels leave at zero
 * after every launch.  The first call on a device also runs a one-off probe of how the
 * device distributes workgroups and waits for it (hip_stream is synchronised once).
 * Must have completed on the device (same stream, or
 * synchronised) before the first call that uses the workspace; needed once, not per
 * call.  A workspace is tied to the shape it was initialised with.
 * With the environment variable VS_DEBUG set, a HIP error behind VS_ERR_HIP from this call
 * is also printed on stderr as text.
 *
 * What the probe is for.  When a bf16 prefill call splits the keys of a row tile over several
 * workgroups, they merge their partial results inside the same launch once the last of them has
 * finished (each its share of the rows; the others wait for the last one, looking at a word in
 * memory a bounded number of times, a few milliseconds at most),
 * through the L2 cache that the compute units of one XCD (accelerator die) share; the library
 * therefore gives all those workgroups ids that the device deals to one XCD, which it learns
 * from the probe (ids go to the XCDs in turn).  Every workgroup of every such launch checks that
 * it really runs on the XCD the probe saw for its id.  If one does not (another partition mode,
 * masked compute units), or if one waits for the last of its row tile in vain (the workgroups of
 * the launch are not all running at once: the device is shared with other work), it sets a word
 * of pinned host memory (64 bytes per device, allocated by
 * the first vs_workspace_init on the device and kept until the process ends).  The next bf16
 * prefill call on that device (vs_frame_prefill_attn, vs_frame_prefill_compact,
 * vs_question_prefill_append, vs_frames_prefill_attn) then launches nothing and returns
 * VS_ERR_PLACEMENT, once: the outputs of the bf16 prefill calls enqueued since the last one that
 * returned VS_OK after a synchronisation are in doubt and should be repeated.  From then on the
 * partial results are merged by a second kernel, which needs no such placement, until a later
 * vs_workspace_init probes the device again.
 */
vs_status vs_workspace_init(const vs_shape *shape, void *workspace, size_t workspace_bytes,
                            void *hip_stream);

/*
 * Frame prefill attention (Section 3.3, prefilling phase; Eq. 1; carrier last in
 * the run, Section 3.2).
 *   q   [n_tokens][Hq][D], k_f / v_f [n_tokens][Hkv][D]: the frame run, visual
 *   tokens first, carrier token last.  out [n_tokens][Hq][D].
 * Row i attends to the cache's `len` rows and to frame rows 0..i.  The cache is
 * only read.  len may be 0.  n_tokens >= 1, n_tokens <= 4096.
 */
vs_status vs_frame_prefill_attn(const vs_shape *shape, const vs_cache *cache, const void *q,
                                const void *k_f, const void *v_f, int32_t n_tokens, void *out,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Carrier compaction and append (Sections 3.2, 3.3: only the carrier's K/V is
 * kept, the visual tokens' K/V are discarded).  Copies row `carrier_index` of k_f
 * and v_f ([n_tokens][Hkv][D]; the method uses n_tokens-1) bit for bit into cache
 * row `len`, stores that row index in *row_written (may be NULL) and increments
 * cache->len.  VS_ERR_CAPACITY if len == capacity.
 */
vs_status vs_carrier_compact_append(const vs_shape *shape, vs_cache *cache, const void *k_f,
                                    const void *v_f, int32_t n_tokens, int32_t carrier_index,
                                    int32_t *row_written, void *hip_stream);

/*
 * Prefill and compaction of one frame in a single launch: same result as
 * vs_frame_prefill_attn followed by vs_carrier_compact_append with
 * carrier_index = n_tokens-1.  Nothing is launched and len is unchanged if the
 * cache is full.
 */
vs_status vs_frame_prefill_compact(const vs_shape *shape, vs_cache *cache, const void *q,
                                   const void *k_f, const void *v_f, int32_t n_tokens, void *out,
                                   int32_t *row_written, void *workspace, size_t workspace_bytes,
                                   void *hip_stream);

/*
 * Compaction for many caches in one launch (all layers of a frame, or many
 * streams).  Caches live in slabs k_slab / v_slab [n_caches][capacity][Hkv][D];
 * frame runs in k_f / v_f [n_caches][n_tokens][Hkv][D].  For every i, row
 * carrier_index of run i goes to row lens[i] of cache i and lens[i] += 1.
 * rows_written (host, [n_caches]) may be NULL.  If any cache is full nothing is
 * done.  With n_caches > 64 (at most 2^20) the kernel reads the old lengths from memory: from
 * rows_written if that is given (it is filled with them before the launch), else from lens.
 * If that array is pinned host memory the kernel reads it in place, so leave rows_written
 * alone until the stream has passed this call; with pinned lens and no rows_written the call
 * waits for the stream, because lens is incremented before the call returns.  Pageable
 * memory is copied into the workspace first (vs_workspace_bytes with n_streams = n_caches;
 * no workspace is needed otherwise).
 */
vs_status vs_carrier_compact_append_batched(const vs_shape *shape, int32_t n_caches, void *k_slab,
                                            void *v_slab, int32_t capacity, int32_t *lens,
                                            const void *k_f, const void *v_f, int32_t n_tokens,
                                            int32_t carrier_index, int32_t *rows_written,
                                            void *workspace, size_t workspace_bytes,
                                            void *hip_stream);

/*
 * The question after the video (Section 3.3, decoding phase: the question's tokens attend
 * over the retained carrier rows before the answer is decoded; Section 3.4: text reaches the
 * frames only through their carriers, which at inference are exactly the rows kept).
 *   q, out [n_tokens][Hq][D]; k_t, v_t [n_tokens][Hkv][D].
 * Token i attends over the cache's `len` rows and tokens 0..i of the question (Eq. 1), as in
 * vs_frame_prefill_attn; then ALL n_tokens K/V rows are copied bit for bit to cache rows
 * len .. len+n_tokens-1 and cache->len grows by n_tokens, so that vs_decode_attn continues on
 * top of them.  The result is what n_tokens decoding steps, one token each, would give.
 * One launch for bf16.  VS_ERR_CAPACITY, with nothing launched and len unchanged, if
 * len + n_tokens > capacity; other errors as vs_frame_prefill_attn.
 */
vs_status vs_question_prefill_append(const vs_shape *shape, vs_cache *cache, const void *q,
                                     const void *k_t, const void *v_t, int32_t n_tokens,
                                     void *out, void *workspace, size_t workspace_bytes,
                                     void *hip_stream);

/*
 * Decode attention (Section 3.3, decoding phase; Eq. 1), one query token for each
 * of n_streams independent streams of one layer.
 *   k_slab / v_slab [n_streams][capacity][Hkv][D], stream s valid up to lens[s].
 *   q [n_streams][Hq][D]; k_new / v_new [n_streams][Hkv][D] or both NULL.
 * If k_new is given, row lens[s] of stream s receives it first and lens[s] += 1;
 * the query then attends over all valid rows, the new one included.  Every stream
 * must end with at least one valid row.  1 <= n_streams <= 1024.
 * Streams are launched in groups of 64.  Should a launch fail (VS_ERR_HIP) after earlier
 * groups have been enqueued, lens has advanced for exactly those earlier groups, whose rows
 * are written and whose outputs are valid; the failed group and the ones behind it are
 * untouched, so the call can be repeated for them alone.
 */
vs_status vs_decode_attn(const vs_shape *shape, int32_t n_streams, void *k_slab, void *v_slab,
                         int32_t capacity, int32_t *lens, const void *q, const void *k_new,
                         const void *v_new, void *out, void *workspace, size_t workspace_bytes,
                         void *hip_stream);

/*
 * vs_decode_attn without a workspace argument, for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid allocation).  Same
 * arguments, same results bit for bit, same errors; the partial results of the row shares go
 * into an array of vs_decode_static_scratch_bytes() = 16 MiB that is part of the library's
 * code object on every device (each GPU the library runs on holds it until the process ends).
 * Neither this call nor anything it calls allocates or frees memory.  VS_ERR_WORKSPACE if the
 * call would need more than the array holds (vs_workspace_bytes(shape, 0, capacity, n_streams)
 * is the measure: 28 query / 4 KV heads of 128 fit with room to spare; 64 query heads per
 * launch group of 64 streams do not).  All calls on one GPU share that GPU's array, which keeps
 * what the last call left in it (nothing in it has to be cleared for this call): two calls
 * that overlap in time on one GPU, on different streams, race; order them.
 */
size_t vs_decode_static_scratch_bytes(void);
vs_status vs_decode_attn_static(const vs_shape *shape, int32_t n_streams, void *k_slab, void *v_slab,
                                int32_t capacity, int32_t *lens, const void *q, const void *k_new,
                                const void *v_new, void *out, void *hip_stream);

/*
 * Carrier embedding (Section 3.3: C^t = (1/N) sum_i E^t_i).  e [n][d] -> c_out [d],
 * storage type `dtype`, fp32 accumulation in row order, one rounding at the end.
 * d must be a multiple of 8 (bf16) or 4 (fp32).
 */
vs_status vs_carrier_mean_pool(const void *e, int32_t n, int32_t d, int32_t dtype, void *c_out,
                               void *hip_stream);

/*
 * A run of several frames in one call, under the semantic-aware mask (Section 3.4: later
 * tokens reach earlier frames only through those frames' semantic carriers; Section 3.2: the
 * carrier is the last token of its frame).  q, out [n_frames][n_tokens][n_q_heads][head_dim],
 * k_f, v_f [n_frames][n_tokens][n_kv_heads][head_dim].  Token i of frame a sees the cache's
 * `len` rows, the carriers (token n_tokens-1) of frames 0..a-1 of the run, and tokens 0..i of
 * its own frame; Eq. 1 over that set.  All carriers are appended to the cache, in frame
 * order, as rows len..len+n_frames-1, and cache->len grows by n_frames: the call computes what
 * n_frames calls of vs_frame_prefill_compact would, one frame after the other.  bf16 only.
 * 1 <= n_frames <= 64, n_frames * n_tokens <= 4096.  workspace: vs_frames_workspace_bytes.
 * Errors as vs_frame_prefill_compact (VS_ERR_CAPACITY if the cache has no room for n_frames
 * rows; VS_ERR_UNSUPPORTED for fp32 storage).
 */
size_t vs_frames_workspace_bytes(const vs_shape *shape, int32_t n_frames, int32_t n_tokens,
                                 int32_t max_cache_rows);
vs_status vs_frames_prefill_attn(const vs_shape *shape, vs_cache *cache, const void *q, const void *k_f,
                                 const void *v_f, int32_t n_frames, int32_t n_tokens, void *out,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Memory bank of the semantic carriers (Section 3.3, memory mechanism): at most
 * `capacity` carriers are kept, oldest first; their embeddings live in `e`, their K/V
 * rows in the layers' caches behind the rows that are not carriers (e.g. a text prefix).
 */
typedef struct {
    void *e;          /* device, [capacity][d], storage type `dtype` */
    int32_t capacity; /* M, 1..1024 */
    int32_t len;      /* carriers held, host-side truth */
    int32_t d;        /* embedding width; d * element size a multiple of 16 bytes */
    int32_t dtype;    /* vs_dtype */
} vs_bank;

/* Bytes of device scratch vs_memory_bank_push needs for a bank of this capacity. */
size_t vs_memory_bank_workspace_bytes(int32_t capacity);

/*
 * A carrier with embedding e_new [d] (device) arrives at the bank (Section 3.3, memory
 * mechanism: embeddings of adjacent carriers are compared, and of the most similar pair
 * the older carrier is dropped).  With room left the embedding is appended, bank->len
 * grows by one and -1 is written to *victim.  With the bank full the cosines of the
 * `capacity` adjacent pairs of the sequence e[0], .., e[capacity-1], e_new are taken
 * (fp64 sums; a vector of norm 0 has cosine 0), the pair (i, i+1) with the largest one
 * names the victim i (of equal cosines the smallest i; policy 1: the i with the largest
 * cosine to e_new instead), row i is removed, the rows behind it move up, e_new becomes the
 * last row, bank->len stays, and i is written to *victim.  `victim` is DEVICE memory (one
 * int32, may not be NULL): the decision is taken on the device and handed to
 * vs_carrier_evict_append through it, with no wait on the host.  workspace: device,
 * 16-byte aligned, vs_memory_bank_workspace_bytes(capacity) bytes, used by this call only.
 * Errors: VS_ERR_NULL, VS_ERR_SHAPE (capacity, len, d, policy out of range),
 * VS_ERR_UNSUPPORTED (dtype), VS_ERR_ALIGN, VS_ERR_WORKSPACE, VS_ERR_HIP.
 */
vs_status vs_memory_bank_push(vs_bank *bank, const void *e_new, int32_t policy, int32_t *victim,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The K/V side of the same step, for n_layers caches at once (n_layers = 1: one layer, as a
 * decoder produces them): cache l receives the carrier's K/V row k_rows + l*layer_stride_bytes,
 * v_rows + l*layer_stride_bytes ([n_kv_heads][head_dim] each, device).  Rows 0..first_row-1
 * of every cache are not carriers and stay.  A cache that holds fewer than bank_capacity
 * carriers (len < first_row + bank_capacity) appends the row and its len grows by one;
 * otherwise carrier row first_row + *victim is removed, the rows behind it move up, the new
 * row becomes the last and len stays (Sections 3.2, 3.3: the bank stores the carriers'
 * associated KV pairs).  `victim` is the DEVICE int32 that vs_memory_bank_push wrote; it is
 * read by the kernel, never by the host.  `caches` is a HOST array; all of them must hold the
 * same number of rows.  Errors as above plus VS_ERR_CAPACITY (first_row + bank_capacity
 * exceeds a cache's capacity); lengths untouched on error.
 */
vs_status vs_carrier_evict_append(const vs_shape *shape, int32_t n_layers, vs_cache *caches,
                                  int32_t first_row, int32_t bank_capacity, const void *k_rows,
                                  const void *v_rows, int64_t layer_stride_bytes, const int32_t *victim,
                                  void *hip_stream);

/*
 * Launch-plan overrides for tuning and for tests that must show a result does not
 * depend on how the keys were split.  Process-wide, not thread-safe; value 0 restores
 * the library's own choice.  Unknown knobs or out-of-range values: VS_ERR_SHAPE.
 *   VS_TUNE_PREFILL_SPLITS    workgroups sharing one row tile's keys, 1..32
 *   VS_TUNE_PREFILL_KV_GROUPS  key groups (sets of 4 wavefronts) per prefill workgroup, 1 or 2
 *   VS_TUNE_DECODE_CHUNK_ROWS rows of a stream per decode workgroup share, a multiple of 32
 *   VS_TUNE_PREFILL_MERGE     1 = split results are merged inside the attention kernel by the last
 *                             workgroup of a row tile to arrive alone (not shared by the tile's
 *                             workgroups); 2 = always by the second kernel, never inside the
 *                             attention kernel; 3 = for tests of the placement guard (see
 *                             vs_workspace_init): the kernels are told the probed XCD order
 *                             rotated by one, so every workgroup reports itself misplaced while
 *                             the results stay correct; 4 = for tests of the bounded wait of the
 *                             shared merge: the workgroups that would wait for the last of their
 *                             tile give up at once and report, as if the workgroups of a tile
 *                             were not running at the same time (that call's output is
 *                             incomplete; the next call returns VS_ERR_PLACEMENT)
 */
typedef enum {
    VS_TUNE_PREFILL_SPLITS = 0,
    VS_TUNE_PREFILL_KV_GROUPS = 1,
    VS_TUNE_DECODE_CHUNK_ROWS = 2,
    VS_TUNE_PREFILL_MERGE = 4
} vs_tune_knob;
vs_status vs_set_tuning(int32_t knob, int32_t value);

/*
 * The frame's rows and their projections in one launch (Section 3.1: Q = X W_Q, K = X W_K,
 * V = X W_V; Section 3.3: the semantic carrier's embedding is the mean of the frame's token
 * embeddings; Section 3.2: the carrier is the frame's last row).  bf16 only.
 *   e      [n_visual][d_model]   the frame's token embeddings, 1 <= n_visual <= 191
 *   w_qkv  [(Hq + 2 Hkv) * D][d_model]   one row of d_model weights per output feature: the
 *          features of W_Q (head by head), then of W_K, then of W_V
 *   q_out  [n_visual + 1][Hq][D],  k_out, v_out  [n_visual + 1][Hkv][D]: rows 0..n_visual-1 belong
 *          to the tokens, row n_visual to the carrier; exactly what vs_frame_prefill_attn and
 *          vs_frame_prefill_compact take as q, k_f, v_f
 *   c_out  [d_model] or NULL: the carrier embedding itself, the same bits as vs_carrier_mean_pool
 * fp32 accumulation, outputs rounded to bf16 once.  The carrier's row is obtained as the mean of
 * the token rows' fp32 sums (the projection is linear), i.e. the mean enters unrounded; c_out is
 * that mean rounded to bf16.  d_model a multiple of 64.  No workspace.  Position encoding is not
 * part of the paper's statement and not applied.
 */
vs_status vs_frame_qkv_project(const vs_shape *shape, const void *e, int32_t n_visual,
                               int32_t d_model, const void *w_qkv, void *q_out, void *k_out,
                               void *v_out, void *c_out, void *hip_stream);

/*
 * The rest of the decoder layer around the attention (Section 4.1 names the backbone the method is
 * built on; Section 3.1 writes Q = X W_Q, K = X W_K, V = X W_V).  The paper gives none of the
 * layer's details; taken here: the pre-norm layer of that backbone family -- RMS norm, projections
 * without bias, a feed-forward gated by SiLU, residual sums -- and no position encoding (the
 * attention entry points take Q and K as they come).  bf16 storage, fp32 arithmetic, one rounding
 * per tensor written.  All for runs of at most 192 rows (one frame: N visual tokens + carrier).
 */

/* out [n_rows][d] = x * gamma / sqrt(mean_j x_j^2 + eps), row by row.  d a multiple of 8. */
vs_status vs_rmsnorm(const void *x, const void *gamma, int32_t n_rows, int32_t d, float eps, void *out,
                     void *hip_stream);

typedef enum {
    VS_LINEAR_STORE = 0,    /* out [n_rows][n] = x w^T */
    VS_LINEAR_RESIDUAL = 1, /* out [n_rows][n] = residual + x w^T */
    VS_LINEAR_GATED = 2     /* out [n_rows][n/2]: out_j = silu(x w_{2j}) * (x w_{2j+1}), silu(g) = g / (1 + exp(-g)):
                               the rows of w alternate gate and value projections */
} vs_linear_mode;

/*
 * out = x w^T for 1 <= n_rows <= 192 rows: x [n_rows][k] (row-major, dense), w [n][k] (one row of k
 * weights per output feature), k a multiple of 64, n a multiple of 2.  `residual` [n_rows][n] is read in
 * mode VS_LINEAR_RESIDUAL only (it may be the same memory as out).  workspace: device,
 * vs_linear_workspace_bytes(n_rows, k, n) bytes (0 for shapes that need none: NULL is accepted then).
 * Errors: VS_ERR_NULL, VS_ERR_SHAPE, VS_ERR_ALIGN, VS_ERR_WORKSPACE, VS_ERR_HIP.
 */
size_t vs_linear_workspace_bytes(int32_t n_rows, int32_t k, int32_t n);
vs_status vs_linear(const void *x, const void *w, int32_t n_rows, int32_t k, int32_t n, int32_t mode,
                    const void *residual, void *out, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Weights of one decoder layer (device pointers, bf16). */
typedef struct {
    const void *norm1;     /* [d_model]                 RMS norm in front of the attention */
    const void *w_qkv;     /* [(Hq + 2 Hkv) D][d_model] features of W_Q, then W_K, then W_V */
    const void *w_o;       /* [d_model][Hq D]           output projection */
    const void *norm2;     /* [d_model]                 RMS norm in front of the feed-forward */
    const void *w_gate_up; /* [2 d_ff][d_model]         rows 2j, 2j+1: gate and value projection of unit j */
    const void *w_down;    /* [d_model][d_ff] */
    int32_t d_model, d_ff; /* multiples of 64 */
    float eps;             /* of both norms */
} vs_layer_weights;

/*
 * One decoder layer for one frame run (Sections 3.2, 3.3: the frame's visual tokens and its carrier,
 * last, pass through the layers once; only the carrier's K/V row of every layer is kept):
 *   x1 = rmsnorm(h_in, norm1);  [q k v] = x1 w_qkv^T;  a = frame prefill attention of (q, k, v) over
 *   the cache, the carrier's K/V row appended to it (vs_frame_prefill_compact);
 *   h1 = h_in + a w_o^T;  x2 = rmsnorm(h1, norm2);  h_out = h1 + (silu(x2 w_gate^T) * (x2 w_up^T)) w_down^T.
 * h_in, h_out [n_tokens][d_model] (may be the same memory), 1 <= n_tokens <= 192, bf16 only.
 * workspace: vs_layer_workspace_bytes (prepared with vs_workspace_init like every workspace that the
 * attention uses).  Errors as vs_frame_prefill_compact and vs_linear; cache->len grows by one on VS_OK.
 * Seven launches on hip_stream.  Where a product's input features are shared out over several
 * workgroups, these add their sums inside the multiplying launch, placed, counted and waited for
 * exactly as the key splits of the attention are (vs_workspace_init); what they report comes back
 * the same way, as VS_ERR_PLACEMENT from the next call, after which second kernels add the sums.
 */
size_t vs_layer_workspace_bytes(const vs_shape *shape, const vs_layer_weights *weights, int32_t n_tokens);
vs_status vs_frame_decoder_layer(const vs_shape *shape, const vs_layer_weights *weights, vs_cache *cache,
                                 const void *h_in, int32_t n_tokens, void *h_out, void *workspace,
                                 size_t workspace_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* VIDEOSCAN_H */
