/*
 * moe.h -- C ABI of the MI355X (gfx950) MoE-layer library.
 *
 * One call of the layer is what the paper's pipeline runs once per micro-batch
 * inside its post-attention task (section 4.1: the O projection, then the MoE FFN):
 * a gating function picks k of the n_e expert feed-forward networks for every
 * token and only those run (section 2.1).  Shape symbols follow the paper's
 * notation table (section 4.2): h1 (here H) model hidden size, h2 (F) expert
 * intermediate size, n_e (E) experts, k, dt (dtype); T is the micro-batch mu
 * of section 3.3.  Expert weights are not dense arrays but fixed-size PAGES
 * found through a PAGE TABLE, as in the paper's memory management (appendix
 * A.1: weights move in pages, the MoE FFN kernel reaches them via a page
 * table; a buffer of twice the streamed weights allows prefetch).
 *
 * General rules
 *  - Plain C types only.  "device" pointers are HIP device memory, "host"
 *    pointers ordinary host memory, "pinned" host memory from hipHostMalloc.
 *  - The caller owns every buffer and every stream.  Hot calls enqueue work on
 *    `stream` (a hipStream_t passed as void*; NULL = the default stream) and
 *    return without waiting for it.  They never allocate or free memory.
 *  - Every function returns MOE_OK (0) or a negative moe_status.  Arguments
 *    are checked on the host before anything is enqueued; on error nothing was
 *    enqueued.  T == 0 is valid and does nothing.
 *  - All arrays are contiguous row-major.  R = T*k is the number of routed rows.
 *  - dtype is the storage type of x, the router, the expert weights and the
 *    intermediate h; logits, gate weights, expert outputs and y are float.
 *
 * Supported shapes: 1 <= k <= E <= MOE_MAX_EXPERTS, H and F multiples of 128,
 * page_bytes a positive multiple of the weight-tile size (moe_tile_bytes).
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_MAX_EXPERTS 64

typedef enum moe_status {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = -1,        /* null pointer, bad shape, bad alignment */
    MOE_ERR_UNSUPPORTED_DTYPE = -2,
    MOE_ERR_WORKSPACE_TOO_SMALL = -3,
    MOE_ERR_PAGE_NOT_RESIDENT = -4,  /* a needed page-table entry is -1 or outside the pool */
    MOE_ERR_HIP = -5                 /* a HIP call failed; see moe_last_hip_error() */
} moe_status;

enum { MOE_DTYPE_F32 = 0, MOE_DTYPE_BF16 = 1 };

typedef struct moe_shape {
    int32_t T;          /* tokens in the micro-batch (mu) */
    int32_t H;          /* h1 */
    int32_t F;          /* h2 */
    int32_t E;          /* n_e */
    int32_t k;          /* experts per token */
    int32_t dtype;      /* MOE_DTYPE_* */
    int64_t page_bytes; /* size of one weight page */
} moe_shape;

const char* moe_status_string(int status);
/* hipError_t value of the most recent failing HIP call on this thread (0 if none). */
int moe_last_hip_error(void);
/* MOE_OK if the shape is one the library supports. */
int moe_validate_shape(const moe_shape* s);

/* ------------------------------------------------------------------ paged weights
 *
 * Page format (this library's reading of the paper's weight pages, appendix
 * A.1; the paper fixes neither page size nor content).  The unit is a TILE of
 * 128 output features x 64 reduction elements (16 KiB bf16, 32 KiB f32).
 *   f32:  128 rows of 256 bytes; the 16-byte chunk with index c (0..15) of row n
 *         is stored at chunk position (c & 8) | ((c & 7) ^ ((n >> 1) & 7)).
 *   bf16: two half-tiles of 8 KiB, one per 32 reduction elements; half-tile c >> 2
 *         holds, in row n of 64 bytes, chunk c (0..7) of that row at chunk position
 *         (c & 3) ^ ((n >> 2) & 2).
 * These are the images the GEMM kernels copy straight into LDS (the bf16 kernel
 * consumes 32 reduction elements per pipeline stage).  The LDS has 64 banks of
 * 4 bytes, a 128-bit LDS read executes in four phases of 16 lanes (for the bf16
 * kernel's operand fetch, one row per lane: rows r and r + 8 of two neighbouring
 * chunks meet in a phase), and the XOR with the row index makes every phase touch
 * every bank once.  A page holds page_bytes / tile_bytes
 * consecutive tiles and never spans experts.  Expert e owns
 * pages_gu + pages_d logical pages:
 *   group GU (logical pages 0 .. pages_gu-1): tiles ordered [f/128][w][h/64],
 *       w = 0 for W1 (gate) rows f..f+127, w = 1 for W3 (up) rows f..f+127;
 *   group D  (logical pages pages_gu .. ): tiles ordered [d/128][f/64] of W2.
 * The last page of a group is zero padded.  page_table[e * pages_per_expert + p]
 * is the slot of logical page p of expert e in the page pool (byte address
 * pool + slot * page_bytes), or -1 if the page is not resident.
 */
int moe_tile_bytes(const moe_shape* s, int64_t* tile_bytes);
int moe_pages_required(const moe_shape* s, int64_t* pages_gu, int64_t* pages_d);

/* Host-side packer.  W1, W3: [E][F][H]; W2: [E][H][F] (host, dtype elements).
 * page_table: host, [E][pages_gu+pages_d], every entry in [0, pool_pages) and
 * all distinct.  pages_out: host (may be pinned), pool_pages * page_bytes. */
int moe_pack_weights(const moe_shape* s, const void* W1, const void* W3, const void* W2,
                     const int32_t* page_table, int64_t pool_pages, void* pages_out);
/* Inverse of moe_pack_weights (host to host); used by tests. */
int moe_unpack_weights(const moe_shape* s, const void* pages, const int32_t* page_table,
                       int64_t pool_pages, void* W1, void* W3, void* W2);
/* Checks a HOST copy of a page table: MOE_ERR_PAGE_NOT_RESIDENT if an entry is
 * negative or >= pool_pages.  (Kernels also guard every entry they use: a bad
 * entry is never dereferenced, the tile reads slot 0 instead and bit 0 of the
 * device status word is set; see moe_workspace_layout.status.) */
int moe_page_table_validate(const moe_shape* s, const int32_t* page_table_host, int64_t pool_pages);

/* ------------------------------------------------------------------ workspace */

typedef struct moe_workspace_layout {
    /* byte offsets into the workspace of moe_layer, each 256-byte aligned */
    size_t status;     /* int32[4]: [0] bit 0 = a page-table entry was not resident; [2], [3]: shader clock in MHz that a
                        * block of the bf16 gate/up and down launch saw (diagnostic, 0 if none reported) */
    size_t topk_ids;   /* int32[T][k] */
    size_t topk_w;     /* float[T][k] */
    size_t counts;     /* int32[E] */
    size_t offsets;    /* int32[E+1] */
    size_t row_src;    /* int32[R] */
    size_t row_of;     /* int32[R] */
    size_t row_w;      /* float[R]: gate weight of each permuted row */
    size_t scan;       /* scratch of the permutation kernels */
    size_t x_perm;     /* dtype[R][H]; moe_layer leaves it unwritten when the gate/up GEMM gathers the rows itself */
    size_t h;          /* dtype[R][F] */
    size_t out;        /* float[R][H] */
    size_t total;      /* bytes needed by moe_layer */
    size_t permute_bytes; /* bytes moe_permute needs in its own workspace argument */
} moe_workspace_layout;

int moe_workspace_layout_get(const moe_shape* s, moe_workspace_layout* out);

/* ------------------------------------------------------------------ the five calls */

/* a1. Router.  logits = x Wr^T (+ bias); topk_ids[t] = the k largest logits in
 * descending order (ties: lower expert index); topk_w[t] = softmax over those k
 * logits.  x: device dtype[T][H]; Wr: device dtype[E][H]; bias: device float[E]
 * or NULL; topk_ids: device int32[T][k]; topk_w: device float[T][k]; logits:
 * device float[T][E] or NULL. */
int moe_route(const moe_shape* s, const void* x, const void* Wr, const float* bias,
              int32_t* topk_ids, float* topk_w, float* logits, void* stream);

/* a2. Permutation by expert: histogram counts[E], exclusive scan offsets[E+1],
 * stable placement (ascending flat index t*k+slot inside an expert):
 * row_of[t*k+slot] = row, row_src[row] = t*k+slot, x_perm[row] = x[t].
 * row_w (device float[R], may be NULL) receives topk_w[row_src[row]] when topk_w
 * is given.  x / x_perm may both be NULL to skip the row copy.  workspace:
 * device, at least moe_workspace_layout.permute_bytes. */
int moe_permute(const moe_shape* s, const int32_t* topk_ids, const float* topk_w, const void* x,
                int32_t* counts, int32_t* offsets, int32_t* row_src, int32_t* row_of,
                float* row_w, void* x_perm, void* workspace, size_t workspace_bytes, void* stream);

/* a3. Grouped SwiGLU expert FFN over paged weights.  For every row r of expert
 * e (offsets[e] <= r < offsets[e+1]):
 *   h[r] = dtype( silu(W1_e x_perm[r]) * (W3_e x_perm[r]) ),  out[r] = W2_e h[r]
 * and out[r] *= row_w[r] when row_w != NULL.  x_perm: device dtype[R][H];
 * offsets: device int32[E+1]; page_table: device int32[E][pages_per_expert];
 * page_pool: device, pool_pages * page_bytes; h_ws: device dtype[R][F];
 * out: device float[R][H]; status: device int32[4] or NULL (see moe_workspace_layout.status).
 * The kernels only ever OR error bits into status[0] and overwrite status[2], status[3];
 * they never clear: the CALLER zeroes the four words before the call (moe_layer does that
 * for its own status words, in one of its kernels). */
int moe_expert_ffn(const moe_shape* s, const void* x_perm, const int32_t* offsets,
                   const int32_t* page_table, const void* page_pool, int64_t pool_pages,
                   const float* row_w, void* h_ws, float* out, int32_t* status, void* stream);

/* a4. Un-permute and combine: y[t] = sum_slot w * out[row_of[t*k+slot]], with
 * w = topk_w[t][slot], or 1 when topk_w == NULL (weight already applied).
 * out: device float[R][H]; y: device float[T][H]. */
int moe_combine(const moe_shape* s, const float* out, const int32_t* row_of,
                const float* topk_w, float* y, void* stream);

/* a5. The whole layer in one call, on one stream, without host synchronisation.
 * Intermediates live in `workspace` at the offsets of moe_workspace_layout_get
 * and may be inspected after the stream has finished.  With bf16 data and option
 * "fuse_gather" = 1 (the default) the gate/up GEMM reads row r of its input as
 * x[row_src[r] / k], and x_perm is not written (needs T * H * 2 < 2^32, else the copy
 * is made). */
int moe_layer(const moe_shape* s, const void* x, const void* Wr, const float* bias,
              const int32_t* page_table, const void* page_pool, int64_t pool_pages,
              float* y, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ streamed pages
 *
 * Expert pages live in pinned host memory; the library copies them, expert by
 * expert, into a two-slot device region (2 * pages_per_expert pages: the
 * paper's double buffer of appendix A.1) on `copy_stream` while the expert
 * GEMMs of the previous expert run on `stream`.  A copy waits only for the GEMMs
 * that last read the slot it fills - also those of an earlier call on the same
 * streamer: calls on one streamer must be issued one after the other (from one
 * host thread or otherwise ordered), and `copy_stream` must be the same stream
 * in all of them, or the copies of two calls could overtake each other.
 */
typedef struct moe_streamer moe_streamer;

/* host_pages: pinned, host_pool_pages * page_bytes; host_page_table: host
 * int32[E][pages_per_expert], slots into host_pages; slots: device,
 * 2 * pages_per_expert * page_bytes; slot_table: device int32[2][pages_per_expert],
 * filled here.  Creates HIP events (not a hot call). */
int moe_stream_create(const moe_shape* s, const void* host_pages, int64_t host_pool_pages,
                      const int32_t* host_page_table, void* slots, int32_t* slot_table,
                      moe_streamer** out);
int moe_stream_destroy(moe_streamer* st);
/* Same results as moe_expert_ffn / moe_layer with all pages resident. */
int moe_expert_ffn_streamed(moe_streamer* st, const void* x_perm, const int32_t* offsets,
                            const float* row_w, void* h_ws, float* out, int32_t* status,
                            void* stream, void* copy_stream);
int moe_layer_streamed(moe_streamer* st, const void* x, const void* Wr, const float* bias,
                       float* y, void* workspace, size_t workspace_bytes,
                       void* stream, void* copy_stream);

/* moe_layer for callers that cannot allocate device memory and have no workspace to hand
 * over (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * the same layer, same kernels and same result bits as moe_layer, with the workspace in a
 * device array that is part of the library itself (MOE_STATIC_SCRATCH_BYTES per GPU the
 * library runs on, held until the process ends).  The call allocates and frees nothing.
 * Shapes whose moe_workspace_layout.total exceeds MOE_STATIC_SCRATCH_BYTES are refused with
 * MOE_ERR_WORKSPACE_TOO_SMALL before anything is enqueued (the Mixtral-8x7B-shaped layer
 * fits up to 256 tokens, a decode micro-batch).  The first call on a device looks the
 * array's address up (no allocation; make that call outside a graph capture).  All calls on
 * one GPU share that GPU's array: it keeps the last call's intermediates, the status words
 * are cleared by the layer's kernels at each call, and two calls that overlap in time on
 * one GPU (different streams) race.  The intermediates are not exposed. */
#define MOE_STATIC_SCRATCH_BYTES (32u << 20)
int moe_layer_static(const moe_shape* s, const void* x, const void* Wr, const float* bias,
                     const int32_t* page_table, const void* page_pool, int64_t pool_pages,
                     float* y, void* stream);

/* ------------------------------------------------------------------ weight paging over several layers
 *
 * The I/O side of the paper's pipeline (section 4.1, its paragraph on paging the
 * weights and scheduling the transfers, and Algorithm 1; double-buffered weight region of
 * appendix A.1; resident fraction r_w of section 4.2) for a stack of n_layers
 * MoE layers of one shape and n micro-batches of shape.T tokens per layer:
 *   - the first resident_pages_per_expert logical pages of every expert of every
 *     layer stay in the device pool for good (r_w = that number / pages per expert);
 *   - the other pages of layer l+1 are copied host -> device on `copy_stream`
 *     while the n micro-batches of layer l are computed on `stream`, cut into n
 *     chunks of whole pages (one chunk per micro-batch), into the half of a double
 *     buffer that layer l-1 has finished with;
 *   - the hidden states of micro-batch j (the paper's transfer D2) are copied host
 *     -> device on the same copy stream BETWEEN the weight chunks, so a small
 *     transfer never queues behind more than one chunk of weights.
 * Layers are taken cyclically: during the last layer the first layer's pages are
 * fetched for the next call (the next decode step); only the very first call
 * waits for a layer's pages with nothing to overlap.  Every y is bit-identical
 * to moe_layer with all pages resident.
 *
 * Device pool layout (pool_pages from moe_pipeline_pool_pages):
 *   n_layers * E * resident pages, then 2 * E * (pages_per_expert - resident) pages.
 */
typedef struct moe_pipeline moe_pipeline;

int moe_pipeline_pool_pages(const moe_shape* s, int32_t n_layers, int32_t resident_pages_per_expert,
                            int64_t* pool_pages);
/* host_pages[l]: pinned host, host_pool_pages[l] * page_bytes; host_page_tables[l]:
 * host int32[E][pages_per_expert] (copied); device_pool: device, device_pool_pages *
 * page_bytes; device_tables: device int32[n_layers][2][E][pages_per_expert], filled
 * here.  Copies the resident pages synchronously and creates HIP events: not a hot
 * call.  The host page arrays must stay valid until moe_pipeline_destroy. */
int moe_pipeline_create(const moe_shape* s, int32_t n_layers, int32_t max_micro_batches,
                        const void* const* host_pages, const int64_t* host_pool_pages,
                        const int32_t* const* host_page_tables, int32_t resident_pages_per_expert,
                        void* device_pool, int64_t device_pool_pages, int32_t* device_tables,
                        moe_pipeline** out);
int moe_pipeline_destroy(moe_pipeline* p);
/* One pass over all layers.  x_host[l * n_micro + j]: pinned host dtype[T][H], the
 * input of layer l for micro-batch j; x_dev: device staging, dtype[n_micro][T][H];
 * Wr[l]: device dtype[E][H]; bias: NULL or [n_layers] of device float[E] / NULL;
 * y[l * n_micro + j]: device float[T][H] (entries may alias each other if the caller
 * does not need every result).  workspace as for moe_layer.  Enqueues only; if a
 * call fails part way the pipeline must be destroyed. */
int moe_pipeline_run(moe_pipeline* p, int32_t n_micro, const void* const* x_host, void* x_dev,
                     const void* const* Wr, const float* const* bias, float* const* y,
                     void* workspace, size_t workspace_bytes, void* stream, void* copy_stream);

/* ------------------------------------------------------------------ the dense neighbours of the layer
 *
 * The paper's GPU tasks around the MoE FFN (section 4.1): the post-attention task (the O
 * projection, then the MoE FFN) and the pre-attention task (layer norm, then the QKV
 * projection) of the next micro-batch.  The paper does not write their arithmetic
 * down; the forms are those of the models it evaluates: bias-free linear maps, RMS
 * normalisation with a learned scale, an f32 residual stream.  bf16 only.
 *
 * A dense weight W[N][K] is paged like an expert's W2: tiles of 128 output features x
 * 64 reduction elements ordered [n/128][k/64], the last page zero padded; page_table is
 * int32[pages] (moe_linear_pages_required).  K and N multiples of 128.
 */
typedef struct moe_linear_shape {
    int32_t T;          /* rows (tokens) */
    int32_t K;          /* input features */
    int32_t N;          /* output features */
    int32_t dtype;      /* MOE_DTYPE_BF16 */
    int64_t page_bytes;
} moe_linear_shape;

#define MOE_LINEAR_WORKSPACE_BYTES 16

int moe_linear_pages_required(const moe_linear_shape* s, int64_t* pages);
/* Host packer.  W: host bf16[N][K]; page_table: host int32[pages], distinct slots in
 * [0, pool_pages); pages_out: host, pool_pages * page_bytes. */
int moe_linear_pack(const moe_linear_shape* s, const void* W, const int32_t* page_table, int64_t pool_pages,
                    void* pages_out);
/* out[t][n] = sum_k x[t][k] W[n][k].  x: device bf16[T][K]; page_table: device
 * int32[pages]; out: device float[T][N]; workspace: device, MOE_LINEAR_WORKSPACE_BYTES;
 * status: device int32[4] or NULL (bit 0 of [0]: a page-table entry outside the pool). */
int moe_linear(const moe_linear_shape* s, const void* x, const int32_t* page_table, const void* page_pool,
               int64_t pool_pages, float* out, void* workspace, size_t workspace_bytes, int32_t* status, void* stream);
/* s = hidden + delta (hidden may be NULL: s = delta), written to hidden_out when not
 * NULL; x_out = bf16(s / sqrt(mean(s^2) + eps) * gamma).  hidden, delta, hidden_out:
 * device float[T][H]; gamma: device float[H]; x_out: device bf16[T][H].  H a multiple
 * of 4, at most 8192. */
int moe_add_rmsnorm(int32_t T, int32_t H, const float* hidden, const float* delta, const float* gamma, float eps,
                    float* hidden_out, void* x_out, void* stream);
/* out = bf16(in), round to nearest even; n a multiple of 4. */
int moe_cast_bf16(int64_t n, const float* in, void* out, void* stream);

/* Post-attention task: o = attn Wo^T; hidden_mid = hidden + o; x_moe = norm(hidden_mid);
 * y = MoE layer(x_moe).  (The caller adds y to hidden_mid, or passes both to
 * moe_pre_attention, which does.)  attn: device bf16[T][o_proj->K]; hidden: device
 * float[T][H]; o_table: device page table of Wo, slots in the SAME pool as the experts';
 * hidden_mid: device float[T][H]; x_moe: device bf16[T][H]; y: device float[T][H];
 * workspace: device, 256-byte aligned, moe_post_attention_workspace_bytes; the MoE
 * layer's intermediates are at its start (moe_workspace_layout_get). */
int moe_post_attention_workspace_bytes(const moe_shape* s, size_t* bytes);
int moe_post_attention(const moe_shape* s, const moe_linear_shape* o_proj, const void* attn, const float* hidden,
                       const int32_t* o_table, const float* norm_gamma, float eps, const void* Wr, const float* bias,
                       const int32_t* page_table, const void* page_pool, int64_t pool_pages,
                       float* hidden_mid, void* x_moe, float* y, void* workspace, size_t workspace_bytes, void* stream);
/* Pre-attention task: hidden_out = hidden + delta; x_norm = norm(hidden_out);
 * qkv = x_norm Wqkv^T (f32), and its bf16 copy when qkv_bf16 != NULL (what goes to the
 * host for the attention).  hidden may be NULL.  workspace: device,
 * MOE_LINEAR_WORKSPACE_BYTES. */
int moe_pre_attention(const moe_linear_shape* qkv_proj, const float* hidden, const float* delta, const float* norm_gamma,
                      float eps, const int32_t* qkv_table, const void* page_pool, int64_t pool_pages,
                      float* hidden_out, void* x_norm, float* qkv, void* qkv_bf16, void* workspace, size_t workspace_bytes,
                      void* stream);

/* ------------------------------------------------------------------ tuning knobs
 * Named integer options for experiments (kernel variants, tile order); unknown
 * names give MOE_ERR_INVALID_ARG.  The options are process-wide and read at launch
 * time without locking: set them before other threads enqueue work.  Defaults are the
 * measured best.  No option changes a result bit.
 *   "xcd_remap"   1: column-tile groups of the expert GEMMs are dealt round robin to the
 *                 8 XCDs; 0: block b computes tile b.                       default 1
 *   "half_tiles"  1: bf16 row tiles with at most 128 rows run shorter loops.   default 1
 *   "down_cols"   column tiles of the bf16 down GEMM: 0 = by grid size, 1 = 128 wide,
 *                 2 = 256 wide.                                              default 0
 *   "gate_cols"   column tiles of the bf16 gate/up GEMM: 0 = by grid size, 1 = 64 features wide,
 *                 2 = 128 features wide.                                     default 0
 *   "tall_tiles"  1: bf16: row tiles may be up to 32 rows higher than 256, so that a small
 *                 remainder of an expert's rows needs no tile of its own.        default 1
 *   "fuse_gather" 1: moe_layer's bf16 gate/up GEMM gathers the rows of x itself (no
 *                 x_perm copy).                                              default 1
 *   "chunked"     tile order of the expert GEMMs: the column tiles of an expert go to the XCDs
 *                 in chunks of about this many tiles (at most 32); 0: one by one.  default 32
 *   "tall_first"  1: inside a chunk the tall row tiles are numbered first.       default 1
 *   "balance"     1: no XCD runs more than an eighth of the tiles of an expert-GEMM launch: one
 *                 that was dealt more gives its last tiles to XCDs with fewer.   default 1
 *   "profile"     1: moe_layer records stage events (see below).  Setting it to 1 creates
 *                 the events (the only option whose setter touches the device; it may
 *                 return MOE_ERR_HIP); the layer calls themselves create nothing.  default 0 */
int moe_set_option(const char* name, int value);
int moe_get_option(const char* name, int* value);

/* ------------------------------------------------------------------ rate probes
 * Measurement helpers for the roofline model's inputs (the paper's performance model, section 4.2, is fed
 * with profiled rates of the hardware): moe_probe_stream_read launches `blocks` blocks that together read
 * `bytes` bytes (a multiple of 16, 16-byte aligned) from device memory at src once and discard them; timing the
 * launch gives the read rate device memory sustains for a kernel of nothing but coalesced loads.  sink: device
 * int32 or NULL (never written for real data).  Enqueue only, no synchronisation. */
int moe_probe_stream_read(const void* src, size_t bytes, int32_t blocks, int32_t* sink, void* stream);

/* ------------------------------------------------------------------ stage timing
 * For measurements only.  While option "profile" is 1, moe_layer records HIP
 * events on its stream around its stages (route, permute, gate/up GEMM, down
 * GEMM, combine); the last MOE_PROFILE_RING calls are kept.  moe_profile_read
 * must be called after the stream has been synchronised: it writes the average
 * duration of each stage in milliseconds to avg_ms[MOE_PROFILE_STAGES], the
 * number of calls averaged to *n_calls, and forgets them. */
#define MOE_PROFILE_STAGES 5
#define MOE_PROFILE_RING 256
int moe_profile_read(double* avg_ms, int* n_calls);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
