/*
 * cascade_attn.h -- C ABI of the block-cascaded self-attention library for MI355X (gfx950).
 *
 * One forward of a block-cascaded video DiT layer: the queries of several in-flight
 * latent-frame blocks, each at its own denoising step, attend to a shared KV pool that
 * holds the clean cache of finished blocks (rolling window, optional sink) and the K/V
 * of the in-flight blocks themselves (paper Sec. 3.2: the blocks of an iteration are batched
 * and attend together; Sec. 3.3: one KV pool that every block reads; Alg. 1).
 *
 * Conventions
 *   - Every function returns int32_t: CA_OK (0) or a negative CA_E* code.  Nothing throws,
 *     aborts or prints.  On error no metadata changes and no GPU work is enqueued.
 *   - "dev" pointers are device (HBM) addresses, everything else is host memory.
 *   - The caller owns every device buffer (the pool included) and the HIP stream.  ca_ctx
 *     owns host metadata only.  Device calls are asynchronous on the given stream (a
 *     hipStream_t passed as void*, NULL = the default stream) and never synchronise; device
 *     buffers must stay valid until that work has run.
 *   - Device calls enqueue kernel launches only (no allocation, no memset, no copy).  The
 *     first bf16 forward / linear call on a device also sets a kernel attribute; after that
 *     warm-up the calls can be recorded into a HIP graph.  Host metadata (slot map, tags)
 *     changes when the call is made, not when a recorded graph replays.
 *   - A context is not thread-safe; calls on one context that overlap on the GPU in
 *     different streams are the caller's to order.
 *   - Tensors are [token, head, dim] with element strides tok_stride / head_stride and unit
 *     stride along dim.  dtype is that of ca_config.dtype (bf16 bit patterns or fp32).
 *   - Token n of a block is at (frame, row, col) = (Fb*g + n / (gh*gw), (n / gw) % gh, n % gw)
 *     for block index g: a block is `frames_per_block` consecutive latent frames (Sec. 3.2).
 *
 * Rotary embedding (not described in the paper; convention of the Wan-family DiT it adapts):
 * head_dim is cut into three runs of consecutive (even, odd) pairs of rope_dim_t, rope_dim_h,
 * rope_dim_w dims for the frame / row / col axes; pair j of an axis with Da dims is rotated
 * by angle pos_a * theta^(-2j/Da): (u, v) -> (u cos - v sin, u sin + v cos).  Positions are
 * absolute and K is stored rotated, so nothing is re-rotated when the window slides.
 *
 * Pool layout.  Slots 0 .. sink+window+max_inflight-1, each holding one block of
 * P = ceil(L / page_tokens) pages per head.  Block g < sink_blocks lives in slot g; any
 * other block in slot sink + ((g - sink) mod (window + max_inflight)).  Page `p` of slot `s`,
 * head `h` is page pair number (s*P + p)*heads + h; a page pair is a K page followed by a
 * V page, each page_tokens*head_dim elements.  Inside a page:
 *   fp32 : K and V row-major [token][dim].
 *   bf16 (head_dim 128, page_tokens 128): 256-byte rows of sixteen 16-byte chunks, chunk c of
 *          row r stored at chunk position c ^ (r & 15) (LDS-bank swizzle kept in HBM so a page
 *          is copied to LDS linearly).  K page: row = token, chunk c = dims 8c..8c+7.
 *          V page: row = dim, chunk c = eight tokens: element e of chunk c is token
 *          16*(c/2) + perm[8*(c%2) + e], perm = {0,1,2,3,8,9,10,11,4,5,6,7,12,13,14,15}
 *          (the order in which an MFMA 32x32 accumulator hands P to the next MFMA).
 *   Rows/tokens past the end of a block's last page are stored as zeros.
 * For bf16 the pool ends with a fixed scratch area (about 35 MB) that cascade_attn_forward uses
 * for partial results; forwards on one context must therefore not overlap on the GPU.
 */
#ifndef CASCADE_ATTN_H
#define CASCADE_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  CA_OK = 0,
  CA_EINVAL = -1,       /* null pointer, bad size/stride, inconsistent config               */
  CA_ENOSPC = -2,       /* the block's slot is still held by another block                  */
  CA_ENOENT = -3,       /* block not resident                                                */
  CA_ESTATE = -4,       /* wrong state: evict a sink, promote a clean block, rewrite a clean */
  CA_EUNSUPPORTED = -5, /* dtype / head_dim / page size the kernels do not cover             */
  CA_ENOPOOL = -6,      /* device work asked of a metadata-only context                      */
  CA_EDEVICE = -7,      /* the HIP runtime refused a launch                                  */
  CA_ETOOBIG = -8       /* cascade_attn_forward_static: more partial tiles than its area holds */
};

enum { CA_F32 = 0, CA_BF16 = 1 };
enum { CA_BIDIRECTIONAL = 0, CA_BLOCK_CAUSAL = 1 };          /* Sec. 3.4 / Sec. 4.2 (the causal P4 variant) */
enum { CA_FREE = 0, CA_NOISY = 1, CA_CLEAN = 2, CA_SINK = 3 };

typedef struct ca_ctx ca_ctx;

typedef struct {
  int32_t heads, head_dim;
  int32_t frames_per_block, grid_h, grid_w;      /* L = frames_per_block*grid_h*grid_w       */
  int32_t rope_dim_t, rope_dim_h, rope_dim_w;    /* even, sum == head_dim                    */
  double  rope_theta;
  int32_t sink_blocks, window_blocks, max_inflight;
  int32_t page_tokens;
  int32_t dtype;                                 /* CA_F32 | CA_BF16                         */
} ca_config;

typedef struct {
  int32_t slot;
  int32_t state;          /* CA_NOISY | CA_CLEAN | CA_SINK                                   */
  int64_t block_id;
  int32_t timestep;       /* denoising timestep the stored K/V were computed at              */
  int32_t prompt_epoch;   /* prompt the block was last tagged with                           */
} ca_slot_info;

/* Bytes of device memory the pool needs for this configuration (0 if the config is invalid). */
size_t ca_pool_bytes(const ca_config* cfg);

/* Create a context over a caller-allocated pool of at least ca_pool_bytes() bytes, 256-byte
 * aligned.  pool_dev == NULL with pool_bytes == 0 creates a metadata-only context: the cache
 * calls keep the slot map and tags but enqueue nothing, and cascade_attn_forward /
 * rope3d_apply return CA_ENOPOOL.  The pool's contents are never cleared by the library. */
int32_t ca_create(const ca_config* cfg, void* pool_dev, size_t pool_bytes, ca_ctx** out);
int32_t ca_destroy(ca_ctx* ctx);

/* Publish one block's K/V to the shared pool (Sec. 3.3): rotate K by the block's positions,
 * store K and V into the pages of the block's slot, tag the entry NOISY(timestep, epoch).
 * A block that is already resident and NOISY is rewritten in place (its next denoising step).
 * k_dev, v_dev: [L, heads, head_dim], K before rotation.  slot_out (optional) gets the slot. */
int32_t kv_cache_append(ca_ctx* ctx, int64_t block_id, int32_t timestep, int32_t prompt_epoch,
                        const void* k_dev, const void* v_dev,
                        int64_t tok_stride, int64_t head_stride,
                        void* hip_stream, int32_t* slot_out);

/* The same for the n_blocks (1 .. 8) blocks in flight in one cascade iteration (Alg. 1: every
 * block of the batch publishes its K/V before the shared attention), as one launch.  Entry i
 * is block_ids[i] at timesteps[i] with K/V k_dev[i] / v_dev[i] (host arrays of device
 * pointers; all tensors share tok_stride / head_stride).  The entries take effect in order and
 * all or none: if any of them would fail as a single call, that code is returned and nothing
 * has changed.  A block id may appear once (CA_EINVAL otherwise).  slots_out (optional) gets
 * n_blocks slots. */
int32_t kv_cache_append_batch(ca_ctx* ctx, int32_t n_blocks, const int64_t* block_ids,
                              const int32_t* timesteps, int32_t prompt_epoch,
                              const void* const* k_dev, const void* const* v_dev,
                              int64_t tok_stride, int64_t head_stride, void* hip_stream,
                              int32_t* slots_out);

/* The block has run its cache step tc (Alg. 1: the step at which b advances): NOISY -> CLEAN, or
 * -> SINK when block_id < sink_blocks (Sec. 3.3, first block kept as sink). */
int32_t kv_cache_promote(ca_ctx* ctx, int64_t block_id);

/* Drop a block from the rolling window (Sec. 2.3 / 3.3); a SINK entry refuses (CA_ESTATE). */
int32_t kv_cache_evict(ca_ctx* ctx, int64_t block_id);

/* Prompt switch without re-caching (Sec. 3.5): NOISY entries take the new prompt epoch;
 * CLEAN/SINK entries, the slot map and all K/V bytes stay as they are. */
int32_t kv_cache_retag(ca_ctx* ctx, int32_t new_prompt_epoch);

/* Occupied slots in ascending slot order.  n_out gets the number of occupied slots even when
 * it exceeds cap (then only cap entries are written). */
int32_t kv_cache_snapshot(const ca_ctx* ctx, ca_slot_info* out, int32_t cap, int32_t* n_out);

/* Physical page-pair number of (block, page, head), the rule stated above under "Pool layout";
 * CA_ENOENT if the block is not resident.  The paper fixes no placement (Sec. 3.3 only asks for one
 * pool that every block reads, a rolling window and a sink): the rule is this library's own and is
 * exposed so that a caller -- or a test -- can find a block's bytes. */
int32_t kv_cache_page_index(const ca_ctx* ctx, int64_t block_id, int32_t page, int32_t head,
                            int64_t* index_out);

/* Rotate n_tokens tokens that are consecutive in the video, starting at the first token of
 * latent frame first_frame (frame-major, then row, then col).  x_dev == y_dev is allowed. */
int32_t rope3d_apply(const ca_ctx* ctx, const void* x_dev, void* y_dev, int64_t n_tokens,
                     int64_t first_frame, int64_t tok_stride, int64_t head_stride,
                     void* hip_stream);

/* The same with strides of its own for the output (elements; the two views must not overlap
 * unless they are identical): e.g. q out of a packed [tokens][3][heads][head_dim] projection
 * result straight into the contiguous tensor cascade_attn_forward takes. */
int32_t rope3d_apply_strided(const ca_ctx* ctx, const void* x_dev, int64_t x_tok_stride, int64_t x_head_stride,
                             void* y_dev, int64_t y_tok_stride, int64_t y_head_stride, int64_t n_tokens,
                             int64_t first_frame, void* hip_stream);

/* Block-cascaded attention.  q_dev / out_dev: [n_inflight*L, heads, head_dim] contiguous,
 * rotated queries of the in-flight blocks in the order of inflight_block_ids, which must be
 * strictly ascending, resident and NOISY (their K/V appended for this step).
 * KV sequence: SINK blocks, CLEAN blocks by ascending id, then the in-flight blocks.  Query
 * block i sees every SINK/CLEAN block, and in-flight block j iff mode == CA_BIDIRECTIONAL or
 * j <= i; inside a visible block pair every token pair is visible (Sec. 3.1).  Softmax scale
 * is 1/sqrt(head_dim).  Pages of invisible blocks are never read. */
int32_t cascade_attn_forward(ca_ctx* ctx, const void* q_dev,
                             const int64_t* inflight_block_ids, int32_t n_inflight,
                             int32_t mode, void* out_dev, void* hip_stream);

/* One device's share of the same forward when the in-flight blocks are spread over several
 * GPUs, one block per GPU, all of which hold the whole pool (temporal parallelism, Sec. 3.3 /
 * 3.4: every GPU denoises its own block and reads the others' K/V).  Arguments and KV sequence
 * as for cascade_attn_forward; only the queries of in-flight blocks first .. first+count-1 (an
 * index range into inflight_block_ids) are computed: q_dev / out_dev hold just those blocks,
 * [count*L, heads, head_dim] contiguous.  Each of those rows gets the result the whole forward
 * gives it up to floating-point summation order.  first < 0, count < 1 or a range past
 * n_inflight is CA_EINVAL. */
int32_t cascade_attn_forward_share(ca_ctx* ctx, const void* q_dev,
                                   const int64_t* inflight_block_ids, int32_t n_inflight,
                                   int32_t first, int32_t count, int32_t mode, void* out_dev,
                                   void* hip_stream);

/* rope3d_apply and cascade_attn_forward in one launch: q_dev holds the queries of the in-flight
 * blocks as they leave the projection, not rotated, [n_inflight*L, heads, head_dim] with element
 * strides q_tok_stride / q_head_stride (e.g. the q part of a packed [tokens][3][heads][head_dim]
 * projection result); the kernel rotates each query by the position of its token (block
 * inflight_block_ids[i] starts at latent frame frames_per_block * id) as it loads it, in fp32, and
 * rounds it to bf16 once, after the softmax scale.  Everything else as cascade_attn_forward, whose
 * result on rope3d_apply's output it matches up to that one rounding of Q fewer.  The blocks need
 * not be consecutive in the video.  bf16 contexts only (CA_EUNSUPPORTED otherwise, and for latent
 * frames or grid sizes of 4096 and beyond). */
int32_t cascade_attn_forward_rope(ca_ctx* ctx, const void* q_dev, int64_t q_tok_stride, int64_t q_head_stride,
                                  const int64_t* inflight_block_ids, int32_t n_inflight,
                                  int32_t mode, void* out_dev, void* hip_stream);

/* cascade_attn_forward for callers that can neither allocate device memory nor spare any of their
 * own for the library's intermediate results: code recorded into a HIP graph by a harness that owns
 * every allocation, tight serving loops, hosts that forbid hipMalloc after start-up.  Arguments,
 * checks, kernels and results are those of cascade_attn_forward (bit for bit on a device with at
 * most 32 CUs per XCD); the one difference is where the partial results of split KV walks go: not
 * the area at the end of the caller's pool but a static device array inside this library, 256
 * partial tiles = 34.6 MB, which every GPU the library runs on holds from the moment the library is
 * loaded on it until the process ends.  The call allocates nothing, frees nothing, copies nothing
 * and sets no memory: it enqueues the same kernel launches.  Nothing in the area has to start at
 * zero (every partial tile is written in full before it is read), and it keeps the last call's
 * contents.  All contexts of a process share one area per GPU: static-scratch forwards that overlap
 * on one GPU (different streams, or different contexts) race and must be ordered by the caller.
 * A forward whose split would need more than 256 partial tiles (possible only on a device with
 * more than 32 CUs per XCD) is refused with CA_ETOOBIG and nothing is enqueued.  The first call on
 * a device (or ca_create with a pool while that device is current) looks up the area's address
 * there and sets the kernel attribute; make it outside stream capture.  fp32 contexts use no
 * scratch at all: for them this is cascade_attn_forward. */
int32_t cascade_attn_forward_static(ca_ctx* ctx, const void* q_dev,
                                    const int64_t* inflight_block_ids, int32_t n_inflight,
                                    int32_t mode, void* out_dev, void* hip_stream);

/* The mask cascade_attn_forward would use: vis[i*n_kv + r] in {0,1} for query block i and
 * KV block r of the KV sequence, kv_block_ids[r] its block id.  cap = capacity of
 * kv_block_ids (and vis holds n_inflight*cap bytes); n_kv_out gets the sequence length. */
int32_t ca_debug_visibility(const ca_ctx* ctx, const int64_t* inflight_block_ids,
                            int32_t n_inflight, int32_t mode, uint8_t* vis,
                            int64_t* kv_block_ids, int32_t cap, int32_t* n_kv_out);

/* ---- The linear maps either side of the attention inside a layer (QKV projection before it,
 * output projection after it).  The paper takes the generator G_theta as given (Sec. 3.1) and says
 * nothing of its layers; the reading taken here is the plain one: no bias, no q/k normalisation,
 * weights stored [out, in], QKV output rows ordered (q|k|v, head, dim).
 * y[m][n] = sum_k x[m][k] * w[n][k], bf16 in and out, fp32
 * accumulation, one rounding to nearest even at the end.  All three matrices are device memory,
 * row-major with row strides ldx, ldw, ldy in elements (multiples of 8, 16-byte aligned bases);
 * nothing is allocated and nothing but y[0..m_rows) x [0..n_out) is written.  The QKV projection
 * writes [tokens][3][heads][head_dim] rows that rope3d_apply and kv_cache_append take as strided
 * views.  Supported shapes: n_out a multiple of 8, k_in a multiple of 128 (CA_EUNSUPPORTED
 * otherwise); m_rows is free (0: nothing is done, CA_OK).  Tiles are 256 x 256: an n_out that is not
 * a multiple of 256 costs the padding of its last column tile. */
int32_t layer_linear_bf16(const void* x_dev, const void* w_dev, void* y_dev, int64_t m_rows, int32_t n_out,
                          int32_t k_in, int64_t ldx, int64_t ldw, int64_t ldy, void* hip_stream);

/* The QKV projection of the blocks in flight and the publication of their K/V (kv_cache_append_batch)
 * as one launch: the projection's epilogue rotates the K columns and writes K and V straight into
 * the pages of the blocks' slots, so that neither ever exists as a [token, head, dim] tensor in
 * HBM (Sec. 3.3: every block's K/V go to the shared pool at every self-attention layer; Alg. 1:
 * the blocks of an iteration are forwarded together).  x_dev: [n_blocks * L, k_in] activations,
 * block i's L tokens at rows i*L .., row stride ldx; w_qkv_dev: [3 * heads * 128, k_in], output
 * rows ordered (q|k|v, head, dim), row stride ldw (the reading stated for layer_linear_bf16).
 * q_out_dev: [n_blocks * L, heads, 128] contiguous, gets the queries as they leave the projection,
 * not rotated: cascade_attn_forward_rope takes them as they are.  Metadata as
 * kv_cache_append_batch: entries NOISY(timestep, epoch), all or none; slots_out optional.
 * The pool bytes are those that layer_linear_bf16 followed by kv_cache_append_batch on its k and v
 * columns would write, byte for byte.  bf16 contexts with an even number of heads and k_in a
 * multiple of 128 (CA_EUNSUPPORTED otherwise); row tiles are counted per block, so the launch
 * computes ceil(L / 256) * 256 rows per block. */
int32_t layer_qkv_publish(ca_ctx* ctx, int32_t n_blocks, const int64_t* block_ids, const int32_t* timesteps,
                          int32_t prompt_epoch, const void* x_dev, int64_t ldx, const void* w_qkv_dev,
                          int64_t ldw, int32_t k_in, void* q_out_dev, void* hip_stream, int32_t* slots_out);

/* ---- Cascade scheduler: the control flow of Algorithm 1, host integers only.
 * State (b, tau, d) = primary block, timestep index of the primary block, cascade depth.  An
 * iteration forwards blocks b .. b + min(d, G-1), block b+i at timesteps[tau - i] (older blocks
 * are cleaner).  timesteps = {t3, t2, t1, t0, tc}: the second-to-last entry is t0 (the step whose
 * prediction is emitted), the last is the cache step tc.  Only n_parallel == n_timesteps and
 * n_blocks >= n_parallel are supported (the listing is not self-consistent otherwise). */
typedef struct ca_sched ca_sched;
typedef struct {
  int64_t block_id;
  int32_t timestep_index;   /* index into timesteps */
  int32_t timestep;
} ca_sched_entry;

int32_t ca_sched_create(int64_t n_blocks, int32_t n_parallel, const int32_t* timesteps,
                        int32_t n_timesteps, ca_sched** out);
/* The same walk with a lag between consecutive blocks: block j enters `lag` iterations after
 * block j-1 and moves one timestep per iteration, so at most ceil(n_timesteps / lag) blocks are in
 * flight.  lag 1 is Algorithm 1; lag = n_timesteps is sequential generation; for the five-entry
 * timestep list, lag 5, 3, 2, 1 give the 1-, 2-, 3- and 5-block cascades of the ablation
 * (Sec. 4.2, Fig. 7).  1 <= lag <= n_timesteps, any n_blocks >= 1. */
int32_t ca_sched_create_lagged(int64_t n_blocks, const int32_t* timesteps, int32_t n_timesteps, int32_t lag,
                               ca_sched** out);
int32_t ca_sched_destroy(ca_sched* s);
/* The batch of the current iteration, oldest block first; *n_out == 0 once the rollout is over. */
int32_t ca_sched_batch(const ca_sched* s, ca_sched_entry* out, int32_t cap, int32_t* n_out);
/* After the forward of the current batch (Alg. 1, lines 12-24): which block ran at t0 and is
 * emitted (-1 if none), which block completed tc (-1 if none); then advance (b, tau, d).
 * ca_sched_state: b = oldest block in flight, tau = its timestep index, d = batch size - 1
 * (-1 once the rollout is over); with lag 1 these are Alg. 1's state variables. */
int32_t ca_sched_advance(ca_sched* s, int64_t* emitted_block, int64_t* completed_block);
int32_t ca_sched_state(const ca_sched* s, int64_t* b, int32_t* tau, int32_t* d, int64_t* iteration);

const char* ca_strerror(int32_t code);

/* Text of the HIP error behind the calling thread's most recent CA_EDEVICE ("" if none): error
 * reporting of this boundary, no counterpart in the paper. */
const char* ca_last_device_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CASCADE_ATTN_H */
