/*
 * libmtla -- Multi-head Temporal Latent Attention (arxiv 2505.13544) hot path
 * for AMD MI355X (gfx950).  Plain C ABI: pointers and sizes only.
 *
 * Notation (the paper's): n_h heads of width d_h, latent width r, decoupled
 * RoPE width d_R (the paper's d_h^R), hyper-network width d_y, temporal stride
 * s.  Token index i is 1-based in the paper; here p = i-1 is the 0-based
 * position, the token's slot is p / s, and a new slot opens when p % s == 0.
 * After T tokens a sequence owns ceil(T/s) slots.
 *
 * Memory.  Every pointer marked "device" is device (HBM) memory owned by the
 * caller for the whole call; the library allocates and frees no device memory
 * and keeps no pointer after a call returns (one exception, stated there:
 * mtla_set_shared_prefix).  `mtla_ctx` owns host memory only.
 * All arrays are row-major with the innermost dimension contiguous and must be
 * 16-byte aligned.  "elem" is the storage type chosen in the config: float
 * (MTLA_F32) or bfloat16 (MTLA_BF16, round-to-nearest-even); all sums are
 * accumulated in fp32 whatever the storage type, and attention outputs are
 * returned as fp32.
 *
 * Asynchrony.  Compute calls validate their arguments on the host, enqueue
 * kernels on `hip_stream` (a hipStream_t passed as void*, NULL = the default
 * stream) and return without synchronising.
 *
 * Errors.  No call aborts or throws.  Host-detectable problems (NULL pointer,
 * batch larger than max_batch, unsupported shape ...) return an error code
 * before anything is enqueued.  Sequence lengths live on the device, so an
 * append that would overflow a sequence's slot capacity is refused on the
 * device: that sequence is left untouched and a sticky flag is raised in the
 * workspace header, to be read with mtla_device_status().
 */
#ifndef MTLA_H_
#define MTLA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MTLA_OK = 0,
  MTLA_ERR_INVALID_ARG = 1, /* NULL where a pointer is required, bad batch/T ...  */
  MTLA_ERR_SHAPE = 2,       /* config fields out of the supported range            */
  MTLA_ERR_CAPACITY = 3,    /* a sequence would exceed max_slots (device status)   */
  MTLA_ERR_UNSUPPORTED = 4, /* valid request that this build has no kernel for     */
  MTLA_ERR_HIP = 5,         /* a HIP runtime call failed (launch, copy)            */
  MTLA_ERR_SCRATCH = 6      /* the context needs more decode workspace than the
                               library's static scratch holds (mtla_decode_step_static) */
} mtla_status;

typedef enum { MTLA_F32 = 0, MTLA_BF16 = 1 } mtla_dtype;

typedef struct mtla_config {
  int32_t n_heads;     /* n_h, 1..64                                               */
  int32_t d_head;      /* d_h, multiple of 32, <= 256                              */
  int32_t r;           /* latent width: 64, 128, 256 or 512                        */
  int32_t d_rope;      /* d_R: 32 or 64                                            */
  int32_t d_hyper;     /* d_y, width of both hyper-network linear maps, 1..256     */
  int32_t stride;      /* s >= 1                                                   */
  int32_t max_batch;   /* largest `batch` any call will pass                       */
  int32_t max_slots;   /* slot capacity per sequence = ceil(max tokens / s)        */
  int32_t dtype;       /* mtla_dtype: storage of caches, inputs and weights        */
  float softmax_scale; /* 0 selects 1/sqrt(d_head), the paper's Eq. (with-rope)    */
  int32_t page_slots;  /* 0: every sequence owns max_slots rows of the caches;
                          else slots per page of paged storage (a power of two
                          >= 16, MTLA_BF16 only), see "Paged slot storage"        */
  int32_t n_pages;     /* pages in the pool (paged storage), else 0               */
} mtla_config;

typedef struct mtla_ctx mtla_ctx; /* opaque; host memory only */

/* Validates the config and builds a context.  Touches no device. */
mtla_status mtla_create(const mtla_config* cfg, mtla_ctx** out);
void mtla_destroy(mtla_ctx* ctx);
const char* mtla_status_str(mtla_status st);
/* Text of the last HIP runtime error a library call met on the calling thread (what lies behind
 * an MTLA_ERR_HIP); "no error" if there was none.  Static storage, never freed by the caller. */
const char* mtla_last_hip_error(void);

/* Sizes in bytes of the caller-allocated device buffers.
 *   cache_c   [max_batch, max_slots, r]      elem   compressed latent cache C_hat
 *   cache_kr  [max_batch, max_slots, d_rope] elem   compressed RoPE-key cache K_hat^R
 *   tail_c    [max_batch, r]                 float  fp32 running value of each
 *             sequence's open (last) slot; lets a bf16 cache row be rounded once
 *             from the fp32 sum instead of once per folded token.  Part of the
 *             sequence state, like the caches and seq_len.
 *   workspace decode scratch (absorbed queries, split partials) behind a
 *             256-byte header holding the device status word.
 * Cache bytes per token are (r + d_rope) * sizeof(elem) / s, the paper's
 * KV-cache accounting (end of the section on decoupled RoPE). */
size_t mtla_cache_c_bytes(const mtla_ctx* ctx);
size_t mtla_cache_kr_bytes(const mtla_ctx* ctx);
size_t mtla_page_table_bytes(const mtla_ctx* ctx); /* paged storage: int32 [max_batch, ceil(max_slots / page_slots)], else 0 */
size_t mtla_tail_bytes(const mtla_ctx* ctx);
size_t mtla_workspace_bytes(const mtla_ctx* ctx);
/* Scratch for one mtla_prefill_attn call of this batch and length (absorbed
 * queries and the partial slot states C_hat' for all T rows). */
size_t mtla_prefill_workspace_bytes(const mtla_ctx* ctx, int32_t batch, int32_t T);

/* Clears the workspace header (device status word).  Call once after
 * allocating a workspace, before its first use.  Enqueues a fill kernel. */
mtla_status mtla_workspace_init(mtla_ctx* ctx, void* workspace /*device*/, void* hip_stream);

/* Synchronises `hip_stream`, copies the sticky device status out of the
 * workspace header and clears it.  *status_out is MTLA_OK, MTLA_ERR_CAPACITY
 * (an append met a full sequence) or MTLA_ERR_INVALID_ARG (a device-side index
 * was out of range: pos0 of a continuing prefill, src_index of a reorder); the
 * last one raised wins. */
mtla_status mtla_device_status(mtla_ctx* ctx, void* workspace /*device*/, void* hip_stream,
                               int32_t* status_out /*host*/);

/* Tuning knob: number of cache slots one decode workgroup scans (a multiple
 * of 32; 0 restores the default picked at mtla_create).  The number of
 * splits per sequence is ceil(max_slots / chunk).  Must not change between
 * mtla_workspace_bytes() and the calls using that workspace. */
mtla_status mtla_set_decode_chunk(mtla_ctx* ctx, int32_t chunk_slots);
int32_t mtla_get_decode_chunk(const mtla_ctx* ctx);

/* Tuning knob: how mtla_decode_attn spreads the cache slots over the compute
 * units (bf16 storage).  1 = static: one workgroup per (sequence, chunk of
 * decode_chunk slots), the low-latency choice for small batches.  2 =
 * balanced: one persistent workgroup per compute unit; the 16-slot tiles of all
 * sequences form one flat list cut into equal ranges, so ragged or large
 * batches keep every compute unit streaming.  0 = automatic (balanced once the
 * batch's slot capacity gives every compute unit at least 8 tiles). */
mtla_status mtla_set_decode_schedule(mtla_ctx* ctx, int32_t schedule);

/* Kernel timing for benchmarks.  After mtla_profile_start(ctx, capacity) every
 * mtla_decode_attn and mtla_prefill_attn call records a HIP event pair around
 * its dominant kernel (the attention pass over the cache slots, or over the
 * unmasked columns of the parallel form) on the call's stream, up to `capacity`
 * calls.  mtla_profile_read synchronises on the recorded events, writes the
 * elapsed milliseconds of each bracketed launch to ms_out (host, room for
 * `capacity` floats), the number of launches to *n_out, and ends profiling.
 * Events are host-side runtime objects; no device memory is allocated.  Do not
 * use while the stream is being captured into a HIP graph. */
mtla_status mtla_profile_start(mtla_ctx* ctx, int32_t capacity);
mtla_status mtla_profile_read(mtla_ctx* ctx, float* ms_out /*host*/, int32_t* n_out /*host*/);

/* Benchmark helper, not part of the method: one plain streaming read of `bytes` (>= 16, a
 * multiple of 16 is read) of device memory at `buf` (16-byte aligned) with 16-byte loads from
 * four workgroups per compute unit.  Timing it (events on `hip_stream`) over a buffer much larger
 * than the last-level cache gives the HBM read rate a kernel can reach on the device at hand,
 * which bench.py reports beside the published peak.  `workspace` is an initialised decode
 * workspace (one spare header word is written). */
mtla_status mtla_probe_stream_read(mtla_ctx* ctx, const void* buf /*device*/, size_t bytes,
                                   void* workspace /*device*/, void* hip_stream);

/*
 * mtla_cache_append -- hyper-network weight and cache update for new tokens
 * (Section "Inference using MTLA", Eq. (infer-linear) and the update rule
 * after it; RoPE-key rule of Section "Decoupled Rotary Position Embedding").
 *
 * For sequence b, tokens t = 0 .. n-1 (n = n_new[b], or n_new_max when n_new
 * is NULL) are appended in order at positions p = seq_len[b] + t:
 *   w   = sigmoid( < hyp_A c + hyp_a , hyp_G[p / s] > )      (or w_override)
 *   p % s == 0 :  C_hat[b, p/s] = w c        K_hat^R[b, p/s] = k^R
 *   otherwise  :  C_hat[b, p/s] += w c       K_hat^R[b, p/s] = k^R  (overwrite)
 * then seq_len[b] += n.  n_new_max == 1 is the decode step; larger values
 * build a prefix cache in one call.  If seq_len[b] + n > max_slots * s the
 * sequence is left untouched and MTLA_ERR_CAPACITY is raised in the
 * workspace header (see mtla_device_status).
 *
 *   cache_c, cache_kr  device, in/out   layouts above
 *   tail_c             device, in/out   float [max_batch, r]; may be NULL for
 *                      MTLA_F32 (the fp32 cache row is then its own running sum)
 *   seq_len            device, in/out   int32 [batch] tokens seen so far
 *   c_new              device  elem  [batch, n_new_max, r]       post-LayerNorm latents
 *   kr_new             device  elem  [batch, n_new_max, d_rope]  rotated shared keys
 *   n_new              device  int32 [batch] or NULL; values are clamped to [0, n_new_max]
 *   hyp_A              device  elem  [d_hyper, r]   Linear(c) weight
 *   hyp_a              device  elem  [d_hyper]      Linear(c) bias, or NULL
 *   hyp_G              device  elem  [max_slots, d_hyper]  row j-1 = Linear(pe_j), slot j 1-based
 *   w_override         device  float [batch, n_new_max] or NULL: merge weights to
 *                      use instead of the hyper-network (hyp_* may then be NULL)
 *   w_out              device  float [batch, n_new_max] or NULL: weights used
 *   slot_out           device  int32 [batch, n_new_max] or NULL: slot index p/s of each token
 */
mtla_status mtla_cache_append(mtla_ctx* ctx, void* cache_c, void* cache_kr, float* tail_c,
                              int32_t* seq_len, const void* c_new, const void* kr_new,
                              const int32_t* n_new, int32_t n_new_max, int32_t batch,
                              const void* hyp_A, const void* hyp_a, const void* hyp_G,
                              const float* w_override, float* w_out, int32_t* slot_out,
                              void* workspace, void* hip_stream);

/*
 * mtla_decode_attn -- one new query per sequence against its live slots
 * (Eq. (obsorb) and Eq. (with-rope), incremental case).  Per head h:
 *   q~   = W_K^(h) q_h                                    (absorption)
 *   e_k  = ( <q~, C_hat[b,k]> + <q^R_h, K_hat^R[b,k]> ) * softmax_scale,
 *          k = 0 .. ceil(seq_len[b]/s) - 1
 *   o~   = softmax(e) C_hat[b, :]         -> out_latent
 *   o    = o~ W_V^(h)                      -> out
 * The output projection W_O is outside this library.  The cache is read
 * once per step for all heads.  A sequence with seq_len[b] == 0 yields zeros
 * and lse = -inf.
 *
 *   q          device elem  [batch, n_heads, d_head]
 *   q_rope     device elem  [batch, n_heads, d_rope]   rotated
 *   w_uk       device elem  [n_heads, r, d_head]   w_uk[h,n,k] = W_K[n, h*d_head + k]  (per-head W_K)
 *   w_uv       device elem  [n_heads, d_head, r]   w_uv[h,k,n] = W_V[n, h*d_head + k]  (per-head W_V^T);
 *              NULL iff out is NULL.  Both keep the contracted index innermost.
 *   cache_c, cache_kr, seq_len  device, read only
 *   out        device float [batch, n_heads, d_head] or NULL
 *   out_latent device float [batch, n_heads, r] or NULL
 *   lse        device float [batch, n_heads] or NULL: natural-log normaliser of the scaled logits
 */
mtla_status mtla_decode_attn(mtla_ctx* ctx, const void* q, const void* q_rope, const void* w_uk,
                             const void* w_uv, const void* cache_c, const void* cache_kr,
                             const int32_t* seq_len, int32_t batch, float* out, float* out_latent,
                             float* lse, void* workspace, void* hip_stream);

/*
 * mtla_decode_step -- one whole step of incremental inference (the section on
 * inference with the compressed cache: the update rule after Eq. (infer-linear),
 * then Eq. (with-rope)): the
 * step's token of every sequence is appended exactly as
 * mtla_cache_append(n_new = NULL, n_new_max = 1, hyper-network weights) does,
 * then the step's query attends over the updated cache exactly as
 * mtla_decode_attn does.  Results are identical to the two calls in that order;
 * with bf16 storage the append and the absorption, which do not depend on each
 * other, share one kernel launch.  Arguments, layouts, ownership and errors are
 * those of the two calls (a sequence that is full is left untouched, raises
 * MTLA_ERR_CAPACITY in the workspace header, and is attended as it stands).
 */
mtla_status mtla_decode_step(mtla_ctx* ctx, void* cache_c, void* cache_kr, float* tail_c,
                             int32_t* seq_len, const void* c_new, const void* kr_new,
                             const void* hyp_A, const void* hyp_a, const void* hyp_G,
                             const void* q, const void* q_rope, const void* w_uk, const void* w_uv,
                             int32_t batch, float* out, float* out_latent, float* lse,
                             void* workspace, void* hip_stream);

/*
 * mtla_decode_step_static -- mtla_decode_step for callers that cannot allocate
 * device memory and so cannot bring a workspace: code that runs where
 * hipMalloc is not allowed (under HIP graph capture, inside a tight serving
 * loop, in a harness that forbids it).  The decode workspace (absorbed-query
 * operand, split partials, tile counts) is a static device array of the
 * library, MTLA_STATIC_SCRATCH_BYTES per GPU, resident on every GPU the
 * library has run this call on until the process ends.  The call allocates
 * and frees no device memory and calls no routine that does.
 *
 * Same arguments, results and errors as mtla_decode_step (same kernels), but:
 *   device_status  device int32, the caller's, required: the sticky status word
 *                  a full sequence raises MTLA_ERR_CAPACITY in (the role of the
 *                  workspace header; zero it before the first call, read and
 *                  clear it yourself)
 * and no workspace.  Returns MTLA_ERR_SCRATCH, before anything is enqueued,
 * when mtla_workspace_bytes(ctx) exceeds MTLA_STATIC_SCRATCH_BYTES (many heads
 * times a wide latent: 32 heads at r = 512 do not fit).  The first call on a
 * device resolves the array's address (hipGetSymbolAddress); make it outside
 * any stream capture.  Every call on one GPU -- any context, any stream --
 * uses the same array: calls that overlap in time on one GPU race, calls in
 * stream order do not.
 */
#define MTLA_STATIC_SCRATCH_BYTES (16u << 20)
mtla_status mtla_decode_step_static(mtla_ctx* ctx, void* cache_c, void* cache_kr, float* tail_c,
                                    int32_t* seq_len, const void* c_new, const void* kr_new,
                                    const void* hyp_A, const void* hyp_a, const void* hyp_G,
                                    const void* q, const void* q_rope, const void* w_uk, const void* w_uv,
                                    int32_t batch, float* out, float* out_latent, float* lse,
                                    int32_t* device_status /*device*/, void* hip_stream);

/*
 * Paged slot storage (config.page_slots > 0) -- what the paper's decoding with
 * beams of 10 to 50 hypotheses needs around the path: the two cache arrays are
 * one pool of n_pages pages of page_slots slots each,
 *   cache_c  [n_pages, page_slots, r]       cache_kr [n_pages, page_slots, d_rope]
 * and a caller-owned table  page_table  device int32 [max_batch, max_pages],
 * max_pages = ceil(max_slots / page_slots), says where a sequence's slots live:
 * slot k of sequence b is row k % page_slots of page page_table[b][k / page_slots].
 * max_slots stays the per-sequence capacity.  The library never hands out pages:
 * before a call that appends, the caller has filled the table entries of every
 * page the new tokens reach (entries beyond may hold anything; every entry read
 * is clamped into [0, n_pages), so a wrong table gives wrong rows, not a fault).
 * Sequences may name the same page: a prompt stored once for all its beams is
 * shared pages, as long as nobody appends into a shared page (complete pages
 * never change: a complete slot depends on its own s tokens only).  The table is
 * passed to every call, nothing is retained.
 *
 * The _paged calls below are the calls of the same name with `page_table` behind
 * the state arguments; everything else (arguments, results, errors) is theirs,
 * and the state they leave is the contiguous calls' state row for row.  A
 * context takes either kind only: the other returns MTLA_ERR_INVALID_ARG.  Paged
 * contexts do not take mtla_cache_reorder (see mtla_cache_fork_paged),
 * mtla_set_shared_prefix together with a paged call (MTLA_ERR_UNSUPPORTED),
 * mtla_decode_step_static or the whole-layer calls.
 */
mtla_status mtla_cache_append_paged(mtla_ctx* ctx, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                                    const int32_t* page_table /*device*/, const void* c_new, const void* kr_new,
                                    const int32_t* n_new, int32_t n_new_max, int32_t batch, const void* hyp_A,
                                    const void* hyp_a, const void* hyp_G, const float* w_override, float* w_out,
                                    int32_t* slot_out, void* workspace, void* hip_stream);
mtla_status mtla_decode_attn_paged(mtla_ctx* ctx, const void* q, const void* q_rope, const void* w_uk, const void* w_uv,
                                   const void* cache_c, const void* cache_kr, const int32_t* seq_len,
                                   const int32_t* page_table /*device*/, int32_t batch, float* out, float* out_latent,
                                   float* lse, void* workspace, void* hip_stream);
mtla_status mtla_decode_step_paged(mtla_ctx* ctx, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                                   const int32_t* page_table /*device*/, const void* c_new, const void* kr_new,
                                   const void* hyp_A, const void* hyp_a, const void* hyp_G, const void* q,
                                   const void* q_rope, const void* w_uk, const void* w_uv, int32_t batch, float* out,
                                   float* out_latent, float* lse, void* workspace, void* hip_stream);
mtla_status mtla_prefill_chunk_attn_paged(mtla_ctx* ctx, const void* cache_c, const void* cache_kr, const float* tail_prev,
                                          const int32_t* pos0, const int32_t* page_table /*device*/, const void* q,
                                          const void* q_rope, const void* c, const void* kr, const float* w,
                                          const int32_t* n_new, int32_t batch, int32_t T, int32_t max_past_slots,
                                          const void* w_uk, const void* w_uv, float* out, void* chunk_workspace,
                                          void* workspace, void* hip_stream);
mtla_status mtla_prefill_step_paged(mtla_ctx* ctx, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                                    const int32_t* page_table /*device*/, const void* q, const void* q_rope,
                                    const void* c, const void* kr, const int32_t* n_new, const void* hyp_A,
                                    const void* hyp_a, const void* hyp_G, const void* w_uk, const void* w_uv,
                                    int32_t batch, int32_t T, int32_t max_past_slots, float* out, float* w_out,
                                    void* scratch, void* workspace, void* hip_stream);

/*
 * mtla_cache_fork_paged -- beam reordering over paged storage (the role of
 * mtla_cache_reorder): destination sequence b continues source sequence
 * src_index[b]; several destinations may continue one source.  With
 * pw = (src_seq_len / s) / page_slots the page the next token will be written to:
 *   dst_table[b][k] = src_table[src][k]   for k < pw   (complete pages, shared by reference)
 *   dst_table[b][pw] = fresh_pages[b], and the source's live rows of page pw (at
 *                      most one page; none when the next token opens the page) are
 *                      copied into it
 *   dst_tail_c[b], dst_seq_len[b] = the source's; entries above pw are left alone.
 * So a reordering moves table rows, one open page per beam and the tail shadows,
 * not the caches.  fresh_pages[b] is a page nobody uses -- or the source's own
 * page pw, for at most one destination of a source that is not continued
 * otherwise: that destination takes the page over and nothing is copied.  Keeping
 * count of who refers to which page is the caller's.
 *
 *   cache_c, cache_kr   device, the pool, read and written
 *   src_table, src_tail_c, src_seq_len   device, read only; dst_*: written for sequences 0 .. batch-1,
 *                       other arrays than the sources (reorder into a second set and swap)
 *   src_index, fresh_pages   device int32 [batch]; an index outside [0, max_batch) leaves the destination
 *                       untouched, a page outside [0, n_pages) is clamped; both raise MTLA_ERR_INVALID_ARG
 *                       in the workspace header (mtla_device_status)
 */
mtla_status mtla_cache_fork_paged(mtla_ctx* ctx, void* cache_c, void* cache_kr, const int32_t* src_table,
                                  const float* src_tail_c, const int32_t* src_seq_len, const int32_t* src_index,
                                  const int32_t* fresh_pages, int32_t batch, int32_t* dst_table, float* dst_tail_c,
                                  int32_t* dst_seq_len, void* workspace, void* hip_stream);

/*
 * mtla_set_shared_prefix -- decoding several beams over one stored copy of what
 * they have in common (the appendix on decoding with beams of 10-50: every
 * hypothesis of an utterance starts from the same tokens).  While set, the
 * decode calls of this context (mtla_decode_attn, mtla_decode_step,
 * mtla_layer_decode_step) and the prefill calls that continue from a cache
 * read slots j < prefix_slots[b] of sequence b from
 * the rows of sequence prefix_owner[b] of the same cache_c / cache_kr instead
 * of its own rows, which then need not hold anything; slots from
 * prefix_slots[b] on, the tail shadow, the length and every write stay the
 * sequence's own.  The attended values are the ones of Eq. (with-rope) as long
 * as the first prefix_slots[b] * s tokens of the two sequences are the same
 * tokens: a slot that is complete depends on its own s tokens only (the update rule),
 * so the owner's row is the row the sequence would have written itself.
 *   prefix_owner, prefix_slots   device int32 [n], the caller's.  AN EXCEPTION to
 *       the rule that the library keeps no pointer: the context remembers these
 *       two addresses, and every decode call and continuing prefill call reads
 *       them until they are replaced, so the arrays have to stay allocated (and
 *       may be rewritten between calls).  Both NULL: every sequence reads its own
 *       rows again (the state after mtla_create).  The setting belongs to the
 *       context, not to a stream: calls on two streams see the same arrays.
 *       prefix_owner[b] = b or prefix_slots[b] = 0 leaves sequence b alone.
 *       The kernels clamp both (owner into [0, max_batch), slots into [0, live
 *       slots]), so no value makes them leave the caches; a prefix that is not
 *       common to the two sequences gives the attention over the rows it
 *       names, nothing worse.
 *   n   entries of the two arrays, 1 .. max_batch.  A later call with
 *       batch > n returns MTLA_ERR_INVALID_ARG before anything is enqueued.
 * bf16 storage only, r in {128, 256, 512} under the balanced schedule (any r the
 * matrix-core path takes under the static one, which mtla_set_decode_schedule
 * can force); a decode call that would have to take another kernel returns
 * MTLA_ERR_UNSUPPORTED before anything is enqueued.  The prefill calls that continue from a cache (mtla_prefill_chunk_attn,
 * mtla_prefill_step, mtla_layer_prefill) read the cached slots of a sequence the
 * same way; mtla_prefill_attn (which reads no cache) and the reorder calls do
 * not look at it.
 * Errors: MTLA_ERR_INVALID_ARG (NULL ctx, one array NULL and the other not, n
 * out of range), MTLA_ERR_UNSUPPORTED (fp32 storage).
 */
mtla_status mtla_set_shared_prefix(mtla_ctx* ctx, const int32_t* prefix_owner /*device*/,
                                   const int32_t* prefix_slots /*device*/, int32_t n);

/*
 * mtla_prefill_attn -- the parallel form over a whole sequence under the
 * stride-aware causal mask (Section "MTLA Training with Stride-aware Causal
 * Mask"; with RoPE, the last paragraph of the decoupled-RoPE section).  A pure
 * function of its inputs; it does not touch the cache.  Row m (0-based)
 * attends to the final states of the m/s completed chunks before its own and
 * to its own chunk's running state C_hat'[m] = sum_{n in chunk, n<=m} w[n] c[n]
 * with key k^R[m]: exactly the columns the mask leaves open, and exactly what
 * step m of incremental decoding sees.
 *
 *   q       device elem  [batch, T, n_heads, d_head]
 *   q_rope  device elem  [batch, T, n_heads, d_rope]  rotated
 *   c       device elem  [batch, T, r]
 *   kr      device elem  [batch, T, d_rope]           rotated, uncompressed
 *   w       device float [batch, T]   merge weights (w_out of mtla_cache_append)
 *   seq_lens device int32 [batch] or NULL: rows m >= seq_lens[b] are padding and produce zeros
 *   out        device float [batch, T, n_heads, d_head]
 *   out_latent device float [batch, T, n_heads, r] or NULL
 *   prefill_workspace device, mtla_prefill_workspace_bytes(ctx, batch, T) bytes
 *
 * With bf16 storage and d_head in {64,128} the keys and values are formed
 * explicitly (k = C_hat' W_K^(h), v = C_hat' W_V^(h), Eq. (with-rope) before
 * absorption), which is the cheaper form for many rows per head; out_latent,
 * if asked for, is then a second pass of the same attention kernel with the
 * partial states C_hat' as values (r a multiple of d_head; otherwise out
 * still comes from the explicit form and out_latent alone from the absorbed
 * one).  Other shapes and MTLA_F32 take the absorbed form of Eq. (obsorb).  Both give the same out and
 * out_latent within the bf16 tolerance.  batch * T may not exceed 2^24;
 * MTLA_F32 storage (and bf16 shapes outside r in {128,256,512}, d_head in
 * {64,128}) is limited to batch * T <= 65535 and returns MTLA_ERR_UNSUPPORTED
 * beyond.
 */
mtla_status mtla_prefill_attn(mtla_ctx* ctx, const void* q, const void* q_rope, const void* c,
                              const void* kr, const float* w, const int32_t* seq_lens,
                              int32_t batch, int32_t T, const void* w_uk, const void* w_uv,
                              float* out, float* out_latent, void* prefill_workspace,
                              void* hip_stream);

/*
 * mtla_prefill_chunk_attn -- the parallel form for sequences that continue: T
 * new tokens per sequence behind pos0[b] earlier ones whose state is in the
 * cache (chunked prefill, or a prompt continued after some decoding).  Row m
 * of the chunk is token p = pos0[b] + m of its sequence and gives what step p
 * of incremental inference gives (the update rule after Eq. (infer-linear),
 * Eq. (with-rope)): it attends
 * to the final states of the p / s slots completed before its own -- slots
 * below pos0[b] / s out of the cache, later ones closed inside the chunk --
 * and to its own slot's running state with key k^R[m]; under the stride-aware
 * causal mask of the section on the parallel form these are the open columns
 * of row p.  When pos0[b] % s != 0 the slot in progress continues from
 * tail_prev[b], its value before the chunk.
 * The cache is only read, and only below slot pos0[b] / s, which appending the
 * chunk does not change: mtla_cache_append of the chunk (which yields w) may
 * run before this call, but tail_prev and pos0 are the tail_c and seq_len
 * from BEFORE that append (copies).
 *
 *   cache_c, cache_kr  device elem, the context's geometry
 *   tail_prev  device float [batch, r]
 *   pos0       device int32 [batch], 0 <= pos0[b] / s <= max_past_slots; outside: the device
 *              status becomes MTLA_ERR_INVALID_ARG and that sequence's rows are meaningless
 *   q, q_rope, c, kr, w   device, [batch, T, ..] as for mtla_prefill_attn: the chunk
 *   n_new      device int32 [batch] or NULL: rows m >= n_new[b] are padding and produce zeros
 *   max_past_slots  host: upper bound of pos0[b] / s over the batch (sizes the scratch;
 *              the keys and values of the past slots are formed anew from the latent cache)
 *   out        device float [batch, T, n_heads, d_head]
 *   chunk_workspace  device, mtla_prefill_chunk_workspace_bytes(ctx, batch, T, max_past_slots)
 *   workspace  device, the context's workspace (status word)
 *
 * bf16 storage, explicit form (shapes: d_head 64 or 128, r a multiple of 64 up to 512);
 * MTLA_ERR_UNSUPPORTED otherwise and when batch * (max_past_slots + T) exceeds 2^24.
 *
 * Accuracy.  Against exact arithmetic on the same bf16 inputs `out` stays within
 * 2e-2 for strides s <= 3.  The columns of the past come out of the bf16 cache, and
 * a cache row is the bf16 rounding of a sum of s weighted latents: its magnitude,
 * and with it the rounding error the logits and the values inherit, grows with s.
 * At s = 4 (the largest of the paper's 2, 3, 4) most shapes still stay inside 2e-2,
 * not all: over seeded random shapes with unit-variance latents the decode output
 * was off by 1.5e-2 at the median, by more than 2e-2 in one shape of five and by
 * 2.41e-2 at worst (s = 3: 1.1e-2 and 1.65e-2).  From s = 4 on the bound is
 * 2e-2 * s / 3.  The same holds for every call that reads the cache; mtla_create
 * accepts any s >= 1.
 */
size_t mtla_prefill_chunk_workspace_bytes(const mtla_ctx* ctx, int32_t batch, int32_t T, int32_t max_past_slots);
mtla_status mtla_prefill_chunk_attn(mtla_ctx* ctx, const void* cache_c, const void* cache_kr, const float* tail_prev,
                                    const int32_t* pos0, const void* q, const void* q_rope, const void* c,
                                    const void* kr, const float* w, const int32_t* n_new, int32_t batch, int32_t T,
                                    int32_t max_past_slots, const void* w_uk, const void* w_uv, float* out,
                                    void* chunk_workspace, void* workspace, void* hip_stream);

/*
 * mtla_prefill_step -- a prefill that also emits the cache: mtla_cache_append of T new tokens per
 * sequence followed by mtla_prefill_chunk_attn over them, in one call that takes the state as it
 * is (empty sequences: a whole prompt; otherwise the prompt continues) and keeps the copies of
 * seq_len and tail_c the attention needs in its own scratch.  Arguments as for the two calls;
 * on return seq_len[b] += n_new[b] and the caches cover the new tokens.
 *
 *   w_out    device float [batch, T] or NULL: the merge weights, if the caller wants them
 *   scratch  device, mtla_prefill_step_scratch_bytes(ctx, batch, T, max_past_slots) bytes
 *
 * bf16 storage only (MTLA_ERR_UNSUPPORTED otherwise); every argument is checked before anything is
 * enqueued.
 */
size_t mtla_prefill_step_scratch_bytes(const mtla_ctx* ctx, int32_t batch, int32_t T, int32_t max_past_slots);
mtla_status mtla_prefill_step(mtla_ctx* ctx, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                              const void* q, const void* q_rope, const void* c, const void* kr,
                              const int32_t* n_new, const void* hyp_A, const void* hyp_a, const void* hyp_G,
                              const void* w_uk, const void* w_uv, int32_t batch, int32_t T,
                              int32_t max_past_slots, float* out, float* w_out, void* scratch, void* workspace,
                              void* hip_stream);

/*
 * mtla_cache_reorder -- beam search around the path (the paper decodes with beams of 10 to 50):
 * destination sequence b becomes a copy of source sequence src_index[b], i.e. its live slots
 * ceil(seq_len / s) of C_hat and K_hat^R, its fp32 tail shadow and its length.  Several destinations
 * may continue the same source.  Source and destination states must not overlap (reorder into a
 * second set of buffers and swap); both have the context's max_batch / max_slots geometry.
 *
 *   src_cache_c, src_cache_kr, src_tail_c (NULL iff MTLA_F32 without tail), src_seq_len   device, read only
 *   src_index   device int32 [batch], each in [0, max_batch); an index outside leaves that
 *               destination untouched and raises MTLA_ERR_INVALID_ARG in the workspace header
 *               (mtla_device_status)
 *   dst_*       device, written for sequences 0 .. batch-1
 */
mtla_status mtla_cache_reorder(mtla_ctx* ctx, const void* src_cache_c, const void* src_cache_kr,
                               const float* src_tail_c, const int32_t* src_seq_len, const int32_t* src_index,
                               int32_t batch, void* dst_cache_c, void* dst_cache_kr, float* dst_tail_c,
                               int32_t* dst_seq_len, void* workspace, void* hip_stream);

/*
 * mtla_cache_reorder_from -- the same gather for beams that share a prefix: slots below first_slot
 * are neither read nor written.  For a beam search whose hypotheses all start from one prompt, whose
 * first first_slot slots (complete ones: first_slot * s tokens or fewer are never touched again)
 * were put into every sequence of BOTH sets of buffers once: each reordering then moves only what
 * was generated since, not the prompt.  first_slot = 0 is mtla_cache_reorder.  Tail shadow and
 * length are copied as there.
 */
mtla_status mtla_cache_reorder_from(mtla_ctx* ctx, const void* src_cache_c, const void* src_cache_kr,
                                    const float* src_tail_c, const int32_t* src_seq_len,
                                    const int32_t* src_index, int32_t batch, int32_t first_slot,
                                    void* dst_cache_c, void* dst_cache_kr, float* dst_tail_c,
                                    int32_t* dst_seq_len, void* workspace, void* hip_stream);

/*
 * mtla_layer_decode_step -- one whole MTLA attention layer for one new token
 * per sequence: the projections in front of the path, mtla_decode_step, and
 * the output projection behind it.  Per sequence b, with p = seq_len[b] the
 * 0-based position of the new token:
 *   q    = W_Q x                                   Eq. (query)
 *   q^R  = RoPE_p(W_QR x)   per head               Section "Decoupled Rotary Position Embedding in MTLA"
 *   c    = LayerNorm(W_r x)                        Eq. (low-rank) and the normalisation applied to it
 *   k^R  = RoPE_p(W_KR x)   one head shared by all query heads
 *   o    = mtla_decode_step(c, k^R, q, q^R)        update rule after Eq. (infer-linear), Eq. (with-rope)
 *   y    = W_O concat_h(o_h)                       Eq. (softmax)
 * RoPE turns the pair (2k, 2k+1) of a d_rope-wide vector by p * rope_base^(-2k/d_rope).  LayerNorm
 * is over the r outputs, y = (v - mean) / sqrt(var + ln_eps) (* gamma + beta when given).  k^R is
 * rounded to the storage type (it is stored in the cache); q, q^R and c stay in fp32 until they are used.
 * W_K and W_V stay separate from W_Q and W_O (the two-stage form of Eq. (obsorb)): at decode batch
 * sizes the products W_Q W_K^T and W_V W_O would be n_h r / (n_h d_h) times more weight bytes per step.
 *
 * MTLA_BF16 storage only (MTLA_ERR_UNSUPPORTED otherwise, and for d_model not a multiple of 32).
 * All weights are output-major:
 *   w_q  device elem [n_heads*d_head, d_model]     w_qr device elem [n_heads*d_rope, d_model]
 *   w_r  device elem [r, d_model]                  w_kr device elem [d_rope, d_model]
 *   w_o  device elem [d_model, n_heads*d_head]     ln_gamma, ln_beta device elem [r] or NULL
 *   x    device elem [batch, d_model]
 *   y    device float [batch, d_model]
 *   out  device float [batch, n_heads, d_head] or NULL: the attention output before W_O
 *   scratch device, mtla_layer_scratch_bytes(ctx, batch) bytes, 16-byte aligned; contents are
 *        undefined afterwards.  Everything else as in mtla_decode_step (which it calls).
 */
typedef struct {
  const void* w_q;
  const void* w_qr;
  const void* w_r;
  const void* w_kr;
  const void* w_o;
  const void* ln_gamma; /* nullable */
  const void* ln_beta;  /* nullable */
  int32_t d_model;
  float ln_eps;    /* 0 selects 1e-5 */
  float rope_base; /* 0 selects 10000 */
} mtla_layer_weights;

size_t mtla_layer_scratch_bytes(const mtla_ctx* ctx, int32_t batch);

mtla_status mtla_layer_decode_step(mtla_ctx* ctx, const mtla_layer_weights* lw, void* cache_c, void* cache_kr,
                                   float* tail_c, int32_t* seq_len, const void* x, const void* hyp_A,
                                   const void* hyp_a, const void* hyp_G, const void* w_uk, const void* w_uv,
                                   int32_t batch, float* y, float* out, void* scratch, void* workspace,
                                   void* hip_stream);

/*
 * mtla_layer_prefill -- the same layer for T new tokens per sequence at once
 * (the parallel form): what T calls of mtla_layer_decode_step would give, row
 * by row, as matrix products.  With p = seq_len[b] + m the position of row m:
 *   Q = X W_Q, Q^R = RoPE_p(X W_QR), C = LayerNorm(X W_r), K^R = RoPE_p(X W_KR)   Eqs. (query), (low-rank)
 *   mtla_cache_append of (C, K^R): merge weights and the cache                     Eq. (infer-linear), update rule
 *   mtla_prefill_chunk_attn: stride-aware causal mask over the cached slots and
 *     the new rows                                  Section "MTLA Training with Stride-aware Causal Mask"
 *   Y = concat_h(O_h) W_O                                                          Eq. (softmax)
 * The sequences may be empty (seq_len 0: a whole prompt) or continue (chunked
 * prefill, a prompt after decoding).  On return the state covers the new
 * tokens: seq_len[b] += n_new[b].
 *
 *   lw          host struct of device pointers, as for mtla_layer_decode_step
 *   cache_c, cache_kr, tail_c, seq_len   device, the sequence state, updated
 *   x           device elem  [batch, T, d_model]
 *   n_new       device int32 [batch] or NULL (T for all): rows m >= n_new[b] are padding, y = 0 there
 *   max_past_slots  host: upper bound of seq_len[b] / s before the call (0 for empty sequences)
 *   y           device float [batch, T, d_model]
 *   scratch     device, mtla_layer_prefill_scratch_bytes(ctx, d_model, batch, T, max_past_slots) bytes
 *   workspace   device, the context's workspace
 *
 * bf16 storage only; shapes as for mtla_prefill_chunk_attn, d_model a multiple of 32,
 * d_hyper a multiple of 16 up to 64 and s <= 16 (the bulk append that folds the
 * unrounded latents; MTLA_ERR_UNSUPPORTED otherwise).
 * The queries reach the attention as fp16 (scaled by log2(e) / sqrt(d_h)), the attention output
 * reaches W_O as fp16; products accumulate in fp32.
 */
size_t mtla_layer_prefill_scratch_bytes(const mtla_ctx* ctx, int32_t d_model, int32_t batch, int32_t T,
                                        int32_t max_past_slots);
mtla_status mtla_layer_prefill(mtla_ctx* ctx, const mtla_layer_weights* lw, void* cache_c, void* cache_kr,
                               float* tail_c, int32_t* seq_len, const void* x, const int32_t* n_new,
                               const void* hyp_A, const void* hyp_a, const void* hyp_G, const void* w_uk,
                               const void* w_uv, int32_t batch, int32_t T, int32_t max_past_slots, float* y,
                               void* scratch, void* workspace, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MTLA_H_ */
