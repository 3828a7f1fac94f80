// Host-visible launch interface between the C-ABI layer and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace mtla {

// Paged slot storage: the cache arrays are then one pool of fixed-size pages, [n_pages, 2^shift slots, width],
// and slot k of sequence b lives in page table[b * max_pages + (k >> shift)], at offset k mod 2^shift.
// table == NULL: contiguous storage, sequence b owns rows b * max_slots ...
struct PageMap {
  const int32_t* table = nullptr;  // device, [batch rows, max_pages]
  int shift = 0;                   // log2 of the slots per page (a page holds whole 16-slot tiles: shift >= 4)
  int max_pages = 0;               // table entries per sequence = ceil(max_slots / slots per page)
  int n_pages = 0;                 // pages in the pool: a table entry is clamped into [0, n_pages)
};
// Row of the cache arrays that holds slot `slot` of sequence b.
__host__ __device__ inline size_t cache_row(const PageMap& pm, int b, int slot, int max_slots) {
  if (!pm.table) return (size_t)b * max_slots + slot;
  int pg = pm.table[(size_t)b * pm.max_pages + (slot >> pm.shift)];
  pg = pg < 0 ? 0 : (pg < pm.n_pages ? pg : pm.n_pages - 1);  // whatever the table holds, the pool is not left
  return ((size_t)pg << pm.shift) + (size_t)(slot & ((1 << pm.shift) - 1));
}

struct AppendArgs {
  void* cache_c;
  void* cache_kr;
  float* tail_c;
  int32_t* seq_len;
  const void* c_new;
  const void* kr_new;
  const int32_t* n_new;
  const void* hyp_A;
  const void* hyp_a;
  const void* hyp_G;
  const float* w_override;
  float* w_out;
  int32_t* slot_out;
  int32_t* status;  // workspace header word
  int r, d_rope, d_hyper, stride, max_slots, n_new_max, batch;
  const float* c_merge_f32 = nullptr;  // bulk append (matrix-core kernel): the same latents unrounded, [batch, n_new_max, r];
                                       // the merge then folds these and rounds the cache row once
  int c_new_f32;    // fused decode front only: c_new holds fp32 latents (cache storage stays bf16) ...
  float ln_eps;     // ... and, if > 0, they are layer-normalised over r first (the normalisation the
  const void* ln_gamma;  //     paper applies to C = X W_r), times gamma plus beta (storage type, [r]) if given
  const void* ln_beta;
  PageMap pages;         // paged storage of cache_c / cache_kr (table NULL: contiguous)
};

// Row source of the attention kernels.  Decode reads the cache; the prefill
// fallback reads the per-row slot states C_hat' and the uncompressed keys.
struct AttnArgs {
  const void* qcat;      // [rows, n_heads, r + d_rope], pre-scaled to the log2 domain; fp32 for
                         // the vector kernel, two bf16 planes (hi, lo) for the matrix-core kernel
  size_t q_plane;        // elements between the two bf16 planes
  const void* lat;       // decode: cache_c [B, max_slots, r]; prefill: C_hat' [B, T, r]
  const void* key;       // decode: cache_kr;                  prefill: kr [B, T, d_rope]
  const int32_t* seq_len;  // decode: tokens per sequence; prefill: valid rows per sequence or NULL
  float* part_o;         // [rows, n_splits, n_heads, r]   unnormalised partial outputs
  float* part_ml;        // [rows, n_splits, n_heads, 2]   (running max in log2 units, sum)
  int n_heads, r, d_rope, stride, max_slots, chunk, n_splits;
  int batch;             // sequences
  int T;                 // prefill only: rows per sequence (0 selects decode addressing)
  int n_persistent;      // > 0: balanced schedule with this many persistent workgroups
  int32_t* tile_prefix;  // balanced: [batch + 1] running work units, written for the combine kernel
  int run_cost = 0;      // balanced, column-split decode kernel: units a sequence with live slots takes before
                         // its tiles (one unit per tile): the fixed cost of a run, in tiles
  int part_f16;          // column-split decode kernel only: partial outputs are written normalised
                         // (o / l) as IEEE half, [piece, n_heads, r], half the bytes of the fp32 form
  // decode, matrix-core kernels only; NULL = every sequence reads its own rows.  Sequence b reads its
  // first prefix_slots[b] slots from the rows of sequence prefix_owner[b] of the same two arrays.
  const int32_t* prefix_owner = nullptr;
  const int32_t* prefix_slots = nullptr;
  int prefix_rows = 0;   // sequences the two cache arrays hold (max_batch): an owner index is clamped into [0, prefix_rows)
  PageMap pages;         // decode, matrix-core kernels only: paged storage of lat / key (table NULL: contiguous)
};

// Decode kernels: a sequence whose first n slots are read from another sequence's rows of the same
// arrays (a prompt stored once for all beams); those rows lie dlat / dkey elements away from its own.
struct SharedPrefix {
  long long dlat, dkey;
  int n;
};

// Decode kernels, paged storage: the page-table row of the sequence being read (pt == NULL: the row
// pointers are the sequence's own rows).  A 16-slot tile lies inside one page.
struct PageRow {
  const int32_t* pt;
  int shift, n_pages;
  // the streaming kernel's cursor: the page in use, and the one behind it requested ahead of time, so that a
  // tile's loads never wait for a table entry (idx = entry the cursor stands on, -1 before the first lookup)
  int last_entry = 0;   // highest table entry that may be read (max_pages - 1)
  int idx = -1, pg = 0, pg_next = 0;
};

struct AbsorbArgs {
  const void* q;       // [rows, n_heads, d_head]
  const void* q_rope;  // [rows, n_heads, d_rope]
  const void* w_uk;    // [n_heads, r, d_head]
  void* qcat;          // [rows, n_heads, r + d_rope], fp32 or bf16 (out_bf16)
  int rows, n_heads, d_head, r, d_rope;
  int out_bf16;        // 1: bf16 hi/lo operand planes for the matrix-core kernel; 0: fp32 (vector kernel)
  int q_f32;           // matrix-core absorb only: q and q_rope hold fp32 (unrounded) values
  size_t plane;        // out_bf16: elements between the hi plane and the lo plane
  float scale_log2;    // softmax_scale * log2(e)
};

struct CombineArgs {
  const float* part_o;
  const float* part_ml;
  const int32_t* seq_len;
  const void* w_uv;   // [n_heads, d_head, r] or NULL
  float* out;         // [rows, n_heads, d_head] or NULL
  float* out_latent;  // [rows, n_heads, r] or NULL
  float* lse;         // [rows, n_heads] or NULL
  int n_heads, r, d_head, stride, chunk, n_splits, batch, T;
  int n_persistent;             // > 0: the partials came from the balanced schedule
  const int32_t* tile_prefix;   // balanced: [batch + 1] running work units
  int run_cost = 0;             // balanced: units before a row's first tile (as the attention kernel counted)
  int part_f16;                 // part_o holds normalised IEEE-half partials (matrix-core combine only)
};

// Parallel form with explicit per-head keys and values (bf16).
struct ExplicitArgs {
  const void* q;       // [B, T, n_heads, d_head]
  const void* q_rope;  // [B, T, n_heads, d_rope]
  const void* cprime;  // [B, T, r] partial slot states (fp16)
  const void* kr;      // [B, T, d_rope]
  const void* w_uk;    // [n_heads, r, d_head]
  const void* w_uv;    // [n_heads, d_head, r]
  const int32_t* seq_len;  // [B] or NULL
  void* w_kT;          // scratch [n_heads, d_head, r] fp16: W_K^(h) with the latent index innermost
  void* w_v16;         // scratch [n_heads, d_head, r] fp16 copy of w_uv
  void* kr16;          // scratch [B, T, d_rope] fp16 copy of kr
  void* kx;            // scratch [B, T, n_heads, d_head] fp16
  void* vx;            // scratch [B, T, n_heads, d_head] fp16
  float* out;          // [B, T, n_heads, d_head]
  int batch, T, n_heads, d_head, r, d_rope, stride;
  float scale_log2;    // softmax_scale * log2(e)
  // Continuing sequences (a chunk of T new tokens behind pos0[b] earlier ones): cprime, kr16, kx and vx
  // then hold past_pitch + T rows per sequence, the final states (and keys) of the slots completed
  // before the chunk in front of the chunk's own rows.  pos0 == NULL: whole sequences, past_pitch 0.
  const int32_t* pos0 = nullptr;
  int past_pitch = 0;
  int kr_staged = 0;       // kr16 (and cprime) were written by the staging kernel: only the weights are converted
  int q_f16 = 0;           // q and q_rope are fp16 and already carry scale_log2 (the layer's own projections)
  void* out16 = nullptr;   // if set: the output goes here as fp16 [B, T, n_heads, d_head] instead of to `out`
  // > 0 (attention launch only): the latent-space output.  The values are the partial states
  // themselves (cprime, the same rows for every head), r / d_head column slices of d_head per job, and
  // `out` is [B, T, n_heads, r].
  int n_slices = 0;
  float* out_latent = nullptr;  // if set (whole sequences only): also softmax . C_hat' [B, T, n_heads, r], by such a launch
};

// C[z] = A W[z]^T on the matrix cores (see gemm_nt_kernel for the ways out).
struct GemmArgs {
  const void* A = nullptr;                 // [M, K]
  const void* W[2] = {nullptr, nullptr};   // [N, K] each
  void* C[2] = {nullptr, nullptr};         // [M, N] each
  int M = 0, N = 0, K = 0, nz = 1;
  int in_bf16 = 0;                         // A and W: 0 fp16, 1 bf16
  int epi = 0;                             // 0 fp16 = scale * acc, 1 fp16 = scale * RoPE(acc), 3 fp32
  float scale = 1.f;
  int wide = -1;                           // tile columns: -1 chosen by the launcher, 0 128, 1 256
  int N1 = 0;                              // epi 1: columns of the second product A W[1]^T -> C[1] bf16 = RoPE(acc)
  const float2* rope_cs = nullptr;         // epi 1: [M, d_rope / 2] (cos, sin) of every row's angles
  int d_rope = 0;
};

struct RopeTableArgs {
  const int32_t* pos0;   // [B] or NULL: row b*T + t sits at position pos0[b] + t
  float2* table;         // [rows, d_rope / 2]
  size_t rows;
  int T, d_rope;
  double rope_freq[32];  // base^(-2k / d_rope)
};

// Rows of a continuing prefill, in front of the key / value product: slot states of the past out of the cache, the
// chunk's partial states (the slot in progress starts from tail_prev) and all RoPE keys, as fp16.
struct ChunkStageArgs {
  const void* cache_c;      // [*, max_slots, r]       bf16; slots below pos0 / s are read
  const void* cache_kr;     // [*, max_slots, d_rope]
  const float* tail_prev;   // [B, r] value of the slot in progress before the chunk (read iff pos0 % s != 0)
  const int32_t* pos0;      // [B] tokens before the chunk, or NULL: whole sequences (past_pitch 0)
  const void* c;            // [B, T, r]      bf16, the chunk
  const float* c32 = nullptr;  // the same unrounded, or NULL
  const void* kr;           // [B, T, d_rope] bf16
  const float* w;           // [B, T] merge weights
  const int32_t* n_new;     // [B] or NULL: rows at and past n_new[b] are padding (their states are written as zeros)
  void* cprime;             // out [B, past_pitch + T, r]      fp16
  void* kr16;               // out [B, past_pitch + T, d_rope] fp16
  int32_t* status;          // sticky device status word
  int batch, T, r, d_rope, stride, max_slots, past_pitch;
  // NULL, or: slots below prefix_slots[b] of sequence b are read from the rows of sequence prefix_owner[b]
  const int32_t* prefix_owner = nullptr;
  const int32_t* prefix_slots = nullptr;
  int prefix_rows = 0;   // sequences the cache arrays hold (max_batch): an owner index is clamped into [0, prefix_rows)
  PageMap pages;         // paged storage of cache_c / cache_kr (table NULL: contiguous)
};

// Row-wise pieces of the whole-layer prefill: LayerNorm of the latent rows; saving the state the
// chunk starts from and converting W_O.
struct LayerRowsArgs {
  const float* raw = nullptr;   // [rows, r] x W_r
  const void* gamma = nullptr;  // [r] bf16 or NULL
  const void* beta = nullptr;
  void* c = nullptr;            // [rows, r] bf16
  float* c32 = nullptr;         // [rows, r] the same unrounded (may be `raw` itself), or NULL
  size_t rows = 0;
  int r = 0;
  float eps = 1e-5f;
  const int32_t* seq_len = nullptr;  // prep: [batch] -> pos0
  const float* tail_c = nullptr;     //       [batch, r] -> tail_prev
  int32_t* pos0 = nullptr;
  float* tail_prev = nullptr;
  const void* w_o = nullptr;         //       [n_wo] bf16 -> w_o16 fp16
  void* w_o16 = nullptr;
  size_t n_wo = 0;
  int batch = 0;
};

// Beam search: destination sequence b continues source sequence src_index[b].
struct ReorderArgs {
  const void* src_c;
  const void* src_kr;
  const float* src_tail;   // or NULL
  const int32_t* src_len;
  const int32_t* src_index;  // [batch]
  void* dst_c;
  void* dst_kr;
  float* dst_tail;         // or NULL
  int32_t* dst_len;
  int32_t* status;         // workspace header word
  int batch, max_batch, max_slots, stride, r, d_rope, elem;  // elem: bytes per stored element
  int first_slot = 0;      // slots below it are left alone (a prefix every beam already holds)
};

// Beam search over paged storage (bf16): destination b continues source src_index[b] by sharing its complete pages.
struct ForkArgs {
  void* cache_c;             // the pool, [n_pages, page slots, r]
  void* cache_kr;            // [n_pages, page slots, d_rope]
  PageMap src;               // the sources' page table
  const float* src_tail;     // [max_batch, r]
  const int32_t* src_len;    // [max_batch]
  const int32_t* src_index;  // [batch]
  const int32_t* fresh;      // [batch] a free page for every destination
  int32_t* dst_table;        // [max_batch, max_pages]
  float* dst_tail;
  int32_t* dst_len;
  int32_t* status;           // workspace header word
  int batch, max_batch, max_slots, stride, r, d_rope;
};

// Projections in front of and behind the decode path (bf16), one token per sequence.
struct LayerFrontArgs {
  const void* x;       // [batch, d_model]
  const void* w_q;     // [n_heads * d_head, d_model]
  const void* w_qr;    // [n_heads * d_rope, d_model]
  const void* w_r;     // [r, d_model]
  const void* w_kr;    // [d_rope, d_model]
  const int32_t* seq_len;  // [batch]: position of the token being appended
  float* q;            // [batch, n_heads, d_head] fp32: the absorption splits it into bf16 hi + lo planes
  float* q_rope;       // [batch, n_heads, d_rope] fp32, rotated
  float* c;            // [batch, r] fp32, before its layer normalisation
  void* kr;            // [batch, d_rope]
  int batch, d_model, n_heads, d_head, r, d_rope;
  double rope_freq[32];  // rope_base^(-2k / d_rope), k < d_rope / 2
};

struct LayerOutArgs {
  const float* o;      // [batch, k] attention output, k = n_heads * d_head
  const void* w_o;     // [d_model, k]
  float* y;            // [batch, d_model]
  int batch, d_model, k;
};

struct PartialStateArgs {
  const void* c;   // [B, T, r]
  const float* w;  // [B, T]
  const int32_t* seq_len = nullptr;  // [B] or NULL: rows at and past seq_len[b] are padding (written as zeros)
  void* cprime;    // [B, T, r], storage type, or fp16 if out_f16
  int batch, T, r, stride;
  int out_f16;     // 1: write IEEE half (the explicit-form prefill works in fp16)
};

// Optional timing of one launch: the events are attached to the kernel's own dispatch, so their
// difference is the kernel's execution time without any queueing or marker latency.
struct EventPair {
  hipEvent_t start = nullptr, stop = nullptr;
};
template <class K, class A>
inline void launch_timed(K kernel, const dim3& grid, const dim3& block, size_t smem, hipStream_t st,
                         const EventPair& ev, const A& a) {
  if (ev.start)
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)smem, st, ev.start, ev.stop, 0, a);
  else
    hipLaunchKernelGGL(kernel, grid, block, smem, st, a);
}

hipError_t launch_fill_zero(int32_t* p, int n, hipStream_t st);
hipError_t launch_reorder(const ReorderArgs& a, hipStream_t st);
hipError_t launch_fork_paged(const ForkArgs& a, hipStream_t st);
hipError_t launch_stream_read(const void* p, size_t bytes, int32_t* out, int workgroups, hipStream_t st);
hipError_t launch_append(const AppendArgs& a, int dtype, hipStream_t st);
// a bulk append of these shapes runs on the matrix cores (the only bulk kernel that reads AppendArgs::c_merge_f32)
bool append_bulk_mfma_supported(const AppendArgs& a, int dtype);
hipError_t launch_absorb(const AbsorbArgs& a, int dtype, hipStream_t st);
// one-token append and matrix-core absorb of a decode step in a single launch (bf16 storage)
bool decode_front_supported(const AppendArgs& ap, const AbsorbArgs& ab);
hipError_t launch_decode_front(const AppendArgs& ap, const AbsorbArgs& ab, hipStream_t st);
hipError_t launch_attn_split(const AttnArgs& a, int dtype, hipStream_t st, const EventPair& ev = EventPair());
// bf16 matrix-core variant of the split pass (decode addressing only)
bool attn_mfma_supported(const AttnArgs& a);
hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t st, const EventPair& ev = EventPair());
// balanced schedule with the wavefronts splitting the latent columns (r >= 128)
bool attn_cols_supported(const AttnArgs& a);
int attn_cols_workgroups_per_cu(const AttnArgs& a);
// parallel form with the same column split: a workgroup per group of query rows
bool attn_cols_rows_supported(const AttnArgs& a);
hipError_t launch_attn_cols_rows(const AttnArgs& a, hipStream_t st, const EventPair& ev = EventPair());
hipError_t launch_attn_cols(const AttnArgs& a, hipStream_t st, const EventPair& ev = EventPair());
// parallel form with explicit keys / values: K, V up-projection GEMM, then attention (timed by ev)
bool layer_supported(const LayerFrontArgs& a);
hipError_t launch_layer_front(const LayerFrontArgs& a, hipStream_t st);
hipError_t launch_layer_out(const LayerOutArgs& a, hipStream_t st);
bool prefill_explicit_supported(const ExplicitArgs& a);
hipError_t launch_prefill_explicit(const ExplicitArgs& a, hipStream_t st, const EventPair& ev = EventPair());
hipError_t launch_chunk_stage(const ChunkStageArgs& a, hipStream_t st);
hipError_t launch_layer_norm_rows(const LayerRowsArgs& a, hipStream_t st);
hipError_t launch_layer_prefill_prep(const LayerRowsArgs& a, hipStream_t st);
bool gemm_nt_supported(const GemmArgs& a);
hipError_t launch_rope_table(const RopeTableArgs& a, hipStream_t st);
hipError_t launch_gemm_nt(const GemmArgs& a, hipStream_t st);
hipError_t launch_combine(const CombineArgs& a, int dtype, hipStream_t st);
bool combine_mfma_supported(const CombineArgs& a);  // bf16 storage; r, d_head and alignment fit
hipError_t launch_combine_mfma(const CombineArgs& a, hipStream_t st);
hipError_t launch_partial_states(const PartialStateArgs& a, int dtype, hipStream_t st);

}  // namespace mtla
