// C-ABI layer of libmtla: context, argument validation, workspace layout and
// kernel dispatch.  Declarations and their contracts are in include/mtla.h.
#include "../../include/mtla.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "mtla_device.h"
#include "mtla_kernels.h"

struct mtla_ctx {
  mtla_config cfg;
  float scale;           // softmax scale actually used
  int default_chunk;     // decode slots per workgroup chosen at create
  int chunk;             // current value (mtla_set_decode_chunk)
  int schedule = 0;      // mtla_set_decode_schedule: 0 auto, 1 static, 2 balanced
  int n_cu = 0;          // compute units of the device, queried at the first decode call
  std::vector<hipEvent_t> ev_start, ev_stop;  // mtla_profile_start .. mtla_profile_read
  int prof_n = 0;
  const int32_t* prefix_owner = nullptr;  // mtla_set_shared_prefix (device arrays, the caller's)
  const int32_t* prefix_slots = nullptr;
  int prefix_n = 0;                       // entries of the two arrays
};

namespace {

using namespace mtla;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t elem_size(int dtype) { return dtype == MTLA_F32 ? 4 : 2; }

inline int n_splits(const mtla_ctx* c) { return (c->cfg.max_slots + c->chunk - 1) / c->chunk; }

// Persistent workgroups of the balanced decode schedule: one per compute unit, at most this many.
constexpr int kMaxPersistent = 1024;
// Balanced column-split schedule: what starting a sequence costs a workgroup, in tiles.  Measured: a
// workgroup's second run costs it as much as four to five tiles (the first tiles' latency is not hidden
// and the partial has to be stored); 6 to 16 time the same at 8 sequences x 8K slots x 32 heads (25.3 us
// against 29.8 us without), 2 to 6 the same at 256 ragged sequences x 16 heads.
constexpr int kRunCost = 6;
constexpr int kBalancedMaxBatch = 2048;  // the running tile counts of a batch live in LDS

// Partials ("pieces") the decode pass can emit: chunks x sequences under the static schedule,
// one per persistent workgroup plus one per sequence under the balanced one.
inline size_t max_pieces(const mtla_ctx* c) {
  const size_t stat = (size_t)c->cfg.max_batch * n_splits(c);
  const size_t bal = (size_t)kMaxPersistent + c->cfg.max_batch;
  return stat > bal ? stat : bal;
}

// Decode workspace:
// [header 256 B][tile_prefix int32 B+1][qcat fp32 B*n_h*E][part_o fp32 P*n_h*r][part_ml fp32 P*n_h*2]
struct DecodeLayout {
  size_t prefix, qcat, part_o, part_ml, total;
};
DecodeLayout decode_layout(const mtla_ctx* c) {
  const mtla_config& g = c->cfg;
  const size_t B = g.max_batch, nh = g.n_heads, E = g.r + g.d_rope, P = max_pieces(c);
  DecodeLayout L;
  L.prefix = kHeaderBytes;
  L.qcat = align_up(L.prefix + (B + 1) * 4, 256);
  L.part_o = align_up(L.qcat + B * nh * E * 4, 256);
  L.part_ml = align_up(L.part_o + P * nh * g.r * 4, 256);
  L.total = align_up(L.part_ml + P * nh * 2 * 4, 256);
  return L;
}

// Prefill workspace: [qcat fp32 rows*n_h*E][cprime elem rows*r][part_o fp32 rows*n_h*r][part_ml rows*n_h*2]
struct PrefillLayout {
  size_t qcat, cprime, part_o, part_ml, total;
};
PrefillLayout prefill_layout(const mtla_ctx* c, size_t rows) {
  const mtla_config& g = c->cfg;
  const size_t nh = g.n_heads, E = g.r + g.d_rope;
  PrefillLayout L;
  L.qcat = 0;
  // the absorbed query operand, or the explicit form's keys, values, converted weights and RoPE keys,
  // whichever is larger (with a small r the explicit form needs more)
  size_t area = rows * nh * E * 4;
  if (g.dtype == MTLA_BF16 && (g.d_head == 64 || g.d_head == 128)) {
    const size_t need = 2 * align_up(rows * nh * g.d_head * 2, 256) + 2 * align_up(nh * g.d_head * g.r * 2, 256) +
                        align_up(rows * g.d_rope * 2, 256);
    area = area > need ? area : need;
  }
  L.cprime = align_up(L.qcat + area, 256);
  L.part_o = align_up(L.cprime + rows * g.r * elem_size(g.dtype), 256);
  L.part_ml = align_up(L.part_o + rows * nh * g.r * 4, 256);
  L.total = align_up(L.part_ml + rows * nh * 2 * 4, 256);
  return L;
}

// Workspace of a continuing prefill: fp16 [rows*r] states, [rows*d_R] RoPE keys, 2 x [rows*n_h*d_h] keys
// and values, 2 x [n_h*d_h*r] weights; rows = batch * (max_past_slots + T)
struct ChunkLayout {
  size_t cprime, kr16, kx, vx, w_kT, w_v16, total;
};
ChunkLayout chunk_layout(const mtla_ctx* c, size_t rows) {
  const mtla_config& g = c->cfg;
  ChunkLayout L;
  L.cprime = 0;
  L.kr16 = align_up(L.cprime + rows * g.r * 2, 256);
  L.kx = align_up(L.kr16 + rows * g.d_rope * 2, 256);
  L.vx = align_up(L.kx + rows * g.n_heads * g.d_head * 2, 256);
  L.w_kT = align_up(L.vx + rows * g.n_heads * g.d_head * 2, 256);
  L.w_v16 = align_up(L.w_kT + (size_t)g.n_heads * g.d_head * g.r * 2, 256);
  L.total = align_up(L.w_v16 + (size_t)g.n_heads * g.d_head * g.r * 2, 256);
  return L;
}

int pick_chunk(const mtla_config& g) {
  // About two workgroups per compute unit (256 CUs) when every sequence is full; a workgroup's
  // four wavefronts take 16-slot tiles round-robin, so chunks are multiples of 64 slots.
  const long long total = (long long)g.max_batch * g.max_slots;
  long long chunk = (total + 511) / 512;
  chunk = (chunk + 63) / 64 * 64;
  if (chunk < 64) chunk = 64;
  if (chunk > 1024) chunk = 1024;
  return (int)chunk;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Paged storage (cfg.page_slots > 0): table entries per sequence, and the map the kernels follow.
inline int max_pages(const mtla_config& g) { return g.page_slots > 0 ? (g.max_slots + g.page_slots - 1) / g.page_slots : 0; }
inline PageMap page_map(const mtla_ctx* c, const int32_t* table) {
  PageMap pm;
  if (table) {
    int sh = 0;
    while ((1 << sh) < c->cfg.page_slots) ++sh;
    pm.table = table;
    pm.shift = sh;
    pm.max_pages = max_pages(c->cfg);
    pm.n_pages = c->cfg.n_pages;
  }
  return pm;
}
// A call brings a page table exactly when the context stores its slots in pages.
inline bool paging_matches(const mtla_ctx* c, const int32_t* table) { return (c->cfg.page_slots > 0) == (table != nullptr); }

}  // namespace

namespace {
// Last HIP runtime error seen by a library call on this thread (hipSuccess if none).
thread_local hipError_t g_last_hip_error = hipSuccess;
inline bool hip_ok(hipError_t e) {
  if (e == hipSuccess) return true;
  g_last_hip_error = e;
  return false;
}

}  // namespace

extern "C" {

const char* mtla_last_hip_error(void) { return hipGetErrorString(g_last_hip_error); }

const char* mtla_status_str(mtla_status st) {
  switch (st) {
    case MTLA_OK: return "ok";
    case MTLA_ERR_INVALID_ARG: return "invalid argument";
    case MTLA_ERR_SHAPE: return "unsupported shape in config";
    case MTLA_ERR_CAPACITY: return "sequence exceeds max_slots";
    case MTLA_ERR_UNSUPPORTED: return "unsupported request";
    case MTLA_ERR_HIP: return "HIP runtime error";
    case MTLA_ERR_SCRATCH: return "decode workspace larger than the library's static scratch";
  }
  return "unknown status";
}

mtla_status mtla_create(const mtla_config* cfg, mtla_ctx** out) {
  if (!cfg || !out) return MTLA_ERR_INVALID_ARG;
  *out = nullptr;
  const mtla_config& g = *cfg;
  if (g.dtype != MTLA_F32 && g.dtype != MTLA_BF16) return MTLA_ERR_UNSUPPORTED;
  if (g.n_heads < 1 || g.n_heads > 64) return MTLA_ERR_SHAPE;
  if (g.d_head < 32 || g.d_head > 256 || g.d_head % 32) return MTLA_ERR_SHAPE;
  if (!(g.r == 64 || g.r == 128 || g.r == 256 || g.r == 512)) return MTLA_ERR_SHAPE;
  if (!(g.d_rope == 32 || g.d_rope == 64)) return MTLA_ERR_SHAPE;
  if (g.d_hyper < 1 || g.d_hyper > 256) return MTLA_ERR_SHAPE;
  if (g.stride < 1) return MTLA_ERR_SHAPE;
  if (g.max_batch < 1 || g.max_batch > 65535) return MTLA_ERR_SHAPE;
  if (g.max_slots < 1 || (long long)g.max_slots * g.stride > 0x7fffffffLL) return MTLA_ERR_SHAPE;
  if (!(g.softmax_scale >= 0.f) || std::isinf(g.softmax_scale)) return MTLA_ERR_INVALID_ARG;
  if (g.page_slots != 0) {  // paged storage: whole 16-slot tiles per page, a power of two; bf16 only
    if (g.page_slots < 16 || (g.page_slots & (g.page_slots - 1)) || g.page_slots > (1 << 20)) return MTLA_ERR_SHAPE;
    if (g.n_pages < 1 || (long long)g.n_pages * g.page_slots > 0x7fffffffLL) return MTLA_ERR_SHAPE;
    if (g.dtype != MTLA_BF16) return MTLA_ERR_UNSUPPORTED;
  } else if (g.n_pages != 0) {
    return MTLA_ERR_SHAPE;
  }
  mtla_ctx* c = new (std::nothrow) mtla_ctx();
  if (!c) return MTLA_ERR_INVALID_ARG;
  c->cfg = g;
  c->scale = g.softmax_scale > 0.f ? g.softmax_scale : 1.0f / std::sqrt((float)g.d_head);
  c->default_chunk = c->chunk = pick_chunk(g);
  *out = c;
  return MTLA_OK;
}

static void drop_events(mtla_ctx* c) {
  for (hipEvent_t e : c->ev_start) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->ev_stop) (void)hipEventDestroy(e);
  c->ev_start.clear();
  c->ev_stop.clear();
  c->prof_n = 0;
}

void mtla_destroy(mtla_ctx* ctx) {
  if (!ctx) return;
  drop_events(ctx);
  delete ctx;
}

mtla_status mtla_profile_start(mtla_ctx* c, int32_t capacity) {
  if (!c || capacity < 1 || capacity > (1 << 20)) return MTLA_ERR_INVALID_ARG;
  drop_events(c);
  for (int i = 0; i < capacity; ++i) {
    hipEvent_t a, b;
    if (!hip_ok(hipEventCreate(&a))) {
      drop_events(c);
      return MTLA_ERR_HIP;
    }
    c->ev_start.push_back(a);
    if (!hip_ok(hipEventCreate(&b))) {
      drop_events(c);
      return MTLA_ERR_HIP;
    }
    c->ev_stop.push_back(b);
  }
  return MTLA_OK;
}

mtla_status mtla_profile_read(mtla_ctx* c, float* ms_out, int32_t* n_out) {
  if (!c || !ms_out || !n_out) return MTLA_ERR_INVALID_ARG;
  mtla_status rc = MTLA_OK;
  for (int i = 0; i < c->prof_n; ++i) {
    if (!hip_ok(hipEventSynchronize(c->ev_stop[i])) ||
        !hip_ok(hipEventElapsedTime(&ms_out[i], c->ev_start[i], c->ev_stop[i]))) {
      rc = MTLA_ERR_HIP;
      break;
    }
  }
  *n_out = c->prof_n;
  drop_events(c);
  return rc;
}

static size_t cache_rows(const mtla_ctx* c) {  // rows of the two cache arrays: the pool when paged
  return c->cfg.page_slots > 0 ? (size_t)c->cfg.n_pages * c->cfg.page_slots : (size_t)c->cfg.max_batch * c->cfg.max_slots;
}
size_t mtla_cache_c_bytes(const mtla_ctx* c) { return c ? cache_rows(c) * c->cfg.r * elem_size(c->cfg.dtype) : 0; }
size_t mtla_cache_kr_bytes(const mtla_ctx* c) { return c ? cache_rows(c) * c->cfg.d_rope * elem_size(c->cfg.dtype) : 0; }
size_t mtla_page_table_bytes(const mtla_ctx* c) { return c ? (size_t)c->cfg.max_batch * max_pages(c->cfg) * 4 : 0; }
size_t mtla_tail_bytes(const mtla_ctx* c) { return c ? (size_t)c->cfg.max_batch * c->cfg.r * 4 : 0; }
size_t mtla_workspace_bytes(const mtla_ctx* c) { return c ? decode_layout(c).total : 0; }
size_t mtla_prefill_workspace_bytes(const mtla_ctx* c, int32_t batch, int32_t T) {
  if (!c || batch < 1 || T < 1) return 0;
  return prefill_layout(c, (size_t)batch * T).total;
}

mtla_status mtla_set_decode_chunk(mtla_ctx* c, int32_t chunk) {
  if (!c) return MTLA_ERR_INVALID_ARG;
  if (chunk == 0) {
    c->chunk = c->default_chunk;
    return MTLA_OK;
  }
  if (chunk < 32 || chunk % 32) return MTLA_ERR_INVALID_ARG;
  c->chunk = chunk;
  return MTLA_OK;
}
int32_t mtla_get_decode_chunk(const mtla_ctx* c) { return c ? c->chunk : 0; }

mtla_status mtla_set_decode_schedule(mtla_ctx* c, int32_t schedule) {
  if (!c || schedule < 0 || schedule > 2) return MTLA_ERR_INVALID_ARG;
  c->schedule = schedule;
  return MTLA_OK;
}

mtla_status mtla_set_shared_prefix(mtla_ctx* c, const int32_t* prefix_owner, const int32_t* prefix_slots, int32_t n) {
  if (!c || (prefix_owner == nullptr) != (prefix_slots == nullptr)) return MTLA_ERR_INVALID_ARG;
  if (prefix_owner && (n < 1 || n > c->cfg.max_batch)) return MTLA_ERR_INVALID_ARG;
  if (prefix_owner && c->cfg.dtype != MTLA_BF16) return MTLA_ERR_UNSUPPORTED;
  c->prefix_owner = prefix_owner;
  c->prefix_slots = prefix_slots;
  c->prefix_n = prefix_owner ? n : 0;
  return MTLA_OK;
}

mtla_status mtla_workspace_init(mtla_ctx* c, void* workspace, void* hip_stream) {
  if (!c || !workspace) return MTLA_ERR_INVALID_ARG;
  hipError_t e = launch_fill_zero(reinterpret_cast<int32_t*>(workspace), kHeaderBytes / 4,
                                  reinterpret_cast<hipStream_t>(hip_stream));
  return hip_ok(e) ? MTLA_OK : MTLA_ERR_HIP;
}

mtla_status mtla_device_status(mtla_ctx* c, void* workspace, void* hip_stream, int32_t* status_out) {
  if (!c || !workspace || !status_out) return MTLA_ERR_INVALID_ARG;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  int32_t word = 0;
  if (!hip_ok(hipMemcpyAsync(&word, workspace, sizeof(word), hipMemcpyDeviceToHost, st)))
    return MTLA_ERR_HIP;
  if (!hip_ok(hipStreamSynchronize(st))) return MTLA_ERR_HIP;
  *status_out = word;
  if (word != 0) {
    if (!hip_ok(launch_fill_zero(reinterpret_cast<int32_t*>(workspace), 1, st))) return MTLA_ERR_HIP;
    if (!hip_ok(hipStreamSynchronize(st))) return MTLA_ERR_HIP;
  }
  return MTLA_OK;
}

// Checks the arguments of an append and fills the launch record.
static mtla_status append_args(mtla_ctx* c, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                               const void* c_new, const void* kr_new, const int32_t* n_new,
                               int32_t n_new_max, int32_t batch, const void* hyp_A, const void* hyp_a,
                               const void* hyp_G, const float* w_override, float* w_out,
                               int32_t* slot_out, void* workspace, AppendArgs& a,
                               const int32_t* page_table = nullptr) {
  if (!c || !cache_c || !cache_kr || !seq_len || !c_new || !kr_new || !workspace)
    return MTLA_ERR_INVALID_ARG;
  if (!paging_matches(c, page_table)) return MTLA_ERR_INVALID_ARG;
  const mtla_config& g = c->cfg;
  if (batch < 1 || batch > g.max_batch || n_new_max < 1) return MTLA_ERR_INVALID_ARG;
  if (!w_override && (!hyp_A || !hyp_G)) return MTLA_ERR_INVALID_ARG;
  if (g.dtype == MTLA_BF16 && !tail_c) return MTLA_ERR_INVALID_ARG;
  if (!aligned16(cache_c) || !aligned16(cache_kr) || !aligned16(c_new) || !aligned16(kr_new) ||
      !aligned16(workspace))
    return MTLA_ERR_INVALID_ARG;
  // a call longer than the whole capacity can never fit, whatever the lengths are
  if ((long long)n_new_max > (long long)g.max_slots * g.stride && !n_new) return MTLA_ERR_CAPACITY;
  if (((long long)n_new_max + g.stride - 2) / g.stride + 1 > 0x7ffffffLL) return MTLA_ERR_INVALID_ARG;
  a.cache_c = cache_c;
  a.cache_kr = cache_kr;
  a.tail_c = tail_c;
  a.seq_len = seq_len;
  a.c_new = c_new;
  a.kr_new = kr_new;
  a.n_new = n_new;
  a.hyp_A = hyp_A;
  a.hyp_a = hyp_a;
  a.hyp_G = hyp_G;
  a.w_override = w_override;
  a.w_out = w_out;
  a.slot_out = slot_out;
  a.status = reinterpret_cast<int32_t*>(workspace);
  a.r = g.r;
  a.d_rope = g.d_rope;
  a.d_hyper = g.d_hyper;
  a.stride = g.stride;
  a.max_slots = g.max_slots;
  a.n_new_max = n_new_max;
  a.batch = batch;
  a.c_new_f32 = 0;
  a.ln_eps = 0.f;
  a.ln_gamma = a.ln_beta = nullptr;
  a.pages = page_map(c, page_table);
  return MTLA_OK;
}

mtla_status mtla_probe_stream_read(mtla_ctx* c, const void* buf, size_t bytes, void* workspace, void* hip_stream) {
  if (!c || !buf || !workspace || bytes < 16 || !aligned16(buf)) return MTLA_ERR_INVALID_ARG;
  int dev = 0, n = 0;
  if (!hip_ok(hipGetDevice(&dev)) || !hip_ok(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev)) ||
      n < 1)
    return MTLA_ERR_HIP;
  // the folded word goes to an unused header word of the workspace (never word 0, the status)
  int32_t* sink = reinterpret_cast<int32_t*>(workspace) + 1;
  return hip_ok(launch_stream_read(buf, bytes, sink, 4 * n, reinterpret_cast<hipStream_t>(hip_stream))) ? MTLA_OK
                                                                                                         : MTLA_ERR_HIP;
}

mtla_status mtla_cache_append_paged(mtla_ctx* c, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                                    const int32_t* page_table, const void* c_new, const void* kr_new,
                                    const int32_t* n_new, int32_t n_new_max, int32_t batch, const void* hyp_A,
                                    const void* hyp_a, const void* hyp_G, const float* w_override, float* w_out,
                                    int32_t* slot_out, void* workspace, void* hip_stream) {
  AppendArgs a;
  const mtla_status ok = append_args(c, cache_c, cache_kr, tail_c, seq_len, c_new, kr_new, n_new, n_new_max, batch,
                                     hyp_A, hyp_a, hyp_G, w_override, w_out, slot_out, workspace, a, page_table);
  if (ok != MTLA_OK) return ok;
  hipError_t e = launch_append(a, c->cfg.dtype, reinterpret_cast<hipStream_t>(hip_stream));
  return hip_ok(e) ? MTLA_OK : MTLA_ERR_HIP;
}

mtla_status mtla_cache_append(mtla_ctx* c, void* cache_c, void* cache_kr, float* tail_c,
                              int32_t* seq_len, const void* c_new, const void* kr_new,
                              const int32_t* n_new, int32_t n_new_max, int32_t batch,
                              const void* hyp_A, const void* hyp_a, const void* hyp_G,
                              const float* w_override, float* w_out, int32_t* slot_out,
                              void* workspace, void* hip_stream) {
  return mtla_cache_append_paged(c, cache_c, cache_kr, tail_c, seq_len, nullptr, c_new, kr_new, n_new, n_new_max, batch,
                                 hyp_A, hyp_a, hyp_G, w_override, w_out, slot_out, workspace, hip_stream);
}

// Attention of one decode step; `ap` (may be NULL) is the append of the step's token that has to
// come first.
static mtla_status decode_core(mtla_ctx* c, const AppendArgs* ap, const void* q, const void* q_rope,
                               const void* w_uk, const void* w_uv, const void* cache_c,
                               const void* cache_kr, const int32_t* seq_len, int32_t batch, float* out,
                               float* out_latent, float* lse, void* workspace, void* hip_stream,
                               const int32_t* page_table = nullptr) {
  if (!c || !q || !q_rope || !w_uk || !cache_c || !cache_kr || !seq_len || !workspace)
    return MTLA_ERR_INVALID_ARG;
  if (!paging_matches(c, page_table)) return MTLA_ERR_INVALID_ARG;
  const mtla_config& g = c->cfg;
  if (batch < 1 || batch > g.max_batch) return MTLA_ERR_INVALID_ARG;
  if (c->prefix_owner && batch > c->prefix_n) return MTLA_ERR_INVALID_ARG;  // mtla_set_shared_prefix: arrays too short
  if ((out != nullptr) != (w_uv != nullptr)) return MTLA_ERR_INVALID_ARG;
  if (!out && !out_latent && !lse) return MTLA_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(q_rope) || !aligned16(w_uk) || !aligned16(cache_c) ||
      !aligned16(cache_kr) || !aligned16(workspace) || (w_uv && !aligned16(w_uv)))
    return MTLA_ERR_INVALID_ARG;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  char* ws = reinterpret_cast<char*>(workspace);
  const DecodeLayout L = decode_layout(c);

  AbsorbArgs ab;
  ab.q = q;
  ab.q_rope = q_rope;
  ab.w_uk = w_uk;
  ab.qcat = ws + L.qcat;
  ab.rows = batch;
  ab.n_heads = g.n_heads;
  ab.d_head = g.d_head;
  ab.r = g.r;
  ab.d_rope = g.d_rope;
  ab.scale_log2 = c->scale * 1.4426950408889634f;
  ab.q_f32 = (ap && ap->c_new_f32) ? 1 : 0;  // the whole-layer call hands q, q^R and c over unrounded

  AttnArgs at;
  at.qcat = ws + L.qcat;
  at.lat = cache_c;
  at.key = cache_kr;
  at.seq_len = seq_len;
  at.part_o = reinterpret_cast<float*>(ws + L.part_o);
  at.part_ml = reinterpret_cast<float*>(ws + L.part_ml);
  at.n_heads = g.n_heads;
  at.r = g.r;
  at.d_rope = g.d_rope;
  at.stride = g.stride;
  at.max_slots = g.max_slots;
  at.chunk = c->chunk;
  at.n_splits = n_splits(c);
  at.batch = batch;
  at.T = 0;
  at.n_persistent = 0;
  at.tile_prefix = reinterpret_cast<int32_t*>(ws + L.prefix);
  const bool use_mfma = g.dtype == MTLA_BF16 && attn_mfma_supported(at);
  ab.out_bf16 = use_mfma ? 1 : 0;
  ab.plane = at.q_plane = (size_t)g.max_batch * g.n_heads * (g.r + g.d_rope);  // two bf16 planes fill the fp32 area
  if (use_mfma && c->schedule != 1 && batch <= kBalancedMaxBatch) {
    if (c->n_cu == 0) {  // first decode call on this context: ask the device once
      int dev = 0, n = 0;
      if (!hip_ok(hipGetDevice(&dev)) ||
          !hip_ok(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev)) || n < 1)
        return MTLA_ERR_HIP;
      c->n_cu = n < kMaxPersistent ? n : kMaxPersistent;
    }
    // balanced pays off once every persistent workgroup has a run of tiles to stream
    const long long cap_tiles = (long long)batch * ((g.max_slots + 15) / 16);
    if (c->schedule == 2 || cap_tiles >= 8LL * c->n_cu) {
      at.n_persistent = c->n_cu;
      if (attn_cols_supported(at)) {
        const int n = c->n_cu * attn_cols_workgroups_per_cu(at);
        at.n_persistent = n < kMaxPersistent ? n : kMaxPersistent;
      }
    }
  }
  if (page_table) {  // paged storage: the matrix-core kernels follow a page table (with pages a shared prompt is shared pages)
    if (!use_mfma || c->prefix_owner) return MTLA_ERR_UNSUPPORTED;
    if (at.n_persistent > 0 && !attn_cols_supported(at)) at.n_persistent = 0;  // r = 64: the static schedule
    at.pages = page_map(c, page_table);
  }
  if (c->prefix_owner) {  // a shared prefix: only the matrix-core kernels know how to follow it
    if (!use_mfma || (at.n_persistent > 0 && !attn_cols_supported(at))) return MTLA_ERR_UNSUPPORTED;
    at.prefix_owner = c->prefix_owner;
    at.prefix_slots = c->prefix_slots;
    at.prefix_rows = g.max_batch;
  }
  at.part_f16 = 0;
  if (use_mfma && attn_cols_supported(at)) {  // half-size partials if the matrix-core combine will read them
    CombineArgs probe;
    probe.r = g.r;
    probe.d_head = g.d_head;
    probe.n_heads = g.n_heads;
    probe.out = out;
    probe.out_latent = out_latent;
    probe.w_uv = w_uv;
    at.part_f16 = combine_mfma_supported(probe) ? 1 : 0;
    at.run_cost = kRunCost;
  }
  if (ap && decode_front_supported(*ap, ab)) {  // append and absorb do not depend on each other: one launch
    if (!hip_ok(launch_decode_front(*ap, ab, st))) return MTLA_ERR_HIP;
  } else if (ap && ap->c_new_f32) {
    return MTLA_ERR_UNSUPPORTED;  // only the fused front reads fp32 latents
  } else {
    if (ap && !hip_ok(launch_append(*ap, g.dtype, st))) return MTLA_ERR_HIP;
    if (!hip_ok(launch_absorb(ab, g.dtype, st))) return MTLA_ERR_HIP;
  }
  const bool timed = c->prof_n < (int)c->ev_start.size();
  EventPair ev;  // attached to the dispatch itself: the kernel's own begin and end
  if (timed) {
    ev.start = c->ev_start[c->prof_n];
    ev.stop = c->ev_stop[c->prof_n++];
  }
  const hipError_t le = !use_mfma ? launch_attn_split(at, g.dtype, st, ev)
                                  : (attn_cols_supported(at) ? launch_attn_cols(at, st, ev) : launch_attn_mfma(at, st, ev));
  if (!hip_ok(le)) return MTLA_ERR_HIP;

  CombineArgs cb;
  cb.part_o = at.part_o;
  cb.part_ml = at.part_ml;
  cb.seq_len = seq_len;
  cb.w_uv = w_uv;
  cb.out = out;
  cb.out_latent = out_latent;
  cb.lse = lse;
  cb.n_heads = g.n_heads;
  cb.r = g.r;
  cb.d_head = g.d_head;
  cb.stride = g.stride;
  cb.chunk = c->chunk;
  cb.n_splits = at.n_splits;
  cb.batch = batch;
  cb.T = 0;
  cb.n_persistent = at.n_persistent;
  cb.tile_prefix = at.tile_prefix;
  cb.run_cost = at.run_cost;
  cb.part_f16 = at.part_f16;
  if (!hip_ok(launch_combine(cb, g.dtype, st))) return MTLA_ERR_HIP;
  return MTLA_OK;
}

mtla_status mtla_decode_attn_paged(mtla_ctx* c, const void* q, const void* q_rope, const void* w_uk, const void* w_uv,
                                   const void* cache_c, const void* cache_kr, const int32_t* seq_len,
                                   const int32_t* page_table, int32_t batch, float* out, float* out_latent, float* lse,
                                   void* workspace, void* hip_stream) {
  return decode_core(c, nullptr, q, q_rope, w_uk, w_uv, cache_c, cache_kr, seq_len, batch, out, out_latent, lse,
                     workspace, hip_stream, page_table);
}

mtla_status mtla_decode_attn(mtla_ctx* c, const void* q, const void* q_rope, const void* w_uk,
                             const void* w_uv, const void* cache_c, const void* cache_kr,
                             const int32_t* seq_len, int32_t batch, float* out, float* out_latent,
                             float* lse, void* workspace, void* hip_stream) {
  return mtla_decode_attn_paged(c, q, q_rope, w_uk, w_uv, cache_c, cache_kr, seq_len, nullptr, batch, out, out_latent, lse,
                                workspace, hip_stream);
}

mtla_status mtla_decode_step_paged(mtla_ctx* c, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                                   const int32_t* page_table, const void* c_new, const void* kr_new, const void* hyp_A,
                                   const void* hyp_a, const void* hyp_G, const void* q, const void* q_rope,
                                   const void* w_uk, const void* w_uv, int32_t batch, float* out, float* out_latent,
                                   float* lse, void* workspace, void* hip_stream) {
  AppendArgs ap;
  const mtla_status ok = append_args(c, cache_c, cache_kr, tail_c, seq_len, c_new, kr_new, nullptr, 1, batch, hyp_A,
                                     hyp_a, hyp_G, nullptr, nullptr, nullptr, workspace, ap, page_table);
  if (ok != MTLA_OK) return ok;
  return decode_core(c, &ap, q, q_rope, w_uk, w_uv, cache_c, cache_kr, seq_len, batch, out, out_latent, lse,
                     workspace, hip_stream, page_table);
}

mtla_status mtla_decode_step(mtla_ctx* c, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                             const void* c_new, const void* kr_new, const void* hyp_A, const void* hyp_a,
                             const void* hyp_G, const void* q, const void* q_rope, const void* w_uk,
                             const void* w_uv, int32_t batch, float* out, float* out_latent, float* lse,
                             void* workspace, void* hip_stream) {
  return mtla_decode_step_paged(c, cache_c, cache_kr, tail_c, seq_len, nullptr, c_new, kr_new, hyp_A, hyp_a, hyp_G, q, q_rope,
                                w_uk, w_uv, batch, out, out_latent, lse, workspace, hip_stream);
}

// Beam search over paged storage: destination b continues source src_index[b].  Its table row takes the
// source's entries below the page the next token will be written to (complete pages, shared by reference);
// that page becomes fresh_pages[b], into which the source's live rows of it are copied.
mtla_status mtla_cache_fork_paged(mtla_ctx* c, void* cache_c, void* cache_kr, const int32_t* src_table,
                                  const float* src_tail_c, const int32_t* src_seq_len, const int32_t* src_index,
                                  const int32_t* fresh_pages, int32_t batch, int32_t* dst_table, float* dst_tail_c,
                                  int32_t* dst_seq_len, void* workspace, void* hip_stream) {
  if (!c || !cache_c || !cache_kr || !src_table || !src_tail_c || !src_seq_len || !src_index || !fresh_pages ||
      !dst_table || !dst_tail_c || !dst_seq_len || !workspace)
    return MTLA_ERR_INVALID_ARG;
  const mtla_config& g = c->cfg;
  if (g.page_slots <= 0) return MTLA_ERR_INVALID_ARG;
  if (batch < 1 || batch > g.max_batch) return MTLA_ERR_INVALID_ARG;
  if (!aligned16(cache_c) || !aligned16(cache_kr) || !aligned16(src_tail_c) || !aligned16(dst_tail_c)) return MTLA_ERR_INVALID_ARG;
  if (src_table == dst_table || src_tail_c == dst_tail_c || src_seq_len == dst_seq_len) return MTLA_ERR_INVALID_ARG;
  ForkArgs a;
  a.cache_c = cache_c;
  a.cache_kr = cache_kr;
  a.src = page_map(c, src_table);
  a.src_tail = src_tail_c;
  a.src_len = src_seq_len;
  a.src_index = src_index;
  a.fresh = fresh_pages;
  a.dst_table = dst_table;
  a.dst_tail = dst_tail_c;
  a.dst_len = dst_seq_len;
  a.status = reinterpret_cast<int32_t*>(workspace);
  a.batch = batch;
  a.max_batch = g.max_batch;
  a.max_slots = g.max_slots;
  a.stride = g.stride;
  a.r = g.r;
  a.d_rope = g.d_rope;
  return hip_ok(launch_fork_paged(a, reinterpret_cast<hipStream_t>(hip_stream))) ? MTLA_OK : MTLA_ERR_HIP;
}

}  // extern "C"

// Decode scratch of mtla_decode_step_static: one array per GPU the library runs on, resident until the
// process ends.  In host code the array's name only stands for the symbol; the memory is reached
// through the per-device address that hipGetSymbolAddress returns.
static __device__ __align__(256) unsigned char g_static_scratch[MTLA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void* g_static_ptr[kMaxDevices] = {};

// Address of the current device's copy of the array, resolved once per device.
mtla_status static_scratch(void** out) {
  int dev = 0;
  if (!hip_ok(hipGetDevice(&dev))) return MTLA_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return MTLA_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    if (!hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch))) || !p) return MTLA_ERR_HIP;
    g_static_ptr[dev] = p;
  }
  *out = g_static_ptr[dev];
  return MTLA_OK;
}
}  // namespace

extern "C" {

mtla_status mtla_decode_step_static(mtla_ctx* c, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                                    const void* c_new, const void* kr_new, const void* hyp_A, const void* hyp_a,
                                    const void* hyp_G, const void* q, const void* q_rope, const void* w_uk,
                                    const void* w_uv, int32_t batch, float* out, float* out_latent, float* lse,
                                    int32_t* device_status, void* hip_stream) {
  if (!c || !device_status) return MTLA_ERR_INVALID_ARG;
  if (decode_layout(c).total > (size_t)MTLA_STATIC_SCRATCH_BYTES) return MTLA_ERR_SCRATCH;
  void* scratch = nullptr;
  const mtla_status got = static_scratch(&scratch);
  if (got != MTLA_OK) return got;
  AppendArgs ap;
  const mtla_status ok = append_args(c, cache_c, cache_kr, tail_c, seq_len, c_new, kr_new, nullptr, 1, batch, hyp_A,
                                     hyp_a, hyp_G, nullptr, nullptr, nullptr, scratch, ap);
  if (ok != MTLA_OK) return ok;
  ap.status = device_status;  // the caller's word: the scratch is shared by every context on this GPU
  // Nothing in the scratch has to start at zero: tile counts, operand planes and partials are
  // written by this call's kernels before they are read.
  return decode_core(c, &ap, q, q_rope, w_uk, w_uv, cache_c, cache_kr, seq_len, batch, out, out_latent, lse, scratch,
                     hip_stream);
}

mtla_status mtla_cache_reorder(mtla_ctx* c, const void* src_cache_c, const void* src_cache_kr,
                               const float* src_tail_c, const int32_t* src_seq_len, const int32_t* src_index,
                               int32_t batch, void* dst_cache_c, void* dst_cache_kr, float* dst_tail_c,
                               int32_t* dst_seq_len, void* workspace, void* hip_stream) {
  return mtla_cache_reorder_from(c, src_cache_c, src_cache_kr, src_tail_c, src_seq_len, src_index, batch, 0, dst_cache_c,
                                 dst_cache_kr, dst_tail_c, dst_seq_len, workspace, hip_stream);
}

mtla_status mtla_cache_reorder_from(mtla_ctx* c, const void* src_cache_c, const void* src_cache_kr,
                                    const float* src_tail_c, const int32_t* src_seq_len, const int32_t* src_index,
                                    int32_t batch, int32_t first_slot, void* dst_cache_c, void* dst_cache_kr,
                                    float* dst_tail_c, int32_t* dst_seq_len, void* workspace, void* hip_stream) {
  if (first_slot < 0) return MTLA_ERR_INVALID_ARG;
  if (!c || !src_cache_c || !src_cache_kr || !src_seq_len || !src_index || !dst_cache_c || !dst_cache_kr ||
      !dst_seq_len || !workspace)
    return MTLA_ERR_INVALID_ARG;
  const mtla_config& g = c->cfg;
  if (g.page_slots > 0) return MTLA_ERR_INVALID_ARG;  // paged storage reorders page tables: mtla_cache_fork_paged
  if (batch < 1 || batch > g.max_batch) return MTLA_ERR_INVALID_ARG;
  if ((src_tail_c == nullptr) != (dst_tail_c == nullptr)) return MTLA_ERR_INVALID_ARG;
  if (g.dtype == MTLA_BF16 && !src_tail_c) return MTLA_ERR_INVALID_ARG;
  if (!aligned16(src_cache_c) || !aligned16(src_cache_kr) || !aligned16(dst_cache_c) || !aligned16(dst_cache_kr) ||
      !aligned16(workspace))
    return MTLA_ERR_INVALID_ARG;
  if (src_cache_c == dst_cache_c || src_cache_kr == dst_cache_kr || src_seq_len == dst_seq_len ||
      (src_tail_c && src_tail_c == dst_tail_c))
    return MTLA_ERR_INVALID_ARG;
  ReorderArgs a;
  a.src_c = src_cache_c;
  a.src_kr = src_cache_kr;
  a.src_tail = src_tail_c;
  a.src_len = src_seq_len;
  a.src_index = src_index;
  a.dst_c = dst_cache_c;
  a.dst_kr = dst_cache_kr;
  a.dst_tail = dst_tail_c;
  a.dst_len = dst_seq_len;
  a.status = reinterpret_cast<int32_t*>(workspace);
  a.batch = batch;
  a.max_batch = g.max_batch;
  a.max_slots = g.max_slots;
  a.stride = g.stride;
  a.r = g.r;
  a.d_rope = g.d_rope;
  a.elem = (int)elem_size(g.dtype);
  a.first_slot = first_slot;
  return hip_ok(launch_reorder(a, reinterpret_cast<hipStream_t>(hip_stream))) ? MTLA_OK : MTLA_ERR_HIP;
}

// scratch of mtla_layer_decode_step: q, q^R, c (fp32), k^R (storage type) and the attention output (fp32)
struct LayerLayout {
  size_t q, q_rope, c, kr, o, total;
};
static LayerLayout layer_layout(const mtla_ctx* c, size_t batch) {
  const mtla_config& g = c->cfg;
  const size_t es = elem_size(g.dtype);
  LayerLayout L;
  size_t off = 0;
  L.q = off;
  off += align_up(batch * g.n_heads * g.d_head * 4, 256);
  L.q_rope = off;
  off += align_up(batch * g.n_heads * g.d_rope * 4, 256);
  L.c = off;
  off += align_up(batch * g.r * 4, 256);
  L.kr = off;
  off += align_up(batch * g.d_rope * es, 256);
  L.o = off;
  off += align_up(batch * g.n_heads * g.d_head * 4, 256);
  L.total = off;
  return L;
}

size_t mtla_layer_scratch_bytes(const mtla_ctx* c, int32_t batch) {
  if (!c || batch < 1) return 0;
  return layer_layout(c, (size_t)batch).total;
}

mtla_status mtla_layer_decode_step(mtla_ctx* c, const mtla_layer_weights* lw, void* cache_c, void* cache_kr,
                                   float* tail_c, int32_t* seq_len, const void* x, const void* hyp_A,
                                   const void* hyp_a, const void* hyp_G, const void* w_uk, const void* w_uv,
                                   int32_t batch, float* y, float* out, void* scratch, void* workspace,
                                   void* hip_stream) {
  if (!c || !lw || !x || !y || !scratch || !seq_len || !w_uk || !w_uv) return MTLA_ERR_INVALID_ARG;
  if (!lw->w_q || !lw->w_qr || !lw->w_r || !lw->w_kr || !lw->w_o) return MTLA_ERR_INVALID_ARG;
  const mtla_config& g = c->cfg;
  if (batch < 1 || batch > g.max_batch) return MTLA_ERR_INVALID_ARG;
  if (!(lw->ln_eps >= 0.f) || !(lw->rope_base >= 0.f) || std::isinf(lw->ln_eps) || std::isinf(lw->rope_base))
    return MTLA_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(y) || !aligned16(scratch) || !aligned16(lw->w_q) || !aligned16(lw->w_qr) ||
      !aligned16(lw->w_r) || !aligned16(lw->w_kr) || !aligned16(lw->w_o) || (out && !aligned16(out)))
    return MTLA_ERR_INVALID_ARG;
  if (g.dtype != MTLA_BF16) return MTLA_ERR_UNSUPPORTED;
  char* sc = reinterpret_cast<char*>(scratch);
  const LayerLayout L = layer_layout(c, (size_t)batch);
  LayerFrontArgs fa;
  fa.x = x;
  fa.w_q = lw->w_q;
  fa.w_qr = lw->w_qr;
  fa.w_r = lw->w_r;
  fa.w_kr = lw->w_kr;
  fa.seq_len = seq_len;
  fa.q = reinterpret_cast<float*>(sc + L.q);
  fa.q_rope = reinterpret_cast<float*>(sc + L.q_rope);
  fa.c = reinterpret_cast<float*>(sc + L.c);
  fa.kr = sc + L.kr;
  fa.batch = batch;
  fa.d_model = lw->d_model;
  fa.n_heads = g.n_heads;
  fa.d_head = g.d_head;
  fa.r = g.r;
  fa.d_rope = g.d_rope;
  for (int k = 0; k < 32; ++k)
    fa.rope_freq[k] = std::pow((double)(lw->rope_base > 0.f ? lw->rope_base : 10000.f), -2.0 * k / g.d_rope);
  if (!layer_supported(fa)) return MTLA_ERR_UNSUPPORTED;
  // argument check of the step before anything is launched
  AppendArgs ap;
  const mtla_status ok = append_args(c, cache_c, cache_kr, tail_c, seq_len, fa.c, fa.kr, nullptr, 1, batch, hyp_A,
                                     hyp_a, hyp_G, nullptr, nullptr, nullptr, workspace, ap);
  if (ok != MTLA_OK) return ok;
  ap.c_new_f32 = 1;
  ap.ln_eps = lw->ln_eps > 0.f ? lw->ln_eps : 1e-5f;
  ap.ln_gamma = lw->ln_gamma;
  ap.ln_beta = lw->ln_beta;
  {  // the fp32 latent is understood by the fused front of the step only
    AbsorbArgs probe;
    probe.r = g.r;
    probe.d_head = g.d_head;
    probe.d_rope = g.d_rope;
    probe.n_heads = g.n_heads;
    probe.rows = batch;
    probe.out_bf16 = 1;
    probe.q_f32 = 1;
    if (!decode_front_supported(ap, probe)) return MTLA_ERR_UNSUPPORTED;
  }
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  if (!hip_ok(launch_layer_front(fa, st))) return MTLA_ERR_HIP;
  float* o = out ? out : reinterpret_cast<float*>(sc + L.o);
  const mtla_status rc = decode_core(c, &ap, fa.q, fa.q_rope, w_uk, w_uv, cache_c, cache_kr, seq_len, batch, o, nullptr,
                                     nullptr, workspace, hip_stream);
  if (rc != MTLA_OK) return rc;
  LayerOutArgs oa;
  oa.o = o;
  oa.w_o = lw->w_o;
  oa.y = y;
  oa.batch = batch;
  oa.d_model = lw->d_model;
  oa.k = g.n_heads * g.d_head;
  return hip_ok(launch_layer_out(oa, st)) ? MTLA_OK : MTLA_ERR_HIP;
}

// Scratch of mtla_prefill_step: the saved state, the merge weights, then the scratch of the continuing prefill.
struct PrefillStepLayout {
  size_t pos0, tail_prev, w, chunk, total;
};
static PrefillStepLayout prefill_step_layout(const mtla_ctx* c, size_t batch, size_t T, size_t past) {
  PrefillStepLayout L;
  L.pos0 = 0;
  L.tail_prev = align_up(batch * 4, 256);
  L.w = align_up(L.tail_prev + batch * c->cfg.r * 4, 256);
  L.chunk = align_up(L.w + batch * T * 4, 256);
  L.total = L.chunk + chunk_layout(c, batch * (past + T)).total;
  return L;
}

size_t mtla_prefill_step_scratch_bytes(const mtla_ctx* c, int32_t batch, int32_t T, int32_t max_past_slots) {
  if (!c || batch < 1 || T < 1 || max_past_slots < 0) return 0;
  return prefill_step_layout(c, (size_t)batch, (size_t)T, (size_t)max_past_slots).total;
}

mtla_status mtla_prefill_step(mtla_ctx* c, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                              const void* q, const void* q_rope, const void* cc, const void* kr, const int32_t* n_new,
                              const void* hyp_A, const void* hyp_a, const void* hyp_G, const void* w_uk,
                              const void* w_uv, int32_t batch, int32_t T, int32_t max_past_slots, float* out,
                              float* w_out, void* scratch, void* workspace, void* hip_stream) {
  return mtla_prefill_step_paged(c, cache_c, cache_kr, tail_c, seq_len, nullptr, q, q_rope, cc, kr, n_new, hyp_A, hyp_a, hyp_G,
                                 w_uk, w_uv, batch, T, max_past_slots, out, w_out, scratch, workspace, hip_stream);
}

mtla_status mtla_prefill_step_paged(mtla_ctx* c, void* cache_c, void* cache_kr, float* tail_c, int32_t* seq_len,
                                    const int32_t* page_table, const void* q, const void* q_rope, const void* cc,
                                    const void* kr, const int32_t* n_new, const void* hyp_A, const void* hyp_a,
                                    const void* hyp_G, const void* w_uk, const void* w_uv, int32_t batch, int32_t T,
                                    int32_t max_past_slots, float* out, float* w_out, void* scratch, void* workspace,
                                    void* hip_stream) {
  if (!c || !tail_c || !seq_len || !scratch || !workspace) return MTLA_ERR_INVALID_ARG;
  if (page_table && c->prefix_owner) return MTLA_ERR_UNSUPPORTED;  // with pages a shared prompt is shared pages
  if (batch < 1 || batch > c->cfg.max_batch || T < 1 || max_past_slots < 0 || max_past_slots > c->cfg.max_slots)
    return MTLA_ERR_INVALID_ARG;
  if (c->prefix_owner && batch > c->prefix_n) return MTLA_ERR_INVALID_ARG;  // mtla_set_shared_prefix: arrays too short
  if (!aligned16(scratch) || !aligned16(tail_c) || (w_out && !aligned16(w_out))) return MTLA_ERR_INVALID_ARG;
  if (c->cfg.dtype != MTLA_BF16) return MTLA_ERR_UNSUPPORTED;
  char* sc = reinterpret_cast<char*>(scratch);
  const PrefillStepLayout L = prefill_step_layout(c, (size_t)batch, (size_t)T, (size_t)max_past_slots);
  int32_t* pos0 = reinterpret_cast<int32_t*>(sc + L.pos0);
  float* tail_prev = reinterpret_cast<float*>(sc + L.tail_prev);
  float* w = w_out ? w_out : reinterpret_cast<float*>(sc + L.w);
  // everything is checked before anything is enqueued: the append's arguments, then the attention's
  AppendArgs ap;
  const mtla_status ok = append_args(c, cache_c, cache_kr, tail_c, seq_len, cc, kr, n_new, T, batch, hyp_A, hyp_a, hyp_G,
                                     nullptr, w, nullptr, workspace, ap, page_table);
  if (ok != MTLA_OK) return ok;
  if (!q || !q_rope || !w_uk || !w_uv || !out) return MTLA_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(q_rope) || !aligned16(w_uk) || !aligned16(w_uv) || !aligned16(out))
    return MTLA_ERR_INVALID_ARG;
  {
    ExplicitArgs probe;
    probe.batch = batch;
    probe.T = T;
    probe.n_heads = c->cfg.n_heads;
    probe.d_head = c->cfg.d_head;
    probe.r = c->cfg.r;
    probe.d_rope = c->cfg.d_rope;
    probe.past_pitch = max_past_slots;
    if (!prefill_explicit_supported(probe) || (size_t)batch * ((size_t)max_past_slots + T) > ((size_t)1 << 24))
      return MTLA_ERR_UNSUPPORTED;
  }
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  LayerRowsArgs prep;  // seq_len -> pos0, tail_c -> tail_prev
  prep.seq_len = seq_len;
  prep.tail_c = tail_c;
  prep.pos0 = pos0;
  prep.tail_prev = tail_prev;
  prep.n_wo = 0;
  prep.batch = batch;
  prep.r = c->cfg.r;
  if (!hip_ok(launch_layer_prefill_prep(prep, st))) return MTLA_ERR_HIP;
  if (!hip_ok(launch_append(ap, c->cfg.dtype, st))) return MTLA_ERR_HIP;
  return mtla_prefill_chunk_attn_paged(c, cache_c, cache_kr, tail_prev, pos0, page_table, q, q_rope, cc, kr, w, n_new, batch,
                                       T, max_past_slots, w_uk, w_uv, out, sc + L.chunk, workspace, hip_stream);
}

// Scratch of a whole-layer prefill: the saved state, the projections' outputs, the merge weights, the
// attention output as fp16, W_O as fp16, and behind them the scratch of the continuing prefill.
struct LayerPrefillLayout {
  size_t pos0, tail_prev, rope_cs, q16, qr16, kr, c_raw, c, w, out16, w_o16, chunk, total;
};
static LayerPrefillLayout layer_prefill_layout(const mtla_ctx* c, size_t d_model, size_t batch, size_t T, size_t past) {
  const mtla_config& g = c->cfg;
  const size_t M = batch * T, nq = (size_t)g.n_heads * g.d_head, nqr = (size_t)g.n_heads * g.d_rope;
  LayerPrefillLayout L;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += align_up(bytes, 256);
    return at;
  };
  L.pos0 = take(batch * 4);
  L.tail_prev = take(batch * g.r * 4);
  L.rope_cs = take(M * (g.d_rope / 2) * 8);
  L.q16 = take(M * nq * 2);
  L.qr16 = take(M * nqr * 2);
  L.kr = take(M * g.d_rope * 2);
  L.c_raw = take(M * g.r * 4);
  L.c = take(M * g.r * 2);
  L.w = take(M * 4);
  L.out16 = take(M * nq * 2);
  L.w_o16 = take(d_model * nq * 2);
  L.chunk = off;
  off += chunk_layout(c, batch * (past + T)).total;
  L.total = off;
  return L;
}

size_t mtla_layer_prefill_scratch_bytes(const mtla_ctx* c, int32_t d_model, int32_t batch, int32_t T,
                                        int32_t max_past_slots) {
  if (!c || d_model < 1 || batch < 1 || T < 1 || max_past_slots < 0) return 0;
  return layer_prefill_layout(c, (size_t)d_model, (size_t)batch, (size_t)T, (size_t)max_past_slots).total;
}

mtla_status mtla_layer_prefill(mtla_ctx* c, const mtla_layer_weights* lw, void* cache_c, void* cache_kr, float* tail_c,
                               int32_t* seq_len, const void* x, const int32_t* n_new, const void* hyp_A,
                               const void* hyp_a, const void* hyp_G, const void* w_uk, const void* w_uv, int32_t batch,
                               int32_t T, int32_t max_past_slots, float* y, void* scratch, void* workspace,
                               void* hip_stream) {
  if (!c || !lw || !x || !y || !scratch || !seq_len || !tail_c || !w_uk || !w_uv || !workspace) return MTLA_ERR_INVALID_ARG;
  if (!lw->w_q || !lw->w_qr || !lw->w_r || !lw->w_kr || !lw->w_o) return MTLA_ERR_INVALID_ARG;
  const mtla_config& g = c->cfg;
  if (batch < 1 || batch > g.max_batch || T < 1 || max_past_slots < 0 || max_past_slots > g.max_slots)
    return MTLA_ERR_INVALID_ARG;
  if (c->prefix_owner && batch > c->prefix_n) return MTLA_ERR_INVALID_ARG;  // mtla_set_shared_prefix: arrays too short
  if (!(lw->ln_eps >= 0.f) || !(lw->rope_base >= 0.f) || std::isinf(lw->ln_eps) || std::isinf(lw->rope_base))
    return MTLA_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(y) || !aligned16(scratch) || !aligned16(lw->w_q) || !aligned16(lw->w_qr) ||
      !aligned16(lw->w_r) || !aligned16(lw->w_kr) || !aligned16(lw->w_o) || !aligned16(w_uk) || !aligned16(w_uv) ||
      !aligned16(tail_c))
    return MTLA_ERR_INVALID_ARG;
  if (g.dtype != MTLA_BF16) return MTLA_ERR_UNSUPPORTED;
  if (lw->d_model < 32 || lw->d_model % 32 != 0 || g.r > 512) return MTLA_ERR_UNSUPPORTED;
  const size_t M = (size_t)batch * T, rows_p = (size_t)batch * ((size_t)max_past_slots + T);
  if (rows_p > ((size_t)1 << 24)) return MTLA_ERR_UNSUPPORTED;
  char* sc = reinterpret_cast<char*>(scratch);
  const LayerPrefillLayout L = layer_prefill_layout(c, (size_t)lw->d_model, (size_t)batch, (size_t)T, (size_t)max_past_slots);
  const int nq = g.n_heads * g.d_head, nqr = g.n_heads * g.d_rope;
  const float scale_log2 = c->scale * 1.4426950408889634f;
  int32_t* pos0 = reinterpret_cast<int32_t*>(sc + L.pos0);
  float* tail_prev = reinterpret_cast<float*>(sc + L.tail_prev);
  float* w = reinterpret_cast<float*>(sc + L.w);

  // ---- the four projections of x: one product each, rotation and scaling on the way out
  GemmArgs gq;
  gq.A = x;
  gq.M = (int)M;
  gq.K = lw->d_model;
  gq.in_bf16 = 1;
  gq.d_rope = g.d_rope;
  RopeTableArgs rt;
  rt.pos0 = pos0;
  rt.table = reinterpret_cast<float2*>(sc + L.rope_cs);
  rt.rows = M;
  rt.T = T;
  rt.d_rope = g.d_rope;
  for (int k = 0; k < 32; ++k)
    rt.rope_freq[k] = std::pow((double)(lw->rope_base > 0.f ? lw->rope_base : 10000.f), -2.0 * k / g.d_rope);
  GemmArgs gqr = gq, gc = gq;
  gq.W[0] = lw->w_q;    // q = x W_Q, times log2(e) / sqrt(d_h), fp16: what the attention multiplies
  gq.C[0] = sc + L.q16;
  gq.N = nq;
  gq.epi = 0;
  gq.scale = scale_log2;
  gqr.W[0] = lw->w_qr;  // q^R = RoPE(x W_QR), same scaling
  gqr.C[0] = sc + L.qr16;
  gqr.N = nqr;
  gqr.epi = 1;
  gqr.scale = scale_log2;
  gqr.rope_cs = rt.table;
  GemmArgs gkr = gqr;   // k^R = RoPE(x W_KR), storage type (it goes into the cache): rides along with q^R when the
  const bool kr_rides = nqr % 256 == 0;  // column blocks allow it, else it is a product of its own
  if (kr_rides) {
    gqr.W[1] = lw->w_kr;
    gqr.C[1] = sc + L.kr;
    gqr.N1 = g.d_rope;
  } else {  // a launch with the second product only
    gkr.W[1] = lw->w_kr;
    gkr.C[1] = sc + L.kr;
    gkr.N1 = g.d_rope;
    gkr.N = 0;
    if (!gemm_nt_supported(gkr)) return MTLA_ERR_UNSUPPORTED;
  }
  gc.W[0] = lw->w_r;    // x W_r in fp32, normalised next
  gc.C[0] = sc + L.c_raw;
  gc.N = g.r;
  gc.epi = 3;
  if (!gemm_nt_supported(gq) || !gemm_nt_supported(gqr) || !gemm_nt_supported(gc)) return MTLA_ERR_UNSUPPORTED;

  // ---- the path: append (merge weights, cache), then the continuing parallel form
  AppendArgs ap;
  const mtla_status ok = append_args(c, cache_c, cache_kr, tail_c, seq_len, sc + L.c, sc + L.kr, n_new, T, batch, hyp_A,
                                     hyp_a, hyp_G, nullptr, w, nullptr, workspace, ap);
  if (ok != MTLA_OK) return ok;
  ap.c_merge_f32 = reinterpret_cast<const float*>(sc + L.c_raw);  // normalised in place by then
  // only the matrix-core bulk append folds the unrounded latents; the other one would merge the rounded
  // copies while the attention below works from the unrounded ones
  if (!append_bulk_mfma_supported(ap, g.dtype)) return MTLA_ERR_UNSUPPORTED;
  const ChunkLayout CL = chunk_layout(c, rows_p);
  char* ws = sc + L.chunk;
  ExplicitArgs ex;
  ex.q = sc + L.q16;
  ex.q_rope = sc + L.qr16;
  ex.q_f16 = 1;
  ex.cprime = ws + CL.cprime;
  ex.kr = nullptr;
  ex.w_uk = w_uk;
  ex.w_uv = w_uv;
  ex.seq_len = n_new;
  ex.kx = ws + CL.kx;
  ex.vx = ws + CL.vx;
  ex.w_kT = ws + CL.w_kT;
  ex.w_v16 = ws + CL.w_v16;
  ex.kr16 = ws + CL.kr16;
  ex.out = nullptr;
  ex.out16 = sc + L.out16;
  ex.batch = batch;
  ex.T = T;
  ex.n_heads = g.n_heads;
  ex.d_head = g.d_head;
  ex.r = g.r;
  ex.d_rope = g.d_rope;
  ex.stride = g.stride;
  ex.scale_log2 = scale_log2;
  ex.pos0 = pos0;
  ex.past_pitch = max_past_slots;
  if (!prefill_explicit_supported(ex)) return MTLA_ERR_UNSUPPORTED;
  GemmArgs gy;          // y = concat_h(o_h) W_O
  gy.A = sc + L.out16;
  gy.W[0] = sc + L.w_o16;
  gy.C[0] = y;
  gy.M = (int)M;
  gy.N = lw->d_model;
  gy.K = nq;
  gy.epi = 3;
  if (!gemm_nt_supported(gy)) return MTLA_ERR_UNSUPPORTED;

  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  LayerRowsArgs prep;
  prep.seq_len = seq_len;
  prep.tail_c = tail_c;
  prep.pos0 = pos0;
  prep.tail_prev = tail_prev;
  prep.w_o = lw->w_o;
  prep.w_o16 = sc + L.w_o16;
  prep.n_wo = (size_t)lw->d_model * nq;
  prep.batch = batch;
  prep.r = g.r;
  if (!hip_ok(launch_layer_prefill_prep(prep, st))) return MTLA_ERR_HIP;
  if (!hip_ok(launch_rope_table(rt, st))) return MTLA_ERR_HIP;
  if (!hip_ok(launch_gemm_nt(gq, st)) || !hip_ok(launch_gemm_nt(gqr, st)) || !hip_ok(launch_gemm_nt(gc, st)))
    return MTLA_ERR_HIP;
  if (!kr_rides && !hip_ok(launch_gemm_nt(gkr, st))) return MTLA_ERR_HIP;
  LayerRowsArgs ln;
  ln.raw = reinterpret_cast<const float*>(sc + L.c_raw);
  ln.gamma = lw->ln_gamma;
  ln.beta = lw->ln_beta;
  ln.c = sc + L.c;
  ln.c32 = reinterpret_cast<float*>(sc + L.c_raw);  // in place: every lane has read its elements before it writes them
  ln.rows = M;
  ln.r = g.r;
  ln.eps = lw->ln_eps > 0.f ? lw->ln_eps : 1e-5f;
  if (!hip_ok(launch_layer_norm_rows(ln, st))) return MTLA_ERR_HIP;
  if (!hip_ok(launch_append(ap, g.dtype, st))) return MTLA_ERR_HIP;
  ChunkStageArgs cs;
  cs.cache_c = cache_c;
  cs.cache_kr = cache_kr;
  cs.tail_prev = tail_prev;
  cs.prefix_owner = c->prefix_owner;  // mtla_set_shared_prefix: past slots of a common prompt come from their owner
  cs.prefix_slots = c->prefix_slots;
  cs.prefix_rows = c->cfg.max_batch;
  cs.pos0 = pos0;
  cs.c = sc + L.c;
  cs.c32 = reinterpret_cast<const float*>(sc + L.c_raw);
  cs.kr = sc + L.kr;
  cs.w = w;
  cs.n_new = n_new;
  cs.cprime = ws + CL.cprime;
  cs.kr16 = ws + CL.kr16;
  cs.status = reinterpret_cast<int32_t*>(workspace);
  cs.batch = batch;
  cs.T = T;
  cs.r = g.r;
  cs.d_rope = g.d_rope;
  cs.stride = g.stride;
  cs.max_slots = g.max_slots;
  cs.past_pitch = max_past_slots;
  if (!hip_ok(launch_chunk_stage(cs, st))) return MTLA_ERR_HIP;
  const bool timed = c->prof_n < (int)c->ev_start.size();
  EventPair ev;
  if (timed) {
    ev.start = c->ev_start[c->prof_n];
    ev.stop = c->ev_stop[c->prof_n++];
  }
  if (!hip_ok(launch_prefill_explicit(ex, st, ev))) return MTLA_ERR_HIP;
  return hip_ok(launch_gemm_nt(gy, st)) ? MTLA_OK : MTLA_ERR_HIP;
}

size_t mtla_prefill_chunk_workspace_bytes(const mtla_ctx* c, int32_t batch, int32_t T, int32_t max_past_slots) {
  if (!c || batch < 1 || T < 1 || max_past_slots < 0) return 0;
  return chunk_layout(c, (size_t)batch * ((size_t)max_past_slots + T)).total;
}

mtla_status mtla_prefill_chunk_attn(mtla_ctx* c, const void* cache_c, const void* cache_kr, const float* tail_prev,
                                    const int32_t* pos0, const void* q, const void* q_rope, const void* cc,
                                    const void* kr, const float* w, const int32_t* n_new, int32_t batch, int32_t T,
                                    int32_t max_past_slots, const void* w_uk, const void* w_uv, float* out,
                                    void* chunk_workspace, void* workspace, void* hip_stream) {
  return mtla_prefill_chunk_attn_paged(c, cache_c, cache_kr, tail_prev, pos0, nullptr, q, q_rope, cc, kr, w, n_new, batch, T,
                                       max_past_slots, w_uk, w_uv, out, chunk_workspace, workspace, hip_stream);
}

mtla_status mtla_prefill_chunk_attn_paged(mtla_ctx* c, const void* cache_c, const void* cache_kr, const float* tail_prev,
                                          const int32_t* pos0, const int32_t* page_table, const void* q,
                                          const void* q_rope, const void* cc, const void* kr, const float* w,
                                          const int32_t* n_new, int32_t batch, int32_t T, int32_t max_past_slots,
                                          const void* w_uk, const void* w_uv, float* out, void* chunk_workspace,
                                          void* workspace, void* hip_stream) {
  if (!c || !cache_c || !cache_kr || !tail_prev || !pos0 || !q || !q_rope || !cc || !kr || !w || !w_uk || !w_uv ||
      !out || !chunk_workspace || !workspace)
    return MTLA_ERR_INVALID_ARG;
  if (!paging_matches(c, page_table)) return MTLA_ERR_INVALID_ARG;
  if (page_table && c->prefix_owner) return MTLA_ERR_UNSUPPORTED;  // with pages a shared prompt is shared pages
  const mtla_config& g = c->cfg;
  if (batch < 1 || batch > g.max_batch || T < 1 || max_past_slots < 0 || max_past_slots > g.max_slots)
    return MTLA_ERR_INVALID_ARG;
  if (c->prefix_owner && batch > c->prefix_n) return MTLA_ERR_INVALID_ARG;  // mtla_set_shared_prefix: arrays too short
  if (!aligned16(cache_c) || !aligned16(cache_kr) || !aligned16(tail_prev) || !aligned16(q) || !aligned16(q_rope) ||
      !aligned16(cc) || !aligned16(kr) || !aligned16(w_uk) || !aligned16(w_uv) || !aligned16(out) ||
      !aligned16(chunk_workspace))
    return MTLA_ERR_INVALID_ARG;
  if (g.dtype != MTLA_BF16) return MTLA_ERR_UNSUPPORTED;
  const size_t rows = (size_t)batch * ((size_t)max_past_slots + T);
  if (rows > ((size_t)1 << 24)) return MTLA_ERR_UNSUPPORTED;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  char* ws = reinterpret_cast<char*>(chunk_workspace);
  const ChunkLayout L = chunk_layout(c, rows);

  ExplicitArgs ex;
  ex.q = q;
  ex.q_rope = q_rope;
  ex.cprime = ws + L.cprime;
  ex.kr = nullptr;
  ex.w_uk = w_uk;
  ex.w_uv = w_uv;
  ex.seq_len = n_new;
  ex.kx = ws + L.kx;
  ex.vx = ws + L.vx;
  ex.w_kT = ws + L.w_kT;
  ex.w_v16 = ws + L.w_v16;
  ex.kr16 = ws + L.kr16;
  ex.out = out;
  ex.batch = batch;
  ex.T = T;
  ex.n_heads = g.n_heads;
  ex.d_head = g.d_head;
  ex.r = g.r;
  ex.d_rope = g.d_rope;
  ex.stride = g.stride;
  ex.scale_log2 = c->scale * 1.4426950408889634f;
  ex.pos0 = pos0;
  ex.past_pitch = max_past_slots;
  if (!prefill_explicit_supported(ex)) return MTLA_ERR_UNSUPPORTED;

  ChunkStageArgs cs;
  cs.cache_c = cache_c;
  cs.cache_kr = cache_kr;
  cs.tail_prev = tail_prev;
  cs.prefix_owner = c->prefix_owner;  // mtla_set_shared_prefix: past slots of a common prompt come from their owner
  cs.prefix_slots = c->prefix_slots;
  cs.prefix_rows = c->cfg.max_batch;
  cs.pages = page_map(c, page_table);
  cs.pos0 = pos0;
  cs.c = cc;
  cs.kr = kr;
  cs.w = w;
  cs.n_new = n_new;
  cs.cprime = ws + L.cprime;
  cs.kr16 = ws + L.kr16;
  cs.status = reinterpret_cast<int32_t*>(workspace);
  cs.batch = batch;
  cs.T = T;
  cs.r = g.r;
  cs.d_rope = g.d_rope;
  cs.stride = g.stride;
  cs.max_slots = g.max_slots;
  cs.past_pitch = max_past_slots;
  if (!hip_ok(launch_chunk_stage(cs, st))) return MTLA_ERR_HIP;
  const bool timed = c->prof_n < (int)c->ev_start.size();
  EventPair ev;
  if (timed) {
    ev.start = c->ev_start[c->prof_n];
    ev.stop = c->ev_stop[c->prof_n++];
  }
  return hip_ok(launch_prefill_explicit(ex, st, ev)) ? MTLA_OK : MTLA_ERR_HIP;
}

mtla_status mtla_prefill_attn(mtla_ctx* c, const void* q, const void* q_rope, const void* cc,
                              const void* kr, const float* w, const int32_t* seq_lens,
                              int32_t batch, int32_t T, const void* w_uk, const void* w_uv,
                              float* out, float* out_latent, void* prefill_workspace,
                              void* hip_stream) {
  if (!c || !q || !q_rope || !cc || !kr || !w || !w_uk || !w_uv || !out || !prefill_workspace)
    return MTLA_ERR_INVALID_ARG;
  const mtla_config& g = c->cfg;
  if (batch < 1 || batch > g.max_batch || T < 1) return MTLA_ERR_INVALID_ARG;
  if ((long long)batch * T > (1LL << 24)) return MTLA_ERR_UNSUPPORTED;
  if (!aligned16(q) || !aligned16(q_rope) || !aligned16(cc) || !aligned16(kr) || !aligned16(w_uk) ||
      !aligned16(w_uv) || !aligned16(out) || !aligned16(prefill_workspace) || (out_latent && !aligned16(out_latent)))
    return MTLA_ERR_INVALID_ARG;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  char* ws = reinterpret_cast<char*>(prefill_workspace);
  const size_t rows = (size_t)batch * T;
  const PrefillLayout L = prefill_layout(c, rows);

  PartialStateArgs ps;
  ps.c = cc;
  ps.w = w;
  ps.cprime = ws + L.cprime;
  ps.batch = batch;
  ps.T = T;
  ps.r = g.r;
  ps.stride = g.stride;
  ps.seq_len = seq_lens;
  ps.out_f16 = 0;

  // With many query rows per head the un-absorbed form is the cheaper one: explicit keys and
  // values for all rows (scratch inside the area the absorbed query operand would take), then
  // attention per head.  The latent-space output, if asked for, comes from a second pass of the
  // attention kernel over the partial states as values.
  bool latent_only = false;  // `out` came from the explicit form, the absorbed form fills out_latent alone
  if (g.dtype == MTLA_BF16) {
    ExplicitArgs ex;
    ex.q = q;
    ex.q_rope = q_rope;
    ex.cprime = ws + L.cprime;
    ex.kr = kr;
    ex.w_uk = w_uk;
    ex.w_uv = w_uv;
    ex.seq_len = seq_lens;
    const size_t kv_bytes = align_up(rows * g.n_heads * g.d_head * 2, 256);
    const size_t w_bytes = align_up((size_t)g.n_heads * g.d_head * g.r * 2, 256);
    ex.kx = ws + L.qcat;
    ex.vx = ws + L.qcat + kv_bytes;
    ex.w_kT = ws + L.qcat + 2 * kv_bytes;
    ex.w_v16 = ws + L.qcat + 2 * kv_bytes + w_bytes;
    const size_t kr_bytes = align_up(rows * g.d_rope * 2, 256);
    ex.kr16 = ws + L.qcat + 2 * kv_bytes + 2 * w_bytes;
    ex.out = out;
    ex.out_latent = out_latent;
    ex.batch = batch;
    ex.T = T;
    ex.n_heads = g.n_heads;
    ex.d_head = g.d_head;
    ex.r = g.r;
    ex.d_rope = g.d_rope;
    ex.stride = g.stride;
    ex.scale_log2 = c->scale * 1.4426950408889634f;
    const size_t need = 2 * kv_bytes + 2 * w_bytes + kr_bytes;
    // The latent-space output asked for at a shape where only `out` can come from the explicit form (r not a
    // multiple of d_head): `out` from the explicit form all the same (fp16 inside: the absorbed form's bf16
    // operands cost `out` up to the whole 2e-2 at stride 4), then the absorbed form below for out_latent alone.
    if (out_latent && !prefill_explicit_supported(ex)) {
      ExplicitArgs only_out = ex;
      only_out.out_latent = nullptr;
      if (prefill_explicit_supported(only_out)) {
        ex = only_out;
        latent_only = true;
      }
    }
    if (prefill_explicit_supported(ex) && L.qcat + need <= L.cprime) {
      // partial states and RoPE keys as fp16 in one pass (the staging kernel of the continuing form,
      // with nothing in front of the rows)
      ChunkStageArgs cs;
      cs.cache_c = cs.cache_kr = nullptr;
      cs.tail_prev = nullptr;
      cs.pos0 = nullptr;
      cs.c = cc;
      cs.kr = kr;
      cs.w = w;
      cs.n_new = seq_lens;
      cs.cprime = ws + L.cprime;
      cs.kr16 = ex.kr16;
      cs.status = nullptr;
      cs.batch = batch;
      cs.T = T;
      cs.r = g.r;
      cs.d_rope = g.d_rope;
      cs.stride = g.stride;
      cs.max_slots = g.max_slots;
      cs.past_pitch = 0;
      ex.kr_staged = 1;
      if (!hip_ok(launch_chunk_stage(cs, st))) return MTLA_ERR_HIP;
      const bool timed = c->prof_n < (int)c->ev_start.size();
      EventPair ev;
      if (timed) {
        ev.start = c->ev_start[c->prof_n];
        ev.stop = c->ev_stop[c->prof_n++];
      }
      if (!hip_ok(launch_prefill_explicit(ex, st, ev))) return MTLA_ERR_HIP;
      if (!latent_only) return MTLA_OK;
      out = nullptr;  // written; what follows reuses the scratch in stream order and fills out_latent
    } else {
      latent_only = false;
    }
  }
  // the vector-ALU kernels (fp32 storage, or shapes the matrix-core kernels do not take) index a
  // grid dimension by the row
  {
    CombineArgs probe;
    probe.r = g.r;
    probe.d_head = g.d_head;
    probe.n_heads = g.n_heads;
    probe.out = out;
    probe.out_latent = out_latent;
    probe.w_uv = w_uv;
    if (rows > 65535 && (g.dtype != MTLA_BF16 || !combine_mfma_supported(probe))) return MTLA_ERR_UNSUPPORTED;
  }
  if (!hip_ok(launch_partial_states(ps, g.dtype, st))) return MTLA_ERR_HIP;

  AbsorbArgs ab;
  ab.q = q;
  ab.q_rope = q_rope;
  ab.w_uk = w_uk;
  ab.qcat = ws + L.qcat;
  ab.rows = (int)rows;
  ab.n_heads = g.n_heads;
  ab.d_head = g.d_head;
  ab.r = g.r;
  ab.d_rope = g.d_rope;
  ab.scale_log2 = c->scale * 1.4426950408889634f;
  ab.q_f32 = 0;

  AttnArgs at;
  at.qcat = ws + L.qcat;
  at.lat = ws + L.cprime;
  at.key = kr;
  at.seq_len = seq_lens;
  at.part_o = reinterpret_cast<float*>(ws + L.part_o);
  at.part_ml = reinterpret_cast<float*>(ws + L.part_ml);
  at.n_heads = g.n_heads;
  at.r = g.r;
  at.d_rope = g.d_rope;
  at.stride = g.stride;
  at.max_slots = 0;
  at.chunk = 1 << 30;  // one wavefront (matrix cores) or workgroup (vector) scans all live columns
  at.n_splits = 1;
  at.batch = batch;
  at.T = T;
  at.n_persistent = 0;
  at.tile_prefix = nullptr;
  at.part_f16 = 0;
  const bool use_mfma = g.dtype == MTLA_BF16 && attn_mfma_supported(at);
  ab.out_bf16 = use_mfma ? 1 : 0;
  ab.plane = at.q_plane = rows * g.n_heads * (g.r + g.d_rope);  // two bf16 planes fill the fp32 area
  if (!hip_ok(launch_absorb(ab, g.dtype, st))) return MTLA_ERR_HIP;
  const bool timed = !latent_only && c->prof_n < (int)c->ev_start.size();
  EventPair ev;  // attached to the dispatch itself: the kernel's own begin and end
  if (timed) {
    ev.start = c->ev_start[c->prof_n];
    ev.stop = c->ev_stop[c->prof_n++];
  }
  const hipError_t le = !use_mfma ? launch_attn_split(at, g.dtype, st, ev)
                                  : (attn_cols_rows_supported(at) ? launch_attn_cols_rows(at, st, ev)
                                                                  : launch_attn_mfma(at, st, ev));
  if (!hip_ok(le)) return MTLA_ERR_HIP;

  CombineArgs cb;
  cb.part_o = at.part_o;
  cb.part_ml = at.part_ml;
  cb.seq_len = seq_lens;
  cb.w_uv = w_uv;
  cb.out = out;
  cb.out_latent = out_latent;
  cb.lse = nullptr;
  cb.n_heads = g.n_heads;
  cb.r = g.r;
  cb.d_head = g.d_head;
  cb.stride = g.stride;
  cb.chunk = at.chunk;
  cb.n_splits = 1;
  cb.batch = batch;
  cb.T = T;
  cb.n_persistent = 0;
  cb.tile_prefix = nullptr;
  cb.part_f16 = 0;
  if (!hip_ok(launch_combine(cb, g.dtype, st))) return MTLA_ERR_HIP;
  return MTLA_OK;
}

}  // extern "C"
