// mtla_cache_append kernels: hyper-network merge weight, then the temporal
// merge of the new latent into the strided cache (Section "Inference using
// MTLA": Eq. (infer-linear) and the update rule; RoPE-key rule of Section
// "Decoupled Rotary Position Embedding").
//
// Every cache row has exactly one writer.  A decode step (one token per sequence) is a single
// launch of `batch` workgroups that also advances seq_len (append_step_kernel).  A bulk append
// (prefix) runs one workgroup per (sequence, group of 16 touched slots) with the hyper-network on
// the matrix cores (append_bulk_mfma_kernel, bf16 storage) or one workgroup per touched slot
// (append_kernel, any storage), and a second tiny kernel advances seq_len once every workgroup has
// read the old value.
#include "absorb_mfma.h"
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

constexpr int kMaxRPerThread = 4;  // r <= 1024 with 256 threads

constexpr int kTPR = 4;                 // lanes sharing one hyper-network row
constexpr int kRowsPerPass = kBlock / kTPR;


// Linear(c): sg[y] = a[y] + sum_n A[y][n] sc[n] for every row y < dy.  Four adjacent lanes
// share a row and take 8-element pieces round-robin (contiguous 64-byte reads of A,
// conflict-free reads of sc); all loads of a pass are issued before the first use.
template <typename T>
__device__ __forceinline__ void hyper_linear(const T* A, const T* ha, const float* sc, float* sg,
                                             int r, int dy, int tid) {
  const int q = tid & (kTPR - 1);
  for (int y0 = 0; y0 < dy; y0 += kRowsPerPass) {
    const int y = y0 + tid / kTPR;
    float dot = 0.f;
    if (y < dy) {
      const T* Arow = A + (size_t)y * r;
      for (int c8 = q; c8 < r / 8; c8 += kTPR) {
        float wv[8];
        load8(Arow + 8 * c8, wv);
#pragma unroll
        for (int j = 0; j < 8; ++j) dot += wv[j] * sc[8 * c8 + j];
      }
    }
    dot += __shfl_xor(dot, 1, kWave);
    dot += __shfl_xor(dot, 2, kWave);
    if (y < dy && q == 0) sg[y] = dot + (ha ? to_f32(ha[y]) : 0.f);
  }
}

// <Linear(c), Linear(pe_j)> = sum_y sg[y] G[slot][y], reduced over the workgroup; red: [4] floats.
template <typename T>
__device__ __forceinline__ float hyper_logit(const float* sg, const T* Grow, float* red, int dy, int tid) {
  float zp = 0.f;
  for (int y = tid; y < dy; y += kBlock) zp += sg[y] * to_f32(Grow[y]);
  zp = wave_sum(zp);
  if ((tid & (kWave - 1)) == 0) red[tid >> 6] = zp;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// 8 consecutive elements of storage type T, kept raw until they are needed.
template <typename T>
struct Chunk8;
template <>
struct Chunk8<bf16> {
  uint4 raw;
  __device__ __forceinline__ void load(const bf16* p) { raw = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void store(bf16* p) const { *reinterpret_cast<uint4*>(p) = raw; }
  __device__ __forceinline__ void unpack(float (&o)[8]) const {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
template <>
struct Chunk8<float> {
  float4 lo, hi;
  __device__ __forceinline__ void load(const float* p) {
    lo = *reinterpret_cast<const float4*>(p);
    hi = *reinterpret_cast<const float4*>(p + 4);
  }
  __device__ __forceinline__ void store(float* p) const {
    *reinterpret_cast<float4*>(p) = lo;
    *reinterpret_cast<float4*>(p + 4) = hi;
  }
  __device__ __forceinline__ void unpack(float (&o)[8]) const {
    o[0] = lo.x; o[1] = lo.y; o[2] = lo.z; o[3] = lo.w;
    o[4] = hi.x; o[5] = hi.y; o[6] = hi.z; o[7] = hi.w;
  }
};

// Decode step: exactly one candidate token per sequence, one workgroup per sequence.
// Nothing but the positional branch G[slot] depends on the sequence position, so the
// length, the latent, the old tail, the key and the thread's pieces of hyp_A are all
// requested at once (NCH = pieces per thread of one hyp_A row, r / 32); Linear(c) is
// finished by the time the length has arrived, and only the G row costs a second trip.
// TC = element type of c_new: the storage type, or float when the caller's projection hands the
// latent over unrounded (the merge and the hyper-network then see it in full precision and the cache
// row is rounded once).
template <typename T, int NCH, typename TC = T>
__device__ __forceinline__ void append_step_block(const AppendArgs& a, int b, float* smem) {
  float* sg = smem;             // [dy] Linear(c)
  float* red = smem + a.d_hyper;  // [4]
  const int tid = threadIdx.x;
  const int s = a.stride, r = a.r, dR = a.d_rope, dy = a.d_hyper;
  const int q = tid & (kTPR - 1), y = tid / kTPR;
  const int p0 = a.seq_len[b];
  const int n = a.n_new ? a.n_new[b] : 1;
  const TC* crow = reinterpret_cast<const TC*>(a.c_new) + (size_t)b * r;
  float* tail = a.tail_c ? a.tail_c + (size_t)b * r : nullptr;
  float told[kMaxRPerThread], cel[kMaxRPerThread];
#pragma unroll
  for (int i = 0; i < kMaxRPerThread; ++i) {
    const int e = tid + i * kBlock;
    told[i] = (tail && e < r) ? tail[e] : 0.f;
    cel[i] = e < r ? to_f32(crow[e]) : 0.f;
  }
  Chunk8<T> krv;
  if (tid < dR / 8) krv.load(reinterpret_cast<const T*>(a.kr_new) + (size_t)b * dR + 8 * tid);
  const bool ln = sizeof(TC) == 4 && a.ln_eps > 0.f;  // whole-layer call: normalise the unrounded latent first
  // [r] the latent as fp32 (normalised in the whole-layer call): the hyper-network's rows read it from
  // here instead of every thread holding its own copy of the pieces it needs (at r = 512 that copy was 64
  // registers, and with them the fused front kernel of a decode step fitted two workgroups per unit)
  float* sc_row = smem + a.d_hyper + 4 + 8;
  const bool hyper = !a.w_override;
  Chunk8<T> ach[NCH];
  const T* A = reinterpret_cast<const T*>(a.hyp_A);
  const T* ha = reinterpret_cast<const T*>(a.hyp_a);
  float bias = 0.f;
  if (hyper) {
    if (y < dy) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) ach[i].load(A + (size_t)y * r + 8 * (q + i * kTPR));
      if (ha) bias = to_f32(ha[y]);
    }
  }
  // Layer normalisation of an unrounded latent (whole-layer call): y = (v - mean) / sqrt(var + eps),
  // two passes over the row in fp32; every thread ends up with the same mean and 1/sigma.
  float ln_mean = 0.f, ln_inv = 1.f;
  const T* ln_g = reinterpret_cast<const T*>(a.ln_gamma);
  const T* ln_b = reinterpret_cast<const T*>(a.ln_beta);
  float g_pre = 0.f;  // ln: this thread's element of the slot's row of G, requested before the normalisation
  if (ln) {
    if (!a.w_override && tid < dy) {
      const int slot_c = p0 / s < a.max_slots ? p0 / s : a.max_slots - 1;  // a full sequence is refused below
      g_pre = to_f32(reinterpret_cast<const T*>(a.hyp_G)[(size_t)slot_c * dy + tid]);
    }
    float* lred = smem + a.d_hyper + 4;  // [8]
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxRPerThread; ++i) part += cel[i];
    part = wave_sum(part);
    if ((tid & (kWave - 1)) == 0) lred[tid / kWave] = part;
    __syncthreads();
    ln_mean = (lred[0] + lred[1] + lred[2] + lred[3]) / r;
    part = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxRPerThread; ++i) {
      const int e = tid + i * kBlock;
      if (e < r) part += (cel[i] - ln_mean) * (cel[i] - ln_mean);
    }
    part = wave_sum(part);
    if ((tid & (kWave - 1)) == 0) lred[4 + tid / kWave] = part;
    __syncthreads();
    ln_inv = 1.0f / sqrtf((lred[4] + lred[5] + lred[6] + lred[7]) / r + a.ln_eps);
#pragma unroll
    for (int i = 0; i < kMaxRPerThread; ++i) {
      const int e = tid + i * kBlock;
      if (e < r) {
        cel[i] = (cel[i] - ln_mean) * ln_inv;
        if (ln_g) cel[i] *= to_f32(ln_g[e]);
        if (ln_b) cel[i] += to_f32(ln_b[e]);
      }
    }
  }
  if (hyper) {
#pragma unroll
    for (int i = 0; i < kMaxRPerThread; ++i) {
      const int e = tid + i * kBlock;
      if (e < r) sc_row[e] = cel[i];
    }
    __syncthreads();
  }
  if (hyper) {
    // ---- Linear(c), rows y < 64 from the registers, further rows (dy > 64) straight from memory
    for (int y0 = 0; y0 < dy; y0 += kRowsPerPass) {
      const int yy = y0 + y;
      float dot = 0.f;
      if (yy < dy) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
          float av[8], cv[8];
          if (y0 == 0) ach[i].unpack(av);
          else load8(A + (size_t)yy * r + 8 * (q + i * kTPR), av);
          load8(sc_row + 8 * (q + i * kTPR), cv);
#pragma unroll
          for (int j = 0; j < 8; ++j) dot += av[j] * cv[j];
        }
      }
      dot += __shfl_xor(dot, 1, kWave);
      dot += __shfl_xor(dot, 2, kWave);
      if (yy < dy && q == 0) sg[yy] = dot + (y0 == 0 ? bias : (ha ? to_f32(ha[yy]) : 0.f));
    }
  }
  __syncthreads();

  if (n < 1) return;
  if ((long long)p0 + 1 > (long long)a.max_slots * s) {  // refuse: sequence untouched
    if (tid == 0) *a.status = 3;                         // MTLA_ERR_CAPACITY
    return;
  }
  const int slot = p0 / s;
  const bool continuing = (p0 - slot * s) != 0;
  float w;
  if (hyper) {
    float z;
    if (ln && dy <= kBlock) {  // same sum as hyper_logit, with the row already in registers
      float zp = tid < dy ? sg[tid] * g_pre : 0.f;
      zp = wave_sum(zp);
      if ((tid & (kWave - 1)) == 0) red[tid >> 6] = zp;
      __syncthreads();
      z = (red[0] + red[1]) + (red[2] + red[3]);
    } else {
      z = hyper_logit(sg, reinterpret_cast<const T*>(a.hyp_G) + (size_t)slot * dy, red, dy, tid);
    }
    w = 1.f / (1.f + expf(-z));
  } else {
    w = a.w_override[b];
  }
  T* crow_out = reinterpret_cast<T*>(a.cache_c) + cache_row(a.pages, b, slot, a.max_slots) * r;
#pragma unroll
  for (int i = 0; i < kMaxRPerThread; ++i) {
    const int e = tid + i * kBlock;
    if (e < r) {
      const float old = continuing ? (tail ? told[i] : to_f32(crow_out[e])) : 0.f;
      const float v = old + w * cel[i];
      crow_out[e] = from_f32<T>(v);
      if (tail) tail[e] = v;
    }
  }
  if (tid < dR / 8) krv.store(reinterpret_cast<T*>(a.cache_kr) + cache_row(a.pages, b, slot, a.max_slots) * dR + 8 * tid);
  if (tid == 0) {
    if (a.w_out) a.w_out[b] = w;
    if (a.slot_out) a.slot_out[b] = slot;
    a.seq_len[b] = p0 + 1;  // every thread took p0 before the barrier
  }
}

template <typename T, int NCH>
__global__ __launch_bounds__(kBlock) void append_step_kernel(AppendArgs a) {
  extern __shared__ float smem[];
  append_step_block<T, NCH>(a, blockIdx.x, smem);
}

// Front of a fused decode step (bf16 storage): the two things the pass over the cache waits
// for, neither of which needs the other -- the append of the step's token (workgroups below
// `batch`) and the absorbed queries (the rest, numbered like the absorb kernel's grid) -- in one
// launch, so a step pays one kernel start and one round trip to memory for both.
// At batch 256 and more a step launches more workgroups than a unit holds at once, and the kernel then
// takes as many rounds as its registers make necessary: five workgroups per unit (96 registers; four for the
// whole-layer call's fp32 operands, which would spill below 128).
template <int NCH, int KK, typename TC>
__global__ __launch_bounds__(kBlock, sizeof(TC) == 4 ? 4 : 5) void decode_front_kernel(AppendArgs ap, AbsorbArgs ab, int gx, int gy) {
  extern __shared__ float smem[];
  const int blk = blockIdx.x;
  if (blk < ap.batch) {
    append_step_block<bf16, NCH, TC>(ap, blk, smem);
    return;
  }
  const int i = blk - ap.batch;
  const int bx = i % gx, rest = i / gx;
  absorb_mfma_block<KK, sizeof(TC) == 4>(ab, bx, rest % gy, rest / gy);  // the whole-layer call hands q, q^R and c over unrounded
}

// One slot of a bulk append: tokens [t_lo, t_hi) of the call fold into `slot` of sequence b.
// Called by every thread of the workgroup (barriers inside).
template <typename T>
__device__ __forceinline__ void append_slot(const AppendArgs& a, int b, int p0, int n, int slot, float* smem) {
  float* sc = smem;              // [r] current token's latent in fp32
  float* sg = smem + a.r;        // [dy] Linear(c)
  float* red = sg + a.d_hyper;   // [4] per-wave partial of the hyper-network logit
  const int tid = threadIdx.x;
  const int s = a.stride, r = a.r, dR = a.d_rope, dy = a.d_hyper;
  const long long slot_first = (long long)slot * s;
  const int t_lo = int((slot_first > p0 ? slot_first : (long long)p0) - p0);
  const long long slot_end = slot_first + s;
  const int t_hi = int((slot_end < (long long)p0 + n ? slot_end : (long long)p0 + n) - p0);

  T* crow_out = reinterpret_cast<T*>(a.cache_c) + cache_row(a.pages, b, slot, a.max_slots) * r;
  float* tail = a.tail_c ? a.tail_c + (size_t)b * r : nullptr;
  const T* A = reinterpret_cast<const T*>(a.hyp_A);
  const T* ha = reinterpret_cast<const T*>(a.hyp_a);
  const T* G = reinterpret_cast<const T*>(a.hyp_G);

  float acc[kMaxRPerThread];
  const bool continuing = slot_first < p0;  // the slot already holds earlier tokens
#pragma unroll
  for (int i = 0; i < kMaxRPerThread; ++i) {
    const int e = tid + i * kBlock;
    acc[i] = 0.f;
    if (continuing && e < r) acc[i] = tail ? tail[e] : to_f32(crow_out[e]);
  }

  for (int t = t_lo; t < t_hi; ++t) {
    const size_t tok = (size_t)b * a.n_new_max + t;
    const T* crow = reinterpret_cast<const T*>(a.c_new) + tok * r;
#pragma unroll
    for (int i = 0; i < kMaxRPerThread; ++i) {
      const int e = tid + i * kBlock;
      if (e < r) sc[e] = to_f32(crow[e]);
    }
    __syncthreads();
    float w;
    if (a.w_override) {
      w = a.w_override[tok];
    } else {
      hyper_linear(A, ha, sc, sg, r, dy, tid);
      __syncthreads();
      const float z = hyper_logit(sg, G + (size_t)slot * dy, red, dy, tid);
      w = 1.f / (1.f + expf(-z));
    }
#pragma unroll
    for (int i = 0; i < kMaxRPerThread; ++i) {
      const int e = tid + i * kBlock;
      if (e < r) acc[i] += w * sc[e];
    }
    if (tid == 0) {
      if (a.w_out) a.w_out[tok] = w;
      if (a.slot_out) a.slot_out[tok] = slot;
    }
    __syncthreads();  // sc / red are rewritten by the next token
  }

  const bool is_open_slot = (t_hi == n);  // last slot touched: remains the sequence's tail
#pragma unroll
  for (int i = 0; i < kMaxRPerThread; ++i) {
    const int e = tid + i * kBlock;
    if (e < r) {
      crow_out[e] = from_f32<T>(acc[i]);
      if (tail && is_open_slot) tail[e] = acc[i];
    }
  }
  // RoPE key: the slot keeps the key of the newest token folded into it.
  const T* kr_src = reinterpret_cast<const T*>(a.kr_new) + ((size_t)b * a.n_new_max + (t_hi - 1)) * dR;
  T* kr_dst = reinterpret_cast<T*>(a.cache_kr) + cache_row(a.pages, b, slot, a.max_slots) * dR;
  for (int e = tid; e < dR; e += kBlock) kr_dst[e] = kr_src[e];
}

// Bulk append, any storage type: one workgroup per (sequence, slot touched), tokens of the slot in
// order.  The tail shadow is read by the first slot of a call and written by the last: workgroup 0
// of the sequence takes both, one after the other, so the read precedes the write.
template <typename T>
__global__ __launch_bounds__(kBlock) void append_kernel(AppendArgs a) {
  extern __shared__ float smem[];
  const int b = blockIdx.y, kslot = blockIdx.x, s = a.stride;
  const int p0 = a.seq_len[b];
  int n = a.n_new ? a.n_new[b] : a.n_new_max;
  n = n < 0 ? 0 : (n > a.n_new_max ? a.n_new_max : n);
  if (n == 0) return;
  if ((long long)p0 + n > (long long)a.max_slots * s) {   // refuse: sequence untouched
    if (kslot == 0 && threadIdx.x == 0) *a.status = 3;    // MTLA_ERR_CAPACITY
    return;
  }
  const int first_slot = p0 / s, last_slot = int(((long long)p0 + n - 1) / s);
  const int slot = first_slot + kslot;
  if (slot < last_slot || (slot == last_slot && kslot == 0)) append_slot<T>(a, b, p0, n, slot, smem);
  if (kslot == 0 && last_slot > first_slot) append_slot<T>(a, b, p0, n, last_slot, smem);
}

// Bulk append on the matrix cores (bf16 storage): one workgroup per (sequence, group of 16 slots).
// Phase 1: Linear(c) of the group's tokens, 16 at a time, is a small dense contraction
//     D[y, token] = sum_n hyp_A[y, n] c[token, n]                 (M = d_y, N = 16 tokens, K = r)
// whose result is dotted with the slot's row of hyp_G in registers; the sigmoid of that is the
// merge weight (Eq. (infer-linear)), parked in LDS.  Phase 2: the temporal merge, 16 threads per slot,
// each summing w_n c_n over the slot's tokens for its 8-element pieces of the row (fp32, starting
// from the tail shadow when the slot already held tokens), then one rounded store of the cache row,
// the tail shadow of the last slot, and the newest RoPE key.
//
// The tail shadow of a sequence is read by the first slot a call touches (when that slot already
// held tokens) and written by the last one.  Both belong to workgroup 0 of the sequence: it takes
// the last slot in a second pass when that slot lies in another group, behind a barrier, so the
// read always precedes the write.  Inside a pass the shadow is copied to LDS ahead of the barrier
// that separates the two phases, because the reading and the writing slot sit in different wavefronts.
// DY16 = d_y / 16.  kBulkSlots slots of at most kBulkMaxStride tokens per pass.
constexpr int kBulkSlots = 16, kBulkMaxStride = 16;

// Positions [pos_lo, pos_hi) of sequence b, all inside slots slot_base .. slot_base + 15.
// Called by every thread of the workgroup (barriers inside).
template <int DY16, bool C32>  // C32: the latents also come unrounded (a.c_merge_f32)
__device__ __forceinline__ void append_bulk_range(const AppendArgs& a, int b, int p0, int n, int slot_base,
                                                  long long pos_lo, long long pos_hi, float* sW, float* sTail) {
  typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
  typedef float float4_t __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int s = a.stride, r = a.r, dR = a.d_rope, dy = 16 * DY16;
  const int t0 = int(pos_lo - p0), cnt = int(pos_hi - pos_lo);  // tokens t0 .. t0 + cnt - 1 of the call
  const uint16_t* c_seq = reinterpret_cast<const uint16_t*>(a.c_new) + (size_t)b * a.n_new_max * r;
  const size_t tok0 = (size_t)b * a.n_new_max + t0;
  float* tail = a.tail_c + (size_t)b * r;
  if ((long long)slot_base * s < p0)  // the range starts inside a slot that already holds tokens
    for (int e = tid; e < r; e += kBlock) sTail[e] = tail[e];

  // ---- phase 1: merge weights of the range's tokens
  if (a.w_override) {
    for (int u = tid; u < cnt; u += kBlock) {
      const float w = a.w_override[tok0 + u];
      sW[u] = w;
      if (a.w_out) a.w_out[tok0 + u] = w;
      if (a.slot_out) a.slot_out[tok0 + u] = int((pos_lo + u) / s);
    }
  } else {
    const uint16_t* A = reinterpret_cast<const uint16_t*>(a.hyp_A);
    const bf16* ha = reinterpret_cast<const bf16*>(a.hyp_a);
    const uint16_t* G = reinterpret_cast<const uint16_t*>(a.hyp_G);
    for (int u0 = 16 * wv; u0 < cnt; u0 += 16 * (kBlock / kWave)) {  // wavefront-uniform: 16 tokens per pass
      const int u = u0 + l16 < cnt ? u0 + l16 : cnt - 1;  // lane's token (clamped duplicates are not stored)
      const uint16_t* crow = c_seq + (size_t)(t0 + u) * r + 8 * g;
      float4_t acc[DY16];
#pragma unroll
      for (int yt = 0; yt < DY16; ++yt) acc[yt] = float4_t{0.f, 0.f, 0.f, 0.f};
      const float* crow32 = C32 ? a.c_merge_f32 + ((size_t)b * a.n_new_max + (size_t)(t0 + u)) * r + 8 * g : nullptr;
      for (int kk = 0; kk < r / 32; ++kk) {
        bf16x8_t cf, cf_lo;
        if constexpr (C32) {  // unrounded latents: hi + lo bf16 planes, two matrix instructions per step
          float v[8];
          load8(crow32 + 32 * kk, v);
          uint4 hi, lo;
          split_bf16x2(v[0], v[1], hi.x, lo.x);
          split_bf16x2(v[2], v[3], hi.y, lo.y);
          split_bf16x2(v[4], v[5], hi.z, lo.z);
          split_bf16x2(v[6], v[7], hi.w, lo.w);
          cf = __builtin_bit_cast(bf16x8_t, hi);
          cf_lo = __builtin_bit_cast(bf16x8_t, lo);
        } else {
          cf = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(crow + 32 * kk));
        }
#pragma unroll
        for (int yt = 0; yt < DY16; ++yt) {
          const bf16x8_t af = __builtin_bit_cast(
              bf16x8_t, *reinterpret_cast<const uint4*>(A + (size_t)(16 * yt + l16) * r + 32 * kk + 8 * g));
          acc[yt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, cf, acc[yt], 0, 0, 0);
          if constexpr (C32) acc[yt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, cf_lo, acc[yt], 0, 0, 0);
        }
      }
      // the lane holds Linear(c)[y], y = 16 yt + 4 g + v, of its token: dot with the slot's row of G
      const int slot = int((pos_lo + u) / s);
      const uint16_t* grow = G + (size_t)slot * dy + 4 * g;
      float z = 0.f;
#pragma unroll
      for (int yt = 0; yt < DY16; ++yt) {
        const uint2 gv = *reinterpret_cast<const uint2*>(grow + 16 * yt);
        const float gf[4] = {__uint_as_float(gv.x << 16), __uint_as_float(gv.x & 0xffff0000u),
                             __uint_as_float(gv.y << 16), __uint_as_float(gv.y & 0xffff0000u)};
#pragma unroll
        for (int v = 0; v < 4; ++v) z += (acc[yt][v] + (ha ? to_f32(ha[16 * yt + 4 * g + v]) : 0.f)) * gf[v];
      }
      z += __shfl_xor(z, 16, kWave);
      z += __shfl_xor(z, 32, kWave);
      const float w = 1.f / (1.f + expf(-z));
      if (g == 0 && u0 + l16 < cnt) {
        sW[u0 + l16] = w;
        if (a.w_out) a.w_out[tok0 + u0 + l16] = w;
        if (a.slot_out) a.slot_out[tok0 + u0 + l16] = slot;
      }
    }
  }
  __syncthreads();

  // ---- phase 2: temporal merge, 16 threads per slot
  const int j = tid >> 4, q = tid & 15, slot = slot_base + j;
  const long long sf = (long long)slot * s;
  const long long lo = sf > pos_lo ? sf : pos_lo, hi = sf + s < pos_hi ? sf + s : pos_hi;
  if (lo < hi) {                                        // slot touched by this range
    const bool continuing = sf < p0;                    // the slot already holds earlier tokens
    const bool is_open_slot = hi == (long long)p0 + n;  // last slot touched: remains the sequence's tail
    uint16_t* crow_out = reinterpret_cast<uint16_t*>(a.cache_c) + cache_row(a.pages, b, slot, a.max_slots) * r;
    for (int c8 = q; c8 < r / 8; c8 += 16) {
      float acc8[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc8[e] = continuing ? sTail[8 * c8 + e] : 0.f;
      for (long long pos = lo; pos < hi; ++pos) {
        const float w = sW[int(pos - pos_lo)];
        float cv[8];
        if constexpr (C32) load8(a.c_merge_f32 + ((size_t)b * a.n_new_max + (size_t)(pos - p0)) * r + 8 * c8, cv);
        else load8(reinterpret_cast<const bf16*>(c_seq) + (size_t)(pos - p0) * r + 8 * c8, cv);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc8[e] += w * cv[e];
      }
      *reinterpret_cast<uint4*>(crow_out + 8 * c8) =
          make_uint4(pack_bf16x2(acc8[0], acc8[1]), pack_bf16x2(acc8[2], acc8[3]), pack_bf16x2(acc8[4], acc8[5]),
                     pack_bf16x2(acc8[6], acc8[7]));
      if (is_open_slot) {
        *reinterpret_cast<float4*>(tail + 8 * c8) = make_float4(acc8[0], acc8[1], acc8[2], acc8[3]);
        *reinterpret_cast<float4*>(tail + 8 * c8 + 4) = make_float4(acc8[4], acc8[5], acc8[6], acc8[7]);
      }
    }
    // RoPE key: the slot keeps the key of the newest token folded into it
    if (q < dR / 8) {
      const uint16_t* kr_src =
          reinterpret_cast<const uint16_t*>(a.kr_new) + ((size_t)b * a.n_new_max + (size_t)(hi - 1 - p0)) * dR;
      uint16_t* kr_dst = reinterpret_cast<uint16_t*>(a.cache_kr) + cache_row(a.pages, b, slot, a.max_slots) * dR;
      *reinterpret_cast<uint4*>(kr_dst + 8 * q) = *reinterpret_cast<const uint4*>(kr_src + 8 * q);
    }
  }
  __syncthreads();  // sW is rewritten, and the tail shadow written, by a following pass
}

template <int DY16, bool C32>
__global__ __launch_bounds__(kBlock) void append_bulk_mfma_kernel(AppendArgs a) {
  __shared__ float sW[kBulkSlots * kBulkMaxStride];
  __shared__ float sTail[kMaxRPerThread * kBlock];
  const int b = blockIdx.y, s = a.stride;
  const int p0 = a.seq_len[b];
  int n = a.n_new ? a.n_new[b] : a.n_new_max;
  n = n < 0 ? 0 : (n > a.n_new_max ? a.n_new_max : n);
  if (n == 0) return;
  if ((long long)p0 + n > (long long)a.max_slots * s) {       // refuse: sequence untouched
    if (blockIdx.x == 0 && threadIdx.x == 0) *a.status = 3;  // MTLA_ERR_CAPACITY
    return;
  }
  const long long end = (long long)p0 + n;
  const int first_slot = p0 / s, last_slot = int((end - 1) / s);
  const bool last_apart = last_slot - first_slot >= kBulkSlots;  // last slot outside workgroup 0's group
  const int slot0 = first_slot + kBulkSlots * blockIdx.x;
  const long long lim = last_apart ? (long long)last_slot * s : end;  // the group's share ends here
  const long long pos_lo = (long long)slot0 * s > p0 ? (long long)slot0 * s : p0;
  const long long pos_hi = (long long)(slot0 + kBulkSlots) * s < lim ? (long long)(slot0 + kBulkSlots) * s : lim;
  if (pos_lo < pos_hi) append_bulk_range<DY16, C32>(a, b, p0, n, slot0, pos_lo, pos_hi, sW, sTail);
  if (blockIdx.x == 0 && last_apart)
    append_bulk_range<DY16, C32>(a, b, p0, n, last_slot, (long long)last_slot * s, end, sW, sTail);
}

__global__ void advance_len_kernel(AppendArgs a) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= a.batch) return;
  const int p0 = a.seq_len[b];
  int n = a.n_new ? a.n_new[b] : a.n_new_max;
  n = n < 0 ? 0 : (n > a.n_new_max ? a.n_new_max : n);
  if ((long long)p0 + n <= (long long)a.max_slots * a.stride) a.seq_len[b] = p0 + n;
}

__global__ void fill_zero_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Plain streaming read for benchmarks: every workgroup walks its own contiguous share of the buffer
// with 16-byte loads, two 16 KB pieces per wavefront in flight, and folds what it reads into one word.
__global__ __launch_bounds__(kBlock) void stream_read_kernel(const uint4* __restrict__ p, size_t n_vec, uint32_t* out) {
  const size_t per = (n_vec + gridDim.x - 1) / gridDim.x;
  const size_t lo = blockIdx.x * per, hi = lo + per < n_vec ? lo + per : n_vec;
  uint32_t acc = 0;
  for (size_t i = lo + threadIdx.x; i < hi; i += 8 * kBlock) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const size_t j = i + (size_t)u * kBlock;
      v[u] = p[j < hi ? j : hi - 1];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u) *out = acc;  // keeps the loads alive; practically never taken
}

}  // namespace

// Beam reordering of the sequence state: a gather of whole sequences.  Workgroup (x, b) copies every
// gridDim.x-th run of 256 16-byte pieces of the live rows of source sequence src_index[b] (four
// loads in flight per thread); workgroup (0, b) also copies the tail shadow and the length.
__global__ __launch_bounds__(kBlock) void reorder_kernel(ReorderArgs a) {
  const int b = blockIdx.y, tid = threadIdx.x;
  const int src = a.src_index[b];
  if (src < 0 || src >= a.max_batch) {  // refuse: destination sequence untouched
    if (blockIdx.x == 0 && tid == 0) *a.status = 1;  // MTLA_ERR_INVALID_ARG
    return;
  }
  const int len = a.src_len[src];
  int live = len > 0 ? (len + a.stride - 1) / a.stride : 0;
  live = live < a.max_slots ? live : a.max_slots;
  const size_t row_c = (size_t)a.max_slots * a.r * a.elem, row_kr = (size_t)a.max_slots * a.d_rope * a.elem;
  const uint4* sc = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.src_c) + src * row_c);
  const uint4* sk = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.src_kr) + src * row_kr);
  uint4* dc = reinterpret_cast<uint4*>(reinterpret_cast<char*>(a.dst_c) + b * row_c);
  uint4* dk = reinterpret_cast<uint4*>(reinterpret_cast<char*>(a.dst_kr) + b * row_kr);
  // slots first_slot .. live-1 (rows are multiples of 16 bytes)
  const int first = a.first_slot < live ? a.first_slot : live;
  const size_t o_c = (size_t)first * a.r * a.elem / 16, o_k = (size_t)first * a.d_rope * a.elem / 16;
  sc += o_c;
  dc += o_c;
  sk += o_k;
  dk += o_k;
  const size_t n_c = (size_t)(live - first) * a.r * a.elem / 16, n_k = (size_t)(live - first) * a.d_rope * a.elem / 16;
  const size_t step = (size_t)gridDim.x * kBlock;
  for (size_t i = (size_t)blockIdx.x * kBlock + tid; i < n_c + n_k; i += 4 * step) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t j = i + u * step;
      if (j < n_c + n_k) v[u] = j < n_c ? sc[j] : sk[j - n_c];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t j = i + u * step;
      if (j < n_c + n_k) {
        if (j < n_c) dc[j] = v[u];
        else dk[j - n_c] = v[u];
      }
    }
  }
  if (blockIdx.x == 0) {
    if (a.src_tail && a.dst_tail)
      for (int e = tid; e < a.r; e += kBlock) a.dst_tail[(size_t)b * a.r + e] = a.src_tail[(size_t)src * a.r + e];
    if (tid == 0) a.dst_len[b] = len;
  }
}

// Beam reordering over paged storage: one workgroup per destination sequence.  Pages below the one the
// next token will be written to are complete and never change again: the destination's table row takes the
// source's entries for them.  That page becomes the destination's fresh page; the source's live rows of it
// (at most one page, none when the next token opens a page) are copied over, unless the destination takes the
// source's own page over (fresh page = the source's page: nothing to copy, for the one destination that does).
__global__ __launch_bounds__(kBlock) void fork_paged_kernel(ForkArgs a) {
  const int b = blockIdx.y, part = blockIdx.x, n_parts = gridDim.x, tid = threadIdx.x;  // the copy is dealt over n_parts workgroups
  const int src = a.src_index[b];
  int fresh = a.fresh[b];
  if (src < 0 || src >= a.max_batch) {  // refuse: destination untouched
    if (part == 0 && tid == 0) *a.status = 1;  // MTLA_ERR_INVALID_ARG
    return;
  }
  const int len = a.src_len[src];
  int live = len > 0 ? (len + a.stride - 1) / a.stride : 0;
  live = live < a.max_slots ? live : a.max_slots;
  const int P = 1 << a.src.shift;
  const int next_slot = len > 0 ? len / a.stride : 0;           // the slot the next token goes into
  const int pw = (next_slot < a.max_slots ? next_slot : a.max_slots - 1) >> a.src.shift;
  const int32_t* srow = a.src.table + (size_t)src * a.src.max_pages;
  int sp = srow[pw];  // requested before it is known whether the page holds live rows (any entry is readable)
  if (fresh < 0 || fresh >= a.src.n_pages) {
    if (part == 0 && tid == 0) *a.status = 1;
    fresh = fresh < 0 ? 0 : a.src.n_pages - 1;
  }
  if (part == 0) {
    int32_t* drow = a.dst_table + (size_t)b * a.src.max_pages;
    for (int k = tid; k < pw; k += kBlock) drow[k] = srow[k];
    if (tid == 0) {
      drow[pw] = fresh;
      a.dst_len[b] = len;
    }
    for (int e = tid; e < a.r; e += kBlock) a.dst_tail[(size_t)b * a.r + e] = a.src_tail[(size_t)src * a.r + e];
  }
  const int n_rows = live - pw * P;  // live rows of the page being written to (<= P)
  if (n_rows <= 0) return;
  sp = sp < 0 ? 0 : (sp < a.src.n_pages ? sp : a.src.n_pages - 1);
  if (sp == fresh) return;           // the destination takes the source's page over
  const size_t n_c = (size_t)n_rows * a.r / 8, n_k = (size_t)n_rows * a.d_rope / 8;  // 16-byte pieces (bf16)
  const uint4* sc = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(a.cache_c) + (size_t)sp * P * a.r);
  const uint4* sk = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(a.cache_kr) + (size_t)sp * P * a.d_rope);
  uint4* dc = reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(a.cache_c) + (size_t)fresh * P * a.r);
  uint4* dk = reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(a.cache_kr) + (size_t)fresh * P * a.d_rope);
  constexpr int U = 8;  // pieces in flight per thread
  const size_t step = (size_t)n_parts * kBlock;
  for (size_t i = (size_t)part * kBlock + tid; i < n_c + n_k; i += U * step) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t j = i + (size_t)u * step;
      if (j < n_c + n_k) v[u] = j < n_c ? sc[j] : sk[j - n_c];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t j = i + (size_t)u * step;
      if (j < n_c + n_k) {
        if (j < n_c) dc[j] = v[u];
        else dk[j - n_c] = v[u];
      }
    }
  }
}

hipError_t launch_fork_paged(const ForkArgs& a, hipStream_t st) {
  const size_t page_bytes = ((size_t)a.r + a.d_rope) * 2 << a.src.shift;
  size_t parts = (page_bytes + (16u << 10) - 1) / (16u << 10);  // about 16 KB of a page per workgroup
  parts = parts < 1 ? 1 : (parts > 16 ? 16 : parts);
  hipLaunchKernelGGL(fork_paged_kernel, dim3((unsigned)parts, a.batch), dim3(kBlock), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_reorder(const ReorderArgs& a, hipStream_t st) {
  const size_t seq_bytes = (size_t)a.max_slots * (a.r + a.d_rope) * a.elem;
  size_t nx = (seq_bytes + (64u << 10) - 1) / (64u << 10);  // about 64 KB per workgroup and pass
  nx = nx < 1 ? 1 : (nx > 64 ? 64 : nx);
  hipLaunchKernelGGL(reorder_kernel, dim3((unsigned)nx, a.batch), dim3(kBlock), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_stream_read(const void* p, size_t bytes, int32_t* out, int workgroups, hipStream_t st) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(kBlock), 0, st, reinterpret_cast<const uint4*>(p),
                     bytes / 16, reinterpret_cast<uint32_t*>(out));
  return hipGetLastError();
}

hipError_t launch_fill_zero(int32_t* p, int n, hipStream_t st) {
  hipLaunchKernelGGL(fill_zero_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, n);
  return hipGetLastError();
}

bool decode_front_supported(const AppendArgs& ap, const AbsorbArgs& ab) {
  const bool nch = ap.r == 64 || ap.r == 128 || ap.r == 256 || ap.r == 512;
  const bool kk = ab.d_head == 32 || ab.d_head == 64 || ab.d_head == 128;
  return nch && kk && ab.out_bf16 && ap.n_new_max == 1 && ab.rows == ap.batch;
}

hipError_t launch_decode_front(const AppendArgs& ap, const AbsorbArgs& ab, hipStream_t st) {
  const int gx = ab.r / 64 + 1, gy = ab.n_heads;
  const int gz = (ab.rows + absorb_rows_per_block(ab.rows) - 1) / absorb_rows_per_block(ab.rows);
  const dim3 grid(ap.batch + gx * gy * gz), block(kBlock);
  const size_t smem = (size_t)(ap.d_hyper + 4 + 8 + ap.r) * sizeof(float);
#define MTLA_FRONT(N, K)                                                                                \
  if (ap.r == 32 * N && ab.d_head == 32 * K) {                                                          \
    if (ap.c_new_f32)                                                                                   \
      hipLaunchKernelGGL((decode_front_kernel<N, K, float>), grid, block, smem, st, ap, ab, gx, gy);    \
    else                                                                                                \
      hipLaunchKernelGGL((decode_front_kernel<N, K, bf16>), grid, block, smem, st, ap, ab, gx, gy);     \
    return hipGetLastError();                                                                           \
  }
  MTLA_FRONT(2, 1) MTLA_FRONT(2, 2) MTLA_FRONT(2, 4)
  MTLA_FRONT(4, 1) MTLA_FRONT(4, 2) MTLA_FRONT(4, 4)
  MTLA_FRONT(8, 1) MTLA_FRONT(8, 2) MTLA_FRONT(8, 4)
  MTLA_FRONT(16, 1) MTLA_FRONT(16, 2) MTLA_FRONT(16, 4)
#undef MTLA_FRONT
  return hipErrorInvalidValue;
}

bool append_bulk_mfma_supported(const AppendArgs& a, int dtype) {
  return dtype != 0 && a.tail_c && a.stride <= kBulkMaxStride && a.d_hyper % 16 == 0 && a.d_hyper <= 64 && a.r % 32 == 0 &&
         a.d_rope % 8 == 0 && a.d_rope <= 128;
}

hipError_t launch_append(const AppendArgs& a, int dtype, hipStream_t st) {
  const size_t smem = (size_t)(a.r + a.d_hyper + 4) * sizeof(float);
  if (a.n_new_max == 1) {  // decode step: one workgroup per sequence, advances seq_len itself
    const size_t smem1 = (size_t)(a.d_hyper + 4 + 8 + a.r) * sizeof(float);
    const dim3 grid(a.batch), block(kBlock);
#define MTLA_STEP(TT, N)                                                            \
  if (a.r == 32 * N) {                                                               \
    hipLaunchKernelGGL((append_step_kernel<TT, N>), grid, block, smem1, st, a);      \
    return hipGetLastError();                                                        \
  }
    if (dtype == 0) {
      MTLA_STEP(float, 2) MTLA_STEP(float, 4) MTLA_STEP(float, 8) MTLA_STEP(float, 16)
    } else {
      MTLA_STEP(bf16, 2) MTLA_STEP(bf16, 4) MTLA_STEP(bf16, 8) MTLA_STEP(bf16, 16)
    }
#undef MTLA_STEP
    return hipErrorInvalidValue;
  }
  // slots a call can touch per sequence: a partly filled first slot plus the rest
  const int n_slots = (a.n_new_max + a.stride - 2) / a.stride + 1;
  const dim3 grid(n_slots, a.batch), block(kBlock);
  if (append_bulk_mfma_supported(a, dtype)) {
    const dim3 grid16((n_slots + kBulkSlots - 1) / kBulkSlots, a.batch);
#define MTLA_BULK(DY)                                                                                           \
  if (a.c_merge_f32) hipLaunchKernelGGL((append_bulk_mfma_kernel<DY, true>), grid16, block, 0, st, a);          \
  else hipLaunchKernelGGL((append_bulk_mfma_kernel<DY, false>), grid16, block, 0, st, a);
    switch (a.d_hyper / 16) {
      case 1: MTLA_BULK(1) break;
      case 2: MTLA_BULK(2) break;
      case 3: MTLA_BULK(3) break;
      default: MTLA_BULK(4) break;
    }
#undef MTLA_BULK
  } else if (dtype == 0)
    hipLaunchKernelGGL(append_kernel<float>, grid, block, smem, st, a);
  else
    hipLaunchKernelGGL(append_kernel<bf16>, grid, block, smem, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(advance_len_kernel, dim3((a.batch + 255) / 256), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace mtla
