// The append of one token per sequence (a decode step): hyper-network merge weight and the update of
// the sequence's open slot, as one workgroup's work.  Shared by the append kernels (append.hip) and
// the one-launch decode step (decode_fused.hip), so that every path leaves bit-identical state.
#pragma once
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
//
// FUSED (the one-launch decode step calls it): the new value of the open slot -- latent row as
// stored, then the RoPE key -- is also published at pub_row ([r + d_rope] bf16) with device-scope
// stores for the workgroup that attends that slot in the same launch (a 16-bit pattern 0xffff
// means "not there yet" to the reader, so that one NaN pattern is written as another), and
// seq_len is left to the caller, who advances it once no workgroup can still read the old value.
__device__ __forceinline__ void publish_bf16(uint16_t* p, uint16_t bits) {
  __hip_atomic_store(p, (uint16_t)(bits == 0xffffu ? 0x7fffu : bits), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename T, int NCH, typename TC = T, bool FUSED = false>
__device__ __forceinline__ void append_step_block(const AppendArgs& a, int b, float* smem, uint16_t* pub_row = nullptr) {
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
  const float* sc_ln = smem + a.d_hyper + 4 + 8;
  const bool hyper = !a.w_override;
  Chunk8<TC> cch[NCH];
  Chunk8<T> ach[NCH];
  const T* A = reinterpret_cast<const T*>(a.hyp_A);
  const T* ha = reinterpret_cast<const T*>(a.hyp_a);
  float bias = 0.f;
  if (hyper) {
#pragma unroll
    for (int i = 0; i < NCH; ++i)
      if (!ln) cch[i].load(crow + 8 * (q + i * kTPR));
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
    float* sc = lred + 8;  // [r] the normalised latent, for the hyper-network's rows
#pragma unroll
    for (int i = 0; i < kMaxRPerThread; ++i) {
      const int e = tid + i * kBlock;
      if (e < r) {
        cel[i] = (cel[i] - ln_mean) * ln_inv;
        if (ln_g) cel[i] *= to_f32(ln_g[e]);
        if (ln_b) cel[i] += to_f32(ln_b[e]);
        sc[e] = cel[i];
      }
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
          if (ln) load8(sc_ln + 8 * (q + i * kTPR), cv);
          else cch[i].unpack(cv);
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
  T* crow_out = reinterpret_cast<T*>(a.cache_c) + ((size_t)b * a.max_slots + slot) * r;
#pragma unroll
  for (int i = 0; i < kMaxRPerThread; ++i) {
    const int e = tid + i * kBlock;
    if (e < r) {
      const float old = continuing ? (tail ? told[i] : to_f32(crow_out[e])) : 0.f;
      const float v = old + w * cel[i];
      crow_out[e] = from_f32<T>(v);
      if (tail) tail[e] = v;
      if constexpr (FUSED) publish_bf16(pub_row + e, f32_to_bf16_bits(v));
    }
  }
  if (tid < dR / 8) {
    krv.store(reinterpret_cast<T*>(a.cache_kr) + ((size_t)b * a.max_slots + slot) * dR + 8 * tid);
    if constexpr (FUSED) {  // bf16 storage only
      const uint32_t w4[4] = {krv.raw.x, krv.raw.y, krv.raw.z, krv.raw.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        publish_bf16(pub_row + r + 8 * tid + 2 * i, (uint16_t)(w4[i] & 0xffffu));
        publish_bf16(pub_row + r + 8 * tid + 2 * i + 1, (uint16_t)(w4[i] >> 16));
      }
    }
  }
  if (tid == 0) {
    if (a.w_out) a.w_out[b] = w;
    if (a.slot_out) a.slot_out[b] = slot;
    if constexpr (!FUSED) a.seq_len[b] = p0 + 1;  // every thread took p0 before the barrier
  }
}

}  // namespace

}  // namespace mtla
