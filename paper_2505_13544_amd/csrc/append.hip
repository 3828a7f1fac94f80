// mtla_cache_append kernels: hyper-network merge weight, then the temporal
// merge of the new latent into the strided cache (Section "Inference using
// MTLA": Eq. (infer-linear) and the update rule; RoPE-key rule of Section
// "Decoupled Rotary Position Embedding").
//
// One workgroup owns one (sequence, slot) pair touched by the call, so every
// cache row has exactly one writer.  A decode step (one token per sequence)
// is a single launch of `batch` workgroups that also advances seq_len
// (append_step_kernel); a bulk append (prefix) launches one workgroup per
// touched slot (append_kernel) and a second tiny kernel advances seq_len once
// every workgroup has read the old value.
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
template <typename T, int NCH>
__device__ __forceinline__ void append_step_block(const AppendArgs& a, int b, float* smem) {
  float* sg = smem;             // [dy] Linear(c)
  float* red = smem + a.d_hyper;  // [4]
  const int tid = threadIdx.x;
  const int s = a.stride, r = a.r, dR = a.d_rope, dy = a.d_hyper;
  const int q = tid & (kTPR - 1), y = tid / kTPR;
  const int p0 = a.seq_len[b];
  const int n = a.n_new ? a.n_new[b] : 1;
  const T* crow = reinterpret_cast<const T*>(a.c_new) + (size_t)b * r;
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
  const bool hyper = !a.w_override;
  Chunk8<T> cch[NCH], ach[NCH];
  const T* A = reinterpret_cast<const T*>(a.hyp_A);
  const T* ha = reinterpret_cast<const T*>(a.hyp_a);
  float bias = 0.f;
  if (hyper) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) cch[i].load(crow + 8 * (q + i * kTPR));
    if (y < dy) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) ach[i].load(A + (size_t)y * r + 8 * (q + i * kTPR));
      if (ha) bias = to_f32(ha[y]);
    }
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
          cch[i].unpack(cv);
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
    const float z = hyper_logit(sg, reinterpret_cast<const T*>(a.hyp_G) + (size_t)slot * dy, red, dy, tid);
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
    }
  }
  if (tid < dR / 8) krv.store(reinterpret_cast<T*>(a.cache_kr) + ((size_t)b * a.max_slots + slot) * dR + 8 * tid);
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
template <int NCH, int KK>
__global__ __launch_bounds__(kBlock) void decode_front_kernel(AppendArgs ap, AbsorbArgs ab, int gx, int gy) {
  extern __shared__ float smem[];
  const int blk = blockIdx.x;
  if (blk < ap.batch) {
    append_step_block<bf16, NCH>(ap, blk, smem);
    return;
  }
  const int i = blk - ap.batch;
  const int bx = i % gx, rest = i / gx;
  absorb_mfma_block<KK>(ab, bx, rest % gy, rest / gy);
}

template <typename T>
__global__ __launch_bounds__(kBlock) void append_kernel(AppendArgs a) {
  extern __shared__ float smem[];
  float* sc = smem;              // [r] current token's latent in fp32
  float* sg = smem + a.r;        // [dy] Linear(c)
  float* red = sg + a.d_hyper;   // [4] per-wave partial of the hyper-network logit

  const int b = blockIdx.y, kslot = blockIdx.x, tid = threadIdx.x;
  const int s = a.stride, r = a.r, dR = a.d_rope, dy = a.d_hyper;

  const int p0 = a.seq_len[b];
  int n = a.n_new ? a.n_new[b] : a.n_new_max;
  n = n < 0 ? 0 : (n > a.n_new_max ? a.n_new_max : n);
  if (n == 0) return;
  if ((long long)p0 + n > (long long)a.max_slots * s) {  // refuse: sequence untouched
    if (kslot == 0 && tid == 0) *a.status = 3;           // MTLA_ERR_CAPACITY
    return;
  }
  const int slot = p0 / s + kslot;
  const long long slot_first = (long long)slot * s;
  const int t_lo = int((slot_first > p0 ? slot_first : (long long)p0) - p0);
  const long long slot_end = slot_first + s;
  const int t_hi = int((slot_end < (long long)p0 + n ? slot_end : (long long)p0 + n) - p0);
  if (t_lo >= t_hi) return;

  T* crow_out = reinterpret_cast<T*>(a.cache_c) + ((size_t)b * a.max_slots + slot) * r;
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
  T* kr_dst = reinterpret_cast<T*>(a.cache_kr) + ((size_t)b * a.max_slots + slot) * dR;
  for (int e = tid; e < dR; e += kBlock) kr_dst[e] = kr_src[e];
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
  const int gz = (ab.rows + kAbsorbRowsPerBlock - 1) / kAbsorbRowsPerBlock;
  const dim3 grid(ap.batch + gx * gy * gz), block(kBlock);
  const size_t smem = (size_t)(ap.d_hyper + 4) * sizeof(float);
#define MTLA_FRONT(N, K)                                                                         \
  if (ap.r == 32 * N && ab.d_head == 32 * K) {                                                   \
    hipLaunchKernelGGL((decode_front_kernel<N, K>), grid, block, smem, st, ap, ab, gx, gy);      \
    return hipGetLastError();                                                                    \
  }
  MTLA_FRONT(2, 1) MTLA_FRONT(2, 2) MTLA_FRONT(2, 4)
  MTLA_FRONT(4, 1) MTLA_FRONT(4, 2) MTLA_FRONT(4, 4)
  MTLA_FRONT(8, 1) MTLA_FRONT(8, 2) MTLA_FRONT(8, 4)
  MTLA_FRONT(16, 1) MTLA_FRONT(16, 2) MTLA_FRONT(16, 4)
#undef MTLA_FRONT
  return hipErrorInvalidValue;
}

hipError_t launch_append(const AppendArgs& a, int dtype, hipStream_t st) {
  const size_t smem = (size_t)(a.r + a.d_hyper + 4) * sizeof(float);
  if (a.n_new_max == 1) {  // decode step: one workgroup per sequence, advances seq_len itself
    const size_t smem1 = (size_t)(a.d_hyper + 4) * sizeof(float);
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
  if (dtype == 0)
    hipLaunchKernelGGL(append_kernel<float>, grid, block, smem, st, a);
  else
    hipLaunchKernelGGL(append_kernel<bf16>, grid, block, smem, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(advance_len_kernel, dim3((a.batch + 255) / 256), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace mtla
