// mtla_cache_append kernels: hyper-network merge weight, then the temporal
// merge of the new latent into the strided cache (Section "Inference using
// MTLA": Eq. (infer-linear) and the update rule; RoPE-key rule of Section
// "Decoupled Rotary Position Embedding").
//
// One workgroup owns one (sequence, slot) pair touched by the call, so every
// cache row has exactly one writer.  A decode step (one token per sequence)
// is a single launch of `batch` workgroups that also advances seq_len; a bulk
// append (prefix) launches one workgroup per touched slot and a second tiny
// kernel advances seq_len once every workgroup has read the old value.
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

constexpr int kMaxRPerThread = 4;  // r <= 1024 with 256 threads

template <typename T>
__global__ __launch_bounds__(kBlock) void append_kernel(AppendArgs a, int update_len) {
  extern __shared__ float smem[];
  float* sc = smem;          // [r] current token's latent in fp32
  float* red = smem + a.r;   // [4] per-wave partial of the hyper-network logit

  const int b = blockIdx.y, kslot = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wv = tid >> 6;
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
      // logit = sum_y G[slot][y] * (a[y] + sum_n A[y][n] c[n]); rows y strided over waves
      float zp = 0.f;
      for (int y = wv; y < dy; y += kBlock / kWave) {
        const T* Arow = A + (size_t)y * r;
        float d = 0.f;
        for (int e = lane; e < r; e += kWave) d += to_f32(Arow[e]) * sc[e];
        d = wave_sum(d);
        const float bias = ha ? to_f32(ha[y]) : 0.f;
        zp += (d + bias) * to_f32(G[(size_t)slot * dy + y]);
      }
      if (lane == 0) red[wv] = zp;
      __syncthreads();
      const float z = (red[0] + red[1]) + (red[2] + red[3]);
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

  if (update_len) {  // single workgroup per sequence: every thread has read p0 above
    __syncthreads();
    if (tid == 0) a.seq_len[b] = p0 + n;
  }
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

}  // namespace

hipError_t launch_fill_zero(int32_t* p, int n, hipStream_t st) {
  hipLaunchKernelGGL(fill_zero_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, n);
  return hipGetLastError();
}

hipError_t launch_append(const AppendArgs& a, int dtype, hipStream_t st) {
  // slots a call can touch per sequence: a partly filled first slot plus the rest
  const int n_slots = (a.n_new_max + a.stride - 2) / a.stride + 1;
  const int single = (n_slots == 1) ? 1 : 0;
  const dim3 grid(n_slots, a.batch), block(kBlock);
  const size_t smem = (size_t)(a.r + 4) * sizeof(float);
  if (dtype == 0)
    hipLaunchKernelGGL(append_kernel<float>, grid, block, smem, st, a, single);
  else
    hipLaunchKernelGGL(append_kernel<bf16>, grid, block, smem, st, a, single);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || single) return e;
  hipLaunchKernelGGL(advance_len_kernel, dim3((a.batch + 255) / 256), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace mtla
