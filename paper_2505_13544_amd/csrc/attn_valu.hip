// fp32 vector-ALU attention kernels.  They carry the MTLA_F32 storage path
// (whose 1e-5 parity bound rules out bf16 matrix-core inputs) and serve as the
// plain fallback for shapes the matrix-core kernels do not cover.
//
//   absorb_kernel        q~_h = W_K^(h) q_h, concatenated with the RoPE query   (Eq. (obsorb))
//   attn_split_kernel    logits, online softmax and the latent-space weighted
//                        sum over one chunk of slots, all heads of a head group
//                        sharing each cache row                                 (Eq. (with-rope))
//   combine_kernel       log-sum-exp merge of the chunk partials, then o = o~ W_V^(h)
//   partial_states_kernel  C_hat'[m] = running in-chunk sum of w_n c_n          (training form)
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

constexpr int kAbsorbRows = 8;
constexpr int kWaves = kBlock / kWave;

template <typename T, typename OutT>
__global__ __launch_bounds__(kBlock) void absorb_kernel(AbsorbArgs a) {
  extern __shared__ float sq[];  // [kAbsorbRows][d_head]
  const int tid = threadIdx.x, n = blockIdx.x * kBlock + tid, h = blockIdx.y;
  const int row0 = blockIdx.z * kAbsorbRows;
  const int dh = a.d_head, r = a.r, dR = a.d_rope, E = r + dR;
  const T* q = reinterpret_cast<const T*>(a.q);
  const T* qr = reinterpret_cast<const T*>(a.q_rope);
  const T* wuk = reinterpret_cast<const T*>(a.w_uk);
  OutT* qcat = reinterpret_cast<OutT*>(a.qcat);

  for (int idx = tid; idx < kAbsorbRows * dh; idx += kBlock) {
    const int rr = idx / dh, k = idx - rr * dh, row = row0 + rr;
    sq[idx] = row < a.rows ? to_f32(q[((size_t)row * a.n_heads + h) * dh + k]) : 0.f;
  }
  __syncthreads();
  if (n < r) {
    float acc[kAbsorbRows];
#pragma unroll
    for (int rr = 0; rr < kAbsorbRows; ++rr) acc[rr] = 0.f;
    const T* wcol = wuk + (size_t)h * dh * r + n;
    for (int k = 0; k < dh; ++k) {
      const float wv = to_f32(wcol[(size_t)k * r]);
#pragma unroll
      for (int rr = 0; rr < kAbsorbRows; ++rr) acc[rr] += sq[rr * dh + k] * wv;
    }
#pragma unroll
    for (int rr = 0; rr < kAbsorbRows; ++rr) {
      const int row = row0 + rr;
      if (row < a.rows) qcat[((size_t)row * a.n_heads + h) * E + n] = from_f32<OutT>(acc[rr] * a.scale_log2);
    }
  } else if (n < E) {
#pragma unroll
    for (int rr = 0; rr < kAbsorbRows; ++rr) {
      const int row = row0 + rr;
      if (row < a.rows)
        qcat[((size_t)row * a.n_heads + h) * E + n] =
            from_f32<OutT>(to_f32(qr[((size_t)row * a.n_heads + h) * dR + (n - r)]) * a.scale_log2);
    }
  }
}

// Live column count of a query row and the mapping from column k to a source row.
struct RowMap {
  int b, m, live, stride, T, max_slots;
  __device__ __forceinline__ size_t src(int k) const {
    if (T == 0) return (size_t)b * max_slots + k;                        // decode: cache slot k
    const int row = (k < live - 1) ? (k * stride + stride - 1) : m;      // prefill: final state of
    return (size_t)b * T + row;                                          // chunk k, or own row
  }
};

__device__ __forceinline__ RowMap make_row_map(int row, const int32_t* seq_len, int stride, int T,
                                               int max_slots) {
  RowMap rm;
  rm.stride = stride;
  rm.T = T;
  rm.max_slots = max_slots;
  if (T == 0) {
    rm.b = row;
    rm.m = 0;
    const int len = seq_len[row];
    rm.live = (len + stride - 1) / stride;
  } else {
    rm.b = row / T;
    rm.m = row - rm.b * T;
    const bool valid = seq_len ? rm.m < seq_len[rm.b] : true;
    rm.live = valid ? rm.m / stride + 1 : 0;
  }
  return rm;
}

template <typename T, int R, int DR, int HG>
__global__ __launch_bounds__(kBlock) void attn_split_kernel(AttnArgs a) {
  constexpr int E = R + DR, RI = R / kWave;
  static_assert(R % kWave == 0 && DR <= kWave, "lane mapping");
  __shared__ float sq[HG][E];
  __shared__ float s_o[HG][R];
  __shared__ float s_m[kWaves][HG], s_l[kWaves][HG];

  const int split = blockIdx.x, row = blockIdx.y, h0 = blockIdx.z * HG;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const RowMap rm = make_row_map(row, a.seq_len, a.stride, a.T, a.max_slots);
  const int k0 = split * a.chunk;
  const int k1 = rm.live < k0 + a.chunk ? rm.live : k0 + a.chunk;
  if (k0 >= k1) return;

  const float* qcat = reinterpret_cast<const float*>(a.qcat);
  for (int idx = tid; idx < HG * E; idx += kBlock) {
    const int hh = idx / E, e = idx - hh * E, h = h0 + hh;
    sq[hh][e] = h < a.n_heads ? qcat[((size_t)row * a.n_heads + h) * E + e] : 0.f;
  }
  __syncthreads();

  const T* lat = reinterpret_cast<const T*>(a.lat);
  const T* key = reinterpret_cast<const T*>(a.key);
  float mrun[HG], lrun[HG], acc[HG][RI];
#pragma unroll
  for (int hh = 0; hh < HG; ++hh) {
    mrun[hh] = -INFINITY;
    lrun[hh] = 0.f;
#pragma unroll
    for (int i = 0; i < RI; ++i) acc[hh][i] = 0.f;
  }

  for (int k = k0 + wv; k < k1; k += kWaves) {
    const size_t src = rm.src(k);
    const T* cr = lat + src * R;
    float cv[RI];
#pragma unroll
    for (int i = 0; i < RI; ++i) cv[i] = to_f32(cr[lane + i * kWave]);
    const float kv = lane < DR ? to_f32(key[src * DR + lane]) : 0.f;
#pragma unroll
    for (int hh = 0; hh < HG; ++hh) {
      float d = lane < DR ? kv * sq[hh][R + lane] : 0.f;
#pragma unroll
      for (int i = 0; i < RI; ++i) d += cv[i] * sq[hh][lane + i * kWave];
      d = wave_sum(d);  // logit in log2 units (the query is pre-scaled)
      const float mn = fmaxf(mrun[hh], d);
      const float alpha = exp2f(mrun[hh] - mn);
      const float p = exp2f(d - mn);
      lrun[hh] = lrun[hh] * alpha + p;
#pragma unroll
      for (int i = 0; i < RI; ++i) acc[hh][i] = acc[hh][i] * alpha + p * cv[i];
      mrun[hh] = mn;
    }
  }

  // merge the four waves' running states
  if (lane == 0) {
#pragma unroll
    for (int hh = 0; hh < HG; ++hh) {
      s_m[wv][hh] = mrun[hh];
      s_l[wv][hh] = lrun[hh];
    }
  }
  __syncthreads();
#pragma unroll
  for (int hh = 0; hh < HG; ++hh) {
    float mstar = s_m[0][hh];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) mstar = fmaxf(mstar, s_m[w][hh]);
    const float f = exp2f(mrun[hh] - mstar);  // 0 for a wave that saw no slot
#pragma unroll
    for (int i = 0; i < RI; ++i) acc[hh][i] *= f;
  }
  for (int w = 0; w < kWaves; ++w) {
    if (wv == w) {
#pragma unroll
      for (int hh = 0; hh < HG; ++hh)
#pragma unroll
        for (int i = 0; i < RI; ++i) {
          if (w == 0)
            s_o[hh][lane + i * kWave] = acc[hh][i];
          else
            s_o[hh][lane + i * kWave] += acc[hh][i];
        }
    }
    __syncthreads();
  }
  const size_t pbase = ((size_t)row * a.n_splits + split) * a.n_heads;
  for (int idx = tid; idx < HG * R; idx += kBlock) {
    const int hh = idx / R, n = idx - hh * R, h = h0 + hh;
    if (h < a.n_heads) a.part_o[(pbase + h) * R + n] = s_o[hh][n];
  }
  if (tid < HG && h0 + tid < a.n_heads) {
    float mstar = s_m[0][tid];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) mstar = fmaxf(mstar, s_m[w][tid]);
    float lstar = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) lstar += s_l[w][tid] * exp2f(s_m[w][tid] - mstar);
    a.part_ml[(pbase + h0 + tid) * 2 + 0] = mstar;
    a.part_ml[(pbase + h0 + tid) * 2 + 1] = lstar;
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void combine_kernel(CombineArgs a) {
  extern __shared__ float smem[];
  float* s_lat = smem;             // [r]
  float* s_red = smem + a.r;       // [kBlock]
  float* s_f = s_red + kBlock;     // [n_splits]
  const int h = blockIdx.x, row = blockIdx.y, tid = threadIdx.x;
  const int r = a.r, dh = a.d_head;
  const RowMap rm = make_row_map(row, a.seq_len, a.stride, a.T, 0);
  float* out = a.out;
  const size_t oh = (size_t)row * a.n_heads + h;

  if (rm.live == 0) {
    if (a.out_latent)
      for (int n = tid; n < r; n += kBlock) a.out_latent[oh * r + n] = 0.f;
    if (out)
      for (int d = tid; d < dh; d += kBlock) out[oh * dh + d] = 0.f;
    if (a.lse && tid == 0) a.lse[oh] = -INFINITY;
    return;
  }
  const int nsp = (rm.live + a.chunk - 1) / a.chunk;
  const size_t pb = (size_t)row * a.n_splits * a.n_heads + h;  // + sp * n_heads
  float mstar = -INFINITY;
  for (int sp = 0; sp < nsp; ++sp) mstar = fmaxf(mstar, a.part_ml[(pb + (size_t)sp * a.n_heads) * 2]);
  for (int sp = tid; sp < nsp; sp += kBlock)
    s_f[sp] = exp2f(a.part_ml[(pb + (size_t)sp * a.n_heads) * 2] - mstar);
  __syncthreads();
  float lstar = 0.f;
  for (int sp = 0; sp < nsp; ++sp) lstar += s_f[sp] * a.part_ml[(pb + (size_t)sp * a.n_heads) * 2 + 1];
  const float inv = 1.f / lstar;
  for (int n = tid; n < r; n += kBlock) {
    float o = 0.f;
    for (int sp = 0; sp < nsp; ++sp) o += s_f[sp] * a.part_o[(pb + (size_t)sp * a.n_heads) * r + n];
    o *= inv;
    s_lat[n] = o;
    if (a.out_latent) a.out_latent[oh * r + n] = o;
  }
  if (a.lse && tid == 0) a.lse[oh] = (mstar + log2f(lstar)) * 0.6931471805599453f;
  if (!out) return;
  __syncthreads();
  // o = o~ W_V^(h): thread (group g, column d) sums rows n = g, g + ngrp, ...
  const T* wuv = reinterpret_cast<const T*>(a.w_uv) + (size_t)h * r * dh;
  const int ngrp = kBlock / dh, g = tid / dh, d = tid - g * dh;
  float part = 0.f;
  if (g < ngrp)
    for (int n = g; n < r; n += ngrp) part += s_lat[n] * to_f32(wuv[(size_t)n * dh + d]);
  s_red[tid] = part;
  __syncthreads();
  if (g == 0) {
    float sum = 0.f;
    for (int gg = 0; gg < ngrp; ++gg) sum += s_red[gg * dh + d];
    out[oh * dh + d] = sum;
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void partial_states_kernel(PartialStateArgs a) {
  const int n_chunks = (a.T + a.stride - 1) / a.stride;
  const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
  const size_t total = (size_t)a.batch * n_chunks * a.r;
  if (idx >= total) return;
  const int e = int(idx % a.r);
  const int ch = int((idx / a.r) % n_chunks);
  const int b = int(idx / ((size_t)a.r * n_chunks));
  const T* c = reinterpret_cast<const T*>(a.c);
  T* cp = reinterpret_cast<T*>(a.cprime);
  float run = 0.f;
  const int n_end = (ch + 1) * a.stride < a.T ? (ch + 1) * a.stride : a.T;
  for (int n = ch * a.stride; n < n_end; ++n) {
    const size_t o = ((size_t)b * a.T + n) * a.r + e;
    run += a.w[(size_t)b * a.T + n] * to_f32(c[o]);
    cp[o] = from_f32<T>(run);
  }
}

template <typename T, int R, int DR>
hipError_t launch_attn_rd(const AttnArgs& a, hipStream_t st) {
  const int rows = a.T ? a.batch * a.T : a.batch;
  if (a.n_heads <= 4) {
    const dim3 grid(a.n_splits, rows, 1);
    hipLaunchKernelGGL((attn_split_kernel<T, R, DR, 4>), grid, dim3(kBlock), 0, st, a);
  } else {
    const dim3 grid(a.n_splits, rows, (a.n_heads + 7) / 8);
    hipLaunchKernelGGL((attn_split_kernel<T, R, DR, 8>), grid, dim3(kBlock), 0, st, a);
  }
  return hipGetLastError();
}

template <typename T>
hipError_t launch_attn_t(const AttnArgs& a, hipStream_t st) {
#define MTLA_CASE(RR, DD) \
  if (a.r == RR && a.d_rope == DD) return launch_attn_rd<T, RR, DD>(a, st);
  MTLA_CASE(64, 32)
  MTLA_CASE(64, 64)
  MTLA_CASE(128, 32)
  MTLA_CASE(128, 64)
  MTLA_CASE(256, 32)
  MTLA_CASE(256, 64)
  MTLA_CASE(512, 32)
  MTLA_CASE(512, 64)
#undef MTLA_CASE
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_absorb(const AbsorbArgs& a, int dtype, hipStream_t st) {
  const int E = a.r + a.d_rope;
  const dim3 grid((E + kBlock - 1) / kBlock, a.n_heads, (a.rows + kAbsorbRows - 1) / kAbsorbRows);
  const size_t smem = (size_t)kAbsorbRows * a.d_head * sizeof(float);
  if (dtype == 0)
    hipLaunchKernelGGL((absorb_kernel<float, float>), grid, dim3(kBlock), smem, st, a);
  else if (a.out_bf16)
    hipLaunchKernelGGL((absorb_kernel<bf16, bf16>), grid, dim3(kBlock), smem, st, a);
  else
    hipLaunchKernelGGL((absorb_kernel<bf16, float>), grid, dim3(kBlock), smem, st, a);
  return hipGetLastError();
}

hipError_t launch_attn_split(const AttnArgs& a, int dtype, hipStream_t st) {
  return dtype == 0 ? launch_attn_t<float>(a, st) : launch_attn_t<bf16>(a, st);
}

hipError_t launch_combine(const CombineArgs& a, int dtype, hipStream_t st) {
  const int rows = a.T ? a.batch * a.T : a.batch;
  const dim3 grid(a.n_heads, rows);
  const size_t smem = (size_t)(a.r + kBlock + a.n_splits) * sizeof(float);
  if (dtype == 0)
    hipLaunchKernelGGL(combine_kernel<float>, grid, dim3(kBlock), smem, st, a);
  else
    hipLaunchKernelGGL(combine_kernel<bf16>, grid, dim3(kBlock), smem, st, a);
  return hipGetLastError();
}

hipError_t launch_partial_states(const PartialStateArgs& a, int dtype, hipStream_t st) {
  const int n_chunks = (a.T + a.stride - 1) / a.stride;
  const size_t total = (size_t)a.batch * n_chunks * a.r;
  const dim3 grid((unsigned)((total + kBlock - 1) / kBlock));
  if (dtype == 0)
    hipLaunchKernelGGL(partial_states_kernel<float>, grid, dim3(kBlock), 0, st, a);
  else
    hipLaunchKernelGGL(partial_states_kernel<bf16>, grid, dim3(kBlock), 0, st, a);
  return hipGetLastError();
}

}  // namespace mtla
