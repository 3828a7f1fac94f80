// fp32 vector-ALU attention kernels.  They carry the MTLA_F32 storage path
// (whose 1e-5 parity bound rules out bf16 matrix-core inputs) and serve as the
// plain fallback for shapes the matrix-core kernels do not cover.
//
//   attn_split_kernel    logits, online softmax and the latent-space weighted
//                        sum over one chunk of slots, all heads of a head group
//                        sharing each cache row                                 (Eq. (with-rope))
//   partial_states_kernel  C_hat'[m] = running in-chunk sum of w_n c_n          (training form)
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

constexpr int kWaves = kBlock / kWave;

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
  _Float16* cp16 = reinterpret_cast<_Float16*>(a.cprime);
  float run = 0.f;
  const int n_end = (ch + 1) * a.stride < a.T ? (ch + 1) * a.stride : a.T;
  const int len = a.seq_len ? a.seq_len[b] : a.T;
  for (int n = ch * a.stride; n < n_end; ++n) {
    const size_t o = ((size_t)b * a.T + n) * a.r + e;
    // padding rows hold zeros: they are multiplied by zero weights in the tiles of live rows
    run = n < len ? run + a.w[(size_t)b * a.T + n] * to_f32(c[o]) : 0.f;
    if (a.out_f16) cp16[o] = static_cast<_Float16>(run);
    else cp[o] = from_f32<T>(run);
  }
}

template <typename T, int R, int DR>
hipError_t launch_attn_rd(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  const int rows = a.T ? a.batch * a.T : a.batch;
  if (a.n_heads <= 4) {
    const dim3 grid(a.n_splits, rows, 1);
    launch_timed(attn_split_kernel<T, R, DR, 4>, grid, dim3(kBlock), 0, st, ev, a);
  } else {
    const dim3 grid(a.n_splits, rows, (a.n_heads + 7) / 8);
    launch_timed(attn_split_kernel<T, R, DR, 8>, grid, dim3(kBlock), 0, st, ev, a);
  }
  return hipGetLastError();
}

template <typename T>
hipError_t launch_attn_t(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
#define MTLA_CASE(RR, DD) \
  if (a.r == RR && a.d_rope == DD) return launch_attn_rd<T, RR, DD>(a, st, ev);
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

hipError_t launch_attn_split(const AttnArgs& a, int dtype, hipStream_t st, const EventPair& ev) {
  return dtype == 0 ? launch_attn_t<float>(a, st, ev) : launch_attn_t<bf16>(a, st, ev);
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
