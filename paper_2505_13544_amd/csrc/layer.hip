// The layer around the decode path, for one new token per sequence (bf16 storage, gfx950):
//   layer_front_kernel   x -> q = x W_Q (Eq. (query)), q^R = RoPE(x W_QR), c = x W_r (Eq. (low-rank); its
//                        layer normalisation is done by the step's append, where a whole row meets in
//                        one workgroup), k^R = RoPE(x W_KR) (Section "Decoupled Rotary Position
//                        Embedding in MTLA"); q, q^R and c leave in fp32 (they are rounded where they are
//                        used), k^R in bf16
//                        (Section "Decoupled Rotary Position Embedding in MTLA")
//   layer_out_kernel     y = concat_h(o_h) W_O (Eq. (softmax))
// Weights are output-major, [out_features, d_in], so that the contracted index is innermost for both
// operands of `D[n, token] = sum_k W[n, k] x[token, k]` (v_mfma_f32_16x16x32_bf16: W rows are the A
// operand, token rows the B operand).  At decode batch sizes these are weight-streaming kernels: a
// wavefront owns 16 outputs and walks the whole contraction for 16 tokens, operands straight from
// memory into the operand layout (the token rows come out of L2 for every wavefront after the first).
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// D[n0 + 4g + v, tok0 + l16] for v = 0..3: one 16 x 16 tile over the whole contraction (K % 32 == 0).
// Rows past the ends are clamped (their results are never stored).  The operands of kBatch K steps
// are requested together, so a contraction of 512 costs one round trip to memory, not sixteen.
constexpr int kBatch = 16;
__device__ __forceinline__ float4_t linear_tile(const uint16_t* W, int n_out, const uint16_t* x, int n_tok, int K,
                                                int n0, int tok0, int l16, int g) {
  const int n = n0 + l16 < n_out ? n0 + l16 : n_out - 1, t = tok0 + l16 < n_tok ? tok0 + l16 : n_tok - 1;
  const uint16_t* wp = W + (size_t)n * K + 8 * g;
  const uint16_t* xp = x + (size_t)t * K + 8 * g;
  float4_t acc = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < K; k0 += 32 * kBatch) {
    uint4 wf[kBatch], xf[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int k = k0 + 32 * i < K ? k0 + 32 * i : k0;  // past the end: a harmless reload
      wf[i] = *reinterpret_cast<const uint4*>(wp + k);
      xf[i] = *reinterpret_cast<const uint4*>(xp + k);
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i)
      if (k0 + 32 * i < K)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wf[i]), __builtin_bit_cast(bf16x8_t, xf[i]),
                                                      acc, 0, 0, 0);
  }
  return acc;
}

// One wavefront per workgroup, one 16 x 16 output tile per wavefront: the tiles spread over as many
// CUs as there are (a CU streams its 32 KB of operands in well under a microsecond; four tiles per
// CU would queue behind each other).  grid = (tiles, ceil(batch / 16)),
// tiles = (n_h d_h + n_h d_R + d_R + r) / 16 in the order q, q^R, k^R, c.
__global__ __launch_bounds__(kWave) void layer_front_kernel(LayerFrontArgs a) {
  const int lane = threadIdx.x, l16 = lane & 15, g = lane >> 4;
  const int tok0 = 16 * blockIdx.y, tok = tok0 + l16, K = a.d_model;
  const uint16_t* x = reinterpret_cast<const uint16_t*>(a.x);
  const int nq = a.n_heads * a.d_head, nqr = a.n_heads * a.d_rope;
  int n0 = 16 * blockIdx.x;
  if (n0 < nq) {  // ---- q
    const float4_t d = linear_tile(reinterpret_cast<const uint16_t*>(a.w_q), nq, x, a.batch, K, n0, tok0, l16, g);
    if (tok < a.batch) *reinterpret_cast<float4_t*>(a.q + (size_t)tok * nq + n0 + 4 * g) = d;
    return;
  }
  n0 -= nq;
  if (n0 < nqr + a.d_rope) {  // ---- q^R (per head) and k^R (one shared head): rotated at the token's position
    const bool is_key = n0 >= nqr;
    if (is_key) n0 -= nqr;
    const int n_out = is_key ? a.d_rope : nqr;
    const float4_t d = linear_tile(reinterpret_cast<const uint16_t*>(is_key ? a.w_kr : a.w_qr), n_out, x, a.batch, K, n0,
                                   tok0, l16, g);
    if (tok < a.batch) {
      const int pos = a.seq_len[tok];  // 0-based position of the token this step appends
      const int j = (n0 + 4 * g) % a.d_rope;  // element inside the head: pairs (j, j+1), (j+2, j+3)
      float e0 = d[0], e1 = d[1], e2 = d[2], e3 = d[3];
      rope_pair(e0, e1, pos, a.rope_freq[j / 2]);
      rope_pair(e2, e3, pos, a.rope_freq[j / 2 + 1]);
      if (is_key)  // the key goes into the cache: storage type
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.kr) + (size_t)tok * n_out + n0 + 4 * g) =
            make_uint2(pack_bf16x2(e0, e1), pack_bf16x2(e2, e3));
      else
        *reinterpret_cast<float4_t*>(a.q_rope + (size_t)tok * n_out + n0 + 4 * g) = float4_t{e0, e1, e2, e3};
    }
    return;
  }
  // ---- c = x W_r, before its normalisation (which the step's append does, where the whole row meets)
  n0 -= nqr + a.d_rope;
  const float4_t d = linear_tile(reinterpret_cast<const uint16_t*>(a.w_r), a.r, x, a.batch, K, n0, tok0, l16, g);
  if (tok < a.batch) *reinterpret_cast<float4_t*>(a.c + (size_t)tok * a.r + n0 + 4 * g) = d;
}

// y[token, n] = sum_k o[token, k] W_O[n, k]; o is fp32 and enters as bf16 hi + lo planes (two matrix
// instructions per step), so that only the weights' own rounding is left.  One wavefront per
// workgroup; grid = (ceil(d_model / 16), ceil(batch / 16)).
__global__ __launch_bounds__(kWave) void layer_out_kernel(LayerOutArgs a) {
  const int lane = threadIdx.x, l16 = lane & 15, g = lane >> 4;
  const int tok0 = 16 * blockIdx.y, n0 = 16 * blockIdx.x, K = a.k;
  const int n = n0 + l16 < a.d_model ? n0 + l16 : a.d_model - 1;
  const int t = tok0 + l16 < a.batch ? tok0 + l16 : a.batch - 1;
  const uint16_t* wp = reinterpret_cast<const uint16_t*>(a.w_o) + (size_t)n * K + 8 * g;
  const float* op = a.o + (size_t)t * K + 8 * g;
  float4_t acc = {0.f, 0.f, 0.f, 0.f};
  constexpr int kOutBatch = 16;  // K steps requested together (three 16-byte loads per step)
  for (int k0 = 0; k0 < K; k0 += 32 * kOutBatch) {
    uint4 wf[kOutBatch];
    float4 o0[kOutBatch], o1[kOutBatch];
#pragma unroll
    for (int i = 0; i < kOutBatch; ++i) {
      const int k = k0 + 32 * i < K ? k0 + 32 * i : k0;
      wf[i] = *reinterpret_cast<const uint4*>(wp + k);
      o0[i] = *reinterpret_cast<const float4*>(op + k);
      o1[i] = *reinterpret_cast<const float4*>(op + k + 4);
    }
#pragma unroll
    for (int i = 0; i < kOutBatch; ++i)
      if (k0 + 32 * i < K) {
        uint4 hi, lo;
        split_bf16x2(o0[i].x, o0[i].y, hi.x, lo.x);
        split_bf16x2(o0[i].z, o0[i].w, hi.y, lo.y);
        split_bf16x2(o1[i].x, o1[i].y, hi.z, lo.z);
        split_bf16x2(o1[i].z, o1[i].w, hi.w, lo.w);
        const bf16x8_t w8 = __builtin_bit_cast(bf16x8_t, wf[i]);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w8, __builtin_bit_cast(bf16x8_t, hi), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w8, __builtin_bit_cast(bf16x8_t, lo), acc, 0, 0, 0);
      }
  }
  if (tok0 + l16 < a.batch && n0 + 4 * g < a.d_model)  // d_model is a multiple of 4
    *reinterpret_cast<float4_t*>(a.y + (size_t)(tok0 + l16) * a.d_model + n0 + 4 * g) = acc;
}

// ---- the rows of a whole-layer prefill around its matrix products ----------------------------------

// c[row, :] = LayerNorm(raw[row, :]) (* gamma + beta) rounded to bf16; one wavefront per row, r <= 512
__global__ __launch_bounds__(kBlock) void layer_norm_rows_kernel(LayerRowsArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const size_t row = (size_t)blockIdx.x * (kBlock / kWave) + (threadIdx.x >> 6);
  if (row >= a.rows) return;
  const float* src = a.raw + row * a.r;
  float v[8];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int e = lane + kWave * i;
    v[i] = e < a.r ? src[e] : 0.f;
    sum += v[i];
  }
  const float mean = wave_sum(sum) / (float)a.r;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int e = lane + kWave * i;
    const float d = e < a.r ? v[i] - mean : 0.f;
    sq += d * d;
  }
  const float rstd = rsqrtf(wave_sum(sq) / (float)a.r + a.eps);
  const bf16* gamma = reinterpret_cast<const bf16*>(a.gamma);
  const bf16* beta = reinterpret_cast<const bf16*>(a.beta);
  uint16_t* dst = reinterpret_cast<uint16_t*>(a.c) + row * a.r;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int e = lane + kWave * i;
    if (e < a.r) {
      float y = (v[i] - mean) * rstd;
      if (gamma) y *= to_f32(gamma[e]);
      if (beta) y += to_f32(beta[e]);
      dst[e] = f32_to_bf16_bits(y);
      if (a.c32) a.c32[row * a.r + e] = y;
    }
  }
}

// the sequence state a continuing prefill starts from, and W_O as fp16
__global__ __launch_bounds__(kBlock) void layer_prefill_prep_kernel(LayerRowsArgs a) {
  const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
  if (idx < (size_t)a.batch) a.pos0[idx] = a.seq_len[idx];
  if (idx < (size_t)a.batch * a.r) a.tail_prev[idx] = a.tail_c[idx];
  if (idx < a.n_wo) {
    const uint16_t v = reinterpret_cast<const uint16_t*>(a.w_o)[idx];
    reinterpret_cast<uint16_t*>(a.w_o16)[idx] = __builtin_bit_cast(uint16_t, static_cast<_Float16>(__uint_as_float(uint32_t(v) << 16)));
  }
}

}  // namespace

hipError_t launch_layer_norm_rows(const LayerRowsArgs& a, hipStream_t st) {
  const size_t per = kBlock / kWave;
  hipLaunchKernelGGL(layer_norm_rows_kernel, dim3((unsigned)((a.rows + per - 1) / per)), dim3(kBlock), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_layer_prefill_prep(const LayerRowsArgs& a, hipStream_t st) {
  size_t n = a.n_wo > (size_t)a.batch * a.r ? a.n_wo : (size_t)a.batch * a.r;
  hipLaunchKernelGGL(layer_prefill_prep_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, a);
  return hipGetLastError();
}

bool layer_supported(const LayerFrontArgs& a) {
  return a.d_model % 32 == 0 && a.d_model >= 32 && a.d_model <= 16384 && a.d_head % 16 == 0 && a.d_rope % 16 == 0 &&
         a.d_rope <= 64 && a.r % 16 == 0 && a.batch <= 16 * 65535;
}

hipError_t launch_layer_front(const LayerFrontArgs& a, hipStream_t st) {
  const int tiles = (a.n_heads * (a.d_head + a.d_rope) + a.d_rope + a.r) / 16;
  hipLaunchKernelGGL(layer_front_kernel, dim3(tiles, (a.batch + 15) / 16), dim3(kWave), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_layer_out(const LayerOutArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(layer_out_kernel, dim3((a.d_model + 15) / 16, (a.batch + 15) / 16), dim3(kWave), 0, st, a);
  return hipGetLastError();
}

}  // namespace mtla
