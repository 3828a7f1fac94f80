// The layer around the decode path, for one new token per sequence (bf16 storage, gfx950):
//   layer_front_kernel   x -> q = x W_Q (Eq. (query)), q^R = RoPE(x W_QR), c = LayerNorm(x W_r)
//                        (Eq. (low-rank) and the normalisation applied to it), k^R = RoPE(x W_KR);
//                        q, q^R and c leave in fp32 (they are rounded where they are used), k^R in bf16
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
// Rows past the ends are clamped (their results are never stored).
__device__ __forceinline__ float4_t linear_tile(const uint16_t* W, int n_out, const uint16_t* x, int n_tok, int K,
                                                int n0, int tok0, int l16, int g) {
  const int n = n0 + l16 < n_out ? n0 + l16 : n_out - 1, t = tok0 + l16 < n_tok ? tok0 + l16 : n_tok - 1;
  const uint16_t* wp = W + (size_t)n * K + 8 * g;
  const uint16_t* xp = x + (size_t)t * K + 8 * g;
  float4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int k = 0; k < K; k += 32)
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(wp + k)),
                                                  __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(xp + k)),
                                                  acc, 0, 0, 0);
  return acc;
}

// The pair (a, b) = elements (2k, 2k+1) of a d-wide vector, turned by pos * base^(-2k/d).  The angle is
// formed in double: positions reach tens of thousands of radians.
__device__ __forceinline__ void rope_pair(float& a, float& b, int pos, int k, int d, float log2_base) {
  const double ang = (double)pos * exp2(-2.0 * k / d * (double)log2_base);
  const float cs = (float)cos(ang), sn = (float)sin(ang);
  const float ra = a * cs - b * sn, rb = a * sn + b * cs;
  a = ra;
  b = rb;
}

// grid = (jobs, ceil(batch / 16)); jobs = n_h d_h / 64 (q) + n_h d_R / 64 (q^R) + 1 (k^R) + 1 (c).
__global__ __launch_bounds__(kBlock) void layer_front_kernel(LayerFrontArgs a) {
  extern __shared__ float sC[];  // c job only: [16 tokens][r + 4]
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int tok0 = 16 * blockIdx.y, tok = tok0 + l16, K = a.d_model;
  const uint16_t* x = reinterpret_cast<const uint16_t*>(a.x);
  const int nq = a.n_heads * a.d_head, nqr = a.n_heads * a.d_rope;
  const int jobs_q = nq / 64, jobs_qr = nqr / 64;
  int job = blockIdx.x;
  if (job < jobs_q) {  // ---- q
    const int n0 = 64 * job + 16 * wv;
    const float4_t d = linear_tile(reinterpret_cast<const uint16_t*>(a.w_q), nq, x, a.batch, K, n0, tok0, l16, g);
    if (tok < a.batch) *reinterpret_cast<float4_t*>(a.q + (size_t)tok * nq + n0 + 4 * g) = d;
    return;
  }
  job -= jobs_q;
  if (job < jobs_qr + 1) {  // ---- q^R (per head) and k^R (one shared head): rotated at the token's position
    const bool is_key = job == jobs_qr;
    const int n_out = is_key ? a.d_rope : nqr, n0 = (is_key ? 0 : 64 * job) + 16 * wv;
    if (n0 >= n_out) return;
    const float4_t d = linear_tile(reinterpret_cast<const uint16_t*>(is_key ? a.w_kr : a.w_qr), n_out, x, a.batch, K, n0, tok0,
                             l16, g);
    if (tok < a.batch) {
      const int pos = a.seq_len[tok];  // 0-based position of the token this step appends
      const int j = (n0 + 4 * g) % a.d_rope;  // element inside the head: pairs (j, j+1), (j+2, j+3)
      float e0 = d[0], e1 = d[1], e2 = d[2], e3 = d[3];
      rope_pair(e0, e1, pos, j / 2, a.d_rope, a.log2_rope_base);
      rope_pair(e2, e3, pos, j / 2 + 1, a.d_rope, a.log2_rope_base);
      if (is_key)  // the key goes into the cache: storage type
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.kr) + (size_t)tok * n_out + n0 + 4 * g) =
            make_uint2(pack_bf16x2(e0, e1), pack_bf16x2(e2, e3));
      else
        *reinterpret_cast<float4_t*>(a.q_rope + (size_t)tok * n_out + n0 + 4 * g) = float4_t{e0, e1, e2, e3};
    }
    return;
  }
  // ---- c: all r outputs of 16 tokens in one workgroup, then the normalisation over r
  const int r = a.r, CS = r + 4;
  for (int n0 = 16 * wv; n0 < r; n0 += 64) {
    const float4_t d = linear_tile(reinterpret_cast<const uint16_t*>(a.w_r), r, x, a.batch, K, n0, tok0, l16, g);
    *reinterpret_cast<float4_t*>(&sC[l16 * CS + n0 + 4 * g]) = d;
  }
  __syncthreads();
  {
    const int t = tid >> 4, q = tid & 15;  // 16 threads per token
    const float* row = sC + t * CS;
    float sum = 0.f;
    for (int e = q; e < r; e += 16) sum += row[e];
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) sum += __shfl_xor(sum, off, kWave);
    const float mean = sum / r;
    float sq = 0.f;
    for (int e = q; e < r; e += 16) sq += (row[e] - mean) * (row[e] - mean);
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) sq += __shfl_xor(sq, off, kWave);
    const float inv = 1.0f / sqrtf(sq / r + a.ln_eps);
    if (tok0 + t < a.batch) {
      float* dst = a.c + (size_t)(tok0 + t) * r;
      const bf16* gm = reinterpret_cast<const bf16*>(a.ln_gamma);
      const bf16* bt = reinterpret_cast<const bf16*>(a.ln_beta);
      for (int e = q; e < r; e += 16) {
        float y = (row[e] - mean) * inv;
        if (gm) y *= to_f32(gm[e]);
        if (bt) y += to_f32(bt[e]);
        dst[e] = y;
      }
    }
  }
}

// y[token, n] = sum_k o[token, k] W_O[n, k]; o is fp32 and enters as bf16 hi + lo planes (two matrix
// instructions per step), so that only the weights' own rounding is left.  grid = (d_model / 64, ceil(batch / 16)).
__global__ __launch_bounds__(kBlock) void layer_out_kernel(LayerOutArgs a) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int tok0 = 16 * blockIdx.y, n0 = 64 * blockIdx.x + 16 * wv, K = a.k;
  if (n0 >= a.d_model) return;
  const int n = n0 + l16 < a.d_model ? n0 + l16 : a.d_model - 1;
  const int t = tok0 + l16 < a.batch ? tok0 + l16 : a.batch - 1;
  const uint16_t* wp = reinterpret_cast<const uint16_t*>(a.w_o) + (size_t)n * K + 8 * g;
  const float* op = a.o + (size_t)t * K + 8 * g;
  float4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
  for (int k = 0; k < K; k += 32) {
    const float4 o0 = *reinterpret_cast<const float4*>(op + k), o1 = *reinterpret_cast<const float4*>(op + k + 4);
    uint4 hi, lo;
    split_bf16x2(o0.x, o0.y, hi.x, lo.x);
    split_bf16x2(o0.z, o0.w, hi.y, lo.y);
    split_bf16x2(o1.x, o1.y, hi.z, lo.z);
    split_bf16x2(o1.z, o1.w, hi.w, lo.w);
    const bf16x8_t wf = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(wp + k));
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, __builtin_bit_cast(bf16x8_t, hi), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, __builtin_bit_cast(bf16x8_t, lo), acc, 0, 0, 0);
  }
  if (tok0 + l16 < a.batch && n0 + 4 * g < a.d_model)  // d_model is a multiple of 4
    *reinterpret_cast<float4_t*>(a.y + (size_t)(tok0 + l16) * a.d_model + n0 + 4 * g) = acc;
}

}  // namespace

bool layer_supported(const LayerFrontArgs& a) {
  return a.d_model % 32 == 0 && a.d_model >= 32 && a.d_model <= 16384 && (a.n_heads * a.d_head) % 64 == 0 &&
         (a.n_heads * a.d_rope) % 64 == 0 && a.d_rope % 16 == 0 && a.r % 64 == 0 && a.batch <= 16 * 65535;
}

hipError_t launch_layer_front(const LayerFrontArgs& a, hipStream_t st) {
  const int jobs = a.n_heads * a.d_head / 64 + a.n_heads * a.d_rope / 64 + 2;
  const dim3 grid(jobs, (a.batch + 15) / 16);
  const size_t smem = (size_t)16 * (a.r + 4) * sizeof(float);
  hipLaunchKernelGGL(layer_front_kernel, grid, dim3(kBlock), smem, st, a);
  return hipGetLastError();
}

hipError_t launch_layer_out(const LayerOutArgs& a, hipStream_t st) {
  const dim3 grid((a.d_model + 63) / 64, (a.batch + 15) / 16);
  hipLaunchKernelGGL(layer_out_kernel, grid, dim3(kBlock), 0, st, a);
  return hipGetLastError();
}

}  // namespace mtla
