// The two small projections either side of the pass over the cache.
//
//   absorb   q~_h = W_K^(h) q_h for every (row, head), written next to the RoPE
//            query as one operand row [q~ | q^R], pre-scaled by
//            softmax_scale * log2(e)                                   (Eq. (obsorb))
//   combine  log-sum-exp merge of the chunk partials of one (row, head), then
//            o = o~ W_V^(h)                                            (Eq. (obsorb), W_V side)
//
// Both weights are stored with the contracted index innermost
// (w_uk [n_h, r, d_h], w_uv [n_h, d_h, r]), so a lane fetches 8 consecutive
// contraction elements with one 16-byte load, which is also the MFMA operand
// layout.  Every kernel issues all of its global loads before the first use:
// at decode batch sizes these kernels are pure latency.
#include "absorb_mfma.h"
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kWaves = kBlock / kWave;



// absorb, bf16 on the matrix cores: grid = (r/64 + 1, n_heads, row groups), body in absorb_mfma.h
template <int KK, bool QF32>
__global__ __launch_bounds__(kBlock) void absorb_mfma_kernel(AbsorbArgs a) {
  absorb_mfma_block<KK, QF32>(a, blockIdx.x, blockIdx.y, blockIdx.z);
}

// absorb, vector ALU, fp32 result (MTLA_F32 storage, or bf16 storage feeding the
// fp32 vector attention kernel).  grid = (ceil(E/256), n_heads, ceil(rows/8)).
constexpr int kAbsorbRows = 8;
template <typename T>
__global__ __launch_bounds__(kBlock) void absorb_valu_kernel(AbsorbArgs a) {
  extern __shared__ float sq[];  // [kAbsorbRows][d_head]
  const int tid = threadIdx.x, n = blockIdx.x * kBlock + tid, h = blockIdx.y;
  const int row0 = blockIdx.z * kAbsorbRows;
  const int dh = a.d_head, r = a.r, dR = a.d_rope, E = r + dR;
  const T* q = reinterpret_cast<const T*>(a.q);
  const T* qr = reinterpret_cast<const T*>(a.q_rope);
  float* qcat = reinterpret_cast<float*>(a.qcat);
  for (int idx = tid; idx < kAbsorbRows * dh; idx += kBlock) {
    const int rr = idx / dh, k = idx - rr * dh, row = row0 + rr;
    sq[idx] = row < a.rows ? to_f32(q[((size_t)row * a.n_heads + h) * dh + k]) : 0.f;
  }
  __syncthreads();
  if (n < r) {
    float acc[kAbsorbRows];
#pragma unroll
    for (int rr = 0; rr < kAbsorbRows; ++rr) acc[rr] = 0.f;
    const T* wrow = reinterpret_cast<const T*>(a.w_uk) + ((size_t)h * r + n) * dh;
    for (int k8 = 0; k8 < dh; k8 += 8) {
      float wv[8];
      load8(wrow + k8, wv);
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int rr = 0; rr < kAbsorbRows; ++rr) acc[rr] += sq[rr * dh + k8 + j] * wv[j];
    }
#pragma unroll
    for (int rr = 0; rr < kAbsorbRows; ++rr) {
      const int row = row0 + rr;
      if (row < a.rows) qcat[((size_t)row * a.n_heads + h) * E + n] = acc[rr] * a.scale_log2;
    }
  } else if (n < E) {
#pragma unroll
    for (int rr = 0; rr < kAbsorbRows; ++rr) {
      const int row = row0 + rr;
      if (row < a.rows)
        qcat[((size_t)row * a.n_heads + h) * E + n] =
            to_f32(qr[((size_t)row * a.n_heads + h) * dR + (n - r)]) * a.scale_log2;
    }
  }
}

// ---------------------------------------------------------------------------
// combine + value up-projection.  grid = (n_heads, rows).
//
// NCH > 0: the thread's NCH 8-element pieces of its W_V row are requested at the top of the
// kernel, together with the sequence length and (INLINE: at most kInlineSplits chunks per
// row) every partial the thread will need, so the whole kernel is one round trip to memory.
// NCH == 0 / !INLINE are the general forms for shapes or split counts that do not fit.
// ---------------------------------------------------------------------------
constexpr int kInlineSplits = 16;
constexpr int kSplitBatch = 8;  // partial loads kept in flight per thread (general form)
constexpr int kCols = 2;        // r <= 512: at most two latent columns per thread

template <typename T>
struct Chunk8;
template <>
struct Chunk8<bf16> {
  uint4 raw;
  __device__ __forceinline__ void load(const bf16* p) { raw = *reinterpret_cast<const uint4*>(p); }
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
  __device__ __forceinline__ void unpack(float (&o)[8]) const {
    o[0] = lo.x; o[1] = lo.y; o[2] = lo.z; o[3] = lo.w;
    o[4] = hi.x; o[5] = hi.y; o[6] = hi.z; o[7] = hi.w;
  }
};

__host__ __device__ inline int lanes_per_out_col(int dh) {  // power of two, kBlock / dh rounded down
  const int t = kBlock / dh;
  return t >= 8 ? 8 : (t >= 4 ? 4 : (t >= 2 ? 2 : 1));
}

template <typename T, int NCH, bool INLINE>
__global__ __launch_bounds__(kBlock) void combine_kernel(CombineArgs a) {
  extern __shared__ float smem[];
  float* s_lat = smem;              // [r]
  float* s_red = smem + a.r;        // [2 * kWaves]
  float* s_f = s_red + 2 * kWaves;  // [pieces of this row] per-piece weights (general form)
  const int h = blockIdx.x, row = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wv = tid >> 6;
  const int r = a.r, dh = a.d_head;
  const size_t oh = (size_t)row * a.n_heads + h;

  // ---- requests that need nothing but the block index
  int len = 0x7fffffff, bseq = row, mrow = 0;
  if (a.T != 0) {
    bseq = row / a.T;
    mrow = row - bseq * a.T;
  }
  if (a.n_persistent == 0 && (a.T == 0 || a.seq_len)) len = a.seq_len[bseq];
  const int tpd = lanes_per_out_col(dh);
  const int d = tid / tpd, qd = tid - d * tpd;
  const T* wrow = reinterpret_cast<const T*>(a.w_uv) + ((size_t)h * dh + (d < dh ? d : 0)) * r;
  Chunk8<T> wreg[NCH > 0 ? NCH : 1];
  if (NCH > 0 && a.out) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) wreg[i].load(wrow + 8 * (qd + i * tpd));
  }

  // ---- which partials belong to this row
  int piece0, nsp, n_avail;  // first piece id, pieces of this row, pieces that are safe to read
  bool empty;
  if (a.n_persistent > 0) {  // balanced schedule: workgroup i emitted piece i + row for its share
    const int p0 = a.tile_prefix[row], p1 = a.tile_prefix[row + 1], total = a.tile_prefix[a.batch];
    const int share = (total + a.n_persistent - 1) / a.n_persistent;
    empty = p1 == p0;
    const int first = empty ? 0 : (p0 + a.run_cost) / share, last = empty ? 0 : (p1 - 1) / share;
    piece0 = first + row;
    nsp = n_avail = last - first + 1;
  } else {                   // static schedule: chunk c of row b is piece b * n_splits + c
    piece0 = row * a.n_splits;
    n_avail = a.n_splits;
    const int live = a.T == 0 ? (len + a.stride - 1) / a.stride : (mrow < len ? mrow / a.stride + 1 : 0);
    empty = live == 0;
    nsp = (live + a.chunk - 1) / a.chunk;
  }
  const size_t pb = (size_t)piece0 * a.n_heads + h;  // + sp * n_heads

  float2 ml[INLINE ? kInlineSplits : 1];
  float pv[kCols][INLINE ? kInlineSplits : 1];
  if (INLINE) {  // requested before the static schedule has even looked at the length
#pragma unroll
    for (int sp = 0; sp < kInlineSplits; ++sp) {
      if (sp < n_avail) {
        ml[sp] = *reinterpret_cast<const float2*>(a.part_ml + (pb + (size_t)sp * a.n_heads) * 2);
#pragma unroll
        for (int c = 0; c < kCols; ++c) {
          const int n = tid + c * kBlock;
          if (n < r) pv[c][sp] = a.part_o[(pb + (size_t)sp * a.n_heads) * r + n];
        }
      }
    }
  }

  if (empty) {
    if (a.out_latent)
      for (int n = tid; n < r; n += kBlock) a.out_latent[oh * r + n] = 0.f;
    if (a.out)
      for (int dd = tid; dd < dh; dd += kBlock) a.out[oh * dh + dd] = 0.f;
    if (a.lse && tid == 0) a.lse[oh] = -INFINITY;
    return;
  }

  float mstar, lstar;
  if (INLINE && nsp <= kInlineSplits) {
    // ---- every thread folds the (m, l) pairs itself: no exchange, no barrier
    mstar = -INFINITY;
#pragma unroll
    for (int sp = 0; sp < kInlineSplits; ++sp)
      if (sp < nsp) mstar = fmaxf(mstar, ml[sp].x);
    lstar = 0.f;
    float o[kCols] = {0.f, 0.f};
#pragma unroll
    for (int sp = 0; sp < kInlineSplits; ++sp) {
      if (sp < nsp) {
        const float f = __builtin_amdgcn_exp2f(ml[sp].x - mstar);
        lstar += f * ml[sp].y;
#pragma unroll
        for (int c = 0; c < kCols; ++c) o[c] += f * pv[c][sp];
      }
    }
    const float inv = 1.f / lstar;
#pragma unroll
    for (int c = 0; c < kCols; ++c) {
      const int n = tid + c * kBlock;
      if (n < r) {
        s_lat[n] = o[c] * inv;
        if (a.out_latent) a.out_latent[oh * r + n] = o[c] * inv;
      }
    }
  } else {
    // ---- m* = max_s m_s, l* = sum_s l_s 2^(m_s - m*), reduced over the workgroup
    float mloc = -INFINITY;
    for (int sp = tid; sp < nsp; sp += kBlock) mloc = fmaxf(mloc, a.part_ml[(pb + (size_t)sp * a.n_heads) * 2]);
    mloc = wave_max(mloc);
    if (lane == 0) s_red[wv] = mloc;
    __syncthreads();
    mstar = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    float lloc = 0.f;
    for (int sp = tid; sp < nsp; sp += kBlock) {
      const float f = exp2f(a.part_ml[(pb + (size_t)sp * a.n_heads) * 2] - mstar);
      s_f[sp] = f;
      lloc += f * a.part_ml[(pb + (size_t)sp * a.n_heads) * 2 + 1];
    }
    lloc = wave_sum(lloc);
    if (lane == 0) s_red[kWaves + wv] = lloc;
    __syncthreads();
    lstar = (s_red[kWaves] + s_red[kWaves + 1]) + (s_red[kWaves + 2] + s_red[kWaves + 3]);
    const float inv = 1.f / lstar;
    for (int n = tid; n < r; n += kBlock) {
      float o = 0.f;
      for (int s0 = 0; s0 < nsp; s0 += kSplitBatch) {
        float v[kSplitBatch];
#pragma unroll
        for (int j = 0; j < kSplitBatch; ++j)
          v[j] = (s0 + j < nsp) ? a.part_o[(pb + (size_t)(s0 + j) * a.n_heads) * r + n] : 0.f;
#pragma unroll
        for (int j = 0; j < kSplitBatch; ++j)
          if (s0 + j < nsp) o += s_f[s0 + j] * v[j];
      }
      o *= inv;
      s_lat[n] = o;
      if (a.out_latent) a.out_latent[oh * r + n] = o;
    }
  }
  if (a.lse && tid == 0) a.lse[oh] = (mstar + log2f(lstar)) * 0.6931471805599453f;
  if (!a.out) return;
  __syncthreads();

  // ---- o[d] = sum_n o~[n] W_V^(h)[n, d]; w_uv is [h][d][n].  tpd lanes share one d and take
  // 8-element pieces of n round-robin, so their LDS and global reads stay contiguous.
  float part = 0.f;
  if (d < dh) {
    if (NCH > 0) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        float wv8[8];
        wreg[i].unpack(wv8);
        const int c8 = qd + i * tpd;
#pragma unroll
        for (int j = 0; j < 8; ++j) part += s_lat[8 * c8 + j] * wv8[j];
      }
    } else {
      for (int c8 = qd; c8 < r / 8; c8 += tpd) {
        float wv8[8];
        load8(wrow + 8 * c8, wv8);
#pragma unroll
        for (int j = 0; j < 8; ++j) part += s_lat[8 * c8 + j] * wv8[j];
      }
    }
  }
  for (int off = 1; off < tpd; off <<= 1) part += __shfl_xor(part, off, kWave);
  if (d < dh && qd == 0) a.out[oh * dh + d] = part;
}

template <typename T, bool INLINE>
void launch_combine_t(const CombineArgs& a, const dim3& grid, size_t smem, hipStream_t st) {
  const int tpd = lanes_per_out_col(a.d_head);
  const int nch = ((a.r / 8) % tpd == 0) ? (a.r / 8) / tpd : 0;
  const int max_nch = sizeof(T) == 2 ? 32 : 8;  // registers: 4 (bf16) or 8 (fp32) per piece
#define MTLA_NCH(N)                                                                              \
  if (nch == N && N <= max_nch) {                                                                \
    hipLaunchKernelGGL((combine_kernel<T, N, INLINE>), grid, dim3(kBlock), smem, st, a);         \
    return;                                                                                      \
  }
  MTLA_NCH(1) MTLA_NCH(2) MTLA_NCH(4) MTLA_NCH(8) MTLA_NCH(16) MTLA_NCH(32)
#undef MTLA_NCH
  hipLaunchKernelGGL((combine_kernel<T, 0, INLINE>), grid, dim3(kBlock), smem, st, a);
}

template <int KK>
void launch_absorb_mfma_kk(const AbsorbArgs& a, hipStream_t st) {
  const dim3 grid(a.r / 64 + 1, a.n_heads, (a.rows + absorb_rows_per_block(a.rows) - 1) / absorb_rows_per_block(a.rows));
  if (a.q_f32) hipLaunchKernelGGL((absorb_mfma_kernel<KK, true>), grid, dim3(kBlock), 0, st, a);
  else hipLaunchKernelGGL((absorb_mfma_kernel<KK, false>), grid, dim3(kBlock), 0, st, a);
}

}  // namespace

hipError_t launch_absorb(const AbsorbArgs& a, int dtype, hipStream_t st) {
  if (a.out_bf16) {  // bf16 storage, matrix-core operand
    switch (a.d_head / 32) {
      case 1: launch_absorb_mfma_kk<1>(a, st); break;
      case 2: launch_absorb_mfma_kk<2>(a, st); break;
      case 3: launch_absorb_mfma_kk<3>(a, st); break;
      case 4: launch_absorb_mfma_kk<4>(a, st); break;
      case 5: launch_absorb_mfma_kk<5>(a, st); break;
      case 6: launch_absorb_mfma_kk<6>(a, st); break;
      case 7: launch_absorb_mfma_kk<7>(a, st); break;
      case 8: launch_absorb_mfma_kk<8>(a, st); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  const int E = a.r + a.d_rope;
  const dim3 grid((E + kBlock - 1) / kBlock, a.n_heads, (a.rows + kAbsorbRows - 1) / kAbsorbRows);
  const size_t smem = (size_t)kAbsorbRows * a.d_head * sizeof(float);
  if (dtype == 0)
    hipLaunchKernelGGL(absorb_valu_kernel<float>, grid, dim3(kBlock), smem, st, a);
  else
    hipLaunchKernelGGL(absorb_valu_kernel<bf16>, grid, dim3(kBlock), smem, st, a);
  return hipGetLastError();
}

hipError_t launch_combine(const CombineArgs& a, int dtype, hipStream_t st) {
  if (dtype != 0 && combine_mfma_supported(a)) return launch_combine_mfma(a, st);
  const int rows = a.T ? a.batch * a.T : a.batch;
  const dim3 grid(a.n_heads, rows);
  // a row's pieces: at most n_splits (static) or one per persistent workgroup (balanced)
  const int max_pieces = a.n_persistent > 0 ? a.n_persistent : a.n_splits;
  const size_t smem = (size_t)(a.r + 2 * kWaves + max_pieces) * sizeof(float);
  const bool inl = (a.n_persistent > 0 || a.n_splits <= kInlineSplits) && a.r <= kCols * kBlock;
  if (dtype == 0) {
    if (inl) launch_combine_t<float, true>(a, grid, smem, st);
    else launch_combine_t<float, false>(a, grid, smem, st);
  } else {
    if (inl) launch_combine_t<bf16, true>(a, grid, smem, st);
    else launch_combine_t<bf16, false>(a, grid, smem, st);
  }
  return hipGetLastError();
}

}  // namespace mtla
