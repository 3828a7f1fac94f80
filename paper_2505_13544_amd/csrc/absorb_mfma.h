// Absorbed query on the matrix cores (bf16 storage): the body of one workgroup, shared by the
// stand-alone absorb kernel and the fused front kernel of a decode step.
#pragma once
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

// Rows (tokens) one workgroup walks, 16 per MFMA.  Few rows (a decode step): short walks and many
// workgroups, since a walk is a chain of load -> multiply -> store round trips (256 rows in one
// workgroup took 17 us at batch 256); many rows (prefill): long walks that keep W_K^(h) in registers.
__host__ __device__ constexpr int absorb_rows_per_block(int rows) { return rows >= 4096 ? 256 : 32; }

// ---------------------------------------------------------------------------
// absorb, bf16 on the matrix cores.  Block coordinates (bx, h, bz) span (r/64 + 1, n_heads, row groups).
// Workgroups x < r/64: wavefront w owns output columns n0 = (4x + w) * 16 of
// head h and walks the rows 16 at a time: D[n, row] = sum_k W[n, k] q[row, k].
// Workgroup x == r/64 copies (and scales) the RoPE query part.  The operand row is written
// as two bf16 planes, hi and lo (a.plane elements apart): the logits are then formed from an
// almost-fp32 query at the price of a second MFMA per K step, which removes the largest
// avoidable error of the bf16 path (rounding the absorbed query) for sequences of few slots.
// ---------------------------------------------------------------------------
// QF32 (= a.q_f32, fixed at compile time so that the registers of the other form do not count against the
// kernel's occupancy: with both forms compiled in, d_head = 128 took 160 registers and a decode step at
// batch 256 ran its 1408 workgroups in almost three rounds).
template <int KK, bool QF32>  // d_head / 32
__device__ __forceinline__ void absorb_mfma_block(const AbsorbArgs& a, int bx, int h, int bz) {
  typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
  typedef float float4_t __attribute__((ext_vector_type(4)));
  constexpr int kWaves = kBlock / kWave;
  constexpr int DH = 32 * KK;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int r = a.r, dR = a.d_rope, E = r + dR;
  const int per_block = absorb_rows_per_block(a.rows);
  const int row_lo = bz * per_block;
  const int row_hi = row_lo + per_block < a.rows ? row_lo + per_block : a.rows;
  uint16_t* qcat = reinterpret_cast<uint16_t*>(a.qcat);

  if (bx == r / 64) {  // RoPE part: qcat[row, h, r + j] = scale * q_rope[row, h, j]
    const uint16_t* qr = reinterpret_cast<const uint16_t*>(a.q_rope);
    const int per_row = dR / 8;
    for (int idx = tid; idx < (row_hi - row_lo) * per_row; idx += kBlock) {
      const int row = row_lo + idx / per_row, j8 = idx % per_row;
      float v[8];
      if (QF32) load8(reinterpret_cast<const float*>(a.q_rope) + ((size_t)row * a.n_heads + h) * dR + 8 * j8, v);
      else load8(reinterpret_cast<const bf16*>(qr) + ((size_t)row * a.n_heads + h) * dR + 8 * j8, v);
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) split_bf16x2(v[2 * i] * a.scale_log2, v[2 * i + 1] * a.scale_log2, hi[i], lo[i]);
      uint16_t* dst = qcat + ((size_t)row * a.n_heads + h) * E + r + 8 * j8;
      *reinterpret_cast<uint4*>(dst) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
      *reinterpret_cast<uint4*>(dst + a.plane) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
    return;
  }

  const int n0 = (bx * kWaves + wv) * 16;
  const uint16_t* w = reinterpret_cast<const uint16_t*>(a.w_uk) + ((size_t)h * r + n0 + l16) * DH + 8 * g;
  const uint16_t* q = reinterpret_cast<const uint16_t*>(a.q);
  uint4 wa[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) wa[kk] = *reinterpret_cast<const uint4*>(w + 32 * kk);
  // two 16-row tiles per pass, their operands requested together
  for (int row0 = row_lo; row0 < row_hi; row0 += 32) {
    int rowt[2];
    bool validt[2];
    uint4 qb[QF32 ? 1 : 2][QF32 ? 1 : KK];
    float qv[QF32 ? 2 : 1][QF32 ? KK : 1][8];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      rowt[t] = row0 + 16 * t + l16;
      validt[t] = rowt[t] < row_hi;
      if constexpr (QF32) {  // unrounded queries
        const float* qf = reinterpret_cast<const float*>(a.q) + ((size_t)(validt[t] ? rowt[t] : row_lo) * a.n_heads + h) * DH + 8 * g;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) load8(qf + 32 * kk, qv[t][kk]);
      } else {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
          qb[t][kk] = validt[t] ? *reinterpret_cast<const uint4*>(q + ((size_t)rowt[t] * a.n_heads + h) * DH + 32 * kk + 8 * g)
                                : make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      if (row0 + 16 * t >= row_hi) break;  // wavefront-uniform
      float4_t acc = {0.f, 0.f, 0.f, 0.f};
      if constexpr (QF32) {  // hi + lo planes, two matrix instructions per K step
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const float (&v)[8] = qv[t][kk];
          uint4 hi, lo;
          split_bf16x2(v[0], v[1], hi.x, lo.x);
          split_bf16x2(v[2], v[3], hi.y, lo.y);
          split_bf16x2(v[4], v[5], hi.z, lo.z);
          split_bf16x2(v[6], v[7], hi.w, lo.w);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wa[kk]), __builtin_bit_cast(bf16x8_t, hi),
                                                        acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wa[kk]), __builtin_bit_cast(bf16x8_t, lo),
                                                        acc, 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wa[kk]),
                                                        __builtin_bit_cast(bf16x8_t, qb[t][kk]), acc, 0, 0, 0);
      }
      if (validt[t]) {  // lane holds columns n0 + 4g .. + 3 of its row
        uint32_t hi0, lo0, hi1, lo1;
        split_bf16x2(acc[0] * a.scale_log2, acc[1] * a.scale_log2, hi0, lo0);
        split_bf16x2(acc[2] * a.scale_log2, acc[3] * a.scale_log2, hi1, lo1);
        uint16_t* dst = qcat + ((size_t)rowt[t] * a.n_heads + h) * E + n0 + 4 * g;
        *reinterpret_cast<uint2*>(dst) = make_uint2(hi0, hi1);
        *reinterpret_cast<uint2*>(dst + a.plane) = make_uint2(lo0, lo1);
      }
    }
  }
}

}  // namespace mtla
