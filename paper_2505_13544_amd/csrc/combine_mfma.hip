// Split combine + value up-projection on the matrix cores (bf16 storage, gfx950).
//
// Eq. (with-rope), last two steps: the partial (m, l, o~) triples of a row are merged with
// weights 2^(m_p - m*), divided by the merged normaliser, and every head's latent output is
// taken through its own W_V^(h):  out[row, h, :] = o~[row, h, :] W_V^(h).
// Heads do not share W_V^(h), rows do, so the up-projection is a dense contraction once 16 rows
// of one head are put side by side:
//     out^T[d, row] = W_V^(h)[d, :] . o~[row, :]^T          (M = d_h, N = 16 rows, K = r)
// A workgroup owns one head and a run of 16-row tiles.  Its W_V^(h) sits in registers for the
// whole run, already in the A-operand layout of v_mfma_f32_16x16x32_bf16 (each wavefront a
// quarter of the d_h output rows).  Per tile, 16 threads per row merge the row's partials (all
// requests of up to PB pieces go out together, before the normaliser is known), write the
// normalised latent row where the caller wants it, and park it in LDS as two bf16 planes
// (hi + lo, an almost-fp32 value) that the four wavefronts read back as the B operand.
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kTileRows = 16;
constexpr int kWaves = kBlock / kWave;

struct Pieces {
  int first, count;
};

// Balanced schedule: workgroup i emitted piece i + row for its share of the row, whose work units are
// [p0, p1) of `total`.
__device__ __forceinline__ Pieces pieces_balanced(const CombineArgs& a, int row, int rows, int p0, int p1, int total) {
  Pieces p{0, 0};
  if (row >= rows || p1 == p0) return p;
  const int share = (total + a.n_persistent - 1) / a.n_persistent;
  const int first = (p0 + a.run_cost) / share, last = (p1 - 1) / share;  // the row's tiles follow its fixed units
  p.first = first + row;
  p.count = last - first + 1;
  return p;
}

// Which partials belong to `row` (see the two attention schedules): none for a row without a
// live column.
__device__ __forceinline__ Pieces pieces_of_row(const CombineArgs& a, int row, int rows, int total) {
  Pieces p{0, 0};
  if (a.n_persistent > 0) {  // balanced: workgroup i emitted piece i + row for its share of the row
    // the row's two counts are requested together, before anything is decided; `total` (the last entry
    // of the list) was read once when the kernel started: one round trip per row, not three
    const int rc = row < rows ? row : rows - 1;
    const int p0 = a.tile_prefix[rc], p1 = a.tile_prefix[rc + 1];
    return pieces_balanced(a, row, rows, p0, p1, total);
  } else {
    if (row >= rows) return p;  // static: chunk c of row b is piece b * n_splits + c
    int live;
    if (a.T == 0) {
      live = (a.seq_len[row] + a.stride - 1) / a.stride;
    } else {
      const int b = row / a.T, m = row - b * a.T;
      const int len = a.seq_len ? a.seq_len[b] : a.T;
      live = m < len ? m / a.stride + 1 : 0;
    }
    p.first = row * a.n_splits;
    p.count = (live + a.chunk - 1) / a.chunk;
  }
  return p;
}

template <int N>  // over aligned groups of N lanes, N a power of two up to the wavefront
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int off = 1; off < N; off <<= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}
template <int N>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int off = 1; off < N; off <<= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// grid = (runs of row tiles, n_heads)
// RPT = rows a workgroup really fills of each 16-row tile.  16 is the dense case; 4 is for small
// batches (decode), where the merge of the partials is the long part and wants more workgroups:
// a row is then merged by a whole wavefront and three quarters of the tile's columns stay zero.
// WKEEP = W_V^(h) is fetched once and kept in registers for the whole run of tiles; otherwise it
// is fetched after the merge, when the registers of the partials are free again (single tile).
// PF16 = the partials are normalised IEEE-half rows (o_p / l_p) from the column-split decode kernel:
// a piece then weighs l_p 2^(m_p - m*) instead of 2^(m_p - m*).
// PS = a few rows of very many pieces (a handful of long sequences under the balanced schedule): one row
// per workgroup (RPT = 1), the row's pieces dealt to the four wavefronts in contiguous quarters, their
// weighted sums added through LDS.  One round of requests instead of one per PB pieces, and four times
// the workgroups.
// HF = the head is the fast grid index: the workgroups that share an XCD (and its L2) then share the
// W_V^(h) of a few heads instead of each XCD fetching all of them.
template <int R, int DH, int RPT, bool WKEEP, bool PF16, bool PS = false, bool HF = PS>
__global__ __launch_bounds__(kBlock) void combine_mfma_kernel(CombineArgs a, int tiles_per_wg) {
  static_assert(!PS || (RPT == 1 && PF16), "piece split: one row per workgroup, half partials");
  constexpr int KK = R / 32;         // K steps
  constexpr int NT = DH / 64;        // 16-row output tiles per wavefront (a quarter of d_h)
  constexpr int TPR = PS ? kWave : kBlock / RPT;  // threads merging one row (piece split: per wavefront)
  constexpr int CJ = R / (4 * TPR);  // float4 pieces of a latent row per thread
  static_assert(CJ >= 1, "a thread merges at least one float4 of its row");
  constexpr int AS = R + 8;          // LDS row stride (bf16 elements)
  // partials requested together per thread: as many as the registers allow (packed halves are cheap)
  // (small batches, four rows per workgroup: 16, so that a row of up to 16 pieces is one round of requests; the
  // headline shape has 9 or 10 pieces per row once it has decoded past 1024 tokens)
  constexpr int PB = PS ? 12 : (WKEEP && R >= 512) ? (HF && PF16 ? 4 : 2) : ((RPT < kTileRows && (PF16 || R <= 256)) ? 16 : 8);
  __shared__ __attribute__((aligned(16))) uint16_t sA[2][kTileRows][AS];  // hi and lo planes
  __shared__ __attribute__((aligned(16))) float sRed[PS ? kWaves - 1 : 1][PS ? R : 4];  // piece split: the other wavefronts' sums

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int h = HF ? blockIdx.x : blockIdx.y;
  const int rows = a.T ? a.batch * a.T : a.batch;
  const int n_tiles = (rows + RPT - 1) / RPT;
  const int t0 = (HF ? blockIdx.y : blockIdx.x) * tiles_per_wg;
  const int t1 = t0 + tiles_per_wg < n_tiles ? t0 + tiles_per_wg : n_tiles;

  // balanced schedule, first tile: a row's counts and the list's total go out together and before the
  // weights (loads return in order, and one count asked for after the other would be a round trip each)
  const int tid0 = threadIdx.x;
  int ps_p0 = 0, ps_p1 = 0, ps_total = 0;
  if (PS || (HF && a.n_persistent > 0)) {
    const int row0 = PS ? t0 : RPT * t0 + tid0 / (kBlock / RPT);
    const int rc = row0 < rows ? row0 : rows - 1;
    ps_p0 = a.tile_prefix[rc];
    ps_p1 = a.tile_prefix[rc + 1];
    ps_total = a.tile_prefix[a.batch];
  }

  // W_V^(h) rows wv*(d_h/4) + 16nt + l16, elements 32kk + 8g .. +7: the A operand
  uint4 wfrag[NT][KK];
  const uint16_t* wsrc =
      reinterpret_cast<const uint16_t*>(a.w_uv) + ((size_t)h * DH + wv * (DH / 4) + l16) * R + 8 * g;
  auto fetch_w = [&]() {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        wfrag[nt][kk] = *reinterpret_cast<const uint4*>(wsrc + (size_t)16 * nt * R + 32 * kk);
  };
  if (WKEEP && a.out) fetch_w();

  if (RPT < kTileRows) {  // tile rows no thread fills stay zero for the whole kernel
    for (int i = tid; i < 2 * kTileRows * AS / 2; i += kBlock) reinterpret_cast<uint32_t*>(&sA[0][0][0])[i] = 0u;
    __syncthreads();
  }

  const int total_tiles = (PS || HF) ? ps_total : (a.n_persistent > 0 ? a.tile_prefix[a.batch] : 0);
  const int rr = PS ? 0 : tid / TPR, sub = tid % TPR;  // merge phase: TPR threads per row
  for (int t = t0; t < t1; ++t) {
    const int row = RPT * t + rr;
    // static schedule: piece ids row*n_splits + 0 .. n_splits-1 are readable whatever the row's
    // length turns out to be, so the requests below do not wait for it
    const bool fixed_ids = a.n_persistent == 0;
    const Pieces pc = (PS || (HF && a.n_persistent > 0 && t == t0)) ? pieces_balanced(a, row, rows, ps_p0, ps_p1, ps_total)
                                                                     : pieces_of_row(a, row, rows, total_tiles);
    const int row_c = row < rows ? row : rows - 1;
    const size_t pb = (size_t)(fixed_ids ? row_c * a.n_splits : pc.first) * a.n_heads + h;  // + p * n_heads
    const int p_last = fixed_ids ? a.n_splits - 1 : (pc.count > 0 ? pc.count - 1 : 0);
    // piece split: this wavefront's quarter of the row's pieces, [pw0, pw0 + cnt)
    const int pq = (pc.count + kWaves - 1) / kWaves;
    const int pw0 = PS ? wv * pq : 0;
    const int cnt = PS ? (pc.count - pw0 < 0 ? 0 : (pc.count - pw0 < pq ? pc.count - pw0 : pq)) : pc.count;

    // ---- first PB pieces: requested before anything is known about m* (any piece id that can
    // come out of pieces_of_row is readable workspace)
    float2 mp[PB];  // (m_p, l_p)
    typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
    float4_t v[PF16 ? 1 : PB][PF16 ? 1 : CJ];   // fp32 partials as loaded
    u32x2_t vh[PF16 ? PB : 1][PF16 ? CJ : 1];   // half partials stay packed until they are used
    auto request = [&](int p0) {
#pragma unroll
      for (int i = 0; i < PB; ++i) {
        const size_t pi = pb + (size_t)(pw0 + p0 + i < p_last ? pw0 + p0 + i : p_last) * a.n_heads;
        mp[i] = *reinterpret_cast<const float2*>(a.part_ml + pi * 2);
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
          if (PF16)
            vh[PF16 ? i : 0][PF16 ? j : 0] = *reinterpret_cast<const u32x2_t*>(
                reinterpret_cast<const uint16_t*>(a.part_o) + pi * R + 4 * sub + 4 * TPR * j);
          else
            v[PF16 ? 0 : i][PF16 ? 0 : j] = *reinterpret_cast<const float4_t*>(a.part_o + pi * R + 4 * sub + 4 * TPR * j);
        }
      }
    };
    request(0);

    // ---- m* = max_p m_p,  l* = sum_p l_p 2^(m_p - m*): piece p is looked at by thread p mod TPR
    float2 ml0 = *reinterpret_cast<const float2*>(a.part_ml + (pb + (size_t)(sub < p_last ? sub : p_last) * a.n_heads) * 2);
    if (sub >= pc.count) ml0 = make_float2(-INFINITY, 0.f);
    float mloc = ml0.x;
    for (int p = sub + TPR; p < pc.count; p += TPR) mloc = fmaxf(mloc, a.part_ml[(pb + (size_t)p * a.n_heads) * 2]);
    const float mstar = group_max<TPR>(mloc);
    float lloc = sub < pc.count ? __builtin_amdgcn_exp2f(ml0.x - mstar) * ml0.y : 0.f;
    for (int p = sub + TPR; p < pc.count; p += TPR) {
      const float2 ml = *reinterpret_cast<const float2*>(a.part_ml + (pb + (size_t)p * a.n_heads) * 2);
      lloc += __builtin_amdgcn_exp2f(ml.x - mstar) * ml.y;
    }
    const float lstar = group_sum<TPR>(lloc);

    // ---- o~ = sum_p 2^(m_p - m*) o_p / l*
    float4_t acc[CJ];
#pragma unroll
    for (int j = 0; j < CJ; ++j) acc[j] = float4_t{0.f, 0.f, 0.f, 0.f};
    for (int p0 = 0; p0 < cnt; p0 += PB) {
      if (p0 > 0) request(p0);
#pragma unroll
      for (int i = 0; i < PB; ++i) {
        if (p0 + i < cnt) {  // a piece beyond the row's own may hold anything: never touched
          const float f = __builtin_amdgcn_exp2f(mp[i].x - mstar) * (PF16 ? mp[i].y : 1.f);
#pragma unroll
          for (int j = 0; j < CJ; ++j) {
            if (PF16) {
              const u32x2_t hv = vh[PF16 ? i : 0][PF16 ? j : 0];
              acc[j] += f * float4_t{f16_lo_to_f32(hv[0]), f16_hi_to_f32(hv[0]), f16_lo_to_f32(hv[1]), f16_hi_to_f32(hv[1])};
            } else {
              acc[j] += f * v[PF16 ? 0 : i][PF16 ? 0 : j];
            }
          }
        }
      }
    }
    if constexpr (PS) {  // wavefront 0 adds the other three sums to its own
      if (wv > 0) {
#pragma unroll
        for (int j = 0; j < CJ; ++j) *reinterpret_cast<float4_t*>(&sRed[wv - 1][4 * sub + 4 * TPR * j]) = acc[j];
      }
      __syncthreads();
      if (wv == 0) {
#pragma unroll
        for (int w = 0; w < kWaves - 1; ++w)
#pragma unroll
          for (int j = 0; j < CJ; ++j) acc[j] += *reinterpret_cast<const float4_t*>(&sRed[w][4 * sub + 4 * TPR * j]);
      }
    }
    const float inv = pc.count > 0 ? 1.f / lstar : 0.f;  // a row with no live column gives zeros
#pragma unroll
    for (int j = 0; j < CJ; ++j) acc[j] *= inv;
    if (row < rows && (!PS || wv == 0)) {
      const size_t oh = (size_t)row * a.n_heads + h;
      if (a.out_latent) {
#pragma unroll
        for (int j = 0; j < CJ; ++j)
          *reinterpret_cast<float4_t*>(a.out_latent + oh * R + 4 * sub + 4 * TPR * j) = acc[j];
      }
      if (a.lse && sub == 0) a.lse[oh] = pc.count > 0 ? (mstar + log2f(lstar)) * 0.6931471805599453f : -INFINITY;
    }
    if (!a.out) continue;

    // ---- park the row as hi + lo bf16 planes
#pragma unroll
    for (int j = 0; j < (!PS || wv == 0 ? CJ : 0); ++j) {
      const uint32_t h01 = pack_bf16x2(acc[j][0], acc[j][1]), h23 = pack_bf16x2(acc[j][2], acc[j][3]);
      const uint32_t l01 = pack_bf16x2(acc[j][0] - __uint_as_float(h01 << 16), acc[j][1] - __uint_as_float(h01 & 0xffff0000u));
      const uint32_t l23 = pack_bf16x2(acc[j][2] - __uint_as_float(h23 << 16), acc[j][3] - __uint_as_float(h23 & 0xffff0000u));
      *reinterpret_cast<uint2*>(&sA[0][rr][4 * sub + 4 * TPR * j]) = make_uint2(h01, h23);
      *reinterpret_cast<uint2*>(&sA[1][rr][4 * sub + 4 * TPR * j]) = make_uint2(l01, l23);
    }
    if (!WKEEP) fetch_w();
    __syncthreads();

    // ---- out^T[d, row] for this wavefront's d_h / 4 output rows
    float4_t o[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) o[nt] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8_t bh = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(&sA[0][l16][32 * kk + 8 * g]));
      const bf16x8_t bl = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(&sA[1][l16][32 * kk + 8 * g]));
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const bf16x8_t wa = __builtin_bit_cast(bf16x8_t, wfrag[nt][kk]);
        o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, bh, o[nt], 0, 0, 0);
        o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, bl, o[nt], 0, 0, 0);
      }
    }
    // lane holds row l16 of the tile, output dims wv*(d_h/4) + 16nt + 4g .. +3
    const int orow = RPT * t + l16;
    if (l16 < RPT && orow < rows) {
      float* dst = a.out + ((size_t)orow * a.n_heads + h) * DH + wv * (DH / 4) + 4 * g;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) *reinterpret_cast<float4_t*>(dst + 16 * nt) = o[nt];
    }
    __syncthreads();  // the planes are rewritten by the next tile
  }
}

template <int R, int DH, bool PF16>
hipError_t launch_rdh_pf(const CombineArgs& a, hipStream_t st) {
  const int rows = a.T ? a.batch * a.T : a.batch;
  if constexpr (R >= 256 && PF16) {
    // a handful of rows of eight or more pieces each (at most n_persistent + rows pieces exist): one row per
    // workgroup, its pieces split over the wavefronts
    if (a.n_persistent > 0 && rows <= 16 && a.n_persistent + rows >= 8 * rows) {
      const dim3 grid(a.n_heads, rows);
      hipLaunchKernelGGL((combine_mfma_kernel<R, DH, 1, true, true, true>), grid, dim3(kBlock), 0, st, a, 1);
      return hipGetLastError();
    }
  }
  if constexpr (R >= 256) {
    if (rows <= 64) {  // small batch: four rows per workgroup, one wavefront merging each
      const dim3 grid((rows + 3) / 4, a.n_heads);
      // up to r = 256 the W_V fragments fit beside the partials: fetched at the top, one round trip
      hipLaunchKernelGGL((combine_mfma_kernel<R, DH, 4, (R <= 256), PF16>), grid, dim3(kBlock), 0, st, a, 1);
      return hipGetLastError();
    }
  }
  const int n_tiles = (rows + kTileRows - 1) / kTileRows;
  // long runs amortise the W_V^(h) fetch; short ones keep every compute unit busy
  long long tpw = (long long)n_tiles * a.n_heads / 2048;
  tpw = tpw < 1 ? 1 : (tpw > 8 ? 8 : tpw);
  const dim3 grid((n_tiles + (int)tpw - 1) / (int)tpw, a.n_heads);
  if constexpr (PF16) {
    // decode over many rows, balanced schedule (a few half-size partials per row): weights requested at the
    // top beside the counts, heads as the fast grid index
    if (tpw == 1 && a.T == 0 && a.n_persistent > 0) {
      hipLaunchKernelGGL((combine_mfma_kernel<R, DH, kTileRows, true, true, false, true>), dim3(a.n_heads, grid.x), dim3(kBlock),
                         0, st, a, 1);
      return hipGetLastError();
    }
  }
  if (tpw == 1)
    hipLaunchKernelGGL((combine_mfma_kernel<R, DH, kTileRows, false, PF16>), grid, dim3(kBlock), 0, st, a, 1);
  else
    hipLaunchKernelGGL((combine_mfma_kernel<R, DH, kTileRows, true, PF16>), grid, dim3(kBlock), 0, st, a, (int)tpw);
  return hipGetLastError();
}

template <int R, int DH>
hipError_t launch_rdh(const CombineArgs& a, hipStream_t st) {
  return a.part_f16 ? launch_rdh_pf<R, DH, true>(a, st) : launch_rdh_pf<R, DH, false>(a, st);
}

}  // namespace

bool combine_mfma_supported(const CombineArgs& a) {
  const bool dims = (a.r == 64 || a.r == 128 || a.r == 256 || a.r == 512) && (a.d_head == 64 || a.d_head == 128);
  const auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  return dims && al16(a.out) && al16(a.out_latent) && al16(a.w_uv) && a.n_heads <= 65535;
}

hipError_t launch_combine_mfma(const CombineArgs& a, hipStream_t st) {
#define MTLA_CASE(RR, DD) \
  if (a.r == RR && a.d_head == DD) return launch_rdh<RR, DD>(a, st);
  MTLA_CASE(64, 64)
  MTLA_CASE(64, 128)
  MTLA_CASE(128, 64)
  MTLA_CASE(128, 128)
  MTLA_CASE(256, 64)
  MTLA_CASE(256, 128)
  MTLA_CASE(512, 64)
  MTLA_CASE(512, 128)
#undef MTLA_CASE
  return hipErrorInvalidValue;
}

}  // namespace mtla
