// bf16 matrix-core decode attention over one chunk of cache slots (gfx950).
//
// Eq. (with-rope), incremental case: all heads of a sequence share each cached
// row (C_hat[k], K_hat^R[k]), so the pass over the cache is two small dense
// contractions per 16-slot tile with the heads as one matrix dimension:
//     S^T[slot, head] = [C_hat | K_hat^R][slot, :] . [q~ | q^R][head, :]      (K = r + d_R)
//     O^T[col,  head] += C_hat^T[col, slot] . P^T[slot, head]                  (K = 16 slots)
// Each of the four wavefronts of a workgroup streams its own 16-slot tiles and
// keeps its own online-softmax state; no workgroup barrier is needed inside the
// loop.  Per tile and wavefront:
//   * the tile is loaded from HBM straight into the A-operand layout of
//     v_mfma_f32_16x16x32_bf16 (lane = slot row, 8 consecutive elements), so
//     the logits need no staging; the query operand comes from LDS;
//   * S^T leaves the matrix core with lane = head column and 4 consecutive slots
//     per lane, which is exactly the B-operand layout of the K=16 bf16 MFMA, so
//     the probabilities never leave registers;
//   * the latent part of the tile is parked in a wavefront-private LDS region
//     and read back transposed (ds_read_b64_tr_b16) as the C_hat^T operand.
// The four wavefront states are merged through LDS at the end and written as
// one unnormalised partial (m, l, o[r]) per (sequence, chunk, head).
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef short4_t __attribute__((address_space(3))) * lds_short4_ptr;

constexpr int kWaves = kBlock / kWave;
constexpr int kTile = 16;  // slots per wavefront tile

template <int R, int DR, int NHT>
struct MfmaCfg {
  static constexpr int E = R + DR;
  static constexpr int HP = 16 * NHT;      // heads padded to whole 16-row tiles
  static constexpr int WPT = kWaves / NHT; // wavefronts sharing one head tile
  static constexpr int KC = R / 32;        // K steps over the latent part
  static constexpr int KR = DR / 32;       // K steps over the RoPE part
  static constexpr int MT = R / 16;        // output column tiles
  static constexpr int QS = E + 8;         // sQ row stride (bf16 elements)
  static constexpr int TS = R + 16;        // tile row stride: 2R+32 bytes, 8 words mod 64 banks
  static constexpr int OS = R + 4;         // merge buffer row stride (floats)
  static constexpr size_t q_bytes = (size_t)HP * QS * 2;
  static constexpr size_t tile_bytes = (size_t)kWaves * kTile * TS * 2;
  static constexpr size_t merge_bytes = (size_t)HP * OS * 4;
  static constexpr size_t body_bytes = tile_bytes > merge_bytes ? tile_bytes : merge_bytes;
  static constexpr size_t ml_bytes = (size_t)2 * kWaves * 16 * 4;
  static constexpr size_t smem_bytes = q_bytes + body_bytes + ml_bytes;
};

// NHT = number of 16-head tiles.  With two head tiles the wavefronts split into
// two pairs, one per head tile, each pair striding over all 16-slot tiles of the
// chunk (a tile is then fetched by one wavefront of each pair; the second fetch
// is served by the cache hierarchy).  One head tile per wavefront keeps the
// output accumulators (r/16 x 4 registers) resident without spilling.
template <int R, int DR, int NHT>
__global__ __launch_bounds__(kBlock) void attn_mfma_kernel(AttnArgs a) {
  using C = MfmaCfg<R, DR, NHT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* sQ = reinterpret_cast<uint16_t*>(smem);
  uint16_t* sT = reinterpret_cast<uint16_t*>(smem + C::q_bytes);
  float* sO = reinterpret_cast<float*>(smem + C::q_bytes);  // aliases sT after the main loop
  float* sM = reinterpret_cast<float*>(smem + C::q_bytes + C::body_bytes);  // [kWaves][16]
  float* sL = sM + kWaves * 16;

  const int split = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int ht = wv / C::WPT, wl = wv - ht * C::WPT;  // head tile of this wavefront, rank inside it
  const int len = a.seq_len[b];
  const int live = (len + a.stride - 1) / a.stride;
  const int k0 = split * a.chunk;
  const int k1 = live < k0 + a.chunk ? live : k0 + a.chunk;
  if (k0 >= k1) return;

  // ---- query operand [q~ | q^R] of every head into LDS; padded heads are zero
  {
    const uint16_t* qcat = reinterpret_cast<const uint16_t*>(a.qcat) + (size_t)b * a.n_heads * C::E;
    constexpr int chunks = C::E / 8;
    for (int idx = tid; idx < C::HP * chunks; idx += kBlock) {
      const int h = idx / chunks, c8 = idx - h * chunks;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (h < a.n_heads) v = *reinterpret_cast<const uint4*>(qcat + (size_t)h * C::E + c8 * 8);
      *reinterpret_cast<uint4*>(sQ + h * C::QS + c8 * 8) = v;
    }
  }
  __syncthreads();

  const uint16_t* lat = reinterpret_cast<const uint16_t*>(a.lat) + (size_t)b * a.max_slots * R;
  const uint16_t* key = reinterpret_cast<const uint16_t*>(a.key) + (size_t)b * a.max_slots * DR;
  uint16_t* sTw = sT + wv * kTile * C::TS;
  const uint16_t* qrow = sQ + (16 * ht + l16) * C::QS + 8 * g;

  float m_run = -INFINITY, l_run = 0.f;
  float4_t acc_o[C::MT];
#pragma unroll
  for (int mt = 0; mt < C::MT; ++mt) acc_o[mt] = float4_t{0.f, 0.f, 0.f, 0.f};

  uint4 xc[C::KC], xr[C::KR];
  auto load_tile = [&](int base) {
    const int slot = base + l16;
    if (slot < k1) {
      const uint16_t* cr = lat + (size_t)slot * R + 8 * g;
      const uint16_t* kr = key + (size_t)slot * DR + 8 * g;
#pragma unroll
      for (int kk = 0; kk < C::KC; ++kk) xc[kk] = *reinterpret_cast<const uint4*>(cr + 32 * kk);
#pragma unroll
      for (int kk = 0; kk < C::KR; ++kk) xr[kk] = *reinterpret_cast<const uint4*>(kr + 32 * kk);
    } else {  // rows past the chunk end contribute exact zeros (0 * garbage could be NaN)
#pragma unroll
      for (int kk = 0; kk < C::KC; ++kk) xc[kk] = make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int kk = 0; kk < C::KR; ++kk) xr[kk] = make_uint4(0, 0, 0, 0);
    }
  };

  int base = k0 + wl * kTile;
  if (base < k1) load_tile(base);
  while (base < k1) {
    // ---- logits S^T[slot, head] for this tile (log2 units: the query is pre-scaled)
    float4_t s = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < C::KC; ++kk) {
      const uint4 qv = *reinterpret_cast<const uint4*>(qrow + 32 * kk);
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xc[kk]),
                                                  __builtin_bit_cast(bf16x8_t, qv), s, 0, 0, 0);
    }
#pragma unroll
    for (int kk = 0; kk < C::KR; ++kk) {
      const uint4 qv = *reinterpret_cast<const uint4*>(qrow + R + 32 * kk);
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xr[kk]),
                                                  __builtin_bit_cast(bf16x8_t, qv), s, 0, 0, 0);
    }
    // ---- park the latent rows in this wavefront's LDS region (row = slot, as loaded)
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int kk = 0; kk < C::KC; ++kk)
      *reinterpret_cast<uint4*>(sTw + l16 * C::TS + 32 * kk + 8 * g) = xc[kk];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // ---- prefetch the next tile of this wavefront while the softmax and PV run
    const int next = base + C::WPT * kTile;
    if (next < k1) load_tile(next);

    // ---- online softmax; lane holds head l16 of its head tile and slots 4g..4g+3
    float sv[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) sv[v] = (base + 4 * g + v < k1) ? s[v] : -INFINITY;
    float mt_ = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    mt_ = fmaxf(mt_, __shfl_xor(mt_, 16, kWave));
    mt_ = fmaxf(mt_, __shfl_xor(mt_, 32, kWave));
    const float m_new = fmaxf(m_run, mt_);  // finite: slot `base` is live
    const float alpha = exp2f(m_run - m_new);
    const bool rescale = m_new > m_run;
    m_run = m_new;
    short4_t pb;
    float ps = 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const uint16_t bits = f32_to_bf16_bits(exp2f(sv[v] - m_new));
      pb[v] = (short)bits;
      ps += __uint_as_float(uint32_t(bits) << 16);  // normaliser from the rounded weights
    }
    ps += __shfl_xor(ps, 16, kWave);
    ps += __shfl_xor(ps, 32, kWave);
    l_run = l_run * alpha + ps;
    if (__any(rescale)) {  // the running maximum settles quickly; most tiles skip this
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) acc_o[mt] *= alpha;
    }

    // ---- O^T[col, head] += C_hat^T[col, slot] P^T[slot, head], transposed operand from LDS.
    // Lane i of each 16-lane group points at row 4g + i/4, columns 4(i%4)..+3 of the column
    // tile; the transposing read hands lane i the four rows of column i.
    const uint16_t* trow = sTw + (4 * g + (l16 >> 2)) * C::TS + 4 * (l16 & 3);
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) {
      const short4_t ct = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(trow + 16 * mt));
      acc_o[mt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ct, pb, acc_o[mt], 0, 0, 0);
    }
    base = next;
  }

  // ---- merge the wavefront states of each head tile
  if (g == 0) {
    sM[wv * 16 + l16] = m_run;
    sL[wv * 16 + l16] = l_run;
  }
  __syncthreads();  // also: every wavefront is done with its tile region, which sO aliases
  {
    float mstar = -INFINITY;
#pragma unroll
    for (int w = 0; w < C::WPT; ++w) mstar = fmaxf(mstar, sM[(ht * C::WPT + w) * 16 + l16]);
    const float f = (m_run == -INFINITY) ? 0.f : exp2f(m_run - mstar);
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) acc_o[mt] *= f;
  }
  for (int w = 0; w < C::WPT; ++w) {
    if (wl == w) {
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) {
        float4_t* dst = reinterpret_cast<float4_t*>(sO + (16 * ht + l16) * C::OS + 16 * mt + 4 * g);
        if (w == 0)
          *dst = acc_o[mt];
        else
          *dst += acc_o[mt];
      }
    }
    __syncthreads();
  }
  const size_t pbase = ((size_t)b * a.n_splits + split) * a.n_heads;
  constexpr int R4 = R / 4;
  for (int idx = tid; idx < a.n_heads * R4; idx += kBlock) {
    const int h = idx / R4, c4 = idx - h * R4;
    *reinterpret_cast<float4_t*>(a.part_o + (pbase + h) * R + 4 * c4) =
        *reinterpret_cast<const float4_t*>(sO + h * C::OS + 4 * c4);
  }
  if (tid < a.n_heads) {
    const int hts = tid >> 4, hl = tid & 15;
    float mstar = -INFINITY;
#pragma unroll
    for (int w = 0; w < C::WPT; ++w) mstar = fmaxf(mstar, sM[(hts * C::WPT + w) * 16 + hl]);
    float lstar = 0.f;
#pragma unroll
    for (int w = 0; w < C::WPT; ++w) {
      const float mw = sM[(hts * C::WPT + w) * 16 + hl];
      lstar += (mw == -INFINITY) ? 0.f : sL[(hts * C::WPT + w) * 16 + hl] * exp2f(mw - mstar);
    }
    a.part_ml[(pbase + tid) * 2 + 0] = mstar;
    a.part_ml[(pbase + tid) * 2 + 1] = lstar;
  }
}

template <int R, int DR, int NHT>
hipError_t launch_one(const AttnArgs& a, hipStream_t st) {
  using C = MfmaCfg<R, DR, NHT>;
  static bool attr_set = false;  // LDS above the 64 KB default needs an explicit opt-in, once
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<R, DR, NHT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::smem_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((attn_mfma_kernel<R, DR, NHT>), dim3(a.n_splits, a.batch), dim3(kBlock),
                     C::smem_bytes, st, a);
  return hipGetLastError();
}

template <int R, int DR>
hipError_t launch_rd(const AttnArgs& a, hipStream_t st) {
  if (a.n_heads <= 16) return launch_one<R, DR, 1>(a, st);
  return launch_one<R, DR, 2>(a, st);
}

}  // namespace

bool attn_mfma_supported(const AttnArgs& a) {
  return a.T == 0 && a.n_heads <= 32 && (a.r == 64 || a.r == 128 || a.r == 256 || a.r == 512) &&
         (a.d_rope == 32 || a.d_rope == 64);
}

hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t st) {
#define MTLA_CASE(RR, DD) \
  if (a.r == RR && a.d_rope == DD) return launch_rd<RR, DD>(a, st);
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

}  // namespace mtla
