// bf16 matrix-core decode attention over one chunk of cache slots (gfx950).
//
// Eq. (with-rope), incremental case: all heads of a sequence share each cached
// row (C_hat[k], K_hat^R[k]), so the pass over the cache is two small dense
// contractions per 16-slot tile with the heads as one matrix dimension:
//     S^T[slot, head] = [C_hat | K_hat^R][slot, :] . [q~ | q^R][head, :]      (K = r + d_R)
//     O^T[col,  head] += C_hat^T[col, slot] . P^T[slot, head]                  (K = 16 slots)
// Each wavefront of a workgroup streams its own 16-slot tiles and keeps its own
// online-softmax state; there is no workgroup barrier inside the loop.  Per
// tile and wavefront:
//   * the tile and the query operand are loaded from memory straight into the
//     operand layouts of v_mfma_f32_16x16x32_bf16 (lane = row, 8 consecutive
//     elements of the contraction), so the logits need no staging at all;
//   * S^T leaves the matrix core with lane = head column and 4 consecutive slots
//     per lane, which is exactly the B-operand layout of the K=16 bf16 MFMA, so
//     the probabilities never leave registers;
//   * the latent part of the tile is parked in a wavefront-private LDS region
//     and read back transposed (ds_read_b64_tr_b16) as the C_hat^T operand.
// At the end every wavefront drops its unnormalised state into LDS and the
// whole workgroup sums the copies into one partial (m, l, o[r]) per
// (sequence, chunk, head).
//
// A single wavefront issues at most one instruction every four cycles, and at
// decode batch sizes a wavefront sees only a tile or two, so the kernel is
// written for a short dynamic instruction stream: one round trip to memory for
// everything whose address does not depend on the sequence length, hardware
// bf16 conversion and exp2, a fixed softmax reference per wavefront instead of
// a running maximum (no accumulator rescaling on the hot path), and a
// single-pass merge.
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
  static constexpr int HP = 16 * NHT;       // heads padded to whole 16-row tiles
  static constexpr int WPT = kWaves / NHT;  // wavefronts sharing one head tile
  static constexpr int KC = R / 32;         // K steps over the latent part
  static constexpr int KR = DR / 32;        // K steps over the RoPE part
  static constexpr int MT = R / 16;         // output column tiles
  static constexpr int TS = R + 16;         // tile row stride: 2R+32 bytes, 8 words mod 64 banks
  static constexpr int OS = R + 4;          // merge row stride (floats)
  static constexpr size_t tile_bytes = (size_t)kWaves * kTile * TS * 2;
  static constexpr size_t merge_bytes = (size_t)kWaves * 16 * OS * 4;  // one copy per wavefront
  static constexpr size_t body_bytes = tile_bytes > merge_bytes ? tile_bytes : merge_bytes;
  static constexpr size_t ml_bytes = (size_t)2 * kWaves * 16 * 4;
  static constexpr int QS = E + 8;          // query row stride in LDS (bf16 elements)
  static constexpr size_t q_bytes = (size_t)HP * QS * 2;
  // the query (when it sits in LDS) follows the tile regions; the merge buffer reuses both
  static constexpr size_t loop_bytes_ql = tile_bytes + q_bytes;
  static constexpr size_t body_bytes_ql = loop_bytes_ql > merge_bytes ? loop_bytes_ql : merge_bytes;
};

// NHT = number of 16-head tiles.  With two head tiles the wavefronts split into
// two pairs, one per head tile, each pair striding over all 16-slot tiles of the
// chunk (a tile is then fetched by one wavefront of each pair; the second fetch
// is served by the cache hierarchy).  One head tile per wavefront keeps the
// output accumulators (r/16 x 4 registers) resident without spilling.
//
// NS = tiles in flight per wavefront (register-staged software pipeline).  QL = the query
// operand lives in LDS instead of registers: with r = 512 the registers are needed for the
// accumulators and the tiles in flight, and a long chunk amortises the extra LDS reads.
template <int R, int DR, int NHT, int NS, bool QL>
__global__ __launch_bounds__(kBlock) void attn_mfma_kernel(AttnArgs a) {
  using C = MfmaCfg<R, DR, NHT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* sT = reinterpret_cast<uint16_t*>(smem);
  float* sO = reinterpret_cast<float*>(smem);  // aliases sT after the main loop
  constexpr size_t kBody = QL ? C::body_bytes_ql : C::body_bytes;
  float* sM = reinterpret_cast<float*>(smem + kBody);  // [kWaves][16]
  float* sL = sM + kWaves * 16;
  uint16_t* sQ = reinterpret_cast<uint16_t*>(smem + C::tile_bytes);  // QL only; dead after the loop

  const int split = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int ht = wv / C::WPT, wl = wv - ht * C::WPT;  // head tile of this wavefront, rank inside it
  const int k0 = split * a.chunk;
  const uint16_t* lat = reinterpret_cast<const uint16_t*>(a.lat) + (size_t)b * a.max_slots * R;
  const uint16_t* key = reinterpret_cast<const uint16_t*>(a.key) + (size_t)b * a.max_slots * DR;

  struct TileRegs {
    uint4 xc[C::KC], xr[C::KR];
    __device__ __forceinline__ void select_live(bool keep) {  // dead rows become exact zeros
      const uint32_t m = keep ? 0xffffffffu : 0u;
#pragma unroll
      for (int kk = 0; kk < C::KC; ++kk) xc[kk] = make_uint4(xc[kk].x & m, xc[kk].y & m, xc[kk].z & m, xc[kk].w & m);
#pragma unroll
      for (int kk = 0; kk < C::KR; ++kk) xr[kk] = make_uint4(xr[kk].x & m, xr[kk].y & m, xr[kk].z & m, xr[kk].w & m);
    }
  };
  TileRegs tl[NS];  // NS tiles in flight per wavefront (register-staged software pipeline)
  // Branch-free fetch: a row index past `last` is clamped to `last`, a row that is readable
  // whatever it holds; its logits are masked to -inf further down, so only NaN/Inf bit patterns
  // in such a row could leak (0 * NaN), and those are cleared with select_live() where the row
  // may be uninitialised memory.
  auto load_tile = [&](TileRegs& t, int base, int last) {
    const int slot = base + l16 < last ? base + l16 : last;
    const uint16_t* cr = lat + (size_t)slot * R + 8 * g;
    const uint16_t* kr = key + (size_t)slot * DR + 8 * g;
#pragma unroll
    for (int kk = 0; kk < C::KC; ++kk) t.xc[kk] = *reinterpret_cast<const uint4*>(cr + 32 * kk);
#pragma unroll
    for (int kk = 0; kk < C::KR; ++kk) t.xr[kk] = *reinterpret_cast<const uint4*>(kr + 32 * kk);
  };

  // Everything whose address does not depend on the sequence length is requested before the
  // length is looked at: the length, the query operand and this wavefront's first NS tiles (any
  // slot below max_slots is readable memory) travel together, one round trip instead of three.
  const int len = a.seq_len[b];
  constexpr int kStep = C::WPT * kTile;  // slots between consecutive tiles of one wavefront
  int base = k0 + wl * kTile;
#pragma unroll
  for (int st = 0; st < NS; ++st) load_tile(tl[st], base + st * kStep, a.max_slots - 1);
  // query operand [q~ | q^R]: lane (head 16*ht + l16, elements 32kk + 8g .. +7); padded heads
  // read the last real head's row and are never stored.
  uint4 qv[QL ? 1 : C::KC + C::KR];
  const uint16_t* qbase = reinterpret_cast<const uint16_t*>(a.qcat) + (size_t)b * a.n_heads * C::E;
  if (!QL) {
    const int h = 16 * ht + l16 < a.n_heads ? 16 * ht + l16 : a.n_heads - 1;
#pragma unroll
    for (int kk = 0; kk < C::KC + C::KR; ++kk)
      qv[kk] = *reinterpret_cast<const uint4*>(qbase + (size_t)h * C::E + 8 * g + 32 * kk);
  } else {
    constexpr int chunks = C::E / 8;
    for (int idx = tid; idx < C::HP * chunks; idx += kBlock) {
      const int hh = idx / chunks, c8 = idx - hh * chunks;
      const int h = hh < a.n_heads ? hh : a.n_heads - 1;
      *reinterpret_cast<uint4*>(sQ + hh * C::QS + c8 * 8) =
          *reinterpret_cast<const uint4*>(qbase + (size_t)h * C::E + c8 * 8);
    }
  }
  const int live = (len + a.stride - 1) / a.stride;
  const int k1 = live < k0 + a.chunk ? live : k0 + a.chunk;
  if (k0 >= k1) return;
  if (QL) __syncthreads();
#pragma unroll
  for (int st = 0; st < NS; ++st)  // the first tiles may have touched rows that were never written
    tl[st].select_live(base + st * kStep + l16 < k1);
  const uint16_t* qrow = sQ + (16 * ht + l16) * C::QS + 8 * g;

  uint16_t* sTw = sT + wv * kTile * C::TS;
  float m_ref = -INFINITY, l_run = 0.f;
  float4_t acc_o[C::MT];
#pragma unroll
  for (int mt = 0; mt < C::MT; ++mt) acc_o[mt] = float4_t{0.f, 0.f, 0.f, 0.f};

  // Every iteration runs all NS stages and every stage refills itself unconditionally (row
  // indices are clamped, dead tiles are masked): with a fixed number of loads between a tile's
  // request and its use, the compiler can wait for exactly that tile and leave the younger
  // requests in flight.  At most NS-1 dead tiles are processed at the end of a chunk.
  const int n_iter = (k1 - base + NS * kStep - 1) / (NS * kStep);  // <= 0 for an idle wavefront
  for (int it = 0; it < n_iter; ++it) {
#pragma unroll
    for (int st = 0; st < NS; ++st) {
      {
        TileRegs& t = tl[st];
        // ---- logits S^T[slot, head] for this tile (log2 units: the query is pre-scaled);
        // two accumulator chains halve the dependent-MFMA latency, and query pieces are
        // fetched from LDS a group at a time so one wait covers kQGroup matrix instructions
        float4_t s0 = float4_t{0.f, 0.f, 0.f, 0.f}, s1 = float4_t{0.f, 0.f, 0.f, 0.f};
        constexpr int kQGroup = 6, KT = C::KC + C::KR;
#pragma unroll
        for (int k0g = 0; k0g < KT; k0g += kQGroup) {
          uint4 qk[kQGroup];
#pragma unroll
          for (int j = 0; j < kQGroup; ++j)
            if (k0g + j < KT) {
              const int kk = k0g + j;  // latent pieces first, then the RoPE pieces (contiguous in a row)
              qk[j] = QL ? *reinterpret_cast<const uint4*>(qrow + 32 * kk) : qv[QL ? 0 : kk];
            }
#pragma unroll
          for (int j = 0; j < kQGroup; ++j)
            if (k0g + j < KT) {
              const int kk = k0g + j;
              const uint4 x = kk < C::KC ? t.xc[kk < C::KC ? kk : 0] : t.xr[kk < C::KC ? 0 : kk - C::KC];
              float4_t& s = (kk & 1) ? s1 : s0;
              s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, x),
                                                          __builtin_bit_cast(bf16x8_t, qk[j]), s, 0, 0, 0);
            }
        }
        // ---- park the latent rows in this wavefront's LDS region (row = slot, as loaded)
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int kk = 0; kk < C::KC; ++kk)
          *reinterpret_cast<uint4*>(sTw + l16 * C::TS + 32 * kk + 8 * g) = t.xc[kk];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- refill this stage NS tiles ahead while the softmax and PV run
        load_tile(t, base + NS * kStep, k1 - 1);

        // ---- online softmax; lane holds head l16 of its head tile and slots 4g..4g+3
        float sv[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) sv[v] = (base + 4 * g + v < k1) ? s0[v] + s1[v] : -INFINITY;
        float mt_ = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
        mt_ = fmaxf(mt_, __shfl_xor(mt_, 16, kWave));
        mt_ = fmaxf(mt_, __shfl_xor(mt_, 32, kWave));
        // Probabilities are taken relative to a reference m_ref fixed at the wavefront's first
        // tile instead of the running maximum: 2^(s - m_ref) has the whole fp32/bf16 exponent
        // range to grow into, so the accumulators are never rescaled on the hot path.  Only
        // when a tile tops the reference by more than 2^kRebase is the state re-based (cold).
        constexpr float kRebase = 40.f;
        if (m_ref == -INFINITY) m_ref = mt_;  // first live tile (mt_ is -inf for a dead tile)
        if (__any(mt_ - m_ref > kRebase)) {
          const float alpha = mt_ - m_ref > kRebase ? __builtin_amdgcn_exp2f(m_ref - mt_) : 1.f;
          if (mt_ - m_ref > kRebase) m_ref = mt_;
          l_run *= alpha;
#pragma unroll
          for (int mt = 0; mt < C::MT; ++mt) acc_o[mt] *= alpha;
        }
        const float m_sub = m_ref == -INFINITY ? 0.f : m_ref;  // no live slot seen yet: p = 2^-inf = 0
        float p[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) p[v] = __builtin_amdgcn_exp2f(sv[v] - m_sub);
        // probabilities as bf16 (hardware round-to-nearest-even); the normaliser sums the rounded values
        const uint32_t p01 = pack_bf16x2(p[0], p[1]), p23 = pack_bf16x2(p[2], p[3]);
        const short4_t pb = __builtin_bit_cast(short4_t, make_uint2(p01, p23));
        float ps = (__uint_as_float(p01 << 16) + __uint_as_float(p01 & 0xffff0000u)) +
                   (__uint_as_float(p23 << 16) + __uint_as_float(p23 & 0xffff0000u));
        ps += __shfl_xor(ps, 16, kWave);
        ps += __shfl_xor(ps, 32, kWave);
        l_run += ps;

        // ---- O^T[col, head] += C_hat^T[col, slot] P^T[slot, head], transposed operand from LDS.
        // Lane i of each 16-lane group points at row 4g + i/4, columns 4(i%4)..+3 of the column
        // tile; the transposing read hands lane i the four rows of column i.
        const uint16_t* trow = sTw + (4 * g + (l16 >> 2)) * C::TS + 4 * (l16 & 3);
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) {
          const short4_t ct = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(trow + 16 * mt));
          acc_o[mt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ct, pb, acc_o[mt], 0, 0, 0);
        }
        base += kStep;
      }
    }
  }

  // ---- merge: every wavefront publishes (m, l, o) as it stands; the workgroup then sums the
  // WPT copies of each head with weights 2^(m_w - m*)
  __syncthreads();  // every wavefront is done with its tile region, which sO aliases
  if (g == 0) {
    sM[wv * 16 + l16] = m_ref;
    sL[wv * 16 + l16] = l_run;
  }
  {
    float* dst = sO + (size_t)(wv * 16 + l16) * C::OS + 4 * g;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) *reinterpret_cast<float4_t*>(dst + 16 * mt) = acc_o[mt];
  }
  __syncthreads();
  const size_t pbase = ((size_t)b * a.n_splits + split) * a.n_heads;
  constexpr int R4 = R / 4;
  for (int idx = tid; idx < a.n_heads * R4; idx += kBlock) {
    const int h = idx / R4, c4 = idx - h * R4;
    const int w0 = (h >> 4) * C::WPT, hl = h & 15;
    float mw[C::WPT], mstar = -INFINITY;
#pragma unroll
    for (int w = 0; w < C::WPT; ++w) {
      mw[w] = sM[(w0 + w) * 16 + hl];
      mstar = fmaxf(mstar, mw[w]);
    }
    float4_t o = float4_t{0.f, 0.f, 0.f, 0.f};
    float lstar = 0.f;
#pragma unroll
    for (int w = 0; w < C::WPT; ++w) {
      const float f = __builtin_amdgcn_exp2f(mw[w] - mstar);  // 0 for a wavefront that saw no slot
      o += f * *reinterpret_cast<const float4_t*>(sO + (size_t)((w0 + w) * 16 + hl) * C::OS + 4 * c4);
      lstar += f * sL[(w0 + w) * 16 + hl];
    }
    *reinterpret_cast<float4_t*>(a.part_o + (pbase + h) * R + 4 * c4) = o;
    if (c4 == 0) {
      a.part_ml[(pbase + h) * 2 + 0] = mstar;
      a.part_ml[(pbase + h) * 2 + 1] = lstar;
    }
  }
}

template <int R, int DR, int NHT, int NS, bool QL>
hipError_t launch_one(const AttnArgs& a, hipStream_t st) {
  using C = MfmaCfg<R, DR, NHT>;
  constexpr size_t smem = (QL ? C::body_bytes_ql : C::body_bytes) + C::ml_bytes;
  static_assert(smem <= 160 * 1024, "LDS budget of one compute unit");
  static bool attr_set = false;  // LDS above the 64 KB default needs an explicit opt-in, once
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<R, DR, NHT, NS, QL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((attn_mfma_kernel<R, DR, NHT, NS, QL>), dim3(a.n_splits, a.batch), dim3(kBlock), smem,
                     st, a);
  return hipGetLastError();
}

// Pipeline depth: a wavefront that will see only a tile or two (decode at small batch) gets the
// short single-stage code with the query in registers; long chunks keep several tiles in flight
// per wavefront, which is what it takes to cover HBM latency with four wavefronts per compute
// unit.
template <int R, int DR>
hipError_t launch_rd(const AttnArgs& a, hipStream_t st) {
  constexpr int kDeep = R >= 512 ? 2 : 3;  // what the 512-register budget per lane allows
  constexpr bool kDeepQL = R >= 512;
  const int nht = a.n_heads <= 16 ? 1 : 2;
  const int tiles_per_wave = a.chunk / (kTile * (kWaves / nht));
  const bool deep = tiles_per_wave >= 2 * kDeep;
  if (nht == 1)
    return deep ? launch_one<R, DR, 1, kDeep, kDeepQL>(a, st) : launch_one<R, DR, 1, 1, false>(a, st);
  return deep ? launch_one<R, DR, 2, kDeep, kDeepQL>(a, st) : launch_one<R, DR, 2, 1, false>(a, st);
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
