// Tile machinery of the bf16 matrix-core decode attention (gfx950): operand layouts, the per-wavefront
// online-softmax state, the streaming loop over 16-slot tiles and the merge of a workgroup's wavefront
// states.  Shared by the kernels of attn_mfma.hip and the one-launch decode step (decode_fused.hip);
// what each piece computes is described at the top of attn_mfma.hip.
#pragma once
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

template <int R_, int DR_, int NHT_>
struct MfmaCfg {
  static constexpr int R = R_, DR = DR_, NHT = NHT_;
  static constexpr int E = R + DR;
  static constexpr int HP = 16 * NHT;       // heads padded to whole 16-row tiles
  static constexpr int WPT = kWaves / NHT;  // wavefronts sharing one head tile
  static constexpr int KC = R / 32;         // K steps over the latent part
  static constexpr int KR = DR / 32;        // K steps over the RoPE part
  static constexpr int KT = KC + KR;
  static constexpr int MT = R / 16;         // output column tiles
  static constexpr int TS = R + 16;         // tile row stride: 2R+32 bytes, 8 words mod 64 banks
  static constexpr int OS = R + 4;          // merge row stride (floats)
  static constexpr int QS = E + 8;          // query row stride in LDS (bf16 elements)
  static constexpr int kStep = WPT * kTile; // slots between consecutive tiles of one wavefront
  static constexpr size_t tile_bytes = (size_t)kWaves * kTile * TS * 2;
  static constexpr size_t merge_bytes = (size_t)kWaves * 16 * OS * 4;  // one copy per wavefront
  static constexpr size_t q_bytes = (size_t)2 * HP * QS * 2;  // hi and lo planes
  // loop phase: tile regions (+ the query when it sits in LDS); merge phase reuses the space
  static constexpr size_t body_bytes(bool ql) {
    const size_t loop = tile_bytes + (ql ? q_bytes : 0);
    return loop > merge_bytes ? loop : merge_bytes;
  }
  static constexpr size_t ml_bytes = (size_t)2 * kWaves * 16 * 4;
};

template <class C>
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

// How a wavefront's column index k maps to a row of the latent / key arrays.
//   decode  (stride == 0): column k is cache slot k.
//   prefill (stride == s): column k < nfin is the final state of chunk k, row k*s + s-1 of
//           C_hat'; the last column is the query row's own running state, row `own`
//           (exactly the columns the stride-aware causal mask leaves open).
struct Cols {
  int step;               // columns between consecutive tiles of this wavefront
  int stride, nfin, own;
  __device__ __forceinline__ int row(int k) const {
    return stride == 0 ? k : (k < nfin ? k * stride + stride - 1 : own);
  }
};

// Branch-free fetch of tile columns base + l16 (clamped to `last`): lane (l16, g) takes elements
// 32kk + 8g .. +7 of its row.  A clamped column is a duplicate of a readable one; its logits are
// masked to -inf in the softmax, so it contributes exact zeros.
template <class C, bool SH = false>
__device__ __forceinline__ void load_tile(TileRegs<C>& t, const uint16_t* lat, const uint16_t* key, int base,
                                          int last, int l16, int g, const Cols& cm,
                                          const SharedPrefix& sp = SharedPrefix{0, 0, 0}) {
  const int slot = cm.row(base + l16 < last ? base + l16 : last);
  const uint16_t* cr = lat + (size_t)slot * C::R + 8 * g;
  const uint16_t* kr = key + (size_t)slot * C::DR + 8 * g;
  if constexpr (SH) {  // decode only (cm.row is the identity there)
    if (slot < sp.n) {
      cr += sp.dlat;
      kr += sp.dkey;
    }
  }
#pragma unroll
  for (int kk = 0; kk < C::KC; ++kk) t.xc[kk] = *reinterpret_cast<const uint4*>(cr + 32 * kk);
#pragma unroll
  for (int kk = 0; kk < C::KR; ++kk) t.xr[kk] = *reinterpret_cast<const uint4*>(kr + 32 * kk);
}

// Per-wavefront attention state over the tiles it has seen.
template <class C>
struct WaveState {
  float m_ref, l_run;  // l_run: this lane's slots only, see l_total()
  float4_t acc_o[C::MT];
  __device__ __forceinline__ float l_total() const {  // normaliser of the lane's head
    float l = l_run + __shfl_xor(l_run, 16, kWave);
    return l + __shfl_xor(l, 32, kWave);
  }
  __device__ __forceinline__ void reset() {
    m_ref = -INFINITY;
    l_run = 0.f;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) acc_o[mt] = float4_t{0.f, 0.f, 0.f, 0.f};
  }
};

// Streams this wavefront's tiles base, base + kStep, ... below k1 through the two contractions.
// tl[0..NS) hold the first NS tiles on entry (register-staged software pipeline).  Every
// iteration runs all NS stages and every stage refills itself unconditionally (row indices are
// clamped, dead tiles are masked): with a fixed number of loads between a tile's request and its
// use, the compiler can wait for exactly that tile and leave the younger requests in flight.  At
// most NS-1 dead tiles are processed at the end.
// QM says where the two query planes live: 0 = both in registers (qv[0..KT) hi, qv[KT..2KT) lo),
// 1 = both in LDS (qrow: hi row, lo row HP*QS further), 2 = hi in registers, lo in LDS (qrow).
constexpr int kQRegs = 0, kQLds = 1, kQMixed = 2;
template <class C, int QM>
struct QRegCount {
  static constexpr int value = QM == kQRegs ? 2 * C::KT : (QM == kQLds ? 1 : C::KT);
};

// Where a wavefront's tile stream continues once its run [base, k1) is used up: the refills of
// the last NS tiles fetch tiles base, base + step, ... of `lat` / `key` (columns clamped to
// `last`) instead of dead duplicates, so the caller finds the first NS tiles of its next run in
// tl[] -- requested a whole tile pass before they are needed.  A caller without a next run points
// it at the current arrays with base > last (every column clamps to a readable row).
struct NextRun {
  const uint16_t* lat;
  const uint16_t* key;
  int base, last;
};

// DEADSKIP: a refill that would only fetch dead duplicates (no next run) is not issued at all.  For
// short runs, where the trip of those loads would be waited for when their registers are reused.
template <class C, int NS, int QM, bool SH = false, bool DEADSKIP = false>  // SH: `sp` applies to this run and to the next one (same sequence)
__device__ __forceinline__ void stream_tiles(TileRegs<C> (&tl)[NS], const uint4 (&qv)[QRegCount<C, QM>::value],
                                             const uint16_t* qrow, uint16_t* sTw, const uint16_t* lat,
                                             const uint16_t* key, int base, int k1, int l16, int g,
                                             const Cols& cm, WaveState<C>& ws, const NextRun& nx,
                                             const SharedPrefix& sp = SharedPrefix{0, 0, 0}) {
  const int n_iter = (k1 - base + NS * cm.step - 1) / (NS * cm.step);  // <= 0 for an idle wavefront
  for (int it = 0; it < n_iter; ++it) {
    const bool tail = it == n_iter - 1;  // this pass refills from the next run
#pragma unroll
    for (int st = 0; st < NS; ++st) {
      TileRegs<C>& t = tl[st];
      // ---- logits S^T[slot, head] for this tile (log2 units: the query is pre-scaled): one
      // accumulator chain for the hi plane of the query and one for the lo plane; query pieces
      // are fetched from LDS a group at a time so one wait covers a group of matrix instructions
      float4_t s0 = float4_t{0.f, 0.f, 0.f, 0.f}, s1 = float4_t{0.f, 0.f, 0.f, 0.f};
      constexpr int kQGroup = 3;
#pragma unroll
      for (int k0g = 0; k0g < C::KT; k0g += kQGroup) {
        uint4 qh[kQGroup], ql[kQGroup];
#pragma unroll
        for (int j = 0; j < kQGroup; ++j)
          if (k0g + j < C::KT) {
            const int kk = k0g + j;  // latent pieces first, then the RoPE pieces (contiguous in a row)
            qh[j] = QM == kQLds ? *reinterpret_cast<const uint4*>(qrow + 32 * kk) : qv[QM == kQLds ? 0 : kk];
            ql[j] = QM == kQRegs ? qv[QM == kQRegs ? C::KT + kk : 0]
                                 : *reinterpret_cast<const uint4*>(qrow + (QM == kQLds ? C::HP * C::QS : 0) + 32 * kk);
          }
#pragma unroll
        for (int j = 0; j < kQGroup; ++j)
          if (k0g + j < C::KT) {
            const int kk = k0g + j;
            const uint4 x = kk < C::KC ? t.xc[kk < C::KC ? kk : 0] : t.xr[kk < C::KC ? 0 : kk - C::KC];
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, x),
                                                         __builtin_bit_cast(bf16x8_t, qh[j]), s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, x),
                                                         __builtin_bit_cast(bf16x8_t, ql[j]), s1, 0, 0, 0);
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
      if (!(DEADSKIP && tail && nx.base + st * cm.step > nx.last))  // wavefront-uniform
        load_tile<C, SH>(t, tail ? nx.lat : lat, tail ? nx.key : key, tail ? nx.base + st * cm.step : base + NS * cm.step,
                         tail ? nx.last : k1 - 1, l16, g, cm, sp);

      // ---- softmax weights; lane holds head l16 of its head tile and slots 4g..4g+3
      float sv[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) sv[v] = (base + 4 * g + v < k1) ? s0[v] + s1[v] : -INFINITY;
      // Weights are taken relative to a reference m_ref fixed at the wavefront's first live tile
      // instead of the running maximum: 2^(s - m_ref) has the whole fp32/bf16 exponent range to
      // grow into, so the accumulators are never rescaled on the hot path, and the hot path needs
      // no cross-lane traffic at all: the four lanes that share a head keep their own partial
      // normaliser (summed by l_total() at the end), and the tile maximum is only formed on the
      // two cold paths -- fixing the reference, and re-basing the state when a tile tops the
      // reference by more than 2^kRebase.
      constexpr float kRebase = 40.f;
      const float mloc = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
      if (__any(ws.m_ref == -INFINITY || mloc - ws.m_ref > kRebase)) {
        float mt_ = fmaxf(mloc, __shfl_xor(mloc, 16, kWave));
        mt_ = fmaxf(mt_, __shfl_xor(mt_, 32, kWave));
        if (ws.m_ref == -INFINITY) {
          ws.m_ref = mt_;  // still -inf if the tile is dead
        } else if (mt_ - ws.m_ref > kRebase) {
          const float alpha = __builtin_amdgcn_exp2f(ws.m_ref - mt_);
          ws.m_ref = mt_;
          ws.l_run *= alpha;
#pragma unroll
          for (int mt = 0; mt < C::MT; ++mt) ws.acc_o[mt] *= alpha;
        }
      }
      const float m_sub = ws.m_ref == -INFINITY ? 0.f : ws.m_ref;  // nothing live yet: p = 2^-inf = 0
      float p[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) p[v] = __builtin_amdgcn_exp2f(sv[v] - m_sub);
      // weights as bf16 (hardware round-to-nearest-even); the normaliser sums the rounded values
      const uint32_t p01 = pack_bf16x2(p[0], p[1]), p23 = pack_bf16x2(p[2], p[3]);
      const short4_t pb = __builtin_bit_cast(short4_t, make_uint2(p01, p23));
      ws.l_run += (__uint_as_float(p01 << 16) + __uint_as_float(p01 & 0xffff0000u)) +
                  (__uint_as_float(p23 << 16) + __uint_as_float(p23 & 0xffff0000u));

      // ---- O^T[col, head] += C_hat^T[col, slot] P^T[slot, head], transposed operand from LDS.
      // Lane i of each 16-lane group points at row 4g + i/4, columns 4(i%4)..+3 of the column
      // tile; the transposing read hands lane i the four rows of column i.
      const uint16_t* trow = sTw + (4 * g + (l16 >> 2)) * C::TS + 4 * (l16 & 3);
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) {
        const short4_t ct = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(trow + 16 * mt));
        ws.acc_o[mt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ct, pb, ws.acc_o[mt], 0, 0, 0);
      }
      base += cm.step;
    }
  }
}

// Merge: every wavefront publishes (m, l, o) as it stands; the workgroup then sums the WPT copies
// of each head with weights 2^(m_w - m*) and writes the piece's partial.  The caller has made sure
// (barrier) that nobody still uses the LDS body, which sO aliases.
template <class C>
__device__ __forceinline__ void merge_store(const WaveState<C>& ws, float* sO, float* sM, float* sL, float* part_o,
                                            float* part_ml, size_t piece, int n_heads, int tid, int wv, int l16,
                                            int g) {
  const float l_head = ws.l_total();
  if (g == 0) {
    sM[wv * 16 + l16] = ws.m_ref;
    sL[wv * 16 + l16] = l_head;
  }
  {
    float* dst = sO + (size_t)(wv * 16 + l16) * C::OS + 4 * g;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) *reinterpret_cast<float4_t*>(dst + 16 * mt) = ws.acc_o[mt];
  }
  __syncthreads();
  const size_t pbase = piece * n_heads;
  constexpr int R4 = C::R / 4;
  for (int idx = tid; idx < n_heads * R4; idx += kBlock) {
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
    *reinterpret_cast<float4_t*>(part_o + (pbase + h) * C::R + 4 * c4) = o;
    if (c4 == 0) {
      part_ml[(pbase + h) * 2 + 0] = mstar;
      part_ml[(pbase + h) * 2 + 1] = lstar;
    }
  }
}

// Query operand [q~ | q^R] of sequence b, hi and lo planes: registers (lane = head 16*ht + l16,
// elements 32kk + 8g .. +7) or LDS rows [plane][head].  Padded heads duplicate the last real
// head and are never stored.  For LDS the fetch is split in two: query_request brings every piece
// of the thread into registers (one round trip, may be issued long before the LDS rows are
// free), query_commit stores them.
template <class C, bool QL>
struct QueryRegs {
  static constexpr int chunks = C::E / 8, total = 2 * C::HP * chunks;
  static constexpr int n = QL ? (total + kBlock - 1) / kBlock : 2 * C::KT;
  uint4 r[n];
};

template <class C, bool QL>
__device__ __forceinline__ void query_request(QueryRegs<C, QL>& q, const uint16_t* qbase, size_t plane, int n_heads,
                                              int ht, int tid, int l16, int g) {
  using Q = QueryRegs<C, QL>;
  if (!QL) {
    const int h = 16 * ht + l16 < n_heads ? 16 * ht + l16 : n_heads - 1;
#pragma unroll
    for (int kk = 0; kk < C::KT; ++kk) {
      q.r[QL ? 0 : kk] = *reinterpret_cast<const uint4*>(qbase + (size_t)h * C::E + 8 * g + 32 * kk);
      q.r[QL ? 0 : C::KT + kk] = *reinterpret_cast<const uint4*>(qbase + plane + (size_t)h * C::E + 8 * g + 32 * kk);
    }
  } else {
#pragma unroll
    for (int i = 0; i < Q::n; ++i) {
      const int idx = tid + i * kBlock;
      const int pl = idx / (C::HP * Q::chunks), rem = idx - pl * C::HP * Q::chunks;
      const int hh = rem / Q::chunks, c8 = rem - hh * Q::chunks;
      const int h = hh < n_heads ? hh : n_heads - 1;
      if (idx < Q::total) q.r[i] = *reinterpret_cast<const uint4*>(qbase + pl * plane + (size_t)h * C::E + c8 * 8);
    }
  }
}

template <class C, bool QL>
__device__ __forceinline__ void query_commit(const QueryRegs<C, QL>& q, uint16_t* sQ, int tid) {
  using Q = QueryRegs<C, QL>;
  if (QL) {
#pragma unroll
    for (int i = 0; i < Q::n; ++i) {
      const int idx = tid + i * kBlock;
      const int pl = idx / (C::HP * Q::chunks), rem = idx - pl * C::HP * Q::chunks;
      const int hh = rem / Q::chunks, c8 = rem - hh * Q::chunks;
      if (idx < Q::total) *reinterpret_cast<uint4*>(sQ + (pl * C::HP + hh) * C::QS + c8 * 8) = q.r[i];
    }
  }
}

}  // namespace

}  // namespace mtla
