// bf16 matrix-core decode attention over the cache slots (gfx950).
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
//     elements of the contraction), so the logits need no staging at all; the
//     query comes as two bf16 planes (hi + lo, an almost-fp32 value), one MFMA
//     chain each, so the only rounding left in the logits is the cache's own;
//   * S^T leaves the matrix core with lane = head column and 4 consecutive slots
//     per lane, which is exactly the B-operand layout of the K=16 bf16 MFMA, so
//     the probabilities never leave registers;
//   * the latent part of the tile is parked in a wavefront-private LDS region
//     and read back transposed (ds_read_b64_tr_b16) as the C_hat^T operand.
// At the end of a piece every wavefront drops its unnormalised state into LDS
// and the whole workgroup sums the copies into one partial (m, l, o[r]) per
// (piece, head).
//
// Where this file is used: the static schedule below is the decode kernel for small batches; for
// large or ragged batches and for the parallel form the column-split kernels take over whenever
// r >= 128, and the balanced and per-row kernels of this file remain for r = 64.
//
// Two schedules share that inner loop:
//   static    grid (chunks, sequences): workgroup (c, b) scans slots
//             [c*chunk, (c+1)*chunk) of sequence b.  For decode at small batch,
//             where a wavefront sees a tile or two and the kernel is all latency:
//             a single wavefront issues at most one instruction every four
//             cycles, so the code is kept short -- one round trip to memory for
//             everything whose address does not depend on the sequence length,
//             hardware bf16 conversion and exp2, a fixed softmax reference per
//             wavefront instead of a running maximum (no accumulator rescaling and no
//             cross-lane traffic on the hot path), and a single-pass merge.
//   balanced  one persistent workgroup per compute unit.  The tiles of all
//             sequences form one flat list that is cut into equal ranges, so
//             ragged batches keep every compute unit streaming until the end; a
//             workgroup emits one partial per sequence its range touches.
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
// PG: paged storage (decode only): lat / key are the pool, and the tile's page comes out of the sequence's
// page-table row with one wavefront-uniform (scalar) load, clamped into the pool.
template <class C, bool SH = false, bool PG = false>
__device__ __forceinline__ void load_tile(TileRegs<C>& t, const uint16_t* lat, const uint16_t* key, int base,
                                          int last, int l16, int g, const Cols& cm,
                                          const SharedPrefix& sp = SharedPrefix{0, 0, 0},
                                          const PageRow& pr = PageRow{nullptr, 0, 0}) {
  const int slot = cm.row(base + l16 < last ? base + l16 : last);
  size_t row = (size_t)slot;
  if constexpr (PG) {
    const int s0 = __builtin_amdgcn_readfirstlane(base < last ? base : last);  // the tile, or the one every lane clamps to
    int pg = load_uniform_i32(pr.pt, s0 >> pr.shift);
    pg = pg < 0 ? 0 : (pg < pr.n_pages ? pg : pr.n_pages - 1);
    row = ((size_t)pg << pr.shift) + (size_t)(slot & ((1 << pr.shift) - 1));
  }
  const uint16_t* cr = lat + row * C::R + 8 * g;
  const uint16_t* kr = key + row * C::DR + 8 * g;
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
  PageRow pr = PageRow{nullptr, 0, 0};  // paged storage: the next run's page-table row
};

template <class C, int NS, int QM, bool SH = false, bool PG = false>  // SH: `sp` applies to this run and to the next one (same sequence)
__device__ __forceinline__ void stream_tiles(TileRegs<C> (&tl)[NS], const uint4 (&qv)[QRegCount<C, QM>::value],
                                             const uint16_t* qrow, uint16_t* sTw, const uint16_t* lat,
                                             const uint16_t* key, int base, int k1, int l16, int g,
                                             const Cols& cm, WaveState<C>& ws, const NextRun& nx,
                                             const SharedPrefix& sp = SharedPrefix{0, 0, 0},
                                             const PageRow& pr = PageRow{nullptr, 0, 0}) {
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
      load_tile<C, SH, PG>(t, tail ? nx.lat : lat, tail ? nx.key : key, tail ? nx.base + st * cm.step : base + NS * cm.step,
                           tail ? nx.last : k1 - 1, l16, g, cm, sp, tail ? nx.pr : pr);

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

// ---------------------------------------------------------------------------
// static schedule
// NHT = number of 16-head tiles.  With two head tiles the wavefronts split into two pairs, one
// per head tile, each pair striding over all 16-slot tiles of the chunk (a tile is then fetched
// by one wavefront of each pair; the second fetch is served by the cache hierarchy).  One head
// tile per wavefront keeps the output accumulators (r/16 x 4 registers) resident.
// NS = tiles in flight per wavefront.  QL = the query operand lives in LDS instead of registers:
// with r = 512 the registers are needed for the accumulators and the tiles in flight.
// ---------------------------------------------------------------------------
// SH: the sequence may read its first slots from another sequence's rows (a.prefix_owner, a.prefix_slots).
// PG: paged storage (a.pages): a.lat / a.key are the pool, the sequence's rows are found through its page-table row.
template <int R, int DR, int NHT, int NS, bool QL, bool SH, bool PG>
__global__ __launch_bounds__(kBlock) void attn_mfma_kernel(AttnArgs a) {
  using C = MfmaCfg<R, DR, NHT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* sT = reinterpret_cast<uint16_t*>(smem);
  float* sO = reinterpret_cast<float*>(smem);  // aliases sT (and sQ) after the main loop
  uint16_t* sQ = reinterpret_cast<uint16_t*>(smem + C::tile_bytes);  // QL only
  float* sM = reinterpret_cast<float*>(smem + C::body_bytes(QL));   // [kWaves][16]
  float* sL = sM + kWaves * 16;

  const int split = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int ht = wv / C::WPT, wl = wv - ht * C::WPT;  // head tile of this wavefront, rank inside it
  const int k0 = split * a.chunk;
  const uint16_t* lat = reinterpret_cast<const uint16_t*>(a.lat) + (PG ? 0 : (size_t)b * a.max_slots * R);
  const uint16_t* key = reinterpret_cast<const uint16_t*>(a.key) + (PG ? 0 : (size_t)b * a.max_slots * DR);
  const PageRow pr{PG ? a.pages.table + (size_t)b * a.pages.max_pages : nullptr, a.pages.shift, a.pages.n_pages};

  // Everything whose address does not depend on the sequence length is requested before the
  // length is looked at: the length, the query operand and this wavefront's first NS tiles (any
  // slot below max_slots is readable memory) travel together, one round trip instead of three.
  const int len = a.seq_len[b];
  SharedPrefix sp{0, 0, 0};
  if constexpr (SH) {  // one more round trip before the first tiles; both values clamped, so that every
                       // address stays inside the caches whatever the two arrays hold
    int owner = a.prefix_owner[b], n = a.prefix_slots[b];
    owner = owner < 0 ? 0 : (owner < a.prefix_rows ? owner : a.prefix_rows - 1);
    sp.n = n < 0 ? 0 : (n < a.max_slots ? n : a.max_slots);
    sp.dlat = (long long)(owner - b) * a.max_slots * R;
    sp.dkey = (long long)(owner - b) * a.max_slots * DR;
  }
  TileRegs<C> tl[NS];
  const int base = k0 + wl * kTile;
  const Cols cm{C::kStep, 0, 0, 0};
#pragma unroll
  for (int st = 0; st < NS; ++st) load_tile<C, SH, PG>(tl[st], lat, key, base + st * C::kStep, a.max_slots - 1, l16, g, cm, sp, pr);
  QueryRegs<C, QL> qr;
  query_request<C, QL>(qr, reinterpret_cast<const uint16_t*>(a.qcat) + (size_t)b * a.n_heads * C::E, a.q_plane,
                       a.n_heads, ht, tid, l16, g);
  const int live = (len + a.stride - 1) / a.stride;
  const int k1 = live < k0 + a.chunk ? live : k0 + a.chunk;
  if (k0 >= k1) return;
  query_commit<C, QL>(qr, sQ, tid);
  if (QL) __syncthreads();
  const uint4 (&qv)[QL ? 1 : 2 * C::KT] = reinterpret_cast<const uint4 (&)[QL ? 1 : 2 * C::KT]>(qr.r);
#pragma unroll
  for (int st = 0; st < NS; ++st)  // the first tiles may have touched rows that were never written
    tl[st].select_live(base + st * C::kStep + l16 < k1);

  WaveState<C> ws;
  ws.reset();
  stream_tiles<C, NS, QL ? kQLds : kQRegs, SH, PG>(tl, qv, sQ + (16 * ht + l16) * C::QS + 8 * g, sT + wv * kTile * C::TS,
                                                   lat, key, base, k1, l16, g, cm, ws, NextRun{lat, key, k1, k1 - 1, pr}, sp, pr);
  __syncthreads();  // every wavefront is done with its tile region (and the query), which sO aliases
  merge_store<C>(ws, sO, sM, sL, a.part_o, a.part_ml, (size_t)b * a.n_splits + split, a.n_heads, tid, wv, l16, g);
}

// ---------------------------------------------------------------------------
// balanced schedule: gridDim.x persistent workgroups, one flat list of tiles.
// Sequence b owns tiles [pre[b], pre[b+1]) with pre the running sum of ceil(live_b / 16);
// workgroup i takes tiles [i*S, (i+1)*S), S = ceil(total / gridDim.x), and emits partial
// number i + b for every sequence b its range touches (ids never collide: moving to the next
// workgroup or to the next sequence both advance the id).  Workgroup 0 publishes pre[] so the
// combine kernel can find each sequence's partials.
// ---------------------------------------------------------------------------
template <int R, int DR, int NHT, int NS, bool QL>
__global__ __launch_bounds__(kBlock) void attn_mfma_balanced_kernel(AttnArgs a) {
  using C = MfmaCfg<R, DR, NHT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* sT = reinterpret_cast<uint16_t*>(smem);
  float* sO = reinterpret_cast<float*>(smem);
  uint16_t* sQ = reinterpret_cast<uint16_t*>(smem + C::tile_bytes);
  float* sM = reinterpret_cast<float*>(smem + C::body_bytes(QL));
  float* sL = sM + kWaves * 16;
  int* sPre = reinterpret_cast<int*>(smem + C::body_bytes(QL) + C::ml_bytes);  // [batch + 1]
  int* sLive = sPre + a.batch + 1;                                             // [batch] live slots
  int* sScan = sLive + a.batch;                                                // [kBlock]

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int ht = wv / C::WPT, wl = wv - ht * C::WPT;
  const int B = a.batch;

  // ---- pre[]: every thread sums a contiguous run of sequences, the run totals are scanned
  const int per = (B + kBlock - 1) / kBlock;
  const int b_lo = tid * per, b_hi = b_lo + per < B ? b_lo + per : B;
  int run = 0;
  for (int bb = b_lo; bb < b_hi; ++bb) run += ((a.seq_len[bb] + a.stride - 1) / a.stride + kTile - 1) / kTile;
  sScan[tid] = run;
  __syncthreads();
  for (int off = 1; off < kBlock; off <<= 1) {  // inclusive Hillis-Steele scan over the 256 run totals
    const int v = tid >= off ? sScan[tid - off] : 0;
    __syncthreads();
    sScan[tid] += v;
    __syncthreads();
  }
  {
    int acc = tid ? sScan[tid - 1] : 0;
    for (int bb = b_lo; bb < b_hi; ++bb) {
      const int lv = (a.seq_len[bb] + a.stride - 1) / a.stride;
      sPre[bb] = acc;
      sLive[bb] = lv;
      acc += (lv + kTile - 1) / kTile;
    }
    if (tid == kBlock - 1) sPre[B] = sScan[kBlock - 1];
  }
  __syncthreads();
  const int total = sPre[B];
  if (blockIdx.x == 0)
    for (int bb = tid; bb <= B; bb += kBlock) a.tile_prefix[bb] = sPre[bb];
  const int share = (total + (int)gridDim.x - 1) / (int)gridDim.x;
  int pos = blockIdx.x * share;
  const int end = pos + share < total ? pos + share : total;
  if (pos >= end) return;

  // ---- first sequence of the range: last b with pre[b] <= pos (sequences without tiles are skipped)
  int b;
  {
    int lo = 0, hi = B;  // invariant: pre[lo] <= pos < pre[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (sPre[mid] <= pos) lo = mid; else hi = mid;
    }
    b = lo;
  }
  uint16_t* sTw = sT + wv * kTile * C::TS;
  const uint16_t* qrow = sQ + (16 * ht + l16) * C::QS + 8 * g;
  const uint16_t* lat_all = reinterpret_cast<const uint16_t*>(a.lat);
  const uint16_t* key_all = reinterpret_cast<const uint16_t*>(a.key);
  const uint16_t* q_all = reinterpret_cast<const uint16_t*>(a.qcat);
  const Cols cm{C::kStep, 0, 0, 0};

  // The workgroup's range is a chain of runs, one per sequence it touches.  The tile stream never
  // drains between them: while a run's last tiles are in the matrix cores the refills already
  // fetch the first tiles of the next run, and the next query is requested before the merge of
  // the finished run, so the only latency a run exposes is the first one's.
  struct Run {
    int b, k0, k1, seg_end;
  };
  auto run_at = [&](int p, int& bb) {  // run starting at flat tile p (p < end); bb: sequence hint
    while (sPre[bb + 1] <= p) ++bb;    // skip sequences that own no tile
    Run r;
    r.b = bb;
    r.seg_end = end < sPre[bb + 1] ? end : sPre[bb + 1];
    const int live = sLive[bb];
    r.k0 = (p - sPre[bb]) * kTile;
    r.k1 = live < (r.seg_end - sPre[bb]) * kTile ? live : (r.seg_end - sPre[bb]) * kTile;
    return r;
  };
  Run cur = run_at(pos, b);
  TileRegs<C> tl[NS];
  QueryRegs<C, QL> qr;
  {
    const uint16_t* lat = lat_all + (size_t)cur.b * a.max_slots * R;
    const uint16_t* key = key_all + (size_t)cur.b * a.max_slots * DR;
#pragma unroll
    for (int st = 0; st < NS; ++st)
      load_tile(tl[st], lat, key, cur.k0 + wl * kTile + st * C::kStep, cur.k1 - 1, l16, g, cm);
    query_request<C, QL>(qr, q_all + (size_t)cur.b * a.n_heads * C::E, a.q_plane, a.n_heads, ht, tid, l16, g);
  }
  while (true) {
    const uint16_t* lat = lat_all + (size_t)cur.b * a.max_slots * R;
    const uint16_t* key = key_all + (size_t)cur.b * a.max_slots * DR;
    const int base = cur.k0 + wl * kTile;
    const bool more = cur.seg_end < end;
    Run nxt = cur;
    NextRun nx{lat, key, cur.k1, cur.k1 - 1};  // no next run: dead refills clamp to a live row
    if (more) {
      nxt = run_at(cur.seg_end, b);
      nx.lat = lat_all + (size_t)nxt.b * a.max_slots * R;
      nx.key = key_all + (size_t)nxt.b * a.max_slots * DR;
      nx.base = nxt.k0 + wl * kTile;
      nx.last = nxt.k1 - 1;
    }
    query_commit<C, QL>(qr, sQ, tid);
    if (QL) __syncthreads();

    WaveState<C> ws;
    ws.reset();
    const uint4 (&qv)[QL ? 1 : 2 * C::KT] = reinterpret_cast<const uint4 (&)[QL ? 1 : 2 * C::KT]>(qr.r);
    stream_tiles<C, NS, QL ? kQLds : kQRegs>(tl, qv, qrow, sTw, lat, key, base, cur.k1, l16, g, cm, ws, nx);
    if (more) {
      if (base >= cur.k1) {  // this wavefront had no tile in the run: nothing was prefetched for it
#pragma unroll
        for (int st = 0; st < NS; ++st) load_tile(tl[st], nx.lat, nx.key, nx.base + st * C::kStep, nx.last, l16, g, cm);
      }
      query_request<C, QL>(qr, q_all + (size_t)nxt.b * a.n_heads * C::E, a.q_plane, a.n_heads, ht, tid, l16, g);
    }
    __syncthreads();  // tile regions and the query are free: sO aliases them
    merge_store<C>(ws, sO, sM, sL, a.part_o, a.part_ml, (size_t)blockIdx.x + cur.b, a.n_heads, tid, wv, l16, g);
    if (!more) break;
    __syncthreads();  // the merge buffer has been read: the next run may overwrite it
    cur = nxt;
  }
}

// ---------------------------------------------------------------------------
// parallel (prefill / training) form: one wavefront per (query row, 16-head tile).
// Row m of a sequence attends the final states of the m/s chunks before its own and its own
// running state C_hat'[m] -- the columns the stride-aware causal mask leaves open -- so the
// wavefront streams columns 0 .. m/s through the same two contractions as the decode pass, with
// the column -> row map of `Cols` standing in for the mask (nothing masked is ever computed).
// The kernel reads C_hat' [B, T, r] and the uncompressed keys [B, T, d_R] and writes one
// unnormalised partial per (row, head), which the combine kernel normalises and up-projects.
// grid = (ceil(T / rows per workgroup), B); the wavefronts of a workgroup take consecutive rows,
// so they walk almost the same columns and share them through the cache hierarchy.
// ---------------------------------------------------------------------------
template <int R, int DR, int NHT, int NS>
__global__ __launch_bounds__(kBlock) void attn_mfma_rows_kernel(AttnArgs a) {
  using C = MfmaCfg<R, DR, NHT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* sT = reinterpret_cast<uint16_t*>(smem);
  uint16_t* sQlo = reinterpret_cast<uint16_t*>(smem + C::tile_bytes);  // [kWaves][16][QS] lo plane

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int ht = wv % NHT, b = blockIdx.y;
  const int m = blockIdx.x * C::WPT + wv / NHT;  // WPT = rows per workgroup here
  if (m >= a.T) return;
  if (a.seq_len && m >= a.seq_len[b]) return;  // padding row: the combine kernel writes zeros

  const uint16_t* lat = reinterpret_cast<const uint16_t*>(a.lat) + (size_t)b * a.T * R;
  const uint16_t* key = reinterpret_cast<const uint16_t*>(a.key) + (size_t)b * a.T * DR;
  const int n_cols = m / a.stride + 1;
  const Cols cm{kTile, a.stride, n_cols - 1, m};
  TileRegs<C> tl[NS];
#pragma unroll
  for (int st = 0; st < NS; ++st) load_tile(tl[st], lat, key, st * kTile, n_cols - 1, l16, g, cm);

  // query planes of head 16*ht + l16: hi stays in registers, lo goes through this wavefront's
  // LDS rows (each lane reads back exactly the pieces it stored)
  const size_t rowg = (size_t)b * a.T + m;
  const int h = 16 * ht + l16 < a.n_heads ? 16 * ht + l16 : a.n_heads - 1;
  const uint16_t* qsrc = reinterpret_cast<const uint16_t*>(a.qcat) + (rowg * a.n_heads + h) * C::E + 8 * g;
  uint16_t* qlo = sQlo + (wv * 16 + l16) * C::QS + 8 * g;
  uint4 qv[C::KT];
#pragma unroll
  for (int kk = 0; kk < C::KT; ++kk) {
    qv[kk] = *reinterpret_cast<const uint4*>(qsrc + 32 * kk);
    *reinterpret_cast<uint4*>(qlo + 32 * kk) = *reinterpret_cast<const uint4*>(qsrc + a.q_plane + 32 * kk);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();

  WaveState<C> ws;
  ws.reset();
  stream_tiles<C, NS, kQMixed>(tl, qv, qlo, sT + wv * kTile * C::TS, lat, key, 0, n_cols, l16, g, cm, ws,
                              NextRun{lat, key, n_cols, n_cols - 1});

  const float l_head = ws.l_total();
  if (16 * ht + l16 < a.n_heads) {  // lane holds head h, columns 16mt + 4g .. +3 of every column tile
    float* po = a.part_o + (rowg * a.n_heads + h) * R + 4 * g;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) *reinterpret_cast<float4_t*>(po + 16 * mt) = ws.acc_o[mt];
    if (g == 0) {
      a.part_ml[(rowg * a.n_heads + h) * 2 + 0] = ws.m_ref;
      a.part_ml[(rowg * a.n_heads + h) * 2 + 1] = l_head;
    }
  }
}

template <int R, int DR, int NHT, int NS>
hipError_t launch_rows(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  using C = MfmaCfg<R, DR, NHT>;
  constexpr size_t smem = C::tile_bytes + (size_t)kWaves * 16 * C::QS * 2;
  static_assert(smem <= 160 * 1024, "LDS budget of one compute unit");
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_rows_kernel<R, DR, NHT, NS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const dim3 grid((a.T + C::WPT - 1) / C::WPT, a.batch);
  launch_timed(attn_mfma_rows_kernel<R, DR, NHT, NS>, grid, dim3(kBlock), smem, st, ev, a);
  return hipGetLastError();
}

template <int R, int DR, int NHT, int NS, bool QL, bool SH, bool PG>
hipError_t launch_static(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  using C = MfmaCfg<R, DR, NHT>;
  constexpr size_t smem = C::body_bytes(QL) + C::ml_bytes;
  static_assert(smem <= 160 * 1024, "LDS budget of one compute unit");
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<R, DR, NHT, NS, QL, SH, PG>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  launch_timed(attn_mfma_kernel<R, DR, NHT, NS, QL, SH, PG>, dim3(a.n_splits, a.batch), dim3(kBlock), smem, st, ev, a);
  return hipGetLastError();
}

template <int R, int DR, int NHT, int NS, bool QL>
hipError_t launch_one(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  using C = MfmaCfg<R, DR, NHT>;
  if (a.n_persistent > 0) {
    if (a.prefix_owner || a.pages.table) return hipErrorInvalidValue;  // shared prefixes, pages: static schedule or the column-split kernel
    const size_t smem = C::body_bytes(QL) + C::ml_bytes + (size_t)(2 * a.batch + 1 + kBlock) * sizeof(int);
    if (smem > 160 * 1024) return hipErrorInvalidValue;
    static bool attr_set = false;  // LDS above the 64 KB default needs an explicit opt-in, once
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_balanced_kernel<R, DR, NHT, NS, QL>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    launch_timed(attn_mfma_balanced_kernel<R, DR, NHT, NS, QL>, dim3(a.n_persistent), dim3(kBlock), smem, st, ev, a);
    return hipGetLastError();
  }
  if (a.pages.table) return a.prefix_owner ? hipErrorInvalidValue : launch_static<R, DR, NHT, NS, QL, false, true>(a, st, ev);
  return a.prefix_owner ? launch_static<R, DR, NHT, NS, QL, true, false>(a, st, ev)
                        : launch_static<R, DR, NHT, NS, QL, false, false>(a, st, ev);
}

// Pipeline depth: a wavefront that will see only a tile or two (decode at small batch) gets the
// short single-stage code with the query in registers; long runs keep several tiles in flight
// per wavefront, which is what it takes to cover HBM latency with four wavefronts per compute
// unit.
template <int R, int DR>
hipError_t launch_rd(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  constexpr int kDeep = R >= 512 ? 2 : 3;  // what the 512-register budget per lane allows
  constexpr bool kDeepQL = R >= 512;
  const int nht = a.n_heads <= 16 ? 1 : 2;
  const int tiles_per_wave = a.chunk / (kTile * (kWaves / nht));
  const bool deep = a.n_persistent > 0 || tiles_per_wave >= 2 * kDeep;
  if (nht == 1)
    return deep ? launch_one<R, DR, 1, kDeep, kDeepQL>(a, st, ev) : launch_one<R, DR, 1, 1, false>(a, st, ev);
  return deep ? launch_one<R, DR, 2, kDeep, kDeepQL>(a, st, ev) : launch_one<R, DR, 2, 1, false>(a, st, ev);
}

}  // namespace

bool attn_mfma_supported(const AttnArgs& a) {
  return a.n_heads <= 32 && a.batch <= 65535 && (a.r == 64 || a.r == 128 || a.r == 256 || a.r == 512) &&
         (a.d_rope == 32 || a.d_rope == 64);
}

hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
#define MTLA_CASE(RR, DD)                                                                       \
  if (a.r == RR && a.d_rope == DD) {                                                            \
    if (a.T == 0) return launch_rd<RR, DD>(a, st, ev);                                              \
    return a.n_heads <= 16 ? launch_rows<RR, DD, 1, 2>(a, st, ev) : launch_rows<RR, DD, 2, 2>(a, st, ev); \
  }
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
