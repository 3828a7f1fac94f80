// bf16 matrix-core decode attention for large or ragged batches: persistent workgroups whose
// four wavefronts split the LATENT COLUMNS of every cache tile instead of the slots (gfx950).
//
// Eq. (with-rope), incremental case, per 16-slot tile and 16-head tile:
//     S^T[slot, head] = sum over columns of [C_hat | K_hat^R][slot, :] . [q~ | q^R][head, :]
//     O^T[col,  head] += C_hat^T[col, slot] . P^T[slot, head]
// Wavefront w owns latent columns [w r/4, (w+1) r/4) and a quarter of the RoPE columns.  Both
// contractions then need only that slice of a cache row: the wavefront contracts its columns
// into a partial S (the four partials meet in LDS, one small exchange and one barrier per tile),
// every wavefront forms the same softmax weights, and the PV product yields exactly the output
// columns the wavefront owns.  Compared with giving each wavefront its own slots this
//   * loads every cache byte once per workgroup whatever the number of heads (two head tiles
//     reuse the slice from registers),
//   * needs a quarter of the output accumulators and of the query operand per wavefront, so
//     the query stays in registers and many more tiles can be in flight,
//   * ends a sequence without any cross-wavefront merge: each wavefront stores its own columns
//     of the partial, and the next sequence's query is already in registers.
// Scheduling is the balanced one: the 16-slot tiles of all sequences form one flat list cut into
// equal ranges, one per persistent workgroup; a workgroup emits partial number i + b for every
// sequence b its range touches, and the tile stream never drains between sequences.
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef short4_t __attribute__((address_space(3))) * lds_short4_ptr;

constexpr int kWaves = kBlock / kWave;
constexpr int kTile = 16;  // slots per tile

template <int R_, int DR_, int NHT_>
struct ColCfg {
  static constexpr int R = R_, DR = DR_, NHT = NHT_;
  static constexpr int E = R + DR;
  static constexpr int RW = R / kWaves;    // latent columns of one wavefront
  static constexpr int KC = RW / 32;       // its K steps over the latent part
  static constexpr int KQ = KC + 1;        // plus one K step holding its RoPE columns (rest zero)
  static constexpr int DRW = DR / kWaves;  // RoPE columns of one wavefront: 8 or 16
  static constexpr int MT = RW / 16;       // its output column tiles
  static constexpr int TS = RW + 16;       // LDS row stride of the parked slice (bf16 elements)
  static_assert(RW % 32 == 0 && (DRW == 8 || DRW == 16), "column split needs r >= 128 and d_R in {32, 64}");
  static constexpr size_t park_bytes = (size_t)kWaves * kTile * TS * 2;
  static constexpr size_t s_bytes = (size_t)2 * kWaves * NHT * kWave * 16;  // two buffers of partial S
};

template <class C>
struct SliceRegs {
  uint4 xc[C::KC], xr;
};

// Slots base + l16 (clamped to `last`, a live slot): lane (l16, g) takes elements 32kk + 8g .. +7
// of the wavefront's latent columns and 8 of its RoPE columns (lanes whose g has no RoPE column
// fetch a duplicate; the query operand is zero there).
template <class C>
__device__ __forceinline__ void load_slice(SliceRegs<C>& t, const uint16_t* lat, const uint16_t* key, int base,
                                           int last, int l16, int g, int wv) {
  const int slot = base + l16 < last ? base + l16 : last;
  const uint16_t* cr = lat + (size_t)slot * C::R + wv * C::RW + 8 * g;
#pragma unroll
  for (int kk = 0; kk < C::KC; ++kk) t.xc[kk] = *reinterpret_cast<const uint4*>(cr + 32 * kk);
  t.xr = *reinterpret_cast<const uint4*>(key + (size_t)slot * C::DR + wv * C::DRW + (8 * g < C::DRW ? 8 * g : 0));
}

// The wavefront's columns of [q~ | q^R] for head 16*ht + l16, hi and lo planes.
template <class C>
struct QSlice {
  uint4 hi[C::NHT][C::KQ], lo[C::NHT][C::KQ];
};

template <class C>
__device__ __forceinline__ void load_query_slice(QSlice<C>& q, const uint16_t* qbase, size_t plane, int n_heads,
                                                 int l16, int g, int wv) {
#pragma unroll
  for (int ht = 0; ht < C::NHT; ++ht) {
    const int h = 16 * ht + l16 < n_heads ? 16 * ht + l16 : n_heads - 1;  // padded heads: never stored
    const uint16_t* src = qbase + (size_t)h * C::E + wv * C::RW + 8 * g;
#pragma unroll
    for (int kk = 0; kk < C::KC; ++kk) {
      q.hi[ht][kk] = *reinterpret_cast<const uint4*>(src + 32 * kk);
      q.lo[ht][kk] = *reinterpret_cast<const uint4*>(src + plane + 32 * kk);
    }
    const bool has = 8 * g < C::DRW;
    const uint16_t* rs = qbase + (size_t)h * C::E + C::R + wv * C::DRW + (has ? 8 * g : 0);
    const uint4 rh = *reinterpret_cast<const uint4*>(rs), rl = *reinterpret_cast<const uint4*>(rs + plane);
    const uint32_t m = has ? 0xffffffffu : 0u;
    q.hi[ht][C::KC] = make_uint4(rh.x & m, rh.y & m, rh.z & m, rh.w & m);
    q.lo[ht][C::KC] = make_uint4(rl.x & m, rl.y & m, rl.z & m, rl.w & m);
  }
}

template <class C>
struct ColState {  // m_ref: identical in all four wavefronts; l_run: this lane's slots only (the
                   // lanes sharing a head are summed when the run ends); acc_o: this wavefront's columns
  float m_ref[C::NHT], l_run[C::NHT];
  float4_t acc_o[C::NHT][C::MT];
  __device__ __forceinline__ void reset() {
#pragma unroll
    for (int ht = 0; ht < C::NHT; ++ht) {
      m_ref[ht] = -INFINITY;
      l_run[ht] = 0.f;
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) acc_o[ht][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
    }
  }
};

struct NextCols {  // where the stream continues after the current run (see the kernel)
  const uint16_t* lat;
  const uint16_t* key;
  int base, last;
};

// One run: tiles base, base + 16, ... below k1 of (lat, key), all four wavefronts in step.
// tl[0..NS) hold the first NS tiles on entry and the first NS tiles of the next run on exit.
// `sbuf` is the parity of the partial-S buffer and carries over from run to run.
template <class C, int NS>
__device__ __forceinline__ void stream_cols(SliceRegs<C> (&tl)[NS], const QSlice<C>& q, uint16_t* sTw, float4_t* sS,
                                            const uint16_t* lat, const uint16_t* key, int base, int k1,
                                            const NextCols& nx, int lane, int l16, int g, int wv, int& sbuf,
                                            ColState<C>& ws) {
  const int n_iter = (k1 - base + NS * kTile - 1) / (NS * kTile);
  for (int it = 0; it < n_iter; ++it) {
    const bool tail = it == n_iter - 1;  // this pass refills from the next run
#pragma unroll
    for (int st = 0; st < NS; ++st) {
      SliceRegs<C>& t = tl[st];
      // ---- this wavefront's share of S^T[slot, head]: hi and lo query planes, one chain each
      float4_t sp[C::NHT];
#pragma unroll
      for (int ht = 0; ht < C::NHT; ++ht) {
        float4_t s0 = float4_t{0.f, 0.f, 0.f, 0.f}, s1 = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < C::KQ; ++kk) {
          const bf16x8_t x = __builtin_bit_cast(bf16x8_t, kk < C::KC ? t.xc[kk < C::KC ? kk : 0] : t.xr);
          s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, __builtin_bit_cast(bf16x8_t, q.hi[ht][kk]), s0, 0, 0, 0);
          s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, __builtin_bit_cast(bf16x8_t, q.lo[ht][kk]), s1, 0, 0, 0);
        }
        sp[ht] = s0 + s1;
      }
      // ---- publish the share; park the latent slice for the transposed PV operand
      float4_t* sSb = sS + (size_t)sbuf * kWaves * C::NHT * kWave;
#pragma unroll
      for (int ht = 0; ht < C::NHT; ++ht) sSb[(wv * C::NHT + ht) * kWave + lane] = sp[ht];
      __builtin_amdgcn_wave_barrier();  // the previous tile's transposed reads come first
#pragma unroll
      for (int kk = 0; kk < C::KC; ++kk)
        *reinterpret_cast<uint4*>(sTw + l16 * C::TS + 32 * kk + 8 * g) = t.xc[kk];

      // ---- refill this stage NS tiles ahead
      load_slice<C>(t, tail ? nx.lat : lat, tail ? nx.key : key, tail ? nx.base + st * kTile : base + NS * kTile,
                    tail ? nx.last : k1 - 1, l16, g, wv);
      __syncthreads();  // all four shares of this tile are in LDS (and this wavefront's slice)

      float4_t* sSr = sSb + lane;
      short4_t pb[C::NHT];
#pragma unroll
      for (int ht = 0; ht < C::NHT; ++ht) {
        float4_t s = sSr[(0 * C::NHT + ht) * kWave];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) s += sSr[(w * C::NHT + ht) * kWave];
        // ---- softmax weights; lane holds head l16 of head tile ht and slots 4g .. 4g+3
        float sv[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) sv[v] = (base + 4 * g + v < k1) ? s[v] : -INFINITY;
        // Weights are taken relative to a reference m_ref fixed at the run's first live tile, so
        // the hot path needs no cross-lane traffic at all: the four lanes that share a head keep
        // their own partial normaliser (summed at the end of the run), and the tile maximum is
        // only formed on the two cold paths -- fixing the reference, and re-basing when a tile
        // tops it by more than 2^kRebase.
        constexpr float kRebase = 40.f;
        const float mloc = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
        if (__any(ws.m_ref[ht] == -INFINITY || mloc - ws.m_ref[ht] > kRebase)) {
          float mt_ = fmaxf(mloc, __shfl_xor(mloc, 16, kWave));
          mt_ = fmaxf(mt_, __shfl_xor(mt_, 32, kWave));
          if (ws.m_ref[ht] == -INFINITY) {
            ws.m_ref[ht] = mt_;  // still -inf if the tile is dead
          } else if (mt_ - ws.m_ref[ht] > kRebase) {
            const float alpha = __builtin_amdgcn_exp2f(ws.m_ref[ht] - mt_);
            ws.m_ref[ht] = mt_;
            ws.l_run[ht] *= alpha;
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) ws.acc_o[ht][mt] *= alpha;
          }
        }
        const float m_sub = ws.m_ref[ht] == -INFINITY ? 0.f : ws.m_ref[ht];
        float p[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) p[v] = __builtin_amdgcn_exp2f(sv[v] - m_sub);
        // weights as bf16 (hardware round-to-nearest-even); the normaliser sums the rounded values
        const uint32_t p01 = pack_bf16x2(p[0], p[1]), p23 = pack_bf16x2(p[2], p[3]);
        pb[ht] = __builtin_bit_cast(short4_t, make_uint2(p01, p23));
        ws.l_run[ht] += (__uint_as_float(p01 << 16) + __uint_as_float(p01 & 0xffff0000u)) +
                        (__uint_as_float(p23 << 16) + __uint_as_float(p23 & 0xffff0000u));
      }
      // ---- O^T[col, head] += C_hat^T[col, slot] P^T[slot, head] over this wavefront's columns
      const uint16_t* trow = sTw + (4 * g + (l16 >> 2)) * C::TS + 4 * (l16 & 3);
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) {
        const short4_t ct = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(trow + 16 * mt));
#pragma unroll
        for (int ht = 0; ht < C::NHT; ++ht)
          ws.acc_o[ht][mt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ct, pb[ht], ws.acc_o[ht][mt], 0, 0, 0);
      }
      sbuf ^= 1;
      base += kTile;
    }
  }
}

template <int R, int DR, int NHT, int NS, int OCC>
__global__ __launch_bounds__(kBlock, OCC) void attn_cols_kernel(AttnArgs a) {
  using C = ColCfg<R, DR, NHT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* sT = reinterpret_cast<uint16_t*>(smem);
  float4_t* sS = reinterpret_cast<float4_t*>(smem + C::park_bytes);
  int* sPre = reinterpret_cast<int*>(smem + C::park_bytes + C::s_bytes);  // [batch + 1]
  int* sLive = sPre + a.batch + 1;                                        // [batch] live slots
  int* sScan = sLive + a.batch;                                           // [kBlock]

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int B = a.batch;

  // ---- pre[]: running tile counts; every thread sums a contiguous run of sequences
  const int per = (B + kBlock - 1) / kBlock;
  const int b_lo = tid * per, b_hi = b_lo + per < B ? b_lo + per : B;
  int run = 0;
  for (int bb = b_lo; bb < b_hi; ++bb) run += ((a.seq_len[bb] + a.stride - 1) / a.stride + kTile - 1) / kTile;
  sScan[tid] = run;
  __syncthreads();
  for (int off = 1; off < kBlock; off <<= 1) {  // inclusive Hillis-Steele scan
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
  const int pos = blockIdx.x * share;
  const int end = pos + share < total ? pos + share : total;
  if (pos >= end) return;

  int b;  // first sequence of the range: last b with pre[b] <= pos
  {
    int lo = 0, hi = B;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (sPre[mid] <= pos) lo = mid; else hi = mid;
    }
    b = lo;
  }
  uint16_t* sTw = sT + wv * kTile * C::TS;
  const uint16_t* lat_all = reinterpret_cast<const uint16_t*>(a.lat);
  const uint16_t* key_all = reinterpret_cast<const uint16_t*>(a.key);
  const uint16_t* q_all = reinterpret_cast<const uint16_t*>(a.qcat);

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
  SliceRegs<C> tl[NS];
  QSlice<C> q, qn;
  {
    const uint16_t* lat = lat_all + (size_t)cur.b * a.max_slots * R;
    const uint16_t* key = key_all + (size_t)cur.b * a.max_slots * DR;
#pragma unroll
    for (int st = 0; st < NS; ++st) load_slice<C>(tl[st], lat, key, cur.k0 + st * kTile, cur.k1 - 1, l16, g, wv);
    load_query_slice<C>(q, q_all + (size_t)cur.b * a.n_heads * C::E, a.q_plane, a.n_heads, l16, g, wv);
  }
  int sbuf = 0;
  while (true) {
    const uint16_t* lat = lat_all + (size_t)cur.b * a.max_slots * R;
    const uint16_t* key = key_all + (size_t)cur.b * a.max_slots * DR;
    const bool more = cur.seg_end < end;
    Run nxt = cur;
    NextCols nx{lat, key, cur.k1, cur.k1 - 1};  // no next run: dead refills clamp to a live slot
    if (more) {
      nxt = run_at(cur.seg_end, b);
      nx.lat = lat_all + (size_t)nxt.b * a.max_slots * R;
      nx.key = key_all + (size_t)nxt.b * a.max_slots * DR;
      nx.base = nxt.k0;
      nx.last = nxt.k1 - 1;
      load_query_slice<C>(qn, q_all + (size_t)nxt.b * a.n_heads * C::E, a.q_plane, a.n_heads, l16, g, wv);
    }
    ColState<C> ws;
    ws.reset();
    stream_cols<C, NS>(tl, q, sTw, sS, lat, key, cur.k0, cur.k1, nx, lane, l16, g, wv, sbuf, ws);

    // ---- this wavefront's columns of the run's partial: lane holds head l16, columns 16mt + 4g .. +3
    const size_t piece = (size_t)blockIdx.x + cur.b;
    float l_head[NHT];
#pragma unroll
    for (int ht = 0; ht < NHT; ++ht) {
      l_head[ht] = ws.l_run[ht] + __shfl_xor(ws.l_run[ht], 16, kWave);
      l_head[ht] += __shfl_xor(l_head[ht], 32, kWave);
    }
#pragma unroll
    for (int ht = 0; ht < NHT; ++ht) {
      const int h = 16 * ht + l16;
      if (h < a.n_heads) {
        float* po = a.part_o + (piece * a.n_heads + h) * R + wv * C::RW + 4 * g;
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) *reinterpret_cast<float4_t*>(po + 16 * mt) = ws.acc_o[ht][mt];
        if (wv == 0 && g == 0) {
          a.part_ml[(piece * a.n_heads + h) * 2 + 0] = ws.m_ref[ht];
          a.part_ml[(piece * a.n_heads + h) * 2 + 1] = l_head[ht];
        }
      }
    }
    if (!more) break;
    cur = nxt;
    q = qn;
  }
}

template <int R, int DR, int NHT, int NS, int OCC>
hipError_t launch_cols(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  using C = ColCfg<R, DR, NHT>;
  const size_t smem = C::park_bytes + C::s_bytes + (size_t)(2 * a.batch + 1 + kBlock) * sizeof(int);
  if (smem > 64 * 1024) return hipErrorInvalidValue;
  launch_timed(attn_cols_kernel<R, DR, NHT, NS, OCC>, dim3(a.n_persistent), dim3(kBlock), smem, st, ev, a);
  return hipGetLastError();
}

}  // namespace

bool attn_cols_supported(const AttnArgs& a) {
  return a.T == 0 && a.n_persistent > 0 && a.n_heads <= 32 && (a.r == 128 || a.r == 256 || a.r == 512) &&
         (a.d_rope == 32 || a.d_rope == 64) && a.batch <= 4096;
}

// Persistent workgroups per compute unit.  One 16-head tile leaves room for two workgroups (two
// wavefronts per SIMD, 256 registers each), which fill each other's stalls; two head tiles need
// the whole register file.
int attn_cols_workgroups_per_cu(const AttnArgs& a) { return a.n_heads <= 16 ? 2 : 1; }

hipError_t launch_attn_cols(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  // Two tiles in flight per wavefront are enough: measured, deeper prefetch does not raise the
  // streaming rate (the memory system is the limit, not the latency a wavefront sees).
#define MTLA_CASE(RR, DD)                                                                 \
  if (a.r == RR && a.d_rope == DD)                                                        \
    return a.n_heads <= 16 ? launch_cols<RR, DD, 1, 2, 2>(a, st, ev) : launch_cols<RR, DD, 2, 2, 1>(a, st, ev);
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
