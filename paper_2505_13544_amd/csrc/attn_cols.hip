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
// Scheduling is the balanced one: the 16-slot tiles of all sequences form one flat list of work
// units (one per tile, after a.run_cost units per sequence for the fixed cost of starting on it) cut
// into equal ranges, one per persistent workgroup; a workgroup emits partial number i + b for every
// sequence b of which its range holds a tile, and the tile stream never drains between sequences.
#include "mtla_device.h"
#include "mtla_kernels.h"

#include <type_traits>

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
  static constexpr size_t park_bytes = (size_t)kWaves * kTile * TS * 2;  // one parked slice per wavefront (two when the logits run a tile ahead)
  static constexpr size_t s_bytes = (size_t)2 * kWaves * NHT * kWave * 16;  // two buffers of partial S
};

template <class C>
struct SliceRegs {
  uint4 xc[C::KC], xr;
};

// Slots base + l16 (clamped to `last`, a live slot): lane (l16, g) takes elements 32kk + 8g .. +7
// of the wavefront's latent columns and 8 of its RoPE columns (lanes whose g has no RoPE column
// fetch a duplicate; the query operand is zero there).
// PG: paged storage: lat / key are the pool, and the tile's page comes out of the sequence's page-table row
// with one wavefront-uniform (scalar) load, clamped into the pool.
// A stream walks a sequence's table entries in order, so the entry behind the one in use is requested when the
// cursor moves (a scalar load that has a whole page of tiles, at least one, to arrive): the tile's own loads
// then never wait for the table.  Anything else (a run's first tile, a clamp back to an earlier page) is
// looked up on the spot.
template <class C, bool SH = false, bool PG = false>
__device__ __forceinline__ void load_slice(SliceRegs<C>& t, const uint16_t* lat, const uint16_t* key, int base,
                                           int last, int l16, int g, int wv, const SharedPrefix& sp, PageRow& pr) {
  const int slot = base + l16 < last ? base + l16 : last;
  size_t row = (size_t)slot;
  if constexpr (PG) {
    const int s0 = __builtin_amdgcn_readfirstlane(base < last ? base : last);  // the tile, or the one every lane clamps to
    const int idx = s0 >> pr.shift;
    if (idx != pr.idx) {  // wavefront-uniform
      int pg = idx == pr.idx + 1 && pr.idx >= 0 ? pr.pg_next : load_uniform_i32(pr.pt, idx);
      pr.pg = pg < 0 ? 0 : (pg < pr.n_pages ? pg : pr.n_pages - 1);
      pr.idx = idx;
      pr.pg_next = load_uniform_i32(pr.pt, idx < pr.last_entry ? idx + 1 : pr.last_entry);
    }
    row = ((size_t)pr.pg << pr.shift) + (size_t)(slot & ((1 << pr.shift) - 1));
  }
  const uint16_t* cr = lat + row * C::R + wv * C::RW + 8 * g;
  const uint16_t* kr = key + row * C::DR + wv * C::DRW + (8 * g < C::DRW ? 8 * g : 0);
  if constexpr (SH) {
    if (slot < sp.n) {
      cr += sp.dlat;
      kr += sp.dkey;
    }
  }
#pragma unroll
  for (int kk = 0; kk < C::KC; ++kk) t.xc[kk] = *reinterpret_cast<const uint4*>(cr + 32 * kk);
  t.xr = *reinterpret_cast<const uint4*>(kr);
}

// The wavefront's columns of [q~ | q^R] for head 16*ht + l16, hi and lo planes.
template <class C>
struct QSlice {
  uint4 hi[C::NHT][C::KQ], lo[C::NHT][C::KQ];
};

// hi/lo planes of one query row's columns for this wavefront: `qhead` points at the row
// [q~ | q^R] of the head (hi plane), the lo plane lies `plane` elements further.
template <class C>
__device__ __forceinline__ void load_query_tile(uint4 (&hi)[C::KQ], uint4 (&lo)[C::KQ], const uint16_t* qhead,
                                                size_t plane, int g, int wv) {
  const uint16_t* src = qhead + wv * C::RW + 8 * g;
#pragma unroll
  for (int kk = 0; kk < C::KC; ++kk) {
    hi[kk] = *reinterpret_cast<const uint4*>(src + 32 * kk);
    lo[kk] = *reinterpret_cast<const uint4*>(src + plane + 32 * kk);
  }
  const bool has = 8 * g < C::DRW;
  const uint16_t* rs = qhead + C::R + wv * C::DRW + (has ? 8 * g : 0);
  const uint4 rh = *reinterpret_cast<const uint4*>(rs), rl = *reinterpret_cast<const uint4*>(rs + plane);
  const uint32_t m = has ? 0xffffffffu : 0u;
  hi[C::KC] = make_uint4(rh.x & m, rh.y & m, rh.z & m, rh.w & m);
  lo[C::KC] = make_uint4(rl.x & m, rl.y & m, rl.z & m, rl.w & m);
}

// decode: query tile ht = heads 16 ht .. 16 ht + 15 of the sequence whose operand rows start at qbase
template <class C>
__device__ __forceinline__ void load_query_slice(QSlice<C>& q, const uint16_t* qbase, size_t plane, int n_heads,
                                                 int l16, int g, int wv) {
#pragma unroll
  for (int ht = 0; ht < C::NHT; ++ht) {
    const int h = 16 * ht + l16 < n_heads ? 16 * ht + l16 : n_heads - 1;  // padded heads: never stored
    load_query_tile<C>(q.hi[ht], q.lo[ht], qbase + (size_t)h * C::E, plane, g, wv);
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
  SharedPrefix sp;
  PageRow pr;
};

// First half of a tile: this wavefront's share of S^T[slot, query tile] over its columns (hi and
// lo query planes, one accumulator chain each) goes to the exchange buffer, and its latent slice
// is parked for the transposed PV operand.
template <class C>
__device__ __forceinline__ void publish_share(const SliceRegs<C>& t, const QSlice<C>& q, float4_t* sSb, uint16_t* sTw,
                                              int lane, int l16, int g, int wv) {
#pragma unroll
  for (int ht = 0; ht < C::NHT; ++ht) {
    float4_t s0 = float4_t{0.f, 0.f, 0.f, 0.f}, s1 = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < C::KQ; ++kk) {
      const bf16x8_t x = __builtin_bit_cast(bf16x8_t, kk < C::KC ? t.xc[kk < C::KC ? kk : 0] : t.xr);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, __builtin_bit_cast(bf16x8_t, q.hi[ht][kk]), s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, __builtin_bit_cast(bf16x8_t, q.lo[ht][kk]), s1, 0, 0, 0);
    }
    sSb[(wv * C::NHT + ht) * kWave + lane] = s0 + s1;
  }
  __builtin_amdgcn_wave_barrier();  // the previous tile's transposed reads come first
#pragma unroll
  for (int kk = 0; kk < C::KC; ++kk) *reinterpret_cast<uint4*>(sTw + l16 * C::TS + 32 * kk + 8 * g) = t.xc[kk];
}

// Second half, after the workgroup barrier: the four shares are summed (same order in every
// wavefront, so all four hold identical logits), the softmax weights are formed and the PV
// product adds this wavefront's output columns.  vmask[ht] bit v says whether slot 4g + v of the
// tile is visible to query tile ht.
template <class C>
struct Shares {  // the four wavefronts' shares of a tile's logits, as this lane reads them
  float4_t s[C::NHT][kWaves];
};
template <class C>
__device__ __forceinline__ void read_shares(Shares<C>& sh, const float4_t* sSb, int lane) {
  const float4_t* sSr = sSb + lane;
#pragma unroll
  for (int ht = 0; ht < C::NHT; ++ht)
#pragma unroll
    for (int w = 0; w < kWaves; ++w) sh.s[ht][w] = sSr[(w * C::NHT + ht) * kWave];
}

template <class C>
__device__ __forceinline__ void finish_tile(const Shares<C>& sh, const uint16_t* sTw, const uint32_t (&vmask)[C::NHT],
                                            ColState<C>& ws, int lane, int l16, int g) {
  short4_t pb[C::NHT];
#pragma unroll
  for (int ht = 0; ht < C::NHT; ++ht) {
    float4_t s = sh.s[ht][0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) s += sh.s[ht][w];
    // ---- softmax weights; lane holds query column l16 of query tile ht and slots 4g .. 4g+3
    float sv[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) sv[v] = (vmask[ht] >> v & 1u) ? s[v] : -INFINITY;
    // Weights are taken relative to a reference m_ref fixed at the first live tile, so the hot
    // path needs no cross-lane traffic at all: the four lanes that share a query column keep
    // their own partial normaliser (summed at the end), and the tile maximum is only formed on
    // the two cold paths -- fixing the reference, and re-basing when a tile tops it by more
    // than 2^kRebase.
    constexpr float kRebase = 40.f;
    const float mloc = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    if (__any(ws.m_ref[ht] == -INFINITY || mloc - ws.m_ref[ht] > kRebase)) {
      float mt_ = fmaxf(mloc, __shfl_xor(mloc, 16, kWave));
      mt_ = fmaxf(mt_, __shfl_xor(mt_, 32, kWave));
      if (ws.m_ref[ht] == -INFINITY) {
        ws.m_ref[ht] = mt_;  // still -inf if nothing of the tile is visible
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
  // ---- O^T[col, query] += C_hat^T[col, slot] P^T[slot, query] over this wavefront's columns
  const uint16_t* trow = sTw + (4 * g + (l16 >> 2)) * C::TS + 4 * (l16 & 3);
  short4_t ct[C::MT];  // all the transposed reads are on their way before the first product waits for one
#pragma unroll
  for (int mt = 0; mt < C::MT; ++mt) ct[mt] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(trow + 16 * mt));
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
    for (int ht = 0; ht < C::NHT; ++ht)
      ws.acc_o[ht][mt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ct[mt], pb[ht], ws.acc_o[ht][mt], 0, 0, 0);
}

// One run: tiles base, base + 16, ... below k1 of (lat, key), all four wavefronts in step.
// tl[0..NS) hold the first NS tiles on entry and the first NS tiles of the next run on exit.
// `sbuf` is the parity of the partial-S buffer and carries over from run to run.
template <class C, int NS, bool SH = false, bool PG = false>
__device__ __forceinline__ void stream_cols(SliceRegs<C> (&tl)[NS], const QSlice<C>& q, uint16_t* sTw, float4_t* sS,
                                            const uint16_t* lat, const uint16_t* key, int base, int k1,
                                            NextCols& nx, int lane, int l16, int g, int wv, int& sbuf,
                                            ColState<C>& ws, const SharedPrefix& sp, PageRow& pr) {
  const int n_iter = (k1 - base + NS * kTile - 1) / (NS * kTile);
  for (int it = 0; it < n_iter; ++it) {
    const bool tail = it == n_iter - 1;  // this pass refills from the next run
#pragma unroll
    for (int st = 0; st < NS; ++st) {
      SliceRegs<C>& t = tl[st];
      float4_t* sSb = sS + (size_t)sbuf * kWaves * C::NHT * kWave;
      publish_share<C>(t, q, sSb, sTw, lane, l16, g, wv);
      // ---- refill this stage NS tiles ahead
      if constexpr (PG) {  // two page cursors: the run's own and the next run's
        if (tail) load_slice<C, SH, PG>(t, nx.lat, nx.key, nx.base + st * kTile, nx.last, l16, g, wv, nx.sp, nx.pr);
        else load_slice<C, SH, PG>(t, lat, key, base + NS * kTile, k1 - 1, l16, g, wv, sp, pr);
      } else {
        load_slice<C, SH, PG>(t, tail ? nx.lat : lat, tail ? nx.key : key, tail ? nx.base + st * kTile : base + NS * kTile,
                              tail ? nx.last : k1 - 1, l16, g, wv, tail ? nx.sp : sp, pr);
      }
      __syncthreads();  // all four shares of this tile are in LDS (and this wavefront's slice)
      uint32_t vmask[C::NHT];
      uint32_t vm = 0;
#pragma unroll
      for (int v = 0; v < 4; ++v) vm |= (base + 4 * g + v < k1 ? 1u : 0u) << v;
#pragma unroll
      for (int ht = 0; ht < C::NHT; ++ht) vmask[ht] = vm;
      Shares<C> sh;
      read_shares<C>(sh, sSb, lane);
      finish_tile<C>(sh, sTw, vmask, ws, lane, l16, g);
      sbuf ^= 1;
      base += kTile;
    }
  }
}

// The same run with the logits one tile ahead: the share of tile j + 1 is formed (and its slice parked in
// the second parking area) between the barrier that makes the shares of tile j visible and their use, so
// the matrix instructions of one tile run while the shares of the other travel from LDS, and a tile
// step is no longer the sum of the two.  One barrier per tile as before: shares and parked slices
// alternate between two areas, and what a wavefront overwrites in step j was last read in step j - 1,
// before the barrier every wavefront has passed.
template <class C, int NS, bool SH = false, bool PG = false>
__device__ __forceinline__ void stream_cols_ahead(SliceRegs<C> (&tl)[NS], const QSlice<C>& q, uint16_t* sTw, float4_t* sS,
                                                  const uint16_t* lat, const uint16_t* key, int base, int k1,
                                                  NextCols& nx, int lane, int l16, int g, int wv, int& sbuf,
                                                  ColState<C>& ws, const SharedPrefix& sp, PageRow& pr) {
  const int n_iter = (k1 - base + NS * kTile - 1) / (NS * kTile), n_all = n_iter * NS;
  const int base0 = base, sb0 = sbuf;
  constexpr size_t kShare = (size_t)kWaves * C::NHT * kWave;   // float4 per share buffer
  constexpr int kPark = kWaves * kTile * C::TS;                // elements per parking area
  // tile j of the run (stage j % NS, known at compile time): share and slice out, stage refilled NS tiles ahead
  auto publish = [&](auto st_, int j) __attribute__((always_inline)) {
    constexpr int st = decltype(st_)::value;
    SliceRegs<C>& t = tl[st];
    const int par = (sb0 ^ j) & 1;
    publish_share<C>(t, q, sS + par * kShare, sTw + par * kPark, lane, l16, g, wv);
    const bool tail = j / NS == n_iter - 1;  // refilled from the next run
    const int bj = base0 + j * kTile;
    if constexpr (PG) {
      if (tail) load_slice<C, SH, PG>(t, nx.lat, nx.key, nx.base + st * kTile, nx.last, l16, g, wv, nx.sp, nx.pr);
      else load_slice<C, SH, PG>(t, lat, key, bj + NS * kTile, k1 - 1, l16, g, wv, sp, pr);
    } else {
      load_slice<C, SH, PG>(t, tail ? nx.lat : lat, tail ? nx.key : key, tail ? nx.base + st * kTile : bj + NS * kTile,
                            tail ? nx.last : k1 - 1, l16, g, wv, tail ? nx.sp : sp, pr);
    }
  };
  // tile j (stage st): its shares in, the share of tile j + 1 out (unless it is the run's last), then softmax
  // and the product with the slice.  Whether a step publishes is fixed where it is written, not
  // tested inside it: the compiler counts the loads in flight along every path, and a refill that
  // may or may not have been issued would make every wait in the loop one for "all of them".
  auto step = [&](auto st_, auto publishes_, int j) __attribute__((always_inline)) {
    constexpr int st = decltype(st_)::value;
    const int par = (sb0 ^ j) & 1;
    __syncthreads();  // all four shares of tile j are in LDS
    Shares<C> sh;
    read_shares<C>(sh, sS + par * kShare, lane);
    if constexpr (decltype(publishes_)::value) publish(std::integral_constant<int, (st + 1) % NS>{}, j + 1);
    uint32_t vmask[C::NHT];
    uint32_t vm = 0;
#pragma unroll
    for (int v = 0; v < 4; ++v) vm |= (base0 + j * kTile + 4 * g + v < k1 ? 1u : 0u) << v;
#pragma unroll
    for (int ht = 0; ht < C::NHT; ++ht) vmask[ht] = vm;
    finish_tile<C>(sh, sTw + par * kPark, vmask, ws, lane, l16, g);
  };
  static_assert(NS == 2, "two stages");
  publish(std::integral_constant<int, 0>{}, 0);
  for (int it = 0; it < n_iter - 1; ++it) {
    step(std::integral_constant<int, 0>{}, std::true_type{}, NS * it);
    step(std::integral_constant<int, 1>{}, std::true_type{}, NS * it + 1);
  }
  step(std::integral_constant<int, 0>{}, std::true_type{}, n_all - 2);
  step(std::integral_constant<int, 1>{}, std::false_type{}, n_all - 1);
  sbuf = (sb0 ^ n_all) & 1;
}

// SH: a sequence may read its first slots from another sequence's rows (a.prefix_owner, a.prefix_slots;
// SharedPrefix): looked up once per run, applied lane by lane where a tile's rows are requested.
// PG: paged storage (a.pages): a.lat / a.key are the pool; a run reads through its sequence's page-table row.
// AH: the logits run one tile ahead of the softmax (stream_cols_ahead; two parking areas in LDS).
template <int R, int DR, int NHT, int NS, int OCC, bool SH, bool PG, bool AH>
__global__ __launch_bounds__(kBlock, OCC) void attn_cols_kernel(AttnArgs a) {
  using C = ColCfg<R, DR, NHT>;
  constexpr size_t kParkBytes = (AH ? 2 : 1) * C::park_bytes;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* sT = reinterpret_cast<uint16_t*>(smem);
  float4_t* sS = reinterpret_cast<float4_t*>(smem + kParkBytes);
  int* sPre = reinterpret_cast<int*>(smem + kParkBytes + C::s_bytes);  // [batch + 1]
  int* sLive = sPre + a.batch + 1;                                        // [batch] live slots
  int* sScan = sLive + a.batch;                                           // [kBlock]

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int B = a.batch;

  // ---- pre[]: running work units.  A sequence with live slots takes rc units for the fixed cost of a run
  // (its query, the first tiles' latency, the partial's stores) and one per tile after them, so that a
  // workgroup whose range starts several sequences gets fewer tiles.  Up to 64 sequences: one
  // wavefront, a shuffle scan, one barrier.
  const int rc = a.run_cost;
  auto units_of = [&](int live) { return live > 0 ? rc + (live + kTile - 1) / kTile : 0; };
  if (B <= kWave) {
    if (wv == 0) {
      const int lv = lane < B ? (a.seq_len[lane] + a.stride - 1) / a.stride : 0;
      const int nt = units_of(lv);
      int inc = nt;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const int v = __shfl_up(inc, off, kWave);
        if (lane >= off) inc += v;
      }
      if (lane < B) {
        sPre[lane] = inc - nt;
        sLive[lane] = lv;
      }
      if (lane == B - 1) sPre[B] = inc;
    }
    __syncthreads();
  } else {  // every thread sums a contiguous run of sequences
    const int per = (B + kBlock - 1) / kBlock;
    const int b_lo = tid * per, b_hi = b_lo + per < B ? b_lo + per : B;
    int run = 0;
    for (int bb = b_lo; bb < b_hi; ++bb) run += units_of((a.seq_len[bb] + a.stride - 1) / a.stride);
    // inclusive scan of the threads' sums: inside each wavefront by shuffles, the wavefronts' totals
    // through LDS (two barriers instead of the sixteen of a scan in LDS over all 256 threads)
    int inc = run;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const int v = __shfl_up(inc, off, kWave);
      if (lane >= off) inc += v;
    }
    if (lane == kWave - 1) sScan[kBlock - kWaves + wv] = inc;  // the wavefront's total, in the array's last entries
    __syncthreads();
    int before = 0;  // units of the wavefronts before this one
#pragma unroll
    for (int w = 0; w < kWaves; ++w) before += w < wv ? sScan[kBlock - kWaves + w] : 0;
    {
      int acc = before + inc - run;  // units before this thread's first sequence
      for (int bb = b_lo; bb < b_hi; ++bb) {
        const int lv = (a.seq_len[bb] + a.stride - 1) / a.stride;
        sPre[bb] = acc;
        sLive[bb] = lv;
        acc += units_of(lv);
      }
      if (tid == kBlock - 1) sPre[B] = before + inc;
    }
    __syncthreads();
  }
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
  while (sPre[b + 1] <= pos) ++b;      // sequences without live slots take no unit
  if (end <= sPre[b] + rc) return;     // the range ends before its only sequence's first tile: nothing to do
  uint16_t* sTw = sT + wv * kTile * C::TS;
  const uint16_t* lat_all = reinterpret_cast<const uint16_t*>(a.lat);
  const uint16_t* key_all = reinterpret_cast<const uint16_t*>(a.key);
  const uint16_t* q_all = reinterpret_cast<const uint16_t*>(a.qcat);

  struct Run {
    int b, k0, k1, seg_end;
    SharedPrefix sp;
  };
  auto rows_of = [&](const uint16_t* all, int bb, int width) {  // where sequence bb's rows start (the pool itself when paged)
    return all + (PG ? 0 : (size_t)bb * a.max_slots * width);
  };
  auto pages_of = [&](int bb) {
    return PageRow{PG ? a.pages.table + (size_t)bb * a.pages.max_pages : nullptr, a.pages.shift, a.pages.n_pages,
                   a.pages.max_pages - 1};
  };
  auto run_at = [&](int p, int& bb) {  // run starting at flat unit p (p < end, and a tile of its sequence lies before end); bb: sequence hint
    while (sPre[bb + 1] <= p) ++bb;    // skip sequences that own no tile
    Run r;
    r.b = bb;
    r.seg_end = end < sPre[bb + 1] ? end : sPre[bb + 1];
    const int live = sLive[bb];
    const int org = sPre[bb] + rc;     // unit of the sequence's first tile
    r.k0 = (p > org ? p - org : 0) * kTile;
    r.k1 = live < (r.seg_end - org) * kTile ? live : (r.seg_end - org) * kTile;
    r.sp = SharedPrefix{0, 0, 0};
    if constexpr (SH) {  // both clamped: whatever the two arrays hold, every address stays inside the caches
      int owner = a.prefix_owner[bb], n = a.prefix_slots[bb];
      owner = owner < 0 ? 0 : (owner < a.prefix_rows ? owner : a.prefix_rows - 1);
      r.sp.n = n < 0 ? 0 : (n < live ? n : live);
      r.sp.dlat = (long long)(owner - bb) * a.max_slots * R;
      r.sp.dkey = (long long)(owner - bb) * a.max_slots * DR;
    }
    return r;
  };
  Run cur = run_at(pos, b);
  PageRow pr_cur = pages_of(cur.b);  // the current run's page cursor
  SliceRegs<C> tl[NS];
  QSlice<C> q, qn;
  {
    const uint16_t* lat = rows_of(lat_all, cur.b, R);
    const uint16_t* key = rows_of(key_all, cur.b, DR);
    // The query first: its loads must be the oldest ones in flight.  The compiler cannot tell the first
    // run from the later ones inside the tile loop, so every wait for a query register there is sized
    // for the first run; with the query requested after the tiles that was "everything in flight",
    // the tile requested a moment ago included (one tile of prefetch instead of NS).
    load_query_slice<C>(q, q_all + (size_t)cur.b * a.n_heads * C::E, a.q_plane, a.n_heads, l16, g, wv);
#pragma unroll
    for (int st = 0; st < NS; ++st)
      load_slice<C, SH, PG>(tl[st], lat, key, cur.k0 + st * kTile, cur.k1 - 1, l16, g, wv, cur.sp, pr_cur);
  }
  int sbuf = 0;
  while (true) {
    const uint16_t* lat = rows_of(lat_all, cur.b, R);
    const uint16_t* key = rows_of(key_all, cur.b, DR);
    const bool more = cur.seg_end + rc < end;  // the next sequence's first tile lies inside the range
    Run nxt = cur;
    NextCols nx{lat, key, cur.k1, cur.k1 - 1, cur.sp, pr_cur};  // no next run: dead refills clamp to a live slot
    if (more) {
      nxt = run_at(cur.seg_end, b);
      nx.lat = rows_of(lat_all, nxt.b, R);
      nx.key = rows_of(key_all, nxt.b, DR);
      nx.base = nxt.k0;
      nx.last = nxt.k1 - 1;
      nx.sp = nxt.sp;
      nx.pr = pages_of(nxt.b);
      load_query_slice<C>(qn, q_all + (size_t)nxt.b * a.n_heads * C::E, a.q_plane, a.n_heads, l16, g, wv);
    }
    ColState<C> ws;
    ws.reset();
    if constexpr (AH) stream_cols_ahead<C, NS, SH, PG>(tl, q, sTw, sS, lat, key, cur.k0, cur.k1, nx, lane, l16, g, wv, sbuf, ws, cur.sp, pr_cur);
    else stream_cols<C, NS, SH, PG>(tl, q, sTw, sS, lat, key, cur.k0, cur.k1, nx, lane, l16, g, wv, sbuf, ws, cur.sp, pr_cur);

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
        if (a.part_f16) {  // normalised by the run's own sum: a convex combination of cache rows, safe in half
          const float inv = l_head[ht] > 0.f ? 1.f / l_head[ht] : 0.f;
          uint16_t* ph = reinterpret_cast<uint16_t*>(a.part_o) + (piece * a.n_heads + h) * R + wv * C::RW + 4 * g;
#pragma unroll
          for (int mt = 0; mt < C::MT; ++mt) {
            const float4_t o = ws.acc_o[ht][mt] * inv;
            *reinterpret_cast<uint2*>(ph + 16 * mt) = make_uint2(pack_f16x2(o[0], o[1]), pack_f16x2(o[2], o[3]));
          }
        } else {
          float* po = a.part_o + (piece * a.n_heads + h) * R + wv * C::RW + 4 * g;
#pragma unroll
          for (int mt = 0; mt < C::MT; ++mt) *reinterpret_cast<float4_t*>(po + 16 * mt) = ws.acc_o[ht][mt];
        }
        if (wv == 0 && g == 0) {
          a.part_ml[(piece * a.n_heads + h) * 2 + 0] = ws.m_ref[ht];
          a.part_ml[(piece * a.n_heads + h) * 2 + 1] = l_head[ht];
        }
      }
    }
    if (!more) break;
    cur = nxt;
    q = qn;
    pr_cur = nx.pr;  // the cursor the last refills left on the next run's first pages
  }
}

template <int R, int DR, int NHT, int NS, int OCC, bool SH, bool PG = false>
hipError_t launch_cols(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  using C = ColCfg<R, DR, NHT>;
  constexpr bool AH = NHT == 2;  // one workgroup per CU: nothing else fills the waits of a tile step (no gain with two)
  const size_t smem = (AH ? 2 : 1) * C::park_bytes + C::s_bytes + (size_t)(2 * a.batch + 1 + kBlock) * sizeof(int);
  if (smem > 64 * 1024) return hipErrorInvalidValue;
  launch_timed(attn_cols_kernel<R, DR, NHT, NS, OCC, SH, PG, AH>, dim3(a.n_persistent), dim3(kBlock), smem, st, ev, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Parallel (prefill / training) form with the same column split.
// A workgroup owns G consecutive query rows m0 .. m0+G-1 of one sequence, all heads: G * (head
// tiles) query tiles share every slice a wavefront loads, so a column tile is fetched once per G
// rows (G = 2 for up to 16 heads, 1 for up to 32).  The columns the stride-aware causal mask leaves open to row m are the final states of
// the chunks that ended before m (rows j*s + s-1 of C_hat', j < m/s) and the row's own running
// state C_hat'[m].  For the whole group that is
//   * the shared columns j < m0/s, open to every row of the group: tiles of 16 with the column
//     -> row map j -> j*s + s-1, and
//   * one last tile holding rows m0 .. m0+G-1 of C_hat' themselves: row m0+i is open to query
//     row m0+gi iff i == gi (own state) or i < gi and m0+i closes a chunk ((m0+i+1) % s == 0).
// Nothing the mask hides is ever multiplied.  Each wavefront writes its columns of one
// unnormalised partial per (row, head); the combine kernel normalises and up-projects.
// grid = (ceil(T / G), B).
// ---------------------------------------------------------------------------
template <int R, int DR, int NHT, int G, int NS, int OCC>
__global__ __launch_bounds__(kBlock, OCC) void attn_cols_rows_kernel(AttnArgs a) {
  using C = ColCfg<R, DR, G * NHT>;  // query tile qt = gi * NHT + ht
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* sT = reinterpret_cast<uint16_t*>(smem);
  float4_t* sS = reinterpret_cast<float4_t*>(smem + C::park_bytes);

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int b = blockIdx.y, m0 = blockIdx.x * G, T = a.T, s = a.stride;
  const int len = a.seq_len ? (a.seq_len[b] < T ? a.seq_len[b] : T) : T;
  if (m0 >= len) return;  // padding rows only: the combine kernel writes zeros

  const uint16_t* lat = reinterpret_cast<const uint16_t*>(a.lat) + (size_t)b * T * R;
  const uint16_t* key = reinterpret_cast<const uint16_t*>(a.key) + (size_t)b * T * DR;
  const int n_sh = m0 / s;                            // shared columns
  const int n_sh_tiles = (n_sh + kTile - 1) / kTile;  // then one tile of the group's own rows
  const int n_tiles = n_sh_tiles + 1;
  auto fetch = [&](SliceRegs<C>& t, int ti) {  // tile ti (beyond the last: a readable duplicate, masked)
    int row;
    if (ti < n_sh_tiles) {
      const int c = kTile * ti + l16 < n_sh ? kTile * ti + l16 : n_sh - 1;
      row = c * s + s - 1;
    } else {
      row = m0 + (l16 < G ? l16 : G - 1);
      row = row < T ? row : T - 1;
    }
    const uint16_t* cr = lat + (size_t)row * R + wv * C::RW + 8 * g;
#pragma unroll
    for (int kk = 0; kk < C::KC; ++kk) t.xc[kk] = *reinterpret_cast<const uint4*>(cr + 32 * kk);
    t.xr = *reinterpret_cast<const uint4*>(key + (size_t)row * DR + wv * C::DRW + (8 * g < C::DRW ? 8 * g : 0));
  };
  SliceRegs<C> tl[NS];
#pragma unroll
  for (int st = 0; st < NS; ++st) fetch(tl[st], st);

  QSlice<C> q;
  const uint16_t* q_all = reinterpret_cast<const uint16_t*>(a.qcat);
#pragma unroll
  for (int gi = 0; gi < G; ++gi) {
    const int m = m0 + gi < T ? m0 + gi : T - 1;
#pragma unroll
    for (int ht = 0; ht < NHT; ++ht) {
      const int h = 16 * ht + l16 < a.n_heads ? 16 * ht + l16 : a.n_heads - 1;
      load_query_tile<C>(q.hi[gi * NHT + ht], q.lo[gi * NHT + ht],
                         q_all + (((size_t)b * T + m) * a.n_heads + h) * C::E, a.q_plane, g, wv);
    }
  }

  // visibility of the group's own rows (last tile): bit v of own_mask[gi] for slot i = 4g + v
  uint32_t own_mask[G];
#pragma unroll
  for (int gi = 0; gi < G; ++gi) {
    uint32_t vm = 0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int i = 4 * g + v;
      const bool open = i < G && (i == gi || (i < gi && (m0 + i + 1) % s == 0));
      vm |= (open ? 1u : 0u) << v;
    }
    own_mask[gi] = vm;
  }

  ColState<C> ws;
  ws.reset();
  uint16_t* sTw = sT + wv * kTile * C::TS;
  int sbuf = 0;
  const int n_iter = (n_tiles + NS - 1) / NS;
  for (int it = 0; it < n_iter; ++it) {
#pragma unroll
    for (int st = 0; st < NS; ++st) {
      const int ti = it * NS + st;
      SliceRegs<C>& t = tl[st];
      float4_t* sSb = sS + (size_t)sbuf * kWaves * C::NHT * kWave;
      publish_share<C>(t, q, sSb, sTw, lane, l16, g, wv);
      fetch(t, ti + NS);
      __syncthreads();
      uint32_t vmask[C::NHT];
      uint32_t shared_vm = 0;
#pragma unroll
      for (int v = 0; v < 4; ++v) shared_vm |= (kTile * ti + 4 * g + v < n_sh ? 1u : 0u) << v;
#pragma unroll
      for (int gi = 0; gi < G; ++gi)
#pragma unroll
        for (int ht = 0; ht < NHT; ++ht)
          vmask[gi * NHT + ht] = ti < n_sh_tiles ? shared_vm : (ti == n_sh_tiles ? own_mask[gi] : 0u);
      Shares<C> sh;
      read_shares<C>(sh, sSb, lane);
      finish_tile<C>(sh, sTw, vmask, ws, lane, l16, g);
      sbuf ^= 1;
    }
  }

  // ---- partial of every live row: this wavefront's columns; lane holds head l16, columns 16mt + 4g .. +3
#pragma unroll
  for (int qt = 0; qt < C::NHT; ++qt) {
    const int gi = qt / NHT, ht = qt % NHT;
    float l_head = ws.l_run[qt] + __shfl_xor(ws.l_run[qt], 16, kWave);
    l_head += __shfl_xor(l_head, 32, kWave);
    const int m = m0 + gi, h = 16 * ht + l16;
    if (m < len && h < a.n_heads) {
      const size_t oh = ((size_t)b * T + m) * a.n_heads + h;
      float* po = a.part_o + oh * R + wv * C::RW + 4 * g;
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) *reinterpret_cast<float4_t*>(po + 16 * mt) = ws.acc_o[qt][mt];
      if (wv == 0 && g == 0) {
        a.part_ml[oh * 2 + 0] = ws.m_ref[qt];
        a.part_ml[oh * 2 + 1] = l_head;
      }
    }
  }
}

template <int R, int DR, int NHT, int G, int NS, int OCC>
hipError_t launch_cols_rows(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  using C = ColCfg<R, DR, G * NHT>;
  constexpr size_t smem = C::park_bytes + C::s_bytes;
  static_assert(smem <= 64 * 1024, "fits the default LDS limit");
  const dim3 grid((a.T + G - 1) / G, a.batch);
  launch_timed(attn_cols_rows_kernel<R, DR, NHT, G, NS, OCC>, grid, dim3(kBlock), smem, st, ev, a);
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
  if (a.pages.table && a.prefix_owner) return hipErrorInvalidValue;  // with pages a shared prompt is shared pages
#define MTLA_CASE(RR, DD)                                                                 \
  if (a.r == RR && a.d_rope == DD) {                                                      \
    if (a.pages.table)                                                                    \
      return a.n_heads <= 16 ? launch_cols<RR, DD, 1, 2, 2, false, true>(a, st, ev) : launch_cols<RR, DD, 2, 2, 1, false, true>(a, st, ev); \
    return a.prefix_owner ? (a.n_heads <= 16 ? launch_cols<RR, DD, 1, 2, 2, true>(a, st, ev) : launch_cols<RR, DD, 2, 2, 1, true>(a, st, ev)) \
                          : (a.n_heads <= 16 ? launch_cols<RR, DD, 1, 2, 2, false>(a, st, ev) : launch_cols<RR, DD, 2, 2, 1, false>(a, st, ev)); \
  }
  MTLA_CASE(128, 32)
  MTLA_CASE(128, 64)
  MTLA_CASE(256, 32)
  MTLA_CASE(256, 64)
  MTLA_CASE(512, 32)
  MTLA_CASE(512, 64)
#undef MTLA_CASE
  return hipErrorInvalidValue;
}

bool attn_cols_rows_supported(const AttnArgs& a) {
  return a.T > 0 && a.n_heads <= 32 && (a.r == 128 || a.r == 256 || a.r == 512) &&
         (a.d_rope == 32 || a.d_rope == 64) && a.batch <= 65535;
}

hipError_t launch_attn_cols_rows(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  // Two query tiles per workgroup (2 rows of up to 16 heads, or 1 row of up to 32) keep a
  // wavefront within 256 registers, so two workgroups share a compute unit and fill each other's
  // stalls: measured, that beats four query tiles at one workgroup per compute unit.
#define MTLA_CASE(RR, DD)                                                                 \
  if (a.r == RR && a.d_rope == DD)                                                        \
    return a.n_heads <= 16 ? launch_cols_rows<RR, DD, 1, 2, 2, 2>(a, st, ev) : launch_cols_rows<RR, DD, 2, 1, 2, 2>(a, st, ev);
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
