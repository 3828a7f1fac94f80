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
#include "attn_tiles.h"
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

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
template <int R, int DR, int NHT, int NS, bool QL, bool SH>
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
  const uint16_t* lat = reinterpret_cast<const uint16_t*>(a.lat) + (size_t)b * a.max_slots * R;
  const uint16_t* key = reinterpret_cast<const uint16_t*>(a.key) + (size_t)b * a.max_slots * DR;

  // Everything whose address does not depend on the sequence length is requested before the
  // length is looked at: the length, the query operand and this wavefront's first NS tiles (any
  // slot below max_slots is readable memory) travel together, one round trip instead of three.
  const int len = a.seq_len[b];
  SharedPrefix sp{0, 0, 0};
  if constexpr (SH) {  // one more round trip before the first tiles; both values clamped, so that every
                       // address stays inside the caches whatever the two arrays hold
    int owner = a.prefix_owner[b], n = a.prefix_slots[b];
    owner = owner < 0 ? 0 : (owner < a.batch ? owner : a.batch - 1);
    sp.n = n < 0 ? 0 : (n < a.max_slots ? n : a.max_slots);
    sp.dlat = (long long)(owner - b) * a.max_slots * R;
    sp.dkey = (long long)(owner - b) * a.max_slots * DR;
  }
  TileRegs<C> tl[NS];
  const int base = k0 + wl * kTile;
  const Cols cm{C::kStep, 0, 0, 0};
#pragma unroll
  for (int st = 0; st < NS; ++st) load_tile<C, SH>(tl[st], lat, key, base + st * C::kStep, a.max_slots - 1, l16, g, cm, sp);
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
  stream_tiles<C, NS, QL ? kQLds : kQRegs, SH>(tl, qv, sQ + (16 * ht + l16) * C::QS + 8 * g, sT + wv * kTile * C::TS,
                                               lat, key, base, k1, l16, g, cm, ws, NextRun{lat, key, k1, k1 - 1}, sp);
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

template <int R, int DR, int NHT, int NS, bool QL, bool SH>
hipError_t launch_static(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  using C = MfmaCfg<R, DR, NHT>;
  constexpr size_t smem = C::body_bytes(QL) + C::ml_bytes;
  static_assert(smem <= 160 * 1024, "LDS budget of one compute unit");
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<R, DR, NHT, NS, QL, SH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  launch_timed(attn_mfma_kernel<R, DR, NHT, NS, QL, SH>, dim3(a.n_splits, a.batch), dim3(kBlock), smem, st, ev, a);
  return hipGetLastError();
}

template <int R, int DR, int NHT, int NS, bool QL>
hipError_t launch_one(const AttnArgs& a, hipStream_t st, const EventPair& ev) {
  using C = MfmaCfg<R, DR, NHT>;
  if (a.n_persistent > 0) {
    if (a.prefix_owner) return hipErrorInvalidValue;  // shared prefixes: static schedule or the column-split kernel
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
  return a.prefix_owner ? launch_static<R, DR, NHT, NS, QL, true>(a, st, ev) : launch_static<R, DR, NHT, NS, QL, false>(a, st, ev);
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
