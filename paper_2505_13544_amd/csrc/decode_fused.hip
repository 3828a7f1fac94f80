// One whole decode step in one launch, for small batches (bf16 storage, gfx950).
//
// Section "Inference using MTLA": the update rule after Eq. (infer-linear), then Eq. (obsorb) and
// Eq. (with-rope) for the step's query.  At small batch the three launches of the step (append +
// absorption, pass over the cache, combine + W_V) are three chains of launch and memory latency; the
// arithmetic and the bytes are nothing.  Here the grid is small enough to be resident all at once
// (G workgroups per sequence, batch * G <= compute units), so the workgroups of a sequence can hand
// results to each other inside the launch:
//
//   every workgroup   requests its first cache tile (addresses do not depend on the length) together
//                     with the length, then
//   absorbers         (one per head) form q~_h = W_K^(h) q_h on the matrix cores and publish it;
//   the appender      (one) runs the step's append exactly as the append kernel does, publishes the
//                     new value of the open slot and, at the very end, advances seq_len;
//   tile workgroups   (all that own a live 16-slot tile: tile u belongs to wavefront u mod 4G) take the
//                     published queries into LDS and run the logits / softmax / PV tile loop of
//                     attn_tiles.h; the wavefront that owns the last tile waits for the appender's row and
//                     patches it in; the four wavefront states are merged and published as one partial;
//   combiners         (the absorbers again) merge the partials of their head, normalise, and take the
//                     latent row through W_V^(h), which has been sitting in registers since the start.
//
// A hand-over costs one trip through memory, not a fence: the producer writes with device-scope
// stores, the consumer polls the data itself with device-scope loads until no element shows the
// "not there yet" pattern (16-bit 0xffff for bf16 planes, 32-bit 0xffffffff for fp32 partials; a
// value that happens to be that NaN is written as another NaN).  Buffers come in two parities of a
// per-sequence epoch; a launch uses one and clears the other for the next.  Every wait is bounded:
// after spin_limit polls the workgroup raises status 7 in the workspace header and goes on without
// the data (its outputs are then not written), so every workgroup always reaches its end.
#include "absorb_mfma.h"
#include "append_step.h"
#include "attn_tiles.h"
#include "mtla_device.h"
#include "mtla_kernels.h"

#ifdef MTLA_FUSED_TRACE
__device__ long long g_fused_trace[1024 * 16];
#define TRACE(k) do { if (threadIdx.x == 0) g_fused_trace[blockIdx.x * 16 + (k)] = wall_clock64(); } while (0)
extern "C" int mtla_debug_read_trace(long long* out) {
  return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_fused_trace), sizeof(long long) * 1024 * 16);
}
#else
#define TRACE(k) do {} while (0)
#endif

namespace mtla {

namespace {

constexpr int kStatusTimeout = 7;  // MTLA_ERR_TIMEOUT

__device__ __forceinline__ uint64_t ld_x8(const void* p) {
  return __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_x8(void* p, uint64_t v) {
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld_x4(const void* p) {
  return __hip_atomic_load(reinterpret_cast<const uint32_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_x4(void* p, uint32_t v) {
  __hip_atomic_store(reinterpret_cast<uint32_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// some 16-bit field of v is 0xffff
__device__ __forceinline__ bool missing16(uint64_t v) {
  const uint64_t x = ~v;
  return ((x - 0x0001000100010001ull) & ~x & 0x8000800080008000ull) != 0;
}
// some 32-bit field of v is 0xffffffff
__device__ __forceinline__ bool missing32(uint64_t v) {
  return (uint32_t)v == 0xffffffffu || (uint32_t)(v >> 32) == 0xffffffffu;
}
// two packed bf16 values; 0xffff (a NaN) becomes 0x7fff (another)
__device__ __forceinline__ uint32_t clean16x2(uint32_t v) {
  if ((v & 0xffffu) == 0xffffu) v &= ~0x8000u;
  if ((v >> 16) == 0xffffu) v &= ~0x80000000u;
  return v;
}
__device__ __forceinline__ uint32_t clean32(float f) {
  const uint32_t v = __float_as_uint(f);
  return v == 0xffffffffu ? 0x7fffffffu : v;
}
__device__ __forceinline__ uint64_t pack_clean32(float a, float b) {
  return (uint64_t)clean32(a) | ((uint64_t)clean32(b) << 32);
}

template <int R, int DR, int DH>
struct FusedCfg {
  using C = MfmaCfg<R, DR, 1>;
  static constexpr int KKA = DH / 32;  // K steps of the absorption
  static constexpr int CT = R / 16;    // 16-column tiles of one head's q~
  static constexpr int MAXU = 4;       // (head, column tile) units of the absorption one wavefront can take
  static constexpr int KKV = R / 32;   // K steps of the W_V product
  static constexpr int NTV = 2;        // 16-row tiles of it one wavefront can take
  static constexpr int TPC = R / 4;    // threads across one latent row (a float4 each)
  static constexpr int NG = kBlock / TPC;  // groups of such threads
  // LDS: [misc: append scratch, row copies][body: tiles + query, later the merge copies, later the combine's]
  static constexpr size_t misc_bytes = 1024 + (size_t)kWaves * C::E * 2;
  static constexpr size_t misc_pad = (misc_bytes + 255) / 256 * 256;
  static constexpr size_t combine_bytes = (size_t)NG * R * 4 + 2 * NG * 4 + (size_t)2 * R * 2 + 64;
  static constexpr size_t body = C::body_bytes(true) > combine_bytes ? C::body_bytes(true) : combine_bytes;
  static constexpr size_t smem = misc_pad + body + C::ml_bytes;
};

template <int R, int DR, int DH>
__global__ __launch_bounds__(kBlock) void decode_fused_kernel(FusedArgs a) {
  using F = FusedCfg<R, DR, DH>;
  using C = typename F::C;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* sApp = reinterpret_cast<float*>(smem);                              // append scratch (d_hyper + 12 floats)
  uint16_t* sRow = reinterpret_cast<uint16_t*>(smem + 1024);                 // [kWaves][E] the new slot row
  unsigned char* body = smem + F::misc_pad;
  uint16_t* sT = reinterpret_cast<uint16_t*>(body);
  uint16_t* sQ = reinterpret_cast<uint16_t*>(body + C::tile_bytes);
  float* sO = reinterpret_cast<float*>(body);                                // aliases sT, sQ after the tile loop
  float* sM = reinterpret_cast<float*>(body + F::body);
  float* sL = sM + kWaves * 16;

  // ---- who am I: consecutive workgroup ids go to consecutive XCDs, so the G workgroups of a
  // sequence are eight ids apart and share one L2
  const int G = a.G, nh = a.n_heads, GT = G - 1;
  const int wg = blockIdx.x, i_x = wg >> 3;
  const int b = (wg & 7) + 8 * (i_x / G), j = i_x % G;
  if (b >= a.batch) return;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  // Roles.  Workgroups 0 .. G-2 absorb and own tiles (wavefront slot 4j + wv of 4 (G - 1)); workgroup G-1
  // appends.  Combining is dealt out from the top, where workgroups are least likely to own a tile: role
  // (head, half of the d_h outputs) goes to workgroup G - 1 - role, two halves per head when there are
  // enough workgroups.  The plan guarantees G >= n_heads + 1.
  const bool is_app = j == GT;
  const int halves = G >= 2 * nh ? 2 : 1;
  const int role = G - 1 - j;
  const bool is_comb = role < nh * halves;
  const int chead = role / halves, chalf = role - chead * halves;
  const FusedLayout& L = a.L;
  TRACE(0);

  // ---- everything whose address is known now is requested now, what is needed first first
  const int len0 = a.ap.seq_len[b];
  uint32_t* ctl = reinterpret_cast<uint32_t*>(a.exch + L.ctl) + (size_t)b * kFusedCtlWords;
  const uint32_t epoch = ctl[0];
  const uint32_t used_a = ctl[kFusedUsedWord], used_b = ctl[kFusedUsedWord + 1];
  const uint32_t magic = *reinterpret_cast<const uint32_t*>(a.exch);
  const uint16_t* lat = reinterpret_cast<const uint16_t*>(a.ap.cache_c) + (size_t)b * a.ap.max_slots * R;
  const uint16_t* key = reinterpret_cast<const uint16_t*>(a.ap.cache_kr) + (size_t)b * a.ap.max_slots * DR;
  const int u = 4 * j + wv;              // this wavefront's slot among the 4 GT that own tiles and absorption units
  const int n_units = nh * F::CT;        // (head, 16-column tile of q~) units, dealt out round-robin
  const Cols cm{4 * GT * kTile, 0, 0, 0};
  uint4 wk[F::MAXU][F::KKA], qb[F::MAXU][F::KKA];
  uint2 qr_raw = make_uint2(0, 0);
  TileRegs<C> tl[1];
  if (!is_app) {
#pragma unroll
    for (int i = 0; i < F::MAXU; ++i) {
      const int unit = u + i * 4 * GT;
      const int uc = unit < n_units ? unit : n_units - 1;  // wavefront-uniform; a clamped unit is computed and dropped
      const int h = uc / F::CT, ct = uc - h * F::CT;
      const uint16_t* w = reinterpret_cast<const uint16_t*>(a.w_uk) + ((size_t)h * R + 16 * ct + l16) * DH + 8 * g;
      const uint16_t* q = reinterpret_cast<const uint16_t*>(a.q) + ((size_t)b * nh + h) * DH + 8 * g;
#pragma unroll
      for (int kk = 0; kk < F::KKA; ++kk) {
        wk[i][kk] = *reinterpret_cast<const uint4*>(w + 32 * kk);
        qb[i][kk] = *reinterpret_cast<const uint4*>(q + 32 * kk);
      }
    }
    if (j < nh && tid < DR / 4)  // the RoPE part of head j's operand row
      qr_raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(a.q_rope) + ((size_t)b * nh + j) * DR + 4 * tid);
    load_tile<C>(tl[0], lat, key, kTile * u, a.ap.max_slots - 1, l16, g, cm);
  }

  if (magic != a.magic) {  // a workspace that was not set up for this context: every workgroup sees the same word
    if (tid == 0) *a.ap.status = 1;
    return;
  }
  const int s = a.ap.stride;
  const bool refused = (long long)len0 + 1 > (long long)a.ap.max_slots * s;  // a full sequence is attended as it stands
  const int live = ((refused ? len0 : len0 + 1) + s - 1) / s;                // >= 1
  const int T = (live + kTile - 1) / kTile, tt = T - 1;
  const int n_act = (T + 3) / 4 < GT ? (T + 3) / 4 : GT;                     // workgroups that own a live tile
  const int par = epoch & 1;
  unsigned char* xb = a.exch + L.data + ((size_t)b * 2 + par) * L.per_seq;   // this launch's buffers
  unsigned char* xo = a.exch + L.data + ((size_t)b * 2 + (par ^ 1)) * L.per_seq;  // the next launch's
  if (tid == 0) st_x4(&ctl[1 + j], epoch + 1);  // "I have read the length and the epoch"
  bool gave_up = false;
  TRACE(1);

  // ---- absorption: q~ = W_K^(h) q, one (head, 16 columns) unit per pass (all 16 MFMA columns carry the
  // same query; column 0 is kept), published as hi + lo bf16 planes
  if (!is_app) {
    uint16_t* qx = reinterpret_cast<uint16_t*>(xb + L.q);
    const size_t plane = (size_t)nh * C::E;
#pragma unroll
    for (int i = 0; i < F::MAXU; ++i) {
      const int unit = u + i * 4 * GT;
      if (unit < n_units) {
        const int h = unit / F::CT, ct = unit - h * F::CT;
        float4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < F::KKA; ++kk)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wk[i][kk]),
                                                        __builtin_bit_cast(bf16x8_t, qb[i][kk]), acc, 0, 0, 0);
        if (l16 == 0) {  // columns 16 ct + 4g .. +3
          uint32_t hi0, lo0, hi1, lo1;
          split_bf16x2(acc[0] * a.scale_log2, acc[1] * a.scale_log2, hi0, lo0);
          split_bf16x2(acc[2] * a.scale_log2, acc[3] * a.scale_log2, hi1, lo1);
          uint16_t* dst = qx + (size_t)h * C::E + 16 * ct + 4 * g;
          st_x8(dst, (uint64_t)clean16x2(hi0) | ((uint64_t)clean16x2(hi1) << 32));
          st_x8(dst + plane, (uint64_t)clean16x2(lo0) | ((uint64_t)clean16x2(lo1) << 32));
        }
      }
    }
    if (j < nh && tid < DR / 4) {
      const float v0 = __uint_as_float(qr_raw.x << 16), v1 = __uint_as_float(qr_raw.x & 0xffff0000u);
      const float v2 = __uint_as_float(qr_raw.y << 16), v3 = __uint_as_float(qr_raw.y & 0xffff0000u);
      uint32_t hi0, lo0, hi1, lo1;
      split_bf16x2(v0 * a.scale_log2, v1 * a.scale_log2, hi0, lo0);
      split_bf16x2(v2 * a.scale_log2, v3 * a.scale_log2, hi1, lo1);
      uint16_t* dst = qx + (size_t)j * C::E + R + 4 * tid;
      st_x8(dst, (uint64_t)clean16x2(hi0) | ((uint64_t)clean16x2(hi1) << 32));
      st_x8(dst + plane, (uint64_t)clean16x2(lo0) | ((uint64_t)clean16x2(lo1) << 32));
    }
  }
  TRACE(2);

  // ---- appender: the step's token goes into the cache (and, for the owner of the last tile, into the exchange)
  if (is_app) append_step_block<bf16, R / 32, bf16, true>(a.ap, b, sApp, reinterpret_cast<uint16_t*>(xb + L.row));
  TRACE(3);

  // ---- tile workgroups
  if (j < n_act) {
    // the absorbed queries of all heads -> LDS (rows of padded heads stay zero)
    constexpr int QC = C::E / 4;                      // 8-byte pieces of one head's row
    constexpr int MAXC = (2 * 16 * QC + kBlock - 1) / kBlock;
    const int total = 2 * nh * QC;
    for (int idx = tid; idx < 2 * 16 * (C::QS / 4); idx += kBlock) reinterpret_cast<uint2*>(sQ)[idx] = make_uint2(0, 0);
    const unsigned char* qx = xb + L.q;
    uint64_t v[MAXC];
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int idx = tid + i * kBlock;
      v[i] = ld_x8(qx + (size_t)(idx < total ? idx : 0) * 8);
    }
    for (int spins = 0;; ++spins) {
      bool ok = true;
#pragma unroll
      for (int i = 0; i < MAXC; ++i) {
        const int idx = tid + i * kBlock;
        if (idx < total && missing16(v[i])) {
          v[i] = ld_x8(qx + (size_t)idx * 8);
          ok = false;
        }
      }
      if (ok) break;
      if (spins >= a.spin_limit) {
        gave_up = true;
        break;
      }
    }
    __syncthreads();  // the zero fill is done
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int idx = tid + i * kBlock;
      if (idx < total) {
        const int pl = idx / (nh * QC), rem = idx - pl * nh * QC;
        const int h = rem / QC, c = rem - h * QC;
        *reinterpret_cast<uint64_t*>(sQ + (size_t)(pl * 16 + h) * C::QS + 4 * c) = v[i];
      }
    }
    gave_up = __syncthreads_or(gave_up);
    TRACE(5);

    WaveState<C> ws;
    ws.reset();
    const uint4 qdummy[1] = {make_uint4(0, 0, 0, 0)};
    const uint16_t* qrow = sQ + (size_t)l16 * C::QS + 8 * g;
    uint16_t* sTw = sT + wv * kTile * C::TS;
    const bool owner = !refused && (tt % (4 * GT)) == u;  // this wavefront attends the slot the token went into
    const int k1r = owner ? kTile * tt : live;            // its other tiles end below that one
    const int base = kTile * u;
    if (base < k1r) tl[0].select_live(base + l16 < k1r);  // rows that were never written become zeros
    stream_tiles<C, 1, kQLds, false, true>(tl, qdummy, qrow, sTw, lat, key, base, k1r, l16, g, cm, ws,
                                           owner ? NextRun{lat, key, kTile * tt, a.ap.max_slots - 1} : NextRun{lat, key, k1r, k1r - 1});
    if (owner) {
      // tl[0] holds the last tile: requested at the start (tt == u, no other tile) or by the loop's last refill.
      // The appender's row: C::E / 4 pieces of 8 bytes, polled by this wavefront into its own LDS copy.
      static_assert(C::E / 4 <= 2 * kWave, "two pieces per lane cover the row");
      const unsigned char* rx = xb + L.row;
      uint16_t* myrow = sRow + (size_t)wv * C::E;
      const bool has0 = lane < C::E / 4, has1 = lane + kWave < C::E / 4;
      const unsigned char* p0 = rx + (size_t)(has0 ? lane : 0) * 8;
      const unsigned char* p1 = rx + (size_t)(has1 ? lane + kWave : 0) * 8;
      uint64_t rv0 = ld_x8(p0), rv1 = ld_x8(p1);
      for (int spins = 0;; ++spins) {
        const bool bad0 = has0 && missing16(rv0), bad1 = has1 && missing16(rv1);
        if (!__any(bad0 || bad1)) break;
        if (spins >= a.spin_limit) {
          gave_up = true;
          break;
        }
        if (bad0) rv0 = ld_x8(p0);
        if (bad1) rv1 = ld_x8(p1);
      }
      if (has0) *reinterpret_cast<uint64_t*>(myrow + 4 * lane) = rv0;
      if (has1) *reinterpret_cast<uint64_t*>(myrow + 4 * (lane + kWave)) = rv1;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (l16 == (live - 1) - kTile * tt) {
#pragma unroll
        for (int kk = 0; kk < C::KC; ++kk) tl[0].xc[kk] = *reinterpret_cast<const uint4*>(myrow + 32 * kk + 8 * g);
#pragma unroll
        for (int kk = 0; kk < C::KR; ++kk) tl[0].xr[kk] = *reinterpret_cast<const uint4*>(myrow + R + 32 * kk + 8 * g);
      }
      tl[0].select_live(kTile * tt + l16 < live);
      stream_tiles<C, 1, kQLds, false, true>(tl, qdummy, qrow, sTw, lat, key, kTile * tt, live, l16, g, cm, ws,
                                             NextRun{lat, key, live, live - 1});
    }
    gave_up = __syncthreads_or(gave_up);  // also: every wavefront is done with the tile regions and the query
    TRACE(6);

    // merge of the four wavefront states (as merge_store) and publication of the partial
    if (!gave_up) {
      const float l_head = ws.l_total();
      if (g == 0) {
        sM[wv * 16 + l16] = ws.m_ref;
        sL[wv * 16 + l16] = l_head;
      }
      float* dst = sO + (size_t)(wv * 16 + l16) * C::OS + 4 * g;
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) *reinterpret_cast<float4_t*>(dst + 16 * mt) = ws.acc_o[mt];
    }
    __syncthreads();
    if (!gave_up) {
      float* po = reinterpret_cast<float*>(xb + L.po) + (size_t)j * nh * R;
      float* pml = reinterpret_cast<float*>(xb + L.pml) + (size_t)j * nh * 2;
      constexpr int R4 = R / 4;
      for (int idx = tid; idx < nh * R4; idx += kBlock) {
        const int h = idx / R4, c4 = idx - h * R4;
        float mw[kWaves], mstar = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          mw[w] = sM[w * 16 + h];
          mstar = fmaxf(mstar, mw[w]);
        }
        float4_t o = float4_t{0.f, 0.f, 0.f, 0.f};
        float lstar = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const float f = __builtin_amdgcn_exp2f(mw[w] - mstar);  // 0 for a wavefront that saw no slot
          o += f * *reinterpret_cast<const float4_t*>(sO + (size_t)(w * 16 + h) * C::OS + 4 * c4);
          lstar += f * sL[w * 16 + h];
        }
        st_x8(po + (size_t)h * R + 4 * c4, pack_clean32(o[0], o[1]));
        st_x8(po + (size_t)h * R + 4 * c4 + 2, pack_clean32(o[2], o[3]));
        if (c4 == 0) st_x8(pml + 2 * h, pack_clean32(mstar, lstar));
      }
    }
    __syncthreads();  // the body is free again
    TRACE(7);
  }

  // ---- combiner: partials of head `chead` from the n_act tile workgroups -> o~ -> this role's rows of W_V^(h)
  if (is_comb) {
    float* sAcc = reinterpret_cast<float*>(body);                  // [NG][R]
    float* sGm = sAcc + F::NG * R;                                 // [NG]
    float* sGl = sGm + F::NG;                                      // [NG]
    uint16_t* sA = reinterpret_cast<uint16_t*>(sGl + F::NG + 8);   // [2][R] hi and lo planes of the latent row
    // W_V rows of this role, requested now: they travel while the partials are waited for
    const int rows_role = DH / halves, n_vt = rows_role / 16;      // 16-row tiles of the role, dealt to the wavefronts
    uint4 wfrag[F::NTV][F::KKV];
#pragma unroll
    for (int t = 0; t < F::NTV; ++t) {
      const int vt = wv + t * kWaves;
      const int vc = vt < n_vt ? vt : 0;
      const uint16_t* wsrc = reinterpret_cast<const uint16_t*>(a.w_uv ? a.w_uv : a.w_uk) +
                             ((size_t)chead * DH + chalf * rows_role + 16 * vc + l16) * R + 8 * g;
#pragma unroll
      for (int kk = 0; kk < F::KKV; ++kk) wfrag[t][kk] = *reinterpret_cast<const uint4*>(wsrc + 32 * kk);
    }
    const int pg = tid / F::TPC, c4 = tid - pg * F::TPC;
    const float* po = reinterpret_cast<const float*>(xb + L.po) + (size_t)chead * R + 4 * c4;
    const float* pml = reinterpret_cast<const float*>(xb + L.pml) + 2 * chead;
    float m_run = -INFINITY, l_run = 0.f;
    float4_t acc = float4_t{0.f, 0.f, 0.f, 0.f};
    constexpr int PB = 4;  // pieces requested together
    for (int p0 = pg; p0 < n_act && !gave_up; p0 += PB * F::NG) {
      uint64_t ml[PB], oa[PB], ob[PB];
#pragma unroll
      for (int i = 0; i < PB; ++i) {
        const int p = p0 + i * F::NG < n_act ? p0 + i * F::NG : p0;
        ml[i] = ld_x8(pml + (size_t)p * nh * 2);
        oa[i] = ld_x8(po + (size_t)p * nh * R);
        ob[i] = ld_x8(po + (size_t)p * nh * R + 2);
      }
      for (int spins = 0;; ++spins) {
        bool ok = true;
#pragma unroll
        for (int i = 0; i < PB; ++i) {
          const int p = p0 + i * F::NG;
          if (p < n_act) {
            if (missing32(ml[i])) {
              ml[i] = ld_x8(pml + (size_t)p * nh * 2);
              ok = false;
            }
            if (missing32(oa[i])) {
              oa[i] = ld_x8(po + (size_t)p * nh * R);
              ok = false;
            }
            if (missing32(ob[i])) {
              ob[i] = ld_x8(po + (size_t)p * nh * R + 2);
              ok = false;
            }
          }
        }
        if (ok) break;
        if (spins >= a.spin_limit) {
          gave_up = true;
          break;
        }
      }
      if (gave_up) break;
#pragma unroll
      for (int i = 0; i < PB; ++i) {
        const int p = p0 + i * F::NG;
        if (p < n_act) {
          const float mp = __uint_as_float((uint32_t)ml[i]), lp = __uint_as_float((uint32_t)(ml[i] >> 32));
          const float mn = fmaxf(m_run, mp);
          const float f_old = __builtin_amdgcn_exp2f(m_run - mn), f_new = __builtin_amdgcn_exp2f(mp - mn);  // m_run = -inf: 0
          const float4_t ov = {__uint_as_float((uint32_t)oa[i]), __uint_as_float((uint32_t)(oa[i] >> 32)),
                               __uint_as_float((uint32_t)ob[i]), __uint_as_float((uint32_t)(ob[i] >> 32))};
          acc = f_old * acc + f_new * ov;
          l_run = f_old * l_run + f_new * lp;
          m_run = mn;
        }
      }
    }
    TRACE(8);
    *reinterpret_cast<float4_t*>(sAcc + (size_t)pg * R + 4 * c4) = acc;
    if (c4 == 0) {
      sGm[pg] = m_run;
      sGl[pg] = l_run;
    }
    gave_up = __syncthreads_or(gave_up);
    if (!gave_up) {
      if (tid < F::TPC) {  // n_act >= 1 and group 0 holds piece 0: m* is finite
        float mstar = -INFINITY;
#pragma unroll
        for (int k = 0; k < F::NG; ++k) mstar = fmaxf(mstar, sGm[k]);
        float lstar = 0.f;
        float4_t o = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < F::NG; ++k) {
          const float f = __builtin_amdgcn_exp2f(sGm[k] - mstar);  // a group without pieces: 0
          lstar += f * sGl[k];
          o += f * *reinterpret_cast<const float4_t*>(sAcc + (size_t)k * R + 4 * tid);
        }
        o *= 1.f / lstar;
        const size_t oh = (size_t)b * nh + chead;
        if (chalf == 0) {
          if (a.out_latent) *reinterpret_cast<float4_t*>(a.out_latent + oh * R + 4 * tid) = o;
          if (a.lse && tid == 0) a.lse[oh] = (mstar + log2f(lstar)) * 0.6931471805599453f;
        }
        const uint32_t h01 = pack_bf16x2(o[0], o[1]), h23 = pack_bf16x2(o[2], o[3]);
        const uint32_t l01 = pack_bf16x2(o[0] - __uint_as_float(h01 << 16), o[1] - __uint_as_float(h01 & 0xffff0000u));
        const uint32_t l23 = pack_bf16x2(o[2] - __uint_as_float(h23 << 16), o[3] - __uint_as_float(h23 & 0xffff0000u));
        *reinterpret_cast<uint2*>(sA + 4 * tid) = make_uint2(h01, h23);
        *reinterpret_cast<uint2*>(sA + R + 4 * tid) = make_uint2(l01, l23);
      }
      __syncthreads();
      if (a.out) {  // out^T[d, column 0] = W_V^(h)[d, :] . o~ (the other columns of the operand are zero)
        const uint32_t keep = l16 == 0 ? 0xffffffffu : 0u;
#pragma unroll
        for (int t = 0; t < F::NTV; ++t) {
          const int vt = wv + t * kWaves;
          if (vt < n_vt) {  // wavefront-uniform
            float4_t o = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < F::KKV; ++kk) {
              uint4 xh = *reinterpret_cast<const uint4*>(sA + 32 * kk + 8 * g), xl = *reinterpret_cast<const uint4*>(sA + R + 32 * kk + 8 * g);
              xh = make_uint4(xh.x & keep, xh.y & keep, xh.z & keep, xh.w & keep);
              xl = make_uint4(xl.x & keep, xl.y & keep, xl.z & keep, xl.w & keep);
              const bf16x8_t wa = __builtin_bit_cast(bf16x8_t, wfrag[t][kk]);
              o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8_t, xh), o, 0, 0, 0);
              o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8_t, xl), o, 0, 0, 0);
            }
            if (l16 == 0)
              *reinterpret_cast<float4_t*>(a.out + ((size_t)b * nh + chead) * DH + chalf * rows_role + 16 * vt + 4 * g) = o;
          }
        }
      }
    }
  }
  TRACE(9);
  if (gave_up && tid == 0) *a.ap.status = kStatusTimeout;

  // ---- clear what the next launch will poll: queries, row, and as many partials as were published
  // under that parity last time (fire and forget: done when the kernel ends)
  {
    const uint32_t used_other = par ? used_a : used_b;   // word kFusedUsedWord + (par ^ 1)
    const size_t head_bytes = L.po;                      // q and row blocks
    const size_t po_bytes = (size_t)used_other * nh * R * 4, pml_bytes = (size_t)used_other * nh * 8;
    const uint4 ones = make_uint4(~0u, ~0u, ~0u, ~0u);
    const size_t t0 = ((size_t)j * kBlock + tid) * 16, ts = (size_t)G * kBlock * 16;
    for (size_t o = t0; o < head_bytes; o += ts) *reinterpret_cast<uint4*>(xo + o) = ones;
    for (size_t o = t0; o < po_bytes; o += ts) *reinterpret_cast<uint4*>(xo + L.po + o) = ones;
    for (size_t o = t0; o < pml_bytes; o += ts) *reinterpret_cast<uint4*>(xo + L.pml + o) = ones;
  }

  // ---- appender, last: once every workgroup of the sequence has read the old length and epoch,
  // advance both and note how many partials this parity holds
  if (is_app) {
    bool late = false;
    if (tid < G) {
      for (int spins = 0; ld_x4(&ctl[1 + tid]) != epoch + 1; ++spins) {
        if (spins >= a.spin_limit) {
          late = true;
          break;
        }
      }
    }
    late = __syncthreads_or(late);
    TRACE(10);
    if (tid == 0) {
      if (late) *a.ap.status = kStatusTimeout;
      if (!refused) a.ap.seq_len[b] = len0 + 1;
      ctl[0] = epoch + 1;
      ctl[kFusedUsedWord + par] = (uint32_t)n_act;
    }
  }
}

__global__ void fused_init_kernel(uint32_t* p, size_t n_words, size_t ctl_lo, size_t ctl_hi, uint32_t magic) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_words) return;
  p[i] = i == 0 ? magic : ((i >= ctl_lo && i < ctl_hi) ? 0u : 0xffffffffu);
}

template <int R, int DR, int DH>
hipError_t launch_rdh(const FusedArgs& a, hipStream_t st, const EventPair& ev, int* blocks_per_cu) {
  using F = FusedCfg<R, DR, DH>;
  static_assert(F::smem <= 160 * 1024, "LDS budget of one compute unit");
  static bool attr_set = false;
  static int per_cu = 0;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_fused_kernel<R, DR, DH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)F::smem);
    if (e != hipSuccess) return e;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_fused_kernel<R, DR, DH>, kBlock, F::smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if (blocks_per_cu) {
    *blocks_per_cu = per_cu;
    return hipSuccess;
  }
  const int groups = (a.batch + 7) / 8;
  launch_timed(decode_fused_kernel<R, DR, DH>, dim3(8 * groups * a.G), dim3(kBlock), F::smem, st, ev, a);
  return hipGetLastError();
}

hipError_t dispatch(const FusedArgs& a, hipStream_t st, const EventPair& ev, int* blocks_per_cu) {
#define MTLA_CASE(RR, DD, HH) \
  if (a.ap.r == RR && a.ap.d_rope == DD && a.d_head == HH) return launch_rdh<RR, DD, HH>(a, st, ev, blocks_per_cu);
  MTLA_CASE(128, 32, 64)
  MTLA_CASE(128, 64, 128)
  MTLA_CASE(256, 32, 64)
  MTLA_CASE(256, 64, 64)
  MTLA_CASE(256, 32, 128)
  MTLA_CASE(256, 64, 128)
#undef MTLA_CASE
  return hipErrorInvalidValue;
}

}  // namespace

bool decode_fused_shape(int r, int d_rope, int d_head) {
  return ((r == 128 || r == 256) && d_rope == 32 && d_head == 64) || ((r == 128 || r == 256) && d_rope == 64 && d_head == 128) ||
         (r == 256 && d_rope == 64 && d_head == 64) || (r == 256 && d_rope == 32 && d_head == 128);
}

uint32_t fused_magic(const FusedLayout& L, int n_heads, int r, int d_rope) {
  uint64_t h = 0x4d544c41ull;  // any mixing will do: the word only has to differ between layouts
  for (uint64_t v : {(uint64_t)L.total, (uint64_t)L.per_seq, (uint64_t)L.g_max, (uint64_t)L.b_max, (uint64_t)n_heads,
                     (uint64_t)r, (uint64_t)d_rope})
    h = (h ^ v) * 0x9e3779b97f4a7c15ull + 0x7f4a7c15ull;
  const uint32_t m = (uint32_t)(h >> 32);
  return m == 0u || m == 0xffffffffu ? 0x4d544c41u : m;
}

hipError_t launch_fused_init(unsigned char* exch, const FusedLayout& L, uint32_t magic, hipStream_t st) {
  const size_t n = L.total / 4;
  hipLaunchKernelGGL(fused_init_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<uint32_t*>(exch), n, L.ctl / 4, L.data / 4, magic);
  return hipGetLastError();
}

int decode_fused_plan(const FusedArgs& a, int n_cu, bool forced) {
  const AppendArgs& ap = a.ap;
  if (a.batch < 1 || a.batch > a.L.b_max || a.n_heads > 16 || ap.n_new_max != 1 || ap.n_new || ap.w_override ||
      ap.c_new_f32 || ap.w_out || ap.slot_out || !ap.tail_c)
    return 0;
  if (ap.d_hyper > kBlock) return 0;
  int per_cu = 0;
  if (dispatch(a, nullptr, EventPair(), &per_cu) != hipSuccess || per_cu < 1) return 0;
  const int groups = (a.batch + 7) / 8;
  long long resident = (long long)per_cu * n_cu;   // every workgroup has to be on the device at once
  int G = (int)(resident / (8 * groups));
  G = G < a.L.g_max ? G : a.L.g_max;
  if (n_cu / (8 * groups) < G) G = n_cu / (8 * groups);  // one workgroup per compute unit: they are latency chains
  if (G < a.n_heads + 1) return 0;
  if (a.n_heads * (ap.r / 16) > 4 * 4 * (G - 1)) return 0;  // absorption units per wavefront
  if (!forced) {
    const int tiles = (ap.max_slots + kTile - 1) / kTile;
    if (tiles > 2 * 4 * (G - 1)) return 0;  // more than two tiles per wavefront: the pipelined kernels stream better
  }
  return G;
}

hipError_t launch_decode_fused(const FusedArgs& a, hipStream_t st, const EventPair& ev) { return dispatch(a, st, ev, nullptr); }

}  // namespace mtla
