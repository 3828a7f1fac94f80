// Parallel (prefill / training-forward) form with explicit per-head keys and values (bf16 storage,
// fp16 inside, gfx950).
//
// Eq. (with-rope) before absorption: k_n^(h) = C_hat'[n] W_K^(h), v_n^(h) = C_hat'[n] W_V^(h), and
// for query row m of head h
//     e_n = ( <q_m^(h), k_n^(h)> + <q_m^R(h), k_n^R> ) / sqrt(d_h),   o_m^(h) = softmax(e) V^(h)
// over the columns the stride-aware causal mask leaves open to m: the final states of the chunks
// that ended before m (rows j*s + s-1, j < m/s) and the row's own running state (row m).  With many
// query rows per head this is the cheaper form (2 (d_h + d_R) + 2 d_h flop per open (row, column)
// pair instead of 2 (r + d_R) + 2 r), it needs neither the absorbed query operand nor the latent
// partials, and every matrix instruction works on 16 real query rows.  The absorbed form remains
// for decode (one row per head) and whenever the latent-space output is asked for.
//
// Everything between the bf16 inputs and the fp32 output is IEEE half: the partial states, the
// keys, the values and the softmax weights each carry 11 significant bits instead of bf16's 8 (the
// intermediate roundings of this form would otherwise use up the whole 2e-2 budget), and all of
// them are of order 1, far inside the half range.  bf16 inputs (queries, RoPE keys, weights)
// convert exactly apart from values below 6e-5.
//
// Three kernels:
//   to_f16_kernel         W_K^(h) with the contracted (latent) index innermost, like W_V^(h), and the
//                         RoPE keys, as fp16
//   kv_up_kernel          K = C_hat' W_K, V = C_hat' W_V for all T rows: a plain fp16 MFMA GEMM,
//                         operands fetched straight into the operand layouts, 128 x 128 tile
//   attn_explicit_kernel  one workgroup per (128 query rows, head, sequence); keys, RoPE keys and
//                         values of 64 columns at a time go through LDS and are shared by the four
//                         wavefronts (32 query rows each, queries in registers)
#include "mtla_device.h"
#include "mtla_kernels.h"

namespace mtla {

namespace {

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));  // staging registers (a plain vector type: promoted reliably)
typedef short4_t __attribute__((address_space(3))) * lds_short4_ptr;

__device__ __forceinline__ uint16_t bf16_bits_to_f16_bits(uint16_t v) {
  return __builtin_bit_cast(uint16_t, static_cast<_Float16>(__uint_as_float(uint32_t(v) << 16)));
}
// 8 bf16 values, each times `scale` -> 8 fp16 values
__device__ __forceinline__ u32x4_t bf16x8_to_f16x8(u32x4_t v, float scale = 1.f) {
  u32x4_t o;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    o[i] = pack_f16x2(__uint_as_float(v[i] << 16) * scale, __uint_as_float(v[i] & 0xffff0000u) * scale);
  return o;
}

// w_kT[h][d][n] = fp16(w_uk[h][n][d]),  w_v16[h][d][n] = fp16(w_uv[h][d][n]),  kr16 = fp16(kr)
__global__ void to_f16_kernel(const uint16_t* w_uk, const uint16_t* w_uv, uint16_t* w_kT, uint16_t* w_v16,
                              const uint16_t* kr, uint16_t* kr16, int n_heads, int r, int dh, size_t n_kr) {
  const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
  const size_t n_w = (size_t)n_heads * r * dh;
  if (idx < n_w) {
    const int n = int(idx % r), d = int((idx / r) % dh), h = int(idx / ((size_t)r * dh));
    w_kT[idx] = bf16_bits_to_f16_bits(w_uk[((size_t)h * r + n) * dh + d]);
    w_v16[idx] = bf16_bits_to_f16_bits(w_uv[idx]);
  } else if (idx - n_w < n_kr) {
    kr16[idx - n_w] = bf16_bits_to_f16_bits(kr[idx - n_w]);
  }
}

// C[row][n] = sum_k A[row][k] W[n][k]   (A [M][K], W [N][K], C [M][N], all fp16, K = 32 KK, K % 64 == 0).
// grid = (ceil(N/128), ceil(M/128), 2): z selects (W0, C0) or (W1, C1).  128 x 128 tile, K walked 64
// at a time through LDS (full 128-byte lines from memory, register-staged so the next slab travels
// while this one is multiplied).  Wavefront (wm, wn) owns a 64 x 64 quarter: W rows are the A
// operand, A rows the B operand, so a lane ends up with four consecutive n of one row (one 8-byte
// store).
template <int KK>
__global__ __launch_bounds__(kBlock) void kv_up_kernel(const uint16_t* A, const uint16_t* W0, const uint16_t* W1,
                                                       uint16_t* C0, uint16_t* C1, int M, int N) {
  constexpr int K = 32 * KK, BK = 64, LS = BK + 8;  // LDS row stride: 36 words, conflict-free operand reads
  static_assert(K % BK == 0, "K is walked 64 at a time");
  __shared__ __attribute__((aligned(16))) uint16_t sA[128 * LS];
  __shared__ __attribute__((aligned(16))) uint16_t sW[128 * LS];
  const uint16_t* W = blockIdx.z ? W1 : W0;
  uint16_t* C = blockIdx.z ? C1 : C0;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int nb = blockIdx.x * 128, rb = blockIdx.y * 128;
  const int wn = 64 * (wv & 1), wm = 64 * (wv >> 1);

  // piece p = tid + 256 i of a slab: row p / 8, 16-byte piece p % 8
  const uint16_t* ap[4];
  const uint16_t* wp[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int p = tid + kBlock * i, row = p >> 3, c = p & 7;
    ap[i] = A + (size_t)(rb + row < M ? rb + row : M - 1) * K + 8 * c;
    wp[i] = W + (size_t)(nb + row < N ? nb + row : N - 1) * K + 8 * c;
  }
  u32x4_t ra[4], rw[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ra[i] = *reinterpret_cast<const u32x4_t*>(ap[i]);
    rw[i] = *reinterpret_cast<const u32x4_t*>(wp[i]);
  }
  float4_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = float4_t{0.f, 0.f, 0.f, 0.f};

  for (int k0 = 0; k0 < K; k0 += BK) {
    __syncthreads();  // the previous slab has been read
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int p = tid + kBlock * i;
      *reinterpret_cast<u32x4_t*>(&sA[(p >> 3) * LS + 8 * (p & 7)]) = ra[i];
      *reinterpret_cast<u32x4_t*>(&sW[(p >> 3) * LS + 8 * (p & 7)]) = rw[i];
    }
    __syncthreads();
    const int kn = k0 + BK < K ? k0 + BK : k0;  // past the end: a harmless reload
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ra[i] = *reinterpret_cast<const u32x4_t*>(ap[i] + kn);
      rw[i] = *reinterpret_cast<const u32x4_t*>(wp[i] + kn);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
      f16x8_t wf[4], af[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        wf[i] = __builtin_bit_cast(f16x8_t, *reinterpret_cast<const u32x4_t*>(&sW[(wn + 16 * i + l16) * LS + 32 * ks + 8 * g]));
        af[i] = __builtin_bit_cast(f16x8_t, *reinterpret_cast<const u32x4_t*>(&sA[(wm + 16 * i + l16) * LS + 32 * ks + 8 * g]));
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[i], af[j], acc[i][j], 0, 0, 0);
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = rb + wm + 16 * j + l16;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = nb + wn + 16 * i + 4 * g;
      if (row < M && n < N)
        *reinterpret_cast<uint2*>(C + (size_t)row * N + n) =
            make_uint2(pack_f16x2(acc[i][j][0], acc[i][j][1]), pack_f16x2(acc[i][j][2], acc[i][j][3]));
    }
  }
}

// Where the 64 columns of tile t of a workgroup come from, and their way into LDS: first the
// shared columns j < n_sh (rows j*s + s-1), then the block's own rows.  Every thread carries
// NK + NV 16-byte pieces of a tile in registers from one tile's compute phase to the next.
template <int DH, int DR>
struct TileSrc {
  static constexpr int BN = 64, VC = DH / 8, RC = DR / 8;  // 16-byte pieces per key / value row, per RoPE key row
  static constexpr int NKV = BN * VC / kBlock, NR = BN * RC / kBlock, N = 2 * NKV + NR;  // pieces per thread
  static_assert(BN * VC % kBlock == 0 && BN * RC % kBlock == 0, "whole pieces per thread");
  const uint16_t* kx;    // keys of this (sequence, head): row stride nh * DH
  const uint16_t* vx;    // values, same stride
  const uint16_t* kr16;  // RoPE keys of the sequence (fp16): row stride DR
  uint32_t kv_stride;
  int s, n_sh, n_sh_tiles, m0, T;
  __device__ __forceinline__ uint32_t src_row(int t, int c_) const {
    const int c = BN * t + c_ < n_sh ? BN * t + c_ : n_sh - 1;  // shared column (unused if there is none)
    const int r_ = m0 + BN * (t - n_sh_tiles) + c_;              // own row
    const int own = r_ < T ? r_ : T - 1;
    return (uint32_t)(t < n_sh_tiles ? c * s + s - 1 : own);
  }
  // stg: [0, NKV) key pieces, [NKV, 2 NKV) value pieces, then the RoPE key pieces.  32-bit element
  // offsets (one sequence's keys stay far below 2^31 elements); no lane-dependent control flow.
  // A tile of 64 shared columns (all but a few tiles of a block) is fetched from wavefront-uniform
  // base addresses plus one per-thread offset that never changes.
  __device__ __forceinline__ void fetch(u32x4_t (&stg)[N], int t, int tid) const {
    if (BN * t + BN <= n_sh) {
      const uint32_t row0 = (uint32_t)(BN * t * s + s - 1);  // source row of the tile's column 0
      const uint32_t thr_kv = (uint32_t)(tid / VC * s) * kv_stride + 8 * (tid % VC);
      const uint32_t thr_r = (uint32_t)(tid / RC * s) * DR + 8 * (tid % RC);
#pragma unroll
      for (int i = 0; i < NKV; ++i) {
        const size_t base = (size_t)(row0 + (uint32_t)(i * (kBlock / VC) * s)) * kv_stride;
        stg[i] = *reinterpret_cast<const u32x4_t*>(kx + base + thr_kv);
        stg[NKV + i] = *reinterpret_cast<const u32x4_t*>(vx + base + thr_kv);
      }
#pragma unroll
      for (int i = 0; i < NR; ++i) {
        const size_t base = (size_t)(row0 + (uint32_t)(i * (kBlock / RC) * s)) * DR;
        stg[2 * NKV + i] = *reinterpret_cast<const u32x4_t*>(kr16 + base + thr_r);
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < NKV; ++i) {
      const int idx = tid + kBlock * i;
      const uint32_t off = src_row(t, idx / VC) * kv_stride + 8 * (idx % VC);
      stg[i] = *reinterpret_cast<const u32x4_t*>(kx + off);
      stg[NKV + i] = *reinterpret_cast<const u32x4_t*>(vx + off);
    }
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      const int idx = tid + kBlock * i;
      stg[2 * NKV + i] = *reinterpret_cast<const u32x4_t*>(kr16 + (src_row(t, idx / RC) * DR + 8 * (idx % RC)));
    }
  }
  template <int KS, int VS>
  __device__ __forceinline__ void commit(const u32x4_t (&stg)[N], uint16_t* sK, uint16_t* sV, int tid) const {
#pragma unroll
    for (int i = 0; i < NKV; ++i) {
      const int idx = tid + kBlock * i;
      *reinterpret_cast<u32x4_t*>(&sK[(idx / VC) * KS + 8 * (idx % VC)]) = stg[i];
      *reinterpret_cast<u32x4_t*>(&sV[(idx / VC) * VS + 8 * (idx % VC)]) = stg[NKV + i];
    }
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      const int idx = tid + kBlock * i;
      *reinterpret_cast<u32x4_t*>(&sK[(idx / RC) * KS + DH + 8 * (idx % RC)]) = stg[2 * NKV + i];
    }
  }
};

// grid = (ceil(ceil(T/128) / 2), n_heads, B)
template <int DH, int DR>
__global__ __launch_bounds__(kBlock, 2) void attn_explicit_kernel(ExplicitArgs a) {
  constexpr int KD = DH / 32, KQ = (DH + DR) / 32, MT = DH / 16;
  constexpr int BM = 128, BN = 64;
  constexpr int KS = DH + DR + 8;  // LDS row stride of [k | k^R] (bf16 elements): 16-byte rows, odd multiple of 4 banks
  constexpr int VS = DH + 16;      // LDS row stride of v
  __shared__ __attribute__((aligned(16))) uint16_t sK[BN * KS];
  __shared__ __attribute__((aligned(16))) uint16_t sV[BN * VS];

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int b = blockIdx.z, h = blockIdx.y, T = a.T, s = a.stride, nh = a.n_heads;
  const int len = a.seq_len ? (a.seq_len[b] < T ? a.seq_len[b] : T) : T;
  float* out = a.out + ((size_t)b * T * nh + h) * DH;  // + row * nh * DH
  // Row block x walks x * BM / (s BN) + 2 tiles.  A workgroup takes block n-1-x and then block x, so
  // every workgroup of the launch walks the same number of tiles (the middle one, if n is odd, half).
  const int n_blocks = (T + BM - 1) / BM;
  for (int pass = 0; pass < 2; ++pass) {
  const int xb = pass == 0 ? n_blocks - 1 - (int)blockIdx.x : (int)blockIdx.x;
  if (pass == 1 && xb >= n_blocks - 1 - (int)blockIdx.x) break;
  const int m0 = xb * BM;
  if (m0 >= len) {  // padding rows only
    const int rows = T - m0 < BM ? T - m0 : BM;
    for (int i = tid; i < rows * (DH / 4); i += kBlock)
      *reinterpret_cast<float4_t*>(out + (size_t)(m0 + i / (DH / 4)) * nh * DH + 4 * (i % (DH / 4))) =
          float4_t{0.f, 0.f, 0.f, 0.f};
    continue;
  }
  const uint16_t* kx = reinterpret_cast<const uint16_t*>(a.kx) + ((size_t)b * T * nh + h) * DH;
  const uint16_t* vx = reinterpret_cast<const uint16_t*>(a.vx) + ((size_t)b * T * nh + h) * DH;
  const uint16_t* kr16 = reinterpret_cast<const uint16_t*>(a.kr16) + (size_t)b * T * DR;

  // ---- the columns: shared ones j < m0/s (rows j*s + s-1), then the block's own 128 rows
  const int n_sh = m0 / s, n_sh_tiles = (n_sh + BN - 1) / BN, n_tiles = n_sh_tiles + BM / BN;
  TileSrc<DH, DR> src;
  src.kx = kx;
  src.vx = vx;
  src.kr16 = kr16;
  src.kv_stride = (uint32_t)(nh * DH);
  src.s = s;
  src.n_sh = n_sh;
  src.n_sh_tiles = n_sh_tiles;
  src.m0 = m0;
  src.T = T;
  u32x4_t stg[TileSrc<DH, DR>::N];
  src.fetch(stg, 0, tid);

  // ---- queries of this wavefront's 32 rows: B operand, lane = row l16 of row tile rt
  u32x4_t qf[2][KQ];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int m = m0 + 32 * wv + 16 * rt + l16;
    const size_t row = (size_t)b * T + (m < T ? m : T - 1);
    const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + (row * nh + h) * DH + 8 * g;
    const uint16_t* qrp = reinterpret_cast<const uint16_t*>(a.q_rope) + (row * nh + h) * DR + 8 * g;
#pragma unroll
    for (int kk = 0; kk < KQ; ++kk)
      qf[rt][kk] = bf16x8_to_f16x8(kk < KD ? *reinterpret_cast<const u32x4_t*>(qp + 32 * kk)
                                           : *reinterpret_cast<const u32x4_t*>(qrp + 32 * (kk - KD)),
                                   a.scale_log2);  // logits come out in units of log2: log2(e) / sqrt(d_h) folded in
  }

  float m_ref[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
  float4_t acc[2][MT];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};

  // bit 4 sub + v of closes_mask[dt]: row m0 + 64 dt + 16 sub + 4g + v of the block closes a chunk
  uint32_t closes_mask[BM / BN];
#pragma unroll
  for (int dt = 0; dt < BM / BN; ++dt) {
    uint32_t cm = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int c = BN * dt + 16 * (i >> 2) + 4 * g + (i & 3);
      cm |= ((m0 + c + 1) % s == 0 ? 1u : 0u) << i;
    }
    closes_mask[dt] = cm;
  }

  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();  // the previous tile has been read
    src.template commit<KS, VS>(stg, sK, sV, tid);
    __syncthreads();
    // the next tile travels while this one is worked on (past the last: a readable duplicate)
    src.fetch(stg, t + 1, tid);

    // Visibility.  A shared tile below n_sh is open to every row; the last shared tile is cut at
    // n_sh; a tile of the block's own rows is open to row rrel at column c iff c == rrel (the row's
    // own running state) or c < rrel and row m0 + c closes a chunk (closes_mask, set up once).
    // Bit 4 sub + v of open_bits[rt]: column 16 sub + 4g + v of the tile is open to the lane's row.
    const bool own = t >= n_sh_tiles;
    const int cbase = own ? BN * (t - n_sh_tiles) : BN * t;
    const bool all_open = !own && cbase + BN <= n_sh;
    uint32_t open_bits[2] = {0xffffu, 0xffffu};
    if (!all_open) {  // workgroup-uniform: at most three tiles per row block come here
      const uint32_t closes = own ? closes_mask[t - n_sh_tiles] : 0xffffu;
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) {
        const int bound = own ? 32 * wv + 16 * rt + l16 : n_sh;  // columns below `bound` may be open
        uint32_t m = 0;
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
          const int d = bound - (cbase + 16 * sub + 4 * g);  // column 4g + v of the group is below iff v < d
          const int dd = d < 0 ? 0 : (d > 4 ? 4 : d);
          const uint32_t lt = (1u << dd) - 1u;
          const uint32_t eq = own ? (uint32_t)((unsigned)d < 4u) << (d & 3) : 0u;
          m |= ((lt & (closes >> (4 * sub))) | eq) << (4 * sub);
        }
        open_bits[rt] = m;
      }
    }

    // ---- two halves of 32 columns: S^T = [k | k^R] [q | q^R]^T, softmax weights, O^T += V^T P^T
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
      float4_t sacc[2][2];
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) sacc[rt][sb] = float4_t{0.f, 0.f, 0.f, 0.f};
      const uint16_t* krow = &sK[(32 * h2 + l16) * KS + 8 * g];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < KQ; ++kk)  // K step outermost: four independent accumulator chains
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
          const f16x8_t kf = __builtin_bit_cast(f16x8_t, *reinterpret_cast<const u32x4_t*>(krow + 16 * sb * KS + 32 * kk));
#pragma unroll
          for (int rt = 0; rt < 2; ++rt)
            sacc[rt][sb] =
                __builtin_amdgcn_mfma_f32_16x16x32_f16(kf, __builtin_bit_cast(f16x8_t, qf[rt][kk]), sacc[rt][sb], 0, 0, 0);
        }
      // issue order: the LDS reads run four ahead of the matrix instructions that use them
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int i = 0; i < 2 * KQ - 4; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
      __builtin_amdgcn_sched_barrier(0);

      // the first value fragments travel while the softmax arithmetic runs
      const uint16_t* vrow = &sV[(32 * h2 + 4 * g + (l16 >> 2)) * VS + 4 * (l16 & 3)];
      constexpr int VPRE = MT / 2;
      u32x4_t vpre[VPRE];
#pragma unroll
      for (int mt = 0; mt < VPRE; ++mt) {
        const short4_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(vrow + 16 * mt));
        const short4_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(vrow + 16 * VS + 16 * mt));
        const uint2 u0 = __builtin_bit_cast(uint2, v0), u1 = __builtin_bit_cast(uint2, v1);
        vpre[mt] = u32x4_t{u0.x, u0.y, u1.x, u1.y};
      }
      __builtin_amdgcn_sched_barrier(0);

      // softmax weights: lane holds row l16 of row tile rt and columns 32 h2 + 16 sb + 4g + v
      u32x4_t pb[2];  // per row tile: B operand of the K = 32 PV product
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) {
        float sv[2][4];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
          for (int v = 0; v < 4; ++v) sv[sb][v] = sacc[rt][sb][v];
        if (!all_open) {
#pragma unroll
          for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int v = 0; v < 4; ++v)
              sv[sb][v] = (open_bits[rt] >> (8 * h2 + 4 * sb + v) & 1u) ? sv[sb][v] : -INFINITY;
        }
        float mloc = -INFINITY;
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
          for (int v = 0; v < 4; ++v) mloc = fmaxf(mloc, sv[sb][v]);
        // fixed reference per row (set at the row's first open columns, re-based only when a half
        // tile tops it by more than 2^kRebase): no accumulator rescaling and no cross-lane traffic
        // per tile.  Weights more than 2^-24 below the reference vanish in fp16; they are that much
        // smaller than weights already summed.
        constexpr float kRebase = 12.f;  // fp16 weights: 2^(s - m_ref) stays far below 65504
        if (__any(mloc - m_ref[rt] > kRebase)) {  // also true while m_ref is -inf and a column is open
          float mt_ = fmaxf(mloc, __shfl_xor(mloc, 16, kWave));
          mt_ = fmaxf(mt_, __shfl_xor(mt_, 32, kWave));
          if (m_ref[rt] == -INFINITY) {
            m_ref[rt] = mt_;
          } else if (mt_ - m_ref[rt] > kRebase) {
            const float alpha = __builtin_amdgcn_exp2f(m_ref[rt] - mt_);
            m_ref[rt] = mt_;
            l_run[rt] *= alpha;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[rt][mt] *= alpha;
          }
        }
        const float m_sub = m_ref[rt] == -INFINITY ? 0.f : m_ref[rt];
        uint32_t pk[2][2];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
          float p[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) p[v] = __builtin_amdgcn_exp2f(sv[sb][v] - m_sub);
          pk[sb][0] = pack_f16x2(p[0], p[1]);
          pk[sb][1] = pack_f16x2(p[2], p[3]);
          l_run[rt] += (p[0] + p[1]) + (p[2] + p[3]);  // fp32 sum; the half rounding of a weight is 2^-12 of it
        }
        // K index 8g + e of the half: e < 4 -> column 4g + e of its first 16, else of its second 16
        pb[rt] = u32x4_t{pk[0][0], pk[0][1], pk[1][0], pk[1][1]};
      }

      // O^T[d, row] += V^T[d, col] P^T[col, row]; V^T comes out of LDS through the transposing read
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        u32x4_t vu;
        if (mt < VPRE) {
          vu = vpre[mt];
        } else {
          const short4_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(vrow + 16 * mt));
          const short4_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(vrow + 16 * VS + 16 * mt));
          const uint2 u0 = __builtin_bit_cast(uint2, v0), u1 = __builtin_bit_cast(uint2, v1);
          vu = u32x4_t{u0.x, u0.y, u1.x, u1.y};
        }
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
          acc[rt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, vu),
                                                               __builtin_bit_cast(f16x8_t, pb[rt]), acc[rt][mt], 0, 0, 0);
      }
      // the remaining reads go out ahead, between the first matrix instructions
#pragma unroll
      for (int i = 0; i < (MT - VPRE) / 2; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * MT - (MT - VPRE), 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- normalise and store: lane holds row l16 of row tile rt, output dims 16 mt + 4g .. +3
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    float l = l_run[rt] + __shfl_xor(l_run[rt], 16, kWave);
    l += __shfl_xor(l, 32, kWave);
    const int m = m0 + 32 * wv + 16 * rt + l16;
    if (m < T) {
      const float inv = m < len ? 1.f / l : 0.f;  // rows past the sequence's length are zeros
      float* po = out + (size_t)m * nh * DH + 4 * g;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) *reinterpret_cast<float4_t*>(po + 16 * mt) = acc[rt][mt] * inv;
    }
  }
  }  // pass
}

template <int DH, int DR>
hipError_t launch_attn_explicit(const ExplicitArgs& a, hipStream_t st, const EventPair& ev) {
  const int n_blocks = (a.T + 127) / 128;
  const dim3 grid((n_blocks + 1) / 2, a.n_heads, a.batch);  // two row blocks per workgroup
  launch_timed(attn_explicit_kernel<DH, DR>, grid, dim3(kBlock), 0, st, ev, a);
  return hipGetLastError();
}

}  // namespace

bool prefill_explicit_supported(const ExplicitArgs& a) {
  return (a.d_head == 64 || a.d_head == 128) && (a.d_rope == 32 || a.d_rope == 64) && a.r % 64 == 0 && a.r >= 64 &&
         a.r <= 512 && a.n_heads <= 65535 && a.batch <= 65535;
}

// partial states must already be in a.cprime (fp16 [B*T, r])
hipError_t launch_prefill_explicit(const ExplicitArgs& a, hipStream_t st, const EventPair& ev) {
  const size_t n_w = (size_t)a.n_heads * a.r * a.d_head;
  const size_t n_kr = (size_t)a.batch * a.T * a.d_rope;
  hipLaunchKernelGGL(to_f16_kernel, dim3((unsigned)((n_w + n_kr + kBlock - 1) / kBlock)), dim3(kBlock), 0, st,
                     reinterpret_cast<const uint16_t*>(a.w_uk), reinterpret_cast<const uint16_t*>(a.w_uv),
                     reinterpret_cast<uint16_t*>(a.w_kT), reinterpret_cast<uint16_t*>(a.w_v16),
                     reinterpret_cast<const uint16_t*>(a.kr), reinterpret_cast<uint16_t*>(a.kr16), a.n_heads, a.r,
                     a.d_head, n_kr);
  const int M = a.batch * a.T, N = a.n_heads * a.d_head;
  const dim3 grid((N + 127) / 128, (M + 127) / 128, 2);
  const uint16_t* A = reinterpret_cast<const uint16_t*>(a.cprime);
  const uint16_t* W0 = reinterpret_cast<const uint16_t*>(a.w_kT);
  const uint16_t* W1 = reinterpret_cast<const uint16_t*>(a.w_v16);
  uint16_t* C0 = reinterpret_cast<uint16_t*>(a.kx);
  uint16_t* C1 = reinterpret_cast<uint16_t*>(a.vx);
  switch (a.r / 32) {
#define MTLA_KK(K_) \
  case K_: hipLaunchKernelGGL(kv_up_kernel<K_>, grid, dim3(kBlock), 0, st, A, W0, W1, C0, C1, M, N); break;
    MTLA_KK(2) MTLA_KK(4) MTLA_KK(6) MTLA_KK(8) MTLA_KK(10) MTLA_KK(12) MTLA_KK(14) MTLA_KK(16)
#undef MTLA_KK
    default: return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.d_head == 64 && a.d_rope == 32) return launch_attn_explicit<64, 32>(a, st, ev);
  if (a.d_head == 64 && a.d_rope == 64) return launch_attn_explicit<64, 64>(a, st, ev);
  if (a.d_head == 128 && a.d_rope == 32) return launch_attn_explicit<128, 32>(a, st, ev);
  if (a.d_head == 128 && a.d_rope == 64) return launch_attn_explicit<128, 64>(a, st, ev);
  return hipErrorInvalidValue;
}

}  // namespace mtla
