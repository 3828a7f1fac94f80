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
// them are of order 1, far inside the half range.  bf16 inputs (RoPE keys, weights) convert exactly
// apart from values below 6e-5; the queries are multiplied by log2(e) / sqrt(d_h) before their one
// rounding to half.
//
// Three kernels:
//   to_f16_kernel         W_K^(h) with the contracted (latent) index innermost, like W_V^(h), and the
//                         RoPE keys, as fp16
//   gemm_nt_kernel        K = C_hat' W_K, V = C_hat' W_V for all T rows: a plain MFMA GEMM, 256 x 128
//                         tile, operands streamed from memory straight into LDS (also the projections
//                         of the whole-layer prefill, with rotation / scaling on the way out)
//   attn_explicit_kernel  one workgroup per pair of 128-row blocks of a (head, sequence); keys, RoPE
//                         keys and values of 32 columns at a time stream from memory straight into
//                         LDS and are shared by the four wavefronts (32 query rows each, queries in
//                         registers)
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

// Continuing sequences: the rows the key / value product and the attention read, 8 elements per thread.
//   part 1  rows k < past_pitch of sequence b: slot k of the cache (latent and RoPE key) if k < pos0 / s,
//           else zeros (never read as columns)
//   part 2  the chunk's partial states: run jl holds the chunk's tokens of slot pos0 / s + jl; the first
//           run continues the slot in progress from tail_prev when pos0 % s != 0
//   part 3  the chunk's RoPE keys
__global__ __launch_bounds__(kBlock) void chunk_stage_kernel(ChunkStageArgs a) {
  const int r8 = a.r / 8, d8 = a.d_rope / 8, s = a.stride, T = a.T, past = a.past_pitch, Tp = past + T;
  const int n_runs = (T + s - 1) / s + 1;
  const size_t n1 = (size_t)a.batch * past * (r8 + d8), n2 = (size_t)a.batch * n_runs * r8, n3 = (size_t)a.batch * T * d8;
  size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
  const uint16_t* cache_c = reinterpret_cast<const uint16_t*>(a.cache_c);
  const uint16_t* cache_kr = reinterpret_cast<const uint16_t*>(a.cache_kr);
  uint16_t* cp = reinterpret_cast<uint16_t*>(a.cprime);
  uint16_t* kr16 = reinterpret_cast<uint16_t*>(a.kr16);
  auto start_of = [&](int b) -> int {  // tokens before the chunk, forced into what the arrays hold
    if (!a.pos0) return 0;             // whole sequences
    const int p0 = a.pos0[b];
    if (p0 < 0 || p0 / s > past || p0 / s > a.max_slots) {
      *a.status = 1;  // MTLA_ERR_INVALID_ARG
      const int lim = past < a.max_slots ? past : a.max_slots;
      return lim * s;
    }
    return p0;
  };
  if (idx < n1) {
    const int piece = int(idx % (r8 + d8)), k = int(idx / (r8 + d8) % past), b = int(idx / ((size_t)(r8 + d8) * past));
    const bool live = k < start_of(b) / s;
    int sb = b;  // the sequence whose rows hold slot k: b itself, or the owner of a prompt it shares
    if (a.prefix_owner && k < a.prefix_slots[b]) {
      const int o = a.prefix_owner[b];
      sb = o < 0 ? 0 : (o < a.prefix_rows ? o : a.prefix_rows - 1);
    }
    u32x4_t v = {0u, 0u, 0u, 0u};
    const size_t src_row = live ? cache_row(a.pages, sb, k, a.max_slots) : 0;
    if (piece < r8) {
      if (live) v = bf16x8_to_f16x8(*reinterpret_cast<const u32x4_t*>(cache_c + src_row * a.r + 8 * piece));
      *reinterpret_cast<u32x4_t*>(cp + ((size_t)b * Tp + k) * a.r + 8 * piece) = v;
    } else {
      const int pd = piece - r8;
      if (live) v = bf16x8_to_f16x8(*reinterpret_cast<const u32x4_t*>(cache_kr + src_row * a.d_rope + 8 * pd));
      *reinterpret_cast<u32x4_t*>(kr16 + ((size_t)b * Tp + k) * a.d_rope + 8 * pd) = v;
    }
    return;
  }
  idx -= n1;
  if (idx < n2) {
    const int piece = int(idx % r8), jl = int(idx / r8 % n_runs), b = int(idx / ((size_t)r8 * n_runs));
    const int ph = start_of(b) % s;
    int n = jl * s - ph;
    const int n_end = n + s < T ? n + s : T;
    float run[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (jl == 0 && ph > 0) load8(a.tail_prev + (size_t)b * a.r + 8 * piece, run);
    if (n < 0) n = 0;
    const bf16* c = reinterpret_cast<const bf16*>(a.c);
    const int len = a.n_new ? a.n_new[b] : T;
    for (; n < n_end; ++n) {
      const size_t row = (size_t)b * T + n;
      u32x4_t o = {0u, 0u, 0u, 0u};  // padding rows hold zeros: they meet zero weights in the tiles of live rows
      if (n < len) {
        float cv[8];
        if (a.c32) load8(a.c32 + row * a.r + 8 * piece, cv);
        else load8(c + row * a.r + 8 * piece, cv);
        const float w = a.w[row];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          run[2 * i] += w * cv[2 * i];
          run[2 * i + 1] += w * cv[2 * i + 1];
          o[i] = pack_f16x2(run[2 * i], run[2 * i + 1]);
        }
      }
      *reinterpret_cast<u32x4_t*>(cp + ((size_t)b * Tp + past + n) * a.r + 8 * piece) = o;
    }
    return;
  }
  idx -= n2;
  if (idx < n3) {
    const int pd = int(idx % d8), n = int(idx / d8 % T), b = int(idx / ((size_t)d8 * T));
    *reinterpret_cast<u32x4_t*>(kr16 + ((size_t)b * Tp + past + n) * a.d_rope + 8 * pd) = bf16x8_to_f16x8(
        *reinterpret_cast<const u32x4_t*>(reinterpret_cast<const uint16_t*>(a.kr) + ((size_t)b * T + n) * a.d_rope + 8 * pd));
  }
}

// ---- memory -> LDS without registers --------------------------------------------------------
//
// Both kernels below stream their operands from memory straight into LDS: 16 bytes per lane, 64
// lanes fill 1 KB of consecutive LDS, several tiles ahead of the one being multiplied, so no
// register carries a tile and one barrier per tile is enough.  Rows are stored without padding;
// each 16-byte piece j of row `row` sits at position j ^ swizzle(row), chosen per region so that
// the reads of the matrix-core operands are free of bank conflicts:
//   swz_rows16   ds_read_b128, 16 lanes = 16 consecutive rows, same logical piece
//   swz_tr       transposing 8-byte reads, 32 lanes = 8 consecutive rows x 32 bytes
// The swizzle is applied on the way in: a lane asks memory for the piece that belongs at its place.
template <int PC>  // pieces per row (4, 8 or 16): 16 / PC rows share 256 bytes
__device__ __forceinline__ int swz_rows16(int row) {
  return (row / (16 / PC)) & (PC - 1);
}
template <int PC>
__device__ __forceinline__ int swz_tr(int row) {
  return ((row / (16 / PC)) & (PC / 2 - 1)) << 1;
}

typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;

// 64 lanes x 16 bytes from memory to 1 KB of LDS starting at byte address `lds_addr` (the same in
// every lane); lane i's 16 bytes land at lds_addr + 16 i.  Counted by vmcnt like any load.  Written
// as an instruction of its own so that the compiler keeps no account of it: the waits for these
// loads are the explicit ones below, and ordinary LDS reads are not held back by loads in flight
// into another buffer.
__device__ __forceinline__ void load_to_lds_16(const void* src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(src) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_loads_but() {  // until at most N of this wavefront's loads are in flight
  static_assert(N >= 0 && N <= 15, "vmcnt field");
  if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ void wait_loads_but(int n) {  // wavefront-uniform n, 0 .. 15
  switch (n) {
#define MTLA_W(N_) case N_: wait_loads_but<N_>(); break;
    MTLA_W(1) MTLA_W(2) MTLA_W(3) MTLA_W(4) MTLA_W(5) MTLA_W(6) MTLA_W(7) MTLA_W(8) MTLA_W(9) MTLA_W(10)
    MTLA_W(11) MTLA_W(12) MTLA_W(13) MTLA_W(14) MTLA_W(15)
#undef MTLA_W
    default: wait_loads_but<0>(); break;
  }
}
// workgroup barrier without a fence: callers order their own memory traffic around it
__device__ __forceinline__ void barrier_only() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// C[row][n] = sum_k A[row][k] W[n][k]   (A [M][K], W [N][K], C [M][N]; A and W both fp16 or both bf16,
// K % 32 == 0, N % 8 == 0), fp32 accumulation, one of four ways out (GemmArgs::epi):
//   0  C fp16 = scale * acc                       (keys, values, queries)
//   1  C fp16 = scale * RoPE(acc)                 (RoPE queries: row b*T + t is turned at pos0[b] + t; the
//      cosines and sines come from a table, rope_cs[row][k]).  With N1 > 0 a second product rides
//      along: columns N .. N + N1 - 1 are A W[1]^T, rotated the same way and stored as bf16 in C[1]
//      ([M, N1]: the shared RoPE key, as it is stored in the cache); N is then a multiple of 128.
//   3  C fp32 = acc
// Jobs = ceil(N/128) * ceil(M/256) * nz workgroups (z selects (W[z], C[z]): products that share A),
// numbered so that the workgroups that read the same rows of A and of W run on one XCD.  256 x 128
// tile; K is walked 32 at a time through three LDS stages of 24 KB.  Wavefront (wm, wn) owns a 128 x 64
// quarter: W rows are the A operand, A rows the B operand, so a lane ends up with four consecutive
// n of one row (two RoPE pairs).
template <bool BF16, int EPI, int BN>  // BN = 128: four wavefronts, two workgroups per CU; 256: eight wavefronts, one
__global__ __launch_bounds__(2 * BN, BN == 128 ? 2 : 1) void gemm_nt_kernel(GemmArgs a) {
  typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
  constexpr int BM = 256, BK = 32, NBUF = 3, PF = NBUF - 1;
  constexpr int NWV = 2 * BN / 64, NT = 64 * NWV, WCOLS = BN / 64;  // wavefronts: 2 row halves x BN/64 column strips
  constexpr int W_BYTES = BN * BK * 2, A_BYTES = BM * BK * 2, STAGE = W_BYTES + A_BYTES;  // 8 or 16 KB + 16 KB
  constexpr int NLW = W_BYTES / 1024 / NWV, NLA = A_BYTES / 1024 / NWV, LOADS = NLW + NLA;  // loads per wavefront and stage
  __shared__ __attribute__((aligned(1024))) unsigned char lds[NBUF * STAGE];

  const int M = a.M, K = a.K;
  const int Nt = a.N + (EPI == 1 ? a.N1 : 0);  // all columns of the launch
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g = lane >> 4;
  // Job order: groups of four column blocks of the weights (1 MB at K = 512 and 128 columns, stays in
  // L2) slowest, then the 256-row blocks of A, then the jobs of one row block inside the group; each
  // XCD takes an eighth of that list.
  const unsigned nz = (unsigned)a.nz;
  const unsigned gx = (unsigned)((Nt + BN - 1) / BN), gy = (unsigned)((M + BM - 1) / BM), jobs = gridDim.x, w = blockIdx.x;
  const unsigned job = jobs % 8 == 0 ? (w >> 3) + (w & 7) * (jobs >> 3) : w;
  // groups of four column blocks, then one group with the blocks that are left
  const unsigned full_jobs = (gx / 4u) * 4u * nz * gy;
  const bool in_full = job < full_jobs;
  const unsigned gsz = in_full ? 4u : gx % 4u, per_group = nz * gsz * gy;
  const unsigned first = in_full ? (job / per_group) * 4u : (gx / 4u) * 4u;
  const unsigned rem = in_full ? job % per_group : job - full_jobs, inner = rem % (nz * gsz);
  const int nb_all = (int)(first + inner / nz) * BN, rb = (int)(rem / (nz * gsz)) * BM;
  const bool seg1 = EPI == 1 && nb_all >= a.N;  // the block belongs to the second product
  const int z = seg1 ? 1 : (int)(inner % nz), nb = seg1 ? nb_all - a.N : nb_all, N = seg1 ? a.N1 : a.N;
  const uint16_t* A = reinterpret_cast<const uint16_t*>(a.A);
  const uint16_t* W = reinterpret_cast<const uint16_t*>(a.W[z]);
  const int wn = 64 * (wv % WCOLS), wm = 128 * (wv / WCOLS);

  // what this thread brings in of every stage: 1 KB chunk c of a region = rows 16 c .. 16 c + 15 (4
  // pieces of 8 k each); wavefront wv fills chunks wv, wv + NWV, ..
  const int prow = lane >> 2;
  const uint32_t psrc = 8 * ((lane & 3) ^ swz_rows16<4>(prow));
  const uint16_t* wsrc[NLW];
  const uint16_t* asrc[NLA];
#pragma unroll
  for (int i = 0; i < NLW; ++i) {
    const int row = nb + 16 * (wv + NWV * i) + prow;
    wsrc[i] = W + (size_t)(row < N ? row : N - 1) * K + psrc;
  }
#pragma unroll
  for (int i = 0; i < NLA; ++i) {
    const int row = rb + 16 * (wv + NWV * i) + prow;
    asrc[i] = A + (size_t)(row < M ? row : M - 1) * K + psrc;
  }
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_byte_ptr)lds;
  auto issue = [&](int st) {  // stage st: k = 32 st ..
    const uint32_t buf = lds_addr + (uint32_t)((st % NBUF) * STAGE);
#pragma unroll
    for (int i = 0; i < NLW; ++i) load_to_lds_16(wsrc[i] + BK * st, buf + (uint32_t)((wv + NWV * i) * 1024));
#pragma unroll
    for (int i = 0; i < NLA; ++i) load_to_lds_16(asrc[i] + BK * st, buf + W_BYTES + (uint32_t)((wv + NWV * i) * 1024));
  };
  // where this lane reads: rows 16 i + l16 of a quarter, logical piece g
  const uint32_t frag_off = (uint32_t)(l16 * 64 + ((g ^ swz_rows16<4>(l16)) << 4));

  float4_t acc[8][4];  // [token tile][n tile]
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[j][i] = float4_t{0.f, 0.f, 0.f, 0.f};

  const int n_stages = K / BK;
#pragma unroll
  for (int st = 0; st < PF; ++st)
    if (st < n_stages) issue(st);
  for (int st = 0; st < n_stages; ++st) {
    const int after = n_stages - 1 - st < PF - 1 ? n_stages - 1 - st : PF - 1;
    wait_loads_but(LOADS * after);
    barrier_only();
    if (st + PF < n_stages) issue(st + PF);  // into the buffer stage st-1 was read from
    const unsigned char* wb = lds + (st % NBUF) * STAGE + wn * 64 + frag_off;
    const unsigned char* ab = lds + (st % NBUF) * STAGE + W_BYTES + wm * 64 + frag_off;
    u32x4_t wf[4], af[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) wf[i] = *reinterpret_cast<const u32x4_t*>(wb + i * 1024);
#pragma unroll
    for (int j = 0; j < 8; ++j) af[j] = *reinterpret_cast<const u32x4_t*>(ab + j * 1024);
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (BF16)
          acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wf[i]),
                                                              __builtin_bit_cast(bf16x8_t, af[j]), acc[j][i], 0, 0, 0);
        else
          acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, wf[i]),
                                                             __builtin_bit_cast(f16x8_t, af[j]), acc[j][i], 0, 0, 0);
      }
  }

  // ---- rotation: the lane's columns n .. n+3 are two pairs of one head
  if constexpr (EPI == 1) {
    const int half = a.d_rope / 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int row = rb + wm + 16 * j + l16;
      row = row < M ? row : M - 1;
      const float4* cs_row = reinterpret_cast<const float4*>(a.rope_cs + (size_t)row * half);  // (cos, sin) per pair
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int jn = (nb + wn + 16 * i + 4 * g) % a.d_rope;  // element inside the head, a multiple of 4
        const float4 cs = cs_row[jn / 4];                      // pairs jn/2 and jn/2 + 1
        const float e0 = acc[j][i][0], e1 = acc[j][i][1], e2 = acc[j][i][2], e3 = acc[j][i][3];
        acc[j][i] = float4_t{e0 * cs.x - e1 * cs.y, e0 * cs.y + e1 * cs.x, e2 * cs.z - e3 * cs.w, e2 * cs.w + e3 * cs.z};
      }
      __builtin_amdgcn_sched_barrier(0);  // one row's table entries in registers at a time
    }
  }

  // ---- the tile leaves through LDS, RP rows at a time (as many as the stage buffers hold), so that
  // memory sees whole row segments of 256 bytes or more
  constexpr int ES = EPI == 3 ? 4 : 2;                       // bytes per output element
  constexpr int CS = ES * BN + 16;                           // LDS row pitch
  constexpr int RP = NBUF * STAGE / CS >= 256 ? 256 : (NBUF * STAGE / CS >= 128 ? 128 : 64);
  static_assert(RP * CS <= NBUF * STAGE, "the rows of a pass fit in the stage buffers");
  constexpr int PPR = BN * ES / 16;                          // 16-byte pieces per row
  static_assert(RP * PPR % NT == 0, "whole rounds of stores");
  unsigned char* Cb = reinterpret_cast<unsigned char*>(a.C[z]);
  const float sc = a.scale;
  barrier_only();  // every wavefront is done with the last stage
#pragma unroll
  for (int pass = 0; pass < BM / RP; ++pass) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int row = wm + 16 * j;                           // wavefront-uniform
      if (row / RP != pass) continue;
      unsigned char* lrow = lds + (row - RP * pass + l16) * CS;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int col = wn + 16 * i + 4 * g;
        if constexpr (EPI == 3) {
          *reinterpret_cast<float4_t*>(lrow + 4 * col) = acc[j][i];
        } else {
          uint2 o;
          if (seg1) o = make_uint2(pack_bf16x2(acc[j][i][0], acc[j][i][1]), pack_bf16x2(acc[j][i][2], acc[j][i][3]));
          else o = make_uint2(pack_f16x2(sc * acc[j][i][0], sc * acc[j][i][1]), pack_f16x2(sc * acc[j][i][2], sc * acc[j][i][3]));
          *reinterpret_cast<uint2*>(lrow + 2 * col) = o;
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < RP * PPR / NT; ++i) {
      const int p_ = tid + NT * i, row = p_ / PPR, c = p_ % PPR;
      const int grow = rb + RP * pass + row, gcol = nb + c * (16 / ES);
      if (grow < M && gcol < N)  // N is a multiple of 8
        *reinterpret_cast<u32x4_t*>(Cb + ((size_t)grow * N + gcol) * ES) = *reinterpret_cast<const u32x4_t*>(lds + row * CS + 16 * c);
    }
    if (pass + 1 < BM / RP) __syncthreads();
  }
}

// ---- attention over explicit keys and values -------------------------------------------------
//
// A tile is 32 columns: their keys [32][d_h] (swz_rows16), RoPE keys [32][d_R] (swz_rows16) and
// values [32][d_h] (swz_tr), fp16, fetched two tiles ahead through three LDS buffers.
template <int DH, int DR>
struct TileGeom {
  static constexpr int BN = 32, VC = DH / 8, RC = DR / 8;  // 16-byte pieces per key / value row, per RoPE key row
  static constexpr int K_BYTES = BN * DH * 2, R_BYTES = BN * DR * 2;
  static constexpr int K_OFF = 0, R_OFF = K_BYTES, V_OFF = K_BYTES + R_BYTES, BYTES = 2 * K_BYTES + R_BYTES;
  static constexpr int NCK = BN * VC / 64, NCR = BN * RC / 64;  // wavefront loads (1 KB) per region
  static_assert(BYTES % 1024 == 0 && K_BYTES % 1024 == 0 && R_BYTES % 1024 == 0, "1 KB per wavefront load");
};

// NW wavefronts of 32 query rows each per workgroup; grid = ceil(ceil(T / (32 NW)) / 2) * n_heads * B.
// NW = 4 is what the launcher uses: two workgroups per CU, whose wavefronts drift apart so that one
// multiplies while the other does softmax arithmetic.  (NW = 8, one workgroup per CU with every
// tile serving twice the rows, halves the L2 traffic but measured 1 - 10 % slower: the two wavefronts
// of a SIMD then walk the phases in step.)
// CONT: the sequences continue from a cache (a.pos0, a.past_pitch); whole sequences are compiled without it.
// LAYER: the whole-layer prefill's operands (queries already fp16 and scaled, output as fp16 for W_O).
template <int DH, int DR, int NW, bool CONT, bool LAYER>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attn_explicit_kernel(ExplicitArgs a) {
  using G = TileGeom<DH, DR>;
  constexpr int KD = DH / 32, KQ = (DH + DR) / 32, MT = DH / 16;
  constexpr int NT = 64 * NW, BM = 32 * NW, BN = G::BN, VC = G::VC, RC = G::RC;
  constexpr int NBUF = 4, PF = NBUF - 1;  // tiles in LDS, tiles requested ahead
  constexpr int NIK = (G::NCK + NW - 1) / NW, NIR = (G::NCR + NW - 1) / NW;  // loads per wavefront and region, at most
  __shared__ __attribute__((aligned(1024))) unsigned char lds[NBUF * G::BYTES];

  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g = lane >> 4;
  const int T = a.T, s = a.stride, nh = a.n_heads;
  // Workgroups are handed to the 8 XCDs in turn.  The row blocks of one (sequence, head) read the
  // same keys and values, so they are numbered to land on one XCD and meet in its L2: workgroup w of
  // the launch takes job (w / 8) + (w % 8) * (jobs / 8), jobs ordered (sequence, head, block pair).
  const int n_blocks = (T + BM - 1) / BM, n_pairs = (n_blocks + 1) / 2;
  const unsigned jobs = gridDim.x, w = blockIdx.x;
  const unsigned job = jobs % 8 == 0 ? (w >> 3) + (w & 7) * (jobs >> 3) : w;
  // Latent-space output (a.n_slices > 0): the values are the partial states themselves, DH of their r
  // columns per job (the same rows for every head), and the output row has r columns per head.
  const int n_sl = LAYER || a.n_slices < 1 ? 1 : a.n_slices;
  const bool lat = !LAYER && a.n_slices > 0;
  const int pair = (int)(job % (unsigned)n_pairs), sl = (int)(job / (unsigned)n_pairs % (unsigned)n_sl),
            h = (int)(job / (unsigned)(n_pairs * n_sl) % (unsigned)nh), b = (int)(job / (unsigned)(n_pairs * n_sl * nh));
  const int len = a.seq_len ? (a.seq_len[b] < T ? a.seq_len[b] : T) : T;
  // A continuing sequence has p0 tokens behind it: the final states of its first p0 / s slots are the
  // first rows of the key / value arrays (one per slot), the chunk's T rows follow at row `past`.
  const int past = CONT ? a.past_pitch : 0, Tp = past + T;
  int p0 = CONT ? a.pos0[b] : 0;
  if (p0 < 0 || p0 / s > past) p0 = past * s;  // out of range (reported by the staging kernel): stay inside the arrays
  const int j0 = p0 / s;
  const size_t out_stride = lat ? (size_t)nh * a.r : (size_t)nh * DH;  // elements per output row
  float* out = lat ? a.out + ((size_t)b * T * nh + h) * a.r + (size_t)sl * DH : a.out + ((size_t)b * T * nh + h) * DH;
  const uint16_t* kx = reinterpret_cast<const uint16_t*>(a.kx) + ((size_t)b * Tp * nh + h) * DH;
  const uint16_t* vx = lat ? reinterpret_cast<const uint16_t*>(a.cprime) + (size_t)b * Tp * a.r + (size_t)sl * DH
                           : reinterpret_cast<const uint16_t*>(a.vx) + ((size_t)b * Tp * nh + h) * DH;
  const uint16_t* kr16 = reinterpret_cast<const uint16_t*>(a.kr16) + (size_t)b * Tp * DR;
  const uint32_t kv_stride = (uint32_t)(nh * DH), v_stride = lat ? (uint32_t)a.r : kv_stride;

  // ---- what this thread brings in of every tile.  Wavefront wv fills the 1 KB chunks wv, wv + NW, ..
  // of a region; lane i of it the chunk's piece i: row and (swizzled) source piece, the same for
  // all of the wavefront's chunks (they lie a multiple of 16 rows apart).
  const int pk = 64 * wv + lane;
  const int row_k = pk / VC, row_r = pk / RC;
  const uint32_t src_k = 8 * ((pk % VC) ^ swz_rows16<VC>(row_k));  // element offset inside the source row
  const uint32_t src_v = 8 * ((pk % VC) ^ swz_tr<VC>(row_k));
  const uint32_t src_r = 8 * ((pk % RC) ^ swz_rows16<RC>(row_r));
  static_assert(NIK == 1 || (64 * NW / VC) % 16 == 0, "same swizzle for all chunks of a wavefront");
  static_assert(NIR == 1, "one RoPE key chunk per wavefront at most");
  int loads = 0;  // loads of this wavefront per tile
#pragma unroll
  for (int i = 0; i < NIK; ++i) loads += wv + NW * i < G::NCK ? 2 : 0;
  loads += wv < G::NCR ? 1 : 0;
  // ---- where this lane reads: key rows 16 sb + l16 (piece 4 kk + g), value rows 4g + l16/4 (+16)
  const uint32_t k_row_off = (uint32_t)(l16 * VC * 16), k_swz = (uint32_t)(swz_rows16<VC>(l16) ^ g) << 4;
  const uint32_t r_row_off = (uint32_t)(l16 * RC * 16), r_swz = (uint32_t)(swz_rows16<RC>(l16) ^ g) << 4;
  const int v_row = 4 * g + (l16 >> 2);
  const uint32_t v_row_off = (uint32_t)(v_row * VC * 16 + 8 * (l16 & 1));
  const uint32_t v_swz = (uint32_t)(swz_tr<VC>(v_row) ^ ((l16 & 3) >> 1)) << 4;

  // Row block x walks x * BM / (s BN) + BM / BN tiles.  A workgroup takes block n-1-x and then block
  // x, so every workgroup of the launch walks the same number of tiles (the middle one, if n is odd,
  // half).
  for (int pass = 0; pass < 2; ++pass) {
    const int xb = pass == 0 ? n_blocks - 1 - pair : pair;
    if (pass == 1 && xb >= n_blocks - 1 - pair) break;
    const int m0 = xb * BM;
    if (m0 >= len) {  // padding rows only
      const int rows = T - m0 < BM ? T - m0 : BM;
      for (int i = tid; i < rows * (DH / 4); i += NT) {
        const size_t row = (size_t)(m0 + i / (DH / 4));
        if constexpr (LAYER)
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out16) + (((size_t)b * T + row) * nh + h) * DH + 4 * (i % (DH / 4))) =
              make_uint2(0u, 0u);
        else
          *reinterpret_cast<float4_t*>(out + row * out_stride + 4 * (i % (DH / 4))) = float4_t{0.f, 0.f, 0.f, 0.f};
      }
      continue;
    }
    // ---- the columns: shared ones, slots j < (p0 + m0) / s (a slot of the past: row j; one closed
    // inside the chunk: the chunk's row j*s + s-1 - p0), then the block's own rows
    const int n_sh = (p0 + m0) / s, n_sh_tiles = (n_sh + BN - 1) / BN, n_tiles = n_sh_tiles + BM / BN;

    // source row of column `row` of tile t (tiles past the last one: a readable duplicate)
    auto src_row = [&](int t, int row) -> uint32_t {
      if (t < n_sh_tiles) {
        const int c = BN * t + row < n_sh ? BN * t + row : n_sh - 1;
        return (uint32_t)(c < j0 ? c : past + c * s + s - 1 - p0);
      }
      const int r_ = m0 + BN * (t - n_sh_tiles) + row;
      return (uint32_t)(past + (r_ < T ? r_ : T - 1));
    };
    // this wavefront's part of tile t on its way into buffer t % NBUF: `loads` loads
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_byte_ptr)lds;
    auto issue = [&](int t) {
      const uint32_t buf = lds_addr + (uint32_t)((t % NBUF) * G::BYTES);
#pragma unroll
      for (int i = 0; i < NIK; ++i)
        if (wv + NW * i < G::NCK) {
          const uint32_t srow = src_row(t, row_k + i * (64 * NW / VC));
          const uint32_t chunk = (uint32_t)((wv + NW * i) * 1024);
          load_to_lds_16(kx + srow * kv_stride + src_k, buf + G::K_OFF + chunk);
          load_to_lds_16(vx + srow * v_stride + src_v, buf + G::V_OFF + chunk);
        }
      if (wv < G::NCR) load_to_lds_16(kr16 + src_row(t, row_r) * DR + src_r, buf + G::R_OFF + (uint32_t)(wv * 1024));
    };

    // ---- queries of this wavefront's 32 rows: B operand, lane = row l16 of row tile rt
    u32x4_t qf[2][KQ];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const int m = m0 + 32 * wv + 16 * rt + l16;
      const size_t row = (size_t)b * T + (m < T ? m : T - 1);
      const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + (row * nh + h) * DH + 8 * g;
      const uint16_t* qrp = reinterpret_cast<const uint16_t*>(a.q_rope) + (row * nh + h) * DR + 8 * g;
#pragma unroll
      for (int kk = 0; kk < KQ; ++kk) {
        const u32x4_t raw = kk < KD ? *reinterpret_cast<const u32x4_t*>(qp + 32 * kk)
                                    : *reinterpret_cast<const u32x4_t*>(qrp + 32 * (kk - KD));
        // logits come out in units of log2: log2(e) / sqrt(d_h) folded in
        qf[rt][kk] = LAYER ? raw : bf16x8_to_f16x8(raw, a.scale_log2);
      }
    }

    float m_ref[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
    float4_t acc[2][MT];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};

    // bit 8 dt + 4 sb + v of closes_mask: row m0 + 32 dt + 16 sb + 4g + v of the block closes a chunk
    unsigned long long closes_mask = 0;
#pragma unroll
    for (int i = 0; i < 8 * NW; ++i) {
      const int c = BN * (i >> 3) + 16 * ((i >> 2) & 1) + 4 * g + (i & 3);
      closes_mask |= (unsigned long long)((p0 + m0 + c + 1) % s == 0 ? 1u : 0u) << i;
    }

    // every wavefront is done with the buffers of the previous block (no tile load is in flight:
    // the last tiles of a block wait for everything)
    wait_loads_but<0>();
    barrier_only();
#pragma unroll
    for (int t = 0; t < PF; ++t)
      if (t < n_tiles) issue(t);

    for (int t = 0; t < n_tiles; ++t) {
      // tile t has landed: this wavefront's part (all but the loads of the tiles after it), then everyone's
      const int after = n_tiles - 1 - t < PF - 1 ? n_tiles - 1 - t : PF - 1;
      wait_loads_but(loads * after);
      barrier_only();
      if (t + PF < n_tiles) issue(t + PF);  // into the buffer tile t-1 was read from: every wavefront is past that

      // Visibility.  A shared tile below n_sh is open to every row; the last shared tile is cut at
      // n_sh; a tile of the block's own rows is open to row rrel at column c iff c == rrel (the row's
      // own running state) or c < rrel and row m0 + c closes a chunk (closes_mask, set up once).
      const bool own = t >= n_sh_tiles;
      const int dt = t - n_sh_tiles;
      if (own && dt > wv) continue;  // all 32 columns lie above this wavefront's rows
      const int cbase = own ? BN * dt : BN * t;
      const bool all_open = !own && cbase + BN <= n_sh;
      // bit 4 sb + v of open_bits[rt]: column 16 sb + 4g + v of the tile is open to the lane's row
      uint32_t open_bits[2] = {0xffu, 0xffu};
      if (!all_open) {  // workgroup-uniform: five tiles per row block at most come here
        const uint32_t closes = own ? (uint32_t)(closes_mask >> (8 * dt)) : 0xffu;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
          const int bound = own ? 32 * wv + 16 * rt + l16 : n_sh;  // columns below `bound` may be open
          uint32_t m = 0;
#pragma unroll
          for (int sb = 0; sb < 2; ++sb) {
            const int d = bound - (cbase + 16 * sb + 4 * g);  // column 4g + v of the group is below iff v < d
            const int dd = d < 0 ? 0 : (d > 4 ? 4 : d);
            const uint32_t lt = (1u << dd) - 1u;
            const uint32_t eq = own ? (uint32_t)((unsigned)d < 4u) << (d & 3) : 0u;
            m |= ((lt & (closes >> (4 * sb)) & 0xfu) | eq) << (4 * sb);
          }
          open_bits[rt] = m;
        }
      }

      const uint32_t buf = (uint32_t)((t % NBUF) * G::BYTES);  // byte offset of the tile in `lds`
      const unsigned char* kb = lds + buf + G::K_OFF + k_row_off;
      const unsigned char* rb = lds + buf + G::R_OFF + r_row_off;
      const unsigned char* vb = lds + buf + G::V_OFF + v_row_off;
      auto read_k = [&](int kk, int sb) -> u32x4_t {  // [k | k^R] rows 16 sb + l16, elements 32 kk + 8g ..
        return kk < KD ? *reinterpret_cast<const u32x4_t*>(kb + sb * (16 * VC * 16) + ((uint32_t)(64 * kk) ^ k_swz))
                       : *reinterpret_cast<const u32x4_t*>(rb + sb * (16 * RC * 16) + ((uint32_t)(64 * (kk - KD)) ^ r_swz));
      };
      auto read_v = [&](int mt) -> u32x4_t {  // V^T rows 16 mt + l16 (dims), columns 8g .. (K index of the PV product)
        const unsigned char* p = vb + ((uint32_t)(32 * mt) ^ v_swz);
        const short4_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)p);
        const short4_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p + 16 * VC * 16));
        const uint2 u0 = __builtin_bit_cast(uint2, v0), u1 = __builtin_bit_cast(uint2, v1);
        return u32x4_t{u0.x, u0.y, u1.x, u1.y};
      };

      // ---- S^T[col, row] = [k | k^R][col, :] . [q | q^R][row, :]: the reads of one half of the K
      // steps are in flight while the other half is multiplied
      constexpr int KH = KQ / 2;
      float4_t sacc[2][2];
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) sacc[rt][sb] = float4_t{0.f, 0.f, 0.f, 0.f};
      u32x4_t ka[KH][2], kc[KQ - KH][2];
#pragma unroll
      for (int kk = 0; kk < KH; ++kk)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) ka[kk][sb] = read_k(kk, sb);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = KH; kk < KQ; ++kk)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) kc[kk - KH][sb] = read_k(kk, sb);
#pragma unroll
      for (int kk = 0; kk < KH; ++kk)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
          for (int rt = 0; rt < 2; ++rt)
            sacc[rt][sb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, ka[kk][sb]),
                                                                  __builtin_bit_cast(f16x8_t, qf[rt][kk]), sacc[rt][sb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      // the first value fragments travel while the second half is multiplied and the softmax runs
      constexpr int VPRE = MT / 2;
      u32x4_t vpre[VPRE];
#pragma unroll
      for (int mt = 0; mt < VPRE; ++mt) vpre[mt] = read_v(mt);
#pragma unroll
      for (int kk = KH; kk < KQ; ++kk)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
          for (int rt = 0; rt < 2; ++rt)
            sacc[rt][sb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, kc[kk - KH][sb]),
                                                                  __builtin_bit_cast(f16x8_t, qf[rt][kk]), sacc[rt][sb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);

      // ---- softmax weights: lane holds row l16 of row tile rt and columns 16 sb + 4g + v
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
            for (int v = 0; v < 4; ++v) sv[sb][v] = (open_bits[rt] >> (4 * sb + v) & 1u) ? sv[sb][v] : -INFINITY;
        }
        float mloc = -INFINITY;
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
          for (int v = 0; v < 4; ++v) mloc = fmaxf(mloc, sv[sb][v]);
        // fixed reference per row (set at the row's first open columns, re-based only when a tile
        // tops it by more than 2^kRebase): no accumulator rescaling and no cross-lane traffic per
        // tile.  Weights more than 2^-24 below the reference vanish in fp16; they are that much
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
        uint32_t pk2[2][2];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
          float p[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) p[v] = __builtin_amdgcn_exp2f(sv[sb][v] - m_sub);
          pk2[sb][0] = pack_f16x2(p[0], p[1]);
          pk2[sb][1] = pack_f16x2(p[2], p[3]);
          l_run[rt] += (p[0] + p[1]) + (p[2] + p[3]);  // fp32 sum; the half rounding of a weight is 2^-12 of it
        }
        // K index 8g + e of the tile: e < 4 -> column 4g + e of its first 16, else of its second 16
        pb[rt] = u32x4_t{pk2[0][0], pk2[0][1], pk2[1][0], pk2[1][1]};
      }

      // ---- O^T[d, row] += V^T[d, col] P^T[col, row]; V^T comes out of LDS through the transposing read
      __builtin_amdgcn_sched_barrier(0);
      u32x4_t vpost[MT - VPRE];
#pragma unroll
      for (int mt = VPRE; mt < MT; ++mt) vpost[mt - VPRE] = read_v(mt);
#pragma unroll
      for (int mt = 0; mt < VPRE; ++mt)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
          acc[rt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, vpre[mt]),
                                                               __builtin_bit_cast(f16x8_t, pb[rt]), acc[rt][mt], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mt = VPRE; mt < MT; ++mt)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
          acc[rt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, vpost[mt - VPRE]),
                                                               __builtin_bit_cast(f16x8_t, pb[rt]), acc[rt][mt], 0, 0, 0);
    }

    // ---- normalise and store: lane holds row l16 of row tile rt, output dims 16 mt + 4g .. +3
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      float l = l_run[rt] + __shfl_xor(l_run[rt], 16, kWave);
      l += __shfl_xor(l, 32, kWave);
      const int m = m0 + 32 * wv + 16 * rt + l16;
      if (m < T) {
        const bool live = m < len;  // rows past the sequence's length are zeros, whatever their inputs held
        const float inv = live ? 1.f / l : 0.f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[rt][mt] = live ? acc[rt][mt] * inv : float4_t{0.f, 0.f, 0.f, 0.f};
        if constexpr (LAYER) {
          uint16_t* po = reinterpret_cast<uint16_t*>(a.out16) + (((size_t)b * T + m) * nh + h) * DH + 4 * g;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const float4_t o = acc[rt][mt];
            *reinterpret_cast<uint2*>(po + 16 * mt) = make_uint2(pack_f16x2(o[0], o[1]), pack_f16x2(o[2], o[3]));
          }
        } else {
          float* po = out + (size_t)m * out_stride + 4 * g;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) *reinterpret_cast<float4_t*>(po + 16 * mt) = acc[rt][mt];
        }
      }
    }
  }  // pass
}

template <int DH, int DR>
hipError_t launch_attn_explicit(const ExplicitArgs& a, hipStream_t st, const EventPair& ev) {
  constexpr int NW = 4;
  const int n_blocks = (a.T + 32 * NW - 1) / (32 * NW);
  const int n_sl = a.n_slices > 0 ? a.n_slices : 1;
  if (a.n_slices > 0 && (a.q_f16 != 0 || a.n_slices * DH != a.r)) return hipErrorInvalidValue;
  const dim3 grid((unsigned)((n_blocks + 1) / 2) * n_sl * a.n_heads * a.batch);  // two row blocks per workgroup
  const bool layer = a.q_f16 != 0;  // comes with out16
  if (layer != (a.out16 != nullptr) || (layer && !a.pos0)) return hipErrorInvalidValue;
  if (layer) launch_timed(attn_explicit_kernel<DH, DR, NW, true, true>, grid, dim3(64 * NW), 0, st, ev, a);
  else if (a.pos0) launch_timed(attn_explicit_kernel<DH, DR, NW, true, false>, grid, dim3(64 * NW), 0, st, ev, a);
  else launch_timed(attn_explicit_kernel<DH, DR, NW, false, false>, grid, dim3(64 * NW), 0, st, ev, a);
  return hipGetLastError();
}

}  // namespace

bool prefill_explicit_supported(const ExplicitArgs& a) {
  return (a.d_head == 64 || a.d_head == 128) && (a.d_rope == 32 || a.d_rope == 64) && a.r % 64 == 0 && a.r >= 64 &&
         a.r <= 512 && a.n_heads <= 65535 && a.batch <= 65535 &&
         (size_t)((a.T + 255) / 256) * a.n_heads * a.batch * (a.out_latent ? a.r / a.d_head : 1) < (size_t)1 << 31 &&  // workgroups of the attention launch
         (!a.out_latent || (a.r % a.d_head == 0 && !a.pos0 && !a.q_f16)) &&
         (size_t)(a.past_pitch + a.T) * a.n_heads * a.d_head < (size_t)1 << 31 &&  // 32-bit element offsets inside one sequence
         (size_t)a.batch * (a.past_pitch + a.T) < (size_t)1 << 31;                 // rows of the key / value product
}

bool gemm_nt_supported(const GemmArgs& a) {
  const int n1 = a.epi == 1 ? a.N1 : 0;
  return a.M >= 1 && (a.N >= 8 || (a.epi == 1 && a.N == 0 && a.N1 >= 8)) && a.N % 8 == 0 && a.K >= 32 && a.K % 32 == 0 && (a.nz == 1 || a.nz == 2) &&
         (size_t)((a.N + n1 + 127) / 128) * ((a.M + 255) / 256) * a.nz < (size_t)1 << 31 &&
         (a.epi == 0 || a.epi == 3 ||
          (a.epi == 1 && a.nz == 1 && a.d_rope % 4 == 0 && a.d_rope >= 4 && a.rope_cs && a.N % a.d_rope == 0 &&
           n1 % 8 == 0 && n1 >= 0 && (n1 == 0 || (a.N % 256 == 0 && n1 % a.d_rope == 0))));
}

// (cos, sin) of pos * freq[k] for row b*T + t at position pos0[b] + t, k < d_rope / 2
__global__ __launch_bounds__(kBlock) void rope_table_kernel(RopeTableArgs a) {
  const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
  const int half = a.d_rope / 2;
  if (idx >= a.rows * half) return;
  const size_t row = idx / half;
  const int k = int(idx % half), b = int(row / a.T);
  const int pos = (a.pos0 ? a.pos0[b] : 0) + int(row - (size_t)b * a.T);
  float cs = 1.f, sn = 0.f;
  rope_pair(cs, sn, pos, a.rope_freq[k]);  // (1, 0) turned by the angle
  a.table[idx] = make_float2(cs, sn);
}

hipError_t launch_rope_table(const RopeTableArgs& a, hipStream_t st) {
  const size_t n = a.rows * (a.d_rope / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_gemm_nt(const GemmArgs& a, hipStream_t st) {
  if (!gemm_nt_supported(a)) return hipErrorInvalidValue;
  const int n_all = a.N + (a.epi == 1 ? a.N1 : 0);
  // 256-column tiles (a third less traffic into LDS per flop) when they fill: whole tiles of both products
  const bool wide = a.wide >= 0 ? (a.wide != 0 && a.N % 256 == 0) : (a.N % 256 == 0 && (a.epi != 1 || a.N1 == 0 || a.N >= 1024));
  const int bn = wide ? 256 : 128;
  const dim3 grid((unsigned)((n_all + bn - 1) / bn) * (unsigned)((a.M + 255) / 256) * (unsigned)a.nz);
#define MTLA_GEMM(BF, EP)                                                                                   \
  if ((a.in_bf16 != 0) == BF && a.epi == EP) {                                                              \
    if (wide) hipLaunchKernelGGL((gemm_nt_kernel<BF, EP, 256>), grid, dim3(512), 0, st, a);                 \
    else hipLaunchKernelGGL((gemm_nt_kernel<BF, EP, 128>), grid, dim3(256), 0, st, a);                      \
  }
  MTLA_GEMM(false, 0)
  MTLA_GEMM(false, 3)
  MTLA_GEMM(true, 0)
  MTLA_GEMM(true, 1)
  MTLA_GEMM(true, 3)
#undef MTLA_GEMM
  return hipGetLastError();
}

hipError_t launch_chunk_stage(const ChunkStageArgs& a, hipStream_t st) {
  const size_t r8 = a.r / 8, d8 = a.d_rope / 8, n_runs = (a.T + a.stride - 1) / a.stride + 1;
  const size_t n = (size_t)a.batch * a.past_pitch * (r8 + d8) + (size_t)a.batch * n_runs * r8 + (size_t)a.batch * a.T * d8;
  hipLaunchKernelGGL(chunk_stage_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, a);
  return hipGetLastError();
}

// partial states must already be in a.cprime (fp16 [B*T, r]); for continuing sequences (a.pos0) the
// staging kernel has filled a.cprime and a.kr16 ([B*(past_pitch + T), ..])
hipError_t launch_prefill_explicit(const ExplicitArgs& a, hipStream_t st, const EventPair& ev) {
  const size_t n_w = (size_t)a.n_heads * a.r * a.d_head;
  const size_t n_kr = (a.pos0 || a.kr_staged) ? 0 : (size_t)a.batch * a.T * a.d_rope;
  hipLaunchKernelGGL(to_f16_kernel, dim3((unsigned)((n_w + n_kr + kBlock - 1) / kBlock)), dim3(kBlock), 0, st,
                     reinterpret_cast<const uint16_t*>(a.w_uk), reinterpret_cast<const uint16_t*>(a.w_uv),
                     reinterpret_cast<uint16_t*>(a.w_kT), reinterpret_cast<uint16_t*>(a.w_v16),
                     reinterpret_cast<const uint16_t*>(a.kr), reinterpret_cast<uint16_t*>(a.kr16), a.n_heads, a.r,
                     a.d_head, n_kr);
  GemmArgs ga;  // K = C_hat' W_K, V = C_hat' W_V for all rows
  ga.A = a.cprime;
  ga.W[0] = a.w_kT;
  ga.W[1] = a.w_v16;
  ga.C[0] = a.kx;
  ga.C[1] = a.vx;
  ga.M = a.batch * (a.past_pitch + a.T);
  ga.N = a.n_heads * a.d_head;
  ga.K = a.r;
  ga.nz = 2;
  hipError_t e = launch_gemm_nt(ga, st);
  if (e != hipSuccess) return e;
  auto attend = [&](const ExplicitArgs& x, const EventPair& e) -> hipError_t {
    if (x.d_head == 64 && x.d_rope == 32) return launch_attn_explicit<64, 32>(x, st, e);
    if (x.d_head == 64 && x.d_rope == 64) return launch_attn_explicit<64, 64>(x, st, e);
    if (x.d_head == 128 && x.d_rope == 32) return launch_attn_explicit<128, 32>(x, st, e);
    if (x.d_head == 128 && x.d_rope == 64) return launch_attn_explicit<128, 64>(x, st, e);
    return hipErrorInvalidValue;
  };
  if (!a.out_latent) return attend(a, ev);
  // The latent-space output is softmax . C_hat' with the same weights: a second pass of the same kernel
  // whose values are the partial states, d_head of their r columns per job (the logits are formed
  // again for every slice).  The timed launch is this one.
  e = attend(a, EventPair());
  if (e != hipSuccess) return e;
  ExplicitArgs l = a;
  l.out = a.out_latent;
  l.out_latent = nullptr;
  l.n_slices = a.r / a.d_head;
  return attend(l, ev);
}

}  // namespace mtla
