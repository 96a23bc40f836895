// bf16 GEMMs of the stage on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
//   NT:  C[M,N] = A[M,K] . B[N,K]^T     both operands contiguous along the reduction axis
//        (forward with the weight copy stored [out,in]; input gradients with the weights as given)
//   TN:  C[M,N] = A[K,M]^T . B[K,N]     both operands strided along the reduction axis, which is
//        the token axis (weight gradients: A = layer input, B = output gradient)
//
// One work-group = 256 threads = 2 x 2 waves computes a BM x BN tile in 64-deep slices.  Slices go
// global -> registers -> LDS (two LDS stages, one barrier per slice).  NT tiles are stored
// [row][64] with the 16-byte chunk index XOR-ed by ((row >> 1) & 7) so that the 16-byte fragment reads
// are bank-conflict free.  TN tiles are stored as they lie in memory,
// [reduction row][BM] (XOR-swizzled), and fragments are fetched with the LDS transpose read
// (ds_read_b64_tr_b16), which hands every lane four reduction-consecutive values of its column.
//
// The MFMA is issued with its operands swapped (A operand <- B tile, B operand <- A tile): the
// accumulator of lane l then holds, for output row m = l % 32, four consecutive output columns per
// register quad, so the epilogue reads bias / residual and writes C with 8-byte (bf16) or 16-byte
// (fp32 accumulate) vectors.
//
// Block index -> tile: consecutive block ids land on different XCDs (8 of them, each with its own
// L2), so block b works on tile (b % 8) * ceil(tiles/8) + b / 8: every XCD owns a contiguous run of
// the tile order, and that order walks groups of four tile-rows column by column.
#include "common.h"
#include "../../include/kfkb.h"
#include <algorithm>
#include <cstdlib>

namespace kfkb {

constexpr int BK = 64;

// position t of the tile order -> tile coordinates: groups of four tile-rows, column by column
__device__ __forceinline__ void tile_from_linear(int t, int tiles_m, int tiles_n, int& tm, int& tn) {
  constexpr int GM = 4;
  const int group = t / (GM * tiles_n);
  const int first_m = group * GM;
  const int gsz = min(GM, tiles_m - first_m);
  const int in_group = t - group * GM * tiles_n;
  tm = first_m + in_group % gsz;
  tn = in_group / gsz;
}
// block -> position in the tile order such that every XCD owns a contiguous run of it
__device__ __forceinline__ int linear_of_block(int total_tiles) {
  const int per_xcd = (total_tiles + 7) / 8;
  return (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
}
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn, bool& valid) {
  const int t = linear_of_block(tiles_m * tiles_n);
  valid = t < tiles_m * tiles_n;
  tile_from_linear(t, tiles_m, tiles_n, tm, tn);
}

template <int EPI>
__device__ __forceinline__ void epilogue_quad(const f32x16& acc, int q, int m, int n, int N, const bf16_t* __restrict__ bias,
                                              const bf16_t* __restrict__ residual, bf16_t* __restrict__ C,
                                              bf16_t* __restrict__ C2, float* __restrict__ Cacc) {
  float v[4] = {acc[q * 4 + 0], acc[q * 4 + 1], acc[q * 4 + 2], acc[q * 4 + 3]};
  const size_t o = (size_t)m * N + n;
  if (EPI == KFKB_EPI_ACCUM) {
    float4* p = reinterpret_cast<float4*>(Cacc + o);
    float4 c = *p;
    c.x += v[0]; c.y += v[1]; c.z += v[2]; c.w += v[3];
    *p = c;
    return;
  }
  if (EPI == KFKB_EPI_BIAS || EPI == KFKB_EPI_BIAS_GELU || EPI == KFKB_EPI_BIAS_RES) {
    const bf16x4 b = *reinterpret_cast<const bf16x4*>(bias + n);
#pragma unroll
    for (int e = 0; e < 4; e++) v[e] += (float)b[e];
  }
  if (EPI == KFKB_EPI_BIAS_RES) {
    const bf16x4 r = *reinterpret_cast<const bf16x4*>(residual + o);
#pragma unroll
    for (int e = 0; e < 4; e++) v[e] += (float)r[e];
  }
  if (EPI == KFKB_EPI_GELU_BWD) {
    const bf16x4 r = *reinterpret_cast<const bf16x4*>(residual + o);
#pragma unroll
    for (int e = 0; e < 4; e++) v[e] *= gelu_grad_f((float)r[e]);
  }
  bf16x4 out;
#pragma unroll
  for (int e = 0; e < 4; e++) out[e] = (bf16_t)v[e];
  *reinterpret_cast<bf16x4*>(C + o) = out;
  if (EPI == KFKB_EPI_BIAS_GELU) {
    bf16x4 g;
#pragma unroll
    for (int e = 0; e < 4; e++) g[e] = (bf16_t)gelu_f((float)out[e]);   // gelu of the stored (rounded) pre-activation
    *reinterpret_cast<bf16x4*>(C2 + o) = g;
  }
}

// ------------------------------------------------------------------------------------------------
// Shared pieces of the two pipelined kernels.
//
// Pipeline (per work-group, NS LDS stages, ONE barrier per 64-deep slice; slice j lives in stage j % NS and
// is requested NS - 1 slices ahead: a 128 x 128 tile spends only ~0.2 us of MFMA time on a slice, far less
// than a trip to L2 / HBM, so several slices have to be in flight):
//   slices are fetched with direct global->LDS loads (global_load_lds_dwordx4: no registers, no LDS
//   store instructions); a wave instruction fills 1 KiB of LDS linearly, so the swizzle is applied on
//   the global side: the lane that owns LDS position p fetches the logical chunk that belongs there.
//   Inside a slice the fragments of k-step s+1 are read while the MFMAs of k-step s issue.  Before the
//   last k-step of slice t every wave waits for its own loads of slice t+1, all waves meet, the loads
//   of slice t+2 are issued into the stage slice t occupied (its last fragments are in registers by
//   then), and the first fragments of slice t+1 are read during the last MFMAs of slice t.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void dma16(const bf16_t* g, bf16_t* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}
// s_waitcnt encodings (gfx9 layout: vmcnt [3:0]+[15:14], expcnt [6:4], lgkmcnt [11:8])
// wait until at most N vector-memory operations (here: direct loads into LDS) of this wave are outstanding;
// LGKM0 additionally waits for all LDS reads
template <int N, bool LGKM0>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0070 | (LGKM0 ? 0 : 0x0F00));
}

template <int TM, int TN>
__device__ __forceinline__ void mfma_step(f32x16 (&acc)[TM][TN], const bf16x8 (&fa)[TM], const bf16x8 (&fb)[TN]) {
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
}

// scheduling hints for one k-step: READS LDS reads (and LOADS direct global->LDS loads) are issued one
// per MFMA at the front of the step, the remaining MFMAs run at the end and cover the LDS latency of the
// last reads before the next step needs them.
template <int I, int SLOTS, int READS, int LOADS>
__device__ __forceinline__ void interleave_slot() {
  if constexpr (I < SLOTS) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, (READS + SLOTS - 1 - I) / SLOTS, 0);
    if constexpr (LOADS > 0) __builtin_amdgcn_sched_group_barrier(0x020, (LOADS + SLOTS - 1 - I) / SLOTS, 0);
    interleave_slot<I + 1, SLOTS, READS, LOADS>();
  }
}
template <int MFMAS, int READS, int LOADS>
__device__ __forceinline__ void interleave_hint() {
  constexpr int SLOTS = READS < MFMAS ? READS : MFMAS - 1;      // MFMAs that carry memory instructions
  interleave_slot<0, SLOTS, READS, LOADS>();
  __builtin_amdgcn_sched_group_barrier(0x008, MFMAS - SLOTS, 0);
}

// ------------------------------------------------------------------------------------------------
// NT kernel.  LDS tile [rows][64]: 8 chunks of 16 bytes per row, chunk index XOR ((row >> 1) & 7): a 16-byte
// fragment read serves 16 lanes (16 consecutive rows) per clock from 64 banks, and two rows fill one 256-byte
// bank window, so the 16 rows have to land on 16 different chunk slots of it.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int EPI, int NS>
__global__ void __launch_bounds__(256) gemm_bf16_nt_kernel(int M, int N, int K, const bf16_t* __restrict__ A,
                                                           const bf16_t* __restrict__ B, const bf16_t* __restrict__ bias,
                                                           const bf16_t* __restrict__ residual, bf16_t* __restrict__ C,
                                                           bf16_t* __restrict__ C2, float* __restrict__ Cacc,
                                                           int tiles_m, int tiles_n) {
  constexpr int TM = BM / 64, TN = BN / 64;          // 32x32 accumulator tiles per wave
  constexpr int GA = BM / 32, GB = BN / 32;          // 8-row groups (1 KiB) each wave fetches per slice
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);                       // [NS][BM][64]
  bf16_t* Bs = As + NS * BM * BK;                                     // [NS][BN][64]

  int tm, tn; bool valid;
  tile_of_block(tiles_m, tiles_n, tm, tn, valid);
  if (!valid) return;
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);

  // LDS position (row, lane & 7) holds logical chunk (lane & 7) ^ ((row >> 1) & 7); wave w fetches the 8-row groups
  // i*4 + w, whose rows start at multiples of 8, so ((row >> 1) & 7) = 4 * (w & 1) + (lrow >> 1)
  const int lrow = lane >> 3, lchunk = (lane & 7) ^ (((wave & 1) << 2) | (lrow >> 1));
  const bf16_t* Ag[GA]; const bf16_t* Bg[GB];
#pragma unroll
  for (int i = 0; i < GA; i++) Ag[i] = A + (size_t)min(m0 + (i * 4 + wave) * 8 + lrow, M - 1) * K + lchunk * 8;
#pragma unroll
  for (int i = 0; i < GB; i++) Bg[i] = B + (size_t)(n0 + (i * 4 + wave) * 8 + lrow) * K + lchunk * 8;
  auto issue = [&](int kt, int st) {
#pragma unroll
    for (int i = 0; i < GA; i++) dma16(Ag[i] + kt * BK, As + st * BM * BK + (i * 4 + wave) * 512);
#pragma unroll
    for (int i = 0; i < GB; i++) dma16(Bg[i] + kt * BK, Bs + st * BN * BK + (i * 4 + wave) * 512);
  };
  const int frow = lane & 31, fhalf = lane >> 5;
  auto read_frags = [&](int st, int ks, bf16x8 (&fa)[TM], bf16x8 (&fb)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; i++) {
      const int r = wm0 + i * 32 + frow;
      fa[i] = *reinterpret_cast<const bf16x8*>(As + ((st * BM + r) * 8 + ((ks * 2 + fhalf) ^ ((r >> 1) & 7))) * 8);
    }
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int r = wn0 + j * 32 + frow;
      fb[j] = *reinterpret_cast<const bf16x8*>(Bs + ((st * BN + r) * 8 + ((ks * 2 + fhalf) ^ ((r >> 1) & 7))) * 8);
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  const int nk = K / BK;
  constexpr int LPS = GA + GB;                       // loads each wave issues per slice
  bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
#pragma unroll
  for (int j = 0; j < NS - 1; j++)
    if (j < nk) issue(j, j);
  if (nk >= NS - 1) wait_vm<(NS - 2) * LPS, false>(); else wait_vm<0, false>();   // slice 0 has landed
  __syncthreads();
  if (NS - 1 < nk) issue(NS - 1, NS - 1);
  read_frags(0, 0, fa0, fb0);
  // one slice; `more` = slice kt+NS exists (request it), `next` = slice kt+1 exists (start on its fragments)
  auto slice = [&](int kt, int cur, bool more, bool next) {
    read_frags(cur, 1, fa1, fb1);
    mfma_step<TM, TN>(acc, fa0, fb0);
    interleave_hint<TM * TN, TM + TN, 0>();
    read_frags(cur, 2, fa0, fb0);
    mfma_step<TM, TN>(acc, fa1, fb1);
    interleave_hint<TM * TN, TM + TN, 0>();
    read_frags(cur, 3, fa1, fb1);
    mfma_step<TM, TN>(acc, fa0, fb0);
    interleave_hint<TM * TN, TM + TN, 0>();
    // own loads of slice kt+1 have landed; the last fragments of slice kt are in registers
    if (more) wait_vm<(NS - 2) * LPS, true>(); else wait_vm<0, true>();
    __syncthreads();
    if (more) issue(kt + NS, cur);
    if (next) read_frags(cur + 1 == NS ? 0 : cur + 1, 0, fa0, fb0);
    mfma_step<TM, TN>(acc, fa1, fb1);
    if (more) interleave_hint<TM * TN, TM + TN, GA + GB>();
    else if (next) interleave_hint<TM * TN, TM + TN, 0>();
  };
  int kt = 0, cur = 0;
  for (; kt + NS < nk; kt++) { slice(kt, cur, true, true); cur = cur + 1 == NS ? 0 : cur + 1; }
  for (; kt + 1 < nk; kt++) { slice(kt, cur, false, true); cur = cur + 1 == NS ? 0 : cur + 1; }
  slice(kt, cur, false, false);

#pragma unroll
  for (int i = 0; i < TM; i++) {
    const int m = m0 + wm0 + i * 32 + frow;
    if (m < M) {
#pragma unroll
      for (int j = 0; j < TN; j++)
#pragma unroll
        for (int q = 0; q < 4; q++)
          epilogue_quad<EPI>(acc[i][j], q, m, n0 + wn0 + j * 32 + q * 8 + fhalf * 4, N, bias, residual, C, C2, Cacc);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// TN kernel, K % 64 == 0.  LDS tile [64 reduction rows][BM] as it lies in memory, the 16-byte chunk
// index XOR 4 * (row & 3).  The LDS of gfx950 has 64 banks (256 bytes per clock): a transpose read serves
// 32 lanes per clock, i.e. 64 contiguous bytes of each of four consecutive rows, and the XOR puts those four
// rows into the four different 64-byte slots of the 256-byte bank window.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ bf16x8 lds_tr_pair(const bf16_t* p, int second_offset) {
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + second_offset));
  union { struct { s16x4 a, b; } s; bf16x8 v; } u;
  u.s.a = lo; u.s.b = hi;
  return u.v;
}

template <int BM, int BN, int EPI, int NS>
__device__ __forceinline__ void tn_tile(int M, int N, int K, const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                        bf16_t* __restrict__ C, float* __restrict__ Cacc, int tm, int tn, char* smem) {
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int CA = BM / 8, CB = BN / 8;            // 16-byte chunks per tile row
  constexpr int RA = 64 / CA, RB = 64 / CB;          // tile rows one wave instruction (1 KiB) covers
  constexpr int GA = BM / 32, GB = BN / 32;          // wave instructions per wave per slice
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);                       // [NS][64][BM]
  bf16_t* Bs = As + NS * BK * BM;                                     // [NS][64][BN]
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);

  // wave instruction g (0 .. 4*GA) of a slice covers tile rows g*RA .. +RA; lane -> (row, physical chunk)
  const bf16_t* Ag[GA]; const bf16_t* Bg[GB];
#pragma unroll
  for (int i = 0; i < GA; i++) {
    const int row = (i * 4 + wave) * RA + lane / CA, pc = lane % CA;
    Ag[i] = A + (size_t)row * M + m0 + (pc ^ (4 * (row & 3))) * 8;
  }
#pragma unroll
  for (int i = 0; i < GB; i++) {
    const int row = (i * 4 + wave) * RB + lane / CB, pc = lane % CB;
    Bg[i] = B + (size_t)row * N + n0 + (pc ^ (4 * (row & 3))) * 8;
  }
  auto issue = [&](int kt, int st) {
#pragma unroll
    for (int i = 0; i < GA; i++) dma16(Ag[i] + (size_t)kt * BK * M, As + st * BK * BM + (i * 4 + wave) * 512);
#pragma unroll
    for (int i = 0; i < GB; i++) dma16(Bg[i] + (size_t)kt * BK * N, Bs + st * BK * BN + (i * 4 + wave) * 512);
  };
  // transpose-read geometry: 16-lane group g covers columns (g & 1) * 16 .. + 16 and the reduction half
  // g >> 1; inside the group lane j points at row j / 4, columns (j % 4) * 4 .. + 4.
  const int g16 = lane >> 4, j16 = lane & 15;
  const int tr_row = (g16 >> 1) * 8 + (j16 >> 2);
  const int tr_col = (g16 & 1) * 16 + (j16 & 3) * 4;
  auto read_frags = [&](int st, int ks, bf16x8 (&fa)[TM], bf16x8 (&fb)[TN]) {
    const int row = ks * 16 + tr_row, sw = 4 * (row & 3);
#pragma unroll
    for (int i = 0; i < TM; i++) {
      const int col = wm0 + i * 32 + tr_col;
      fa[i] = lds_tr_pair(As + (st * BK + row) * BM + (((col >> 3) ^ sw) << 3) + (col & 7), 4 * BM);
    }
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int col = wn0 + j * 32 + tr_col;
      fb[j] = lds_tr_pair(Bs + (st * BK + row) * BN + (((col >> 3) ^ sw) << 3) + (col & 7), 4 * BN);
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  const int nk = K / BK;
  constexpr int LPS = GA + GB;                       // loads each wave issues per slice
  bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
#pragma unroll
  for (int j = 0; j < NS - 1; j++)
    if (j < nk) issue(j, j);
  if (nk >= NS - 1) wait_vm<(NS - 2) * LPS, false>(); else wait_vm<0, false>();   // slice 0 has landed
  __syncthreads();
  if (NS - 1 < nk) issue(NS - 1, NS - 1);
  read_frags(0, 0, fa0, fb0);
  // one slice; `more` = slice kt+NS exists (request it), `next` = slice kt+1 exists (start on its fragments)
  auto slice = [&](int kt, int cur, bool more, bool next) {
    read_frags(cur, 1, fa1, fb1);
    mfma_step<TM, TN>(acc, fa0, fb0);
    interleave_hint<TM * TN, 2 * (TM + TN), 0>();
    read_frags(cur, 2, fa0, fb0);
    mfma_step<TM, TN>(acc, fa1, fb1);
    interleave_hint<TM * TN, 2 * (TM + TN), 0>();
    read_frags(cur, 3, fa1, fb1);
    mfma_step<TM, TN>(acc, fa0, fb0);
    interleave_hint<TM * TN, 2 * (TM + TN), 0>();
    // own loads of slice kt+1 have landed; the last fragments of slice kt are in registers
    if (more) wait_vm<(NS - 2) * LPS, true>(); else wait_vm<0, true>();
    __syncthreads();
    if (more) issue(kt + NS, cur);
    if (next) read_frags(cur + 1 == NS ? 0 : cur + 1, 0, fa0, fb0);
    mfma_step<TM, TN>(acc, fa1, fb1);
    if (more) interleave_hint<TM * TN, 2 * (TM + TN), GA + GB>();
    else if (next) interleave_hint<TM * TN, 2 * (TM + TN), 0>();
  };
  int kt = 0, cur = 0;
  for (; kt + NS < nk; kt++) { slice(kt, cur, true, true); cur = cur + 1 == NS ? 0 : cur + 1; }
  for (; kt + 1 < nk; kt++) { slice(kt, cur, false, true); cur = cur + 1 == NS ? 0 : cur + 1; }
  slice(kt, cur, false, false);

  const int frow = lane & 31, fhalf = lane >> 5;
#pragma unroll
  for (int i = 0; i < TM; i++) {
    const int m = m0 + wm0 + i * 32 + frow;
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int q = 0; q < 4; q++)
        epilogue_quad<EPI>(acc[i][j], q, m, n0 + wn0 + j * 32 + q * 8 + fhalf * 4, N, nullptr, nullptr, C, nullptr, Cacc);
  }
}

template <int BM, int BN, int EPI, int NS>
__global__ void __launch_bounds__(256) gemm_bf16_tn_kernel(int M, int N, int K, const bf16_t* __restrict__ A,
                                                           const bf16_t* __restrict__ B, bf16_t* __restrict__ C,
                                                           float* __restrict__ Cacc, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int tm, tn; bool valid;
  tile_of_block(tiles_m, tiles_n, tm, tn, valid);
  if (!valid) return;
  tn_tile<BM, BN, EPI, NS>(M, N, K, A, B, C, Cacc, tm, tn, smem);
}

// Several weight-gradient products that share the reduction length K (the token axis) in one launch:
// a backward pass of one block has four of them, each too small to fill the chip on its own.
struct TnProblem { int M, N, tiles_m, tiles_n, first_tile; const bf16_t* A; const bf16_t* B; float* Cacc; };
struct TnGroup { int count, K, total_tiles; TnProblem p[4]; };

template <int BM, int BN, int NS>
__global__ void __launch_bounds__(256) gemm_bf16_tn_grouped_kernel(TnGroup grp) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int t = linear_of_block(grp.total_tiles);
  if (t >= grp.total_tiles) return;
  int i = 0;
#pragma unroll
  for (int q = 1; q < 4; q++) if (q < grp.count && t >= grp.p[q].first_tile) i = q;
  const TnProblem pr = grp.p[i];
  int tm, tn;
  tile_from_linear(t - pr.first_tile, pr.tiles_m, pr.tiles_n, tm, tn);
  tn_tile<BM, BN, KFKB_EPI_ACCUM, NS>(pr.M, pr.N, grp.K, pr.A, pr.B, nullptr, pr.Cacc, tm, tn, smem);
}

// ------------------------------------------------------------------------------------------------
// TN kernel, register-staged variant: accepts a ragged reduction length K (zero-fills the tail).
// Tiles are stored [reduction row][BM + 32].
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ bf16x8 lds_tr_frag(const bf16_t* p, int row_stride) {
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * row_stride));
  union { struct { s16x4 a, b; } s; bf16x8 v; } u;
  u.s.a = lo; u.s.b = hi;
  return u.v;
}

template <int BM, int BN, int EPI>
__global__ void __launch_bounds__(256) gemm_bf16_tn_staged_kernel(int M, int N, int K, const bf16_t* __restrict__ A,
                                                           const bf16_t* __restrict__ B, bf16_t* __restrict__ C,
                                                           float* __restrict__ Cacc, int tiles_m, int tiles_n) {
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int SA = BM + 32, SB = BN + 32;          // LDS row strides (elements): +64 bytes per row
  constexpr int CA = BM / 8, CB = BN / 8;            // 16-byte chunks per tile row
  constexpr int LA = BM / 32, LB = BN / 32;          // chunks per thread per slice
  extern __shared__ __attribute__((aligned(16))) char smem[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);                       // [2][64][SA]
  bf16_t* Bs = As + 2 * BK * SA;                                      // [2][64][SB]

  int tm, tn; bool valid;
  tile_of_block(tiles_m, tiles_n, tm, tn, valid);
  if (!valid) return;
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);

  bf16x8 ra[LA], rb[LB];
  auto load_global = [&](int kt) {
#pragma unroll
    for (int i = 0; i < LA; i++) {
      const int c = tid % CA, r = tid / CA + (256 / CA) * i;
      const int k = kt * BK + r;
      bf16x8 z;
#pragma unroll
      for (int e = 0; e < 8; e++) z[e] = (bf16_t)0.f;
      ra[i] = (k < K) ? *reinterpret_cast<const bf16x8*>(A + (size_t)k * M + m0 + c * 8) : z;
    }
#pragma unroll
    for (int i = 0; i < LB; i++) {
      const int c = tid % CB, r = tid / CB + (256 / CB) * i;
      const int k = kt * BK + r;
      bf16x8 z;
#pragma unroll
      for (int e = 0; e < 8; e++) z[e] = (bf16_t)0.f;
      rb[i] = (k < K) ? *reinterpret_cast<const bf16x8*>(B + (size_t)k * N + n0 + c * 8) : z;
    }
  };
  auto store_lds = [&](int st) {
#pragma unroll
    for (int i = 0; i < LA; i++) {
      const int c = tid % CA, r = tid / CA + (256 / CA) * i;
      *reinterpret_cast<bf16x8*>(As + (st * BK + r) * SA + c * 8) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < LB; i++) {
      const int c = tid % CB, r = tid / CB + (256 / CB) * i;
      *reinterpret_cast<bf16x8*>(Bs + (st * BK + r) * SB + c * 8) = rb[i];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  // transpose-read geometry: 16-lane group g covers columns (g & 1) * 16 .. + 16 and the reduction
  // half g >> 1; inside the group lane j points at row j / 4, columns (j % 4) * 4 .. + 4.
  const int g16 = lane >> 4, j16 = lane & 15;
  const int tr_row = (g16 >> 1) * 8 + (j16 >> 2);
  const int tr_col = (g16 & 1) * 16 + (j16 & 3) * 4;

  const int nk = (K + BK - 1) / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < nk; kt++) {
    const int cur = kt & 1;
    if (kt + 1 < nk) load_global(kt + 1);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ks++) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; i++)
        fa[i] = lds_tr_frag(As + (cur * BK + ks * 16 + tr_row) * SA + wm0 + i * 32 + tr_col, SA);
#pragma unroll
      for (int j = 0; j < TN; j++)
        fb[j] = lds_tr_frag(Bs + (cur * BK + ks * 16 + tr_row) * SB + wn0 + j * 32 + tr_col, SB);
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_lds(cur ^ 1);
    __syncthreads();
  }

  const int frow = lane & 31, fhalf = lane >> 5;
#pragma unroll
  for (int i = 0; i < TM; i++) {
    const int m = m0 + wm0 + i * 32 + frow;
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int q = 0; q < 4; q++)
        epilogue_quad<EPI>(acc[i][j], q, m, n0 + wn0 + j * 32 + q * 8 + fhalf * 4, N, nullptr, nullptr, C, nullptr, Cacc);
  }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
const char* gemm_bf16_check(const GemmArgs& g) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return "bf16 GEMM: empty shape";
  if (g.kind == KFKB_GEMM_NT) {
    if (g.N % 128 != 0) return "bf16 NT GEMM needs N % 128 == 0";
    if (g.K % 64 != 0) return "bf16 NT GEMM needs K % 64 == 0";
  } else if (g.kind == KFKB_GEMM_TN) {
    if (g.M % 128 != 0 || g.N % 128 != 0) return "bf16 TN GEMM needs M % 128 == 0 and N % 128 == 0";
    if (g.epilogue != KFKB_EPI_ACCUM && g.epilogue != KFKB_EPI_NONE) return "bf16 TN GEMM supports epilogues NONE and ACCUM";
  } else {
    return "bf16 GEMM supports the NT and TN forms";
  }
  return nullptr;
}

// Pipeline depth of the 128 x 128 tiles (32 KiB of LDS per stage).  KFKB_STAGES_128 = 2, 3 or 4 overrides
// the default for experiments.
static int stages_128() {
  static int v = 0;
  if (v == 0) {
    const char* e = getenv("KFKB_STAGES_128");
    v = e ? atoi(e) : 2;
    if (v < 2 || v > 4) v = 2;
  }
  return v;
}

template <int BM, int BN, int EPI, int NS>
static hipError_t launch_nt_ns(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = g.N / BN;
  const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
  const size_t smem = (size_t)NS * (BM + BN) * BK * sizeof(bf16_t);
  auto kern = gemm_bf16_nt_kernel<BM, BN, EPI, NS>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  klaunch(kern, dim3(grid), dim3(256), smem, s, PK_GEMM_NT + (BM == 256 ? 100 : 0) + EPI, 2.0 * g.M * g.N * g.K, g.M, g.N, g.K,
          (const bf16_t*)g.A, (const bf16_t*)g.B, (const bf16_t*)g.bias, (const bf16_t*)g.residual, (bf16_t*)g.C,
          (bf16_t*)g.C2, g.Cacc, tiles_m, tiles_n);
  return hipGetLastError();
}
template <int BM, int BN, int EPI>
static hipError_t launch_nt(const GemmArgs& g, hipStream_t s) {
  if (BM == 256) return launch_nt_ns<BM, BN, EPI, 2>(g, s);
  switch (stages_128()) {
    case 2: return launch_nt_ns<BM, BN, EPI, 2>(g, s);
    case 3: return launch_nt_ns<BM, BN, EPI, 3>(g, s);
    default: return launch_nt_ns<BM, BN, EPI, (BM == 256 ? 2 : 4)>(g, s);   // 4 stages
  }
}

template <int BM, int BN, int EPI>
static hipError_t launch_tn_staged(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = g.M / BM, tiles_n = g.N / BN;
  const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
  const size_t smem = (size_t)2 * BK * (BM + 32 + BN + 32) * sizeof(bf16_t);
  auto kern = gemm_bf16_tn_staged_kernel<BM, BN, EPI>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  klaunch(kern, dim3(grid), dim3(256), smem, s, PK_GEMM_TN + 200 + (BM == 256 ? 100 : 0) + EPI, 2.0 * g.M * g.N * g.K, g.M, g.N, g.K,
          (const bf16_t*)g.A, (const bf16_t*)g.B, (bf16_t*)g.C, g.Cacc, tiles_m, tiles_n);
  return hipGetLastError();
}

template <int BM, int BN, int EPI, int NS>
static hipError_t launch_tn_ns(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = g.M / BM, tiles_n = g.N / BN;
  const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
  const size_t smem = (size_t)NS * BK * (BM + BN) * sizeof(bf16_t);
  auto kern = gemm_bf16_tn_kernel<BM, BN, EPI, NS>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  klaunch(kern, dim3(grid), dim3(256), smem, s, PK_GEMM_TN + (BM == 256 ? 100 : 0) + EPI, 2.0 * g.M * g.N * g.K, g.M, g.N, g.K,
          (const bf16_t*)g.A, (const bf16_t*)g.B, (bf16_t*)g.C, g.Cacc, tiles_m, tiles_n);
  return hipGetLastError();
}

template <int BM, int BN, int EPI>
static hipError_t launch_tn(const GemmArgs& g, hipStream_t s) {
  if (g.K % BK != 0) return launch_tn_staged<BM, BN, EPI>(g, s);
  if (BM == 256) return launch_tn_ns<BM, BN, EPI, 2>(g, s);
  switch (stages_128()) {
    case 2: return launch_tn_ns<BM, BN, EPI, 2>(g, s);
    case 3: return launch_tn_ns<BM, BN, EPI, 3>(g, s);
    default: return launch_tn_ns<BM, BN, EPI, (BM == 256 ? 2 : 4)>(g, s);
  }
}

template <int BM, int BN, int NS>
static hipError_t launch_group_ns(const TnGroup& grp, double flops, hipStream_t s) {
  const int grid = ((grp.total_tiles + 7) / 8) * 8;
  const size_t smem = (size_t)NS * BK * (BM + BN) * sizeof(bf16_t);
  auto kern = gemm_bf16_tn_grouped_kernel<BM, BN, NS>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  klaunch(kern, dim3(grid), dim3(256), smem, s, PK_GEMM_TN + (BM == 256 ? 301 : 300), flops, grp);
  return hipGetLastError();
}

// fewest 256 x 256 tiles a launch must have before they are preferred over 128 x 128 tiles
// (KFKB_BIG_TILE_MIN overrides it for experiments)
static long big_tile_min() {
  static long v = -1;
  if (v < 0) { const char* e = getenv("KFKB_BIG_TILE_MIN"); v = e ? atol(e) : 192; }
  return v;
}

hipError_t launch_gemm_bf16_tn_group(const GemmArgs* g, int n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  bool groupable = n <= 4;
  for (int i = 0; i < n; i++)
    groupable = groupable && g[i].kind == KFKB_GEMM_TN && g[i].epilogue == KFKB_EPI_ACCUM && g[i].K == g[0].K &&
                g[i].K % BK == 0 && g[i].M % 128 == 0 && g[i].N % 128 == 0;
  if (!groupable) {
    for (int i = 0; i < n; i++) {
      hipError_t e = launch_gemm_bf16(g[i], s);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  // 256 x 256 tiles when every problem divides into them and the group still gives every CU a tile
  long big_tiles = 0;
  bool big = true;
  for (int i = 0; i < n; i++) {
    big = big && g[i].M % 256 == 0 && g[i].N % 256 == 0;
    big_tiles += (long)(g[i].M / 256) * (g[i].N / 256);
  }
  big = big && big_tiles >= big_tile_min();
  const int BT = big ? 256 : 128;
  TnGroup grp{};
  grp.count = n; grp.K = g[0].K;
  double flops = 0;
  for (int i = 0; i < n; i++) {
    TnProblem& p = grp.p[i];
    p.M = g[i].M; p.N = g[i].N; p.tiles_m = g[i].M / BT; p.tiles_n = g[i].N / BT; p.first_tile = grp.total_tiles;
    p.A = (const bf16_t*)g[i].A; p.B = (const bf16_t*)g[i].B; p.Cacc = g[i].Cacc;
    grp.total_tiles += p.tiles_m * p.tiles_n;
    flops += 2.0 * g[i].M * g[i].N * g[i].K;
  }
  if (big) return launch_group_ns<256, 256, 2>(grp, flops, s);
  return launch_group_ns<128, 128, 2>(grp, flops, s);
}

// Large tiles when they still give every CU a tile; small tiles otherwise.
static bool use_big_tiles(int M, int N, bool m_must_divide) {
  if (N % 256 != 0) return false;
  if (m_must_divide && M % 256 != 0) return false;
  const long tiles = (long)((M + 255) / 256) * (N / 256);
  return tiles >= big_tile_min();
}

template <int EPI>
static hipError_t launch_nt_epi(const GemmArgs& g, hipStream_t s) {
  if (use_big_tiles(g.M, g.N, false)) return launch_nt<256, 256, EPI>(g, s);
  return launch_nt<128, 128, EPI>(g, s);
}

hipError_t launch_gemm_bf16(const GemmArgs& g, hipStream_t s) {
  if (g.kind == KFKB_GEMM_NT) {
    switch (g.epilogue) {
      case KFKB_EPI_NONE: return launch_nt_epi<KFKB_EPI_NONE>(g, s);
      case KFKB_EPI_BIAS: return launch_nt_epi<KFKB_EPI_BIAS>(g, s);
      case KFKB_EPI_BIAS_GELU: return launch_nt_epi<KFKB_EPI_BIAS_GELU>(g, s);
      case KFKB_EPI_BIAS_RES: return launch_nt_epi<KFKB_EPI_BIAS_RES>(g, s);
      case KFKB_EPI_ACCUM: return launch_nt_epi<KFKB_EPI_ACCUM>(g, s);
      default: return launch_nt_epi<KFKB_EPI_GELU_BWD>(g, s);
    }
  }
  const bool big = use_big_tiles(g.M, g.N, true);
  if (g.epilogue == KFKB_EPI_ACCUM)
    return big ? launch_tn<256, 256, KFKB_EPI_ACCUM>(g, s) : launch_tn<128, 128, KFKB_EPI_ACCUM>(g, s);
  return big ? launch_tn<256, 256, KFKB_EPI_NONE>(g, s) : launch_tn<128, 128, KFKB_EPI_NONE>(g, s);
}

}  // namespace kfkb
