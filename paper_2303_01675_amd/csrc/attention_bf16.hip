// Fused causal attention, bf16 storage, fp32 softmax, on v_mfma_f32_32x32x16_bf16.
//
//   forward   per (sample, head, 128 query rows): stream 64-key tiles, online softmax, write O and the
//             log-sum-exp of every row; the T x T score matrix never exists in memory.
//   backward  two kernels so that every output element has exactly one writer (no atomics: results
//             are bit-reproducible):
//               dq kernel   per 128 query rows, streams key tiles:   dQ = scale * dS K
//               dkv kernel  per 128 key rows, streams query tiles:   dV = P^T dO,  dK = scale * dS^T Q
//             both recompute P = exp(scale * Q K^T - lse) and dS = P o (dO V^T - dsum),
//             dsum = rowsum(dO o O), formed by the dq kernel (which runs first) and read by the dkv kernel.
//
// Register / lane plan (one wave owns 32 "own" rows and streams the other operand):
//   the score tile is produced transposed with respect to the streamed rows, i.e. with the wave's own
//   row index on the lane (accumulator column = lane % 32) and the streamed rows spread over the 16
//   accumulator registers.  Per-own-row softmax quantities are then per-lane scalars, and the bf16
//   rounded tile is, as it sits in registers, the B operand of the next MFMA whose reduction runs
//   over the streamed rows.  The A operand of that MFMA is a tile read "down the columns" of the
//   streamed operand in LDS, which the LDS transpose read (ds_read_b64_tr_b16) delivers.
//   Reduction slot s of lane half hh in a 16-row sub-block corresponds to streamed row
//   (s / 4) * 8 + hh * 4 + s % 4 on both operands.
//
// LDS tiles are [64 rows][D] with the 16-byte chunk index XOR-ed with a function of the row (TileIO::sw).
#include "common.h"
#include <cstdlib>

namespace kfkb {
// Built once per 16-bit storage type: this file as it is for bf16, through attention_f16.hip (which defines
// KFKB_H16_IS_F16) for fp16; everything type-dependent lives in a namespace of its own.
#ifdef KFKB_H16_IS_F16
namespace f16k {
typedef f16_t h16_t;
typedef f16x8 h16x8;
typedef f16x4 h16x4;
#define KFKB_MFMA_H16(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0)
#else
namespace bf16k {
typedef bf16_t h16_t;
typedef bf16x8 h16x8;
typedef bf16x4 h16x4;
#define KFKB_MFMA_H16(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)
#endif


constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int D>
struct TileIO {
  static constexpr int CH = D / 8;            // 16-byte chunks per row
  // Swizzle: the chunk index is XOR-ed with sw(row).  The LDS has 64 banks (256 bytes per clock).  A 16-byte
  // fragment read serves 16 consecutive rows per clock and needs them on 16 different chunk slots of the
  // 256-byte window; a transpose read serves 64 contiguous bytes of 4 consecutive rows per clock and needs
  // those on 4 different 64-byte slots.  D = 64 (two rows per window): sw = row bit 1 -> chunk bit 2, row bits
  // 3:2 -> chunk bits 1:0.  D = 128 (one row per window): sw = row bits 1:0 -> chunk bits 3:2, row bits 3:2 ->
  // chunk bits 1:0.
  static __device__ __forceinline__ int sw(int row) {
    return D == 64 ? ((((row >> 1) & 1) << 2) | ((row >> 2) & 3)) : (((row & 3) << 2) | ((row >> 2) & 3));
  }
  static constexpr int NL = D / 32;           // chunks per thread for a 64-row tile
  // rows row0 .. row0+63 of a [*, ld] matrix, clamped to row_max, columns col0 .. col0+D
  static __device__ __forceinline__ void load(h16x8 (&r)[NL], const h16_t* __restrict__ src, size_t ld, int row0,
                                              int row_max, int col0) {
    const int c = threadIdx.x % CH;
#pragma unroll
    for (int i = 0; i < NL; i++) {
      const int row = min(row0 + (int)threadIdx.x / CH + (256 / CH) * i, row_max);
      r[i] = *reinterpret_cast<const h16x8*>(src + (size_t)row * ld + col0 + c * 8);
    }
  }
  static __device__ __forceinline__ void store(h16_t* tile, const h16x8 (&r)[NL]) {
    const int c = threadIdx.x % CH;
#pragma unroll
    for (int i = 0; i < NL; i++) {
      const int row = threadIdx.x / CH + (256 / CH) * i;
      *reinterpret_cast<h16x8*>(tile + (row * CH + (c ^ sw(row))) * 8) = r[i];
    }
  }
  // The same tile filled by loads that write LDS (no staging registers, no LDS stores).  One instruction of a wave
  // fills 64 consecutive 16-byte places of the tile; place P holds chunk (P % CH) ^ sw(P / CH) of row P / CH, so the
  // swizzle is applied on the global side.  A tile is NI instructions per wave: instruction i of wave w covers places
  // (i * 4 + w) * 64 ... + 63.  voff(): this lane's byte offset from the first row of the tile; rows at or past the
  // resource's end read as zero.
  static constexpr int NI = (64 * CH) / 256;
  static __device__ __forceinline__ int dma_voff(int i, int wave, int lane, size_t ld) {
    const int place = (i * 4 + wave) * 64 + lane;
    const int row = place / CH, c = (place % CH) ^ sw(row);
    return (int)((size_t)row * ld * sizeof(h16_t)) + c * 16;
  }
  static __device__ __forceinline__ void dma_tile(const i32x4& rsrc, const int (&voff)[NI], int soff, unsigned lds_tile, int wave) {
#pragma unroll
    for (int i = 0; i < NI; i++) dma16b(rsrc, voff[i], soff, lds_tile + (unsigned)((i * 4 + wave) * 1024));
  }
  // 8 reduction-contiguous values of row `row`, chunk `chunk`
  static __device__ __forceinline__ h16x8 frag(const h16_t* tile, int row, int chunk) {
    return *reinterpret_cast<const h16x8*>(tile + (row * CH + (chunk ^ sw(row))) * 8);
  }
  // transpose read: this lane points at (row, col .. col+4) and (row + 8, col .. col+4)
  static __device__ __forceinline__ h16x8 frag_tr(const h16_t* tile, int row, int col) {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const h16_t* p = tile + (row * CH + ((col >> 3) ^ sw(row))) * 8 + (col & 7);
    const h16_t* p8 = tile + ((row + 8) * CH + ((col >> 3) ^ sw(row + 8))) * 8 + (col & 7);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p8);
    union { struct { s16x4 a, b; } s; h16x8 v; } u;
    u.s.a = lo; u.s.b = hi;
    return u.v;
  }
};

__device__ __forceinline__ h16x8 pack8(const f32x16& a, int first) {
  h16x8 v;
#pragma unroll
  for (int s = 0; s < 8; s++) v[s] = (h16_t)a[first + s];
  return v;
}
__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int e = 0; e < 16; e++) z[e] = 0.f;
  return z;
}
// 2^x through the hardware instruction alone: arguments here are <= 0 (or -inf), results that would be
// denormal flush to zero, which is what a softmax weight that small should be
__device__ __forceinline__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

// streamed-row offset (inside a 32-row tile) of accumulator register r for lane half hh
__device__ __forceinline__ int acc_row(int r, int hh) { return (r >> 2) * 8 + hh * 4 + (r & 3); }

// Block -> (row block, sample*head).  Work per block grows with the row-block index (causal), and consecutive
// block ids are dealt round-robin to the 8 XCDs, each with its own L2.  All row blocks of one (sample, head)
// are therefore given to ONE XCD (its K and V, or Q and dO, then stay in that L2), longest first, and every XCD
// gets the same mix of short and long blocks.  Falls back to a rotation when sample*head does not divide by 8.
// `pair` (set by the host when an XCD's blocks are exactly two per CU, all resident at once): the hardware hands an
// XCD's blocks to its 32 CUs in turn, so blocks n and n + 32 share a CU; the second half of the sequence is then
// dealt shortest first, and every CU gets a long and a short block (measured: 16 % off the forward kernel and 13 %
// off the backward kernels of the 1024-token stage; longest-first is better as soon as blocks queue up).
__device__ __forceinline__ void block_to_work(int& rb, int& bh, int pair) {
  const int gx = gridDim.x, gy = gridDim.y;
  if (gy % 8 == 0) {
    const int lin = blockIdx.y * gx + blockIdx.x;
    const int xcd = lin & 7, n = lin >> 3;
    const int half = (gx * (gy >> 3)) >> 1;         // half of this XCD's blocks
    int h, r;
    if (pair && n >= half) { const int i = n - half; h = (half / gx) + i / gx; r = i % gx; }
    else { h = n / gx; r = gx - 1 - n % gx; }
    bh = xcd + 8 * h;
    rb = r;
  } else {
    bh = blockIdx.y;
    rb = (blockIdx.x + blockIdx.y) % gx;
  }
}

// ------------------------------------------------------------------------------------------------
// forward
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256, 2) attn_fwd_h16_kernel(const h16_t* __restrict__ qkv, h16_t* __restrict__ o,
                                                            float* __restrict__ lse, int T, int H, int heads,
                                                            int causal, float scale_log2, int pair) {
  using IO = TileIO<D>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  h16_t* Ks = reinterpret_cast<h16_t*>(smem);     // [2][64][D]
  h16_t* Vs = Ks + 2 * 64 * D;                     // [2][64][D]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hh = lane >> 5, l32 = lane & 31;
  const int tr_row = hh * 4 + ((lane & 15) >> 2);
  const int tr_col = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  int qb, bh;
  block_to_work(qb, bh, pair);
  const int bi = bh / heads, hd = bh % heads;
  const size_t ld = 3 * (size_t)H;
  const h16_t* base = qkv + (size_t)bi * T * ld;
  const int q0 = qb * 128, qw0 = q0 + wave * 32;
  const int i = qw0 + l32;
  const int ic = min(i, T - 1);

  h16x8 qf[D / 16];
#pragma unroll
  for (int ds = 0; ds < D / 16; ds++)
    qf[ds] = *reinterpret_cast<const h16x8*>(base + (size_t)ic * ld + hd * D + ds * 16 + hh * 8);

  const int nkv_all = (T + 63) / 64;
  const int nkv = causal ? min(nkv_all, (min(q0 + 127, T - 1)) / 64 + 1) : nkv_all;

  f32x16 oacc[D / 32];
#pragma unroll
  for (int t = 0; t < D / 32; t++) oacc[t] = zero16();
  float mrun = -INFINITY, lsum = 0.f;

  // K and V tiles arrive through loads that write LDS; rows past the end of the sequence read as zero (they are
  // masked below, and a zero V row times a zero weight stays zero)
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const size_t row_bytes = ld * sizeof(h16_t);
  const i32x4 rk = make_rsrc(base + H + hd * D, (size_t)(T - 1) * row_bytes + D * sizeof(h16_t));
  const i32x4 rv = make_rsrc(base + 2 * H + hd * D, (size_t)(T - 1) * row_bytes + D * sizeof(h16_t));
  int voff[IO::NI];
#pragma unroll
  for (int q = 0; q < IO::NI; q++) voff[q] = IO::dma_voff(q, wv, lane, ld);
  const unsigned lds_k = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
  const unsigned lds_v = lds_k + 2 * 64 * D * (unsigned)sizeof(h16_t);
  constexpr unsigned TILE_B = 64 * D * sizeof(h16_t);
  IO::dma_tile(rk, voff, 0, lds_k, wv);
  IO::dma_tile(rv, voff, 0, lds_v, wv);
  wait_vmcnt<0>();
  __syncthreads();
  for (int kb = 0; kb < nkv; kb++) {
    const int cur = kb & 1, j0 = kb * 64;
    if (kb + 1 < nkv) {                              // the other buffer was last read before the barrier that ended step kb - 1
      const int soff = (int)((size_t)(j0 + 64) * row_bytes);
      IO::dma_tile(rk, voff, soff, lds_k + (cur ^ 1) * TILE_B, wv);
      IO::dma_tile(rv, voff, soff, lds_v + (cur ^ 1) * TILE_B, wv);
    }
    const h16_t* Kt = Ks + cur * 64 * D;
    const h16_t* Vt = Vs + cur * 64 * D;
    if (!(causal && j0 > qw0 + 31)) {               // wave-uniform: some key of the tile is visible
      f32x16 st[2] = {zero16(), zero16()};
#pragma unroll
      for (int jt = 0; jt < 2; jt++) {
        h16x8 ka[D / 16];                            // requested together, ahead of their MFMAs
#pragma unroll
        for (int ds = 0; ds < D / 16; ds++) ka[ds] = IO::frag(Kt, jt * 32 + l32, ds * 2 + hh);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ds = 0; ds < D / 16; ds++) st[jt] = KFKB_MFMA_H16(ka[ds], qf[ds], st[jt]);
        __builtin_amdgcn_sched_barrier(0);
      }
      // masking is needed only where the tile crosses the diagonal or the end of the sequence
      if (j0 + 63 >= T || (causal && j0 + 63 > qw0)) {
#pragma unroll
        for (int jt = 0; jt < 2; jt++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int j = j0 + jt * 32 + acc_row(r, hh);
            if (j >= T || (causal && j > i)) st[jt][r] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int r = 0; r < 16; r++) mx = fmaxf(mx, st[jt][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;      // scale > 0: max commutes with it
      const float mnew = fmaxf(fmaxf(mrun, mx), -1e30f);
      const float alpha = exp2_raw(mrun - mnew);
      if (__any(alpha != 1.0f)) {                    // the running maximum settles after a few tiles
#pragma unroll
        for (int t = 0; t < D / 32; t++)
#pragma unroll
          for (int e = 0; e < 16; e++) oacc[t][e] *= alpha;
      }
      // Sixteen keys at a time: exponentials, then the P.V MFMAs of those keys.  An MFMA runs on after it has been
      // issued, so the exponentials of the next sixteen keys, next in program order, execute under it.
      float ps = 0.f;
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int t16 = 0; t16 < 2; t16++) {
          h16x8 vt[D / 32];
#pragma unroll
          for (int t = 0; t < D / 32; t++) vt[t] = IO::frag_tr(Vt, jt * 32 + t16 * 16 + tr_row, t * 32 + tr_col);
#pragma unroll
          for (int r = t16 * 8; r < t16 * 8 + 8; r++) {
            const float p = exp2_raw(fmaf(st[jt][r], scale_log2, -mnew));
            st[jt][r] = p;
            ps += p;
          }
          const h16x8 pb = pack8(st[jt], t16 * 8);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int t = 0; t < D / 32; t++) oacc[t] = KFKB_MFMA_H16(vt[t], pb, oacc[t]);
          __builtin_amdgcn_sched_barrier(0);
        }
      lsum = lsum * alpha + ps;
      mrun = mnew;
    }
    wait_vmcnt<0>();                                 // this wave's part of the next tiles has landed
    __syncthreads();
  }
  lsum += __shfl_xor(lsum, 32, 64);
  if (i < T) {
    const float inv = 1.0f / lsum;
    h16_t* orow = o + ((size_t)bi * T + i) * H + hd * D;
#pragma unroll
    for (int t = 0; t < D / 32; t++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        h16x4 v;
#pragma unroll
        for (int e = 0; e < 4; e++) v[e] = (h16_t)(oacc[t][q * 4 + e] * inv);
        *reinterpret_cast<h16x4*>(orow + t * 32 + q * 8 + hh * 4) = v;
      }
    if (hh == 0) lse[((size_t)bi * heads + hd) * T + i] = (mrun + log2f(lsum)) * kLn2;
  }
}

// ------------------------------------------------------------------------------------------------
// backward, dQ: own rows = queries, streamed rows = keys
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256, 2) attn_bwd_dq_h16_kernel(const h16_t* __restrict__ qkv, const h16_t* __restrict__ o,
                                                               const h16_t* __restrict__ d_o,
                                                               const float* __restrict__ lse, float* __restrict__ dsum,
                                                               h16_t* __restrict__ dqkv, int T, int H, int heads,
                                                               int causal, float scale, int pair) {
  using IO = TileIO<D>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  h16_t* Ks = reinterpret_cast<h16_t*>(smem);
  h16_t* Vs = Ks + 2 * 64 * D;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hh = lane >> 5, l32 = lane & 31;
  const int tr_row = hh * 4 + ((lane & 15) >> 2);
  const int tr_col = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  int qb, bh;
  block_to_work(qb, bh, pair);
  const int bi = bh / heads, hd = bh % heads;
  const size_t ld = 3 * (size_t)H;
  const h16_t* base = qkv + (size_t)bi * T * ld;
  const int q0 = qb * 128, qw0 = q0 + wave * 32;
  const int i = qw0 + l32;
  const int ic = min(i, T - 1);
  const float scale_log2 = scale * kLog2e;

  h16x8 qf[D / 16], dof[D / 16];
#pragma unroll
  for (int ds = 0; ds < D / 16; ds++) {
    qf[ds] = *reinterpret_cast<const h16x8*>(base + (size_t)ic * ld + hd * D + ds * 16 + hh * 8);
    dof[ds] = *reinterpret_cast<const h16x8*>(d_o + ((size_t)bi * T + ic) * H + hd * D + ds * 16 + hh * 8);
  }
  const float lse_i = lse[((size_t)bi * heads + hd) * T + ic] * kLog2e;
  // dsum_i = sum_t dO[i,t] O[i,t]: this kernel owns the query rows, so it forms the sum (each lane half holds
  // half of the row) and publishes it for the dK/dV kernel, which runs after this one
  float dpart = 0.f;
#pragma unroll
  for (int ds = 0; ds < D / 16; ds++) {
    const h16x8 of = *reinterpret_cast<const h16x8*>(o + ((size_t)bi * T + ic) * H + hd * D + ds * 16 + hh * 8);
#pragma unroll
    for (int e = 0; e < 8; e++) dpart += (float)of[e] * (float)dof[ds][e];
  }
  const float dsum_i = dpart + __shfl_xor(dpart, 32, 64);
  if (hh == 0 && i < T) dsum[((size_t)bi * heads + hd) * T + i] = dsum_i;

  const int nkv_all = (T + 63) / 64;
  const int nkv = causal ? min(nkv_all, (min(q0 + 127, T - 1)) / 64 + 1) : nkv_all;
  f32x16 dq[D / 32];
#pragma unroll
  for (int t = 0; t < D / 32; t++) dq[t] = zero16();

  // K and V tiles arrive through loads that write LDS, as in the forward kernel
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const size_t row_bytes = ld * sizeof(h16_t);
  const i32x4 rk = make_rsrc(base + H + hd * D, (size_t)(T - 1) * row_bytes + D * sizeof(h16_t));
  const i32x4 rv = make_rsrc(base + 2 * H + hd * D, (size_t)(T - 1) * row_bytes + D * sizeof(h16_t));
  int voff[IO::NI];
#pragma unroll
  for (int q = 0; q < IO::NI; q++) voff[q] = IO::dma_voff(q, wv, lane, ld);
  const unsigned lds_k = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
  const unsigned lds_v = lds_k + 2 * 64 * D * (unsigned)sizeof(h16_t);
  constexpr unsigned TILE_B = 64 * D * sizeof(h16_t);
  IO::dma_tile(rk, voff, 0, lds_k, wv);
  IO::dma_tile(rv, voff, 0, lds_v, wv);
  wait_vmcnt<0>();
  __syncthreads();
  for (int kb = 0; kb < nkv; kb++) {
    const int cur = kb & 1, j0 = kb * 64;
    if (kb + 1 < nkv) {
      const int soff = (int)((size_t)(j0 + 64) * row_bytes);
      IO::dma_tile(rk, voff, soff, lds_k + (cur ^ 1) * TILE_B, wv);
      IO::dma_tile(rv, voff, soff, lds_v + (cur ^ 1) * TILE_B, wv);
    }
    const h16_t* Kt = Ks + cur * 64 * D;
    const h16_t* Vt = Vs + cur * 64 * D;
    if (!(causal && j0 > qw0 + 31)) {
      f32x16 st[2] = {zero16(), zero16()}, dp[2] = {zero16(), zero16()};
      // fragments are requested eight at a time, ahead of the MFMAs that use them: one LDS latency per eight
      // MFMAs instead of one per MFMA
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int d0 = 0; d0 < D / 16; d0 += 4) {
          h16x8 ka[4], va[4];
#pragma unroll
          for (int ds = 0; ds < 4; ds++) {
            ka[ds] = IO::frag(Kt, jt * 32 + l32, (d0 + ds) * 2 + hh);
            va[ds] = IO::frag(Vt, jt * 32 + l32, (d0 + ds) * 2 + hh);
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int ds = 0; ds < 4; ds++) {
            st[jt] = KFKB_MFMA_H16(ka[ds], qf[d0 + ds], st[jt]);
            dp[jt] = KFKB_MFMA_H16(va[ds], dof[d0 + ds], dp[jt]);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      if (j0 + 63 >= T || (causal && j0 + 63 > qw0)) {
#pragma unroll
        for (int jt = 0; jt < 2; jt++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int j = j0 + jt * 32 + acc_row(r, hh);
            if (j >= T || (causal && j > i)) st[jt][r] = -INFINITY;
          }
      }
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const float p = exp2_raw(fmaf(st[jt][r], scale_log2, -lse_i));
          st[jt][r] = p * (dp[jt][r] - dsum_i);
        }
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int t16 = 0; t16 < 2; t16++) {
          h16x8 kt[D / 32];
#pragma unroll
          for (int t = 0; t < D / 32; t++) kt[t] = IO::frag_tr(Kt, jt * 32 + t16 * 16 + tr_row, t * 32 + tr_col);
          const h16x8 dsb = pack8(st[jt], t16 * 8);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int t = 0; t < D / 32; t++) dq[t] = KFKB_MFMA_H16(kt[t], dsb, dq[t]);
          __builtin_amdgcn_sched_barrier(0);
        }
    }
    wait_vmcnt<0>();
    __syncthreads();
  }
  if (i < T) {
    h16_t* row = dqkv + ((size_t)bi * T + i) * ld + hd * D;
#pragma unroll
    for (int t = 0; t < D / 32; t++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        h16x4 v;
#pragma unroll
        for (int e = 0; e < 4; e++) v[e] = (h16_t)(dq[t][q * 4 + e] * scale);
        *reinterpret_cast<h16x4*>(row + t * 32 + q * 8 + hh * 4) = v;
      }
  }
}

// ------------------------------------------------------------------------------------------------
// backward, dK and dV: own rows = keys, streamed rows = queries
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256) attn_bwd_dkv_h16_kernel(const h16_t* __restrict__ qkv, const h16_t* __restrict__ d_o,
                                                                const float* __restrict__ lse, const float* __restrict__ dsum,
                                                                h16_t* __restrict__ dqkv, int T, int H, int heads,
                                                                int causal, float scale, int pair) {
  using IO = TileIO<D>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  h16_t* Qs = reinterpret_cast<h16_t*>(smem);     // [2][64][D]
  h16_t* Os = Qs + 2 * 64 * D;                     // [2][64][D]   (dO tiles)
  float* Ls = reinterpret_cast<float*>(Os + 2 * 64 * D);   // [2][64] lse * log2(e)
  float* Ss = Ls + 2 * 64;                                 // [2][64] dsum
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hh = lane >> 5, l32 = lane & 31;
  const int tr_row = hh * 4 + ((lane & 15) >> 2);
  const int tr_col = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  int kb, bh;
  block_to_work(kb, bh, pair);
  kb = gridDim.x - 1 - kb;                          // for keys the early blocks are the long ones
  const int bi = bh / heads, hd = bh % heads;
  const size_t ld = 3 * (size_t)H;
  const h16_t* base = qkv + (size_t)bi * T * ld;
  const h16_t* dobase = d_o + (size_t)bi * T * H;
  const float* lbase = lse + ((size_t)bi * heads + hd) * T;
  const float* sbase = dsum + ((size_t)bi * heads + hd) * T;
  const int j0 = kb * 128, jw0 = j0 + wave * 32;
  const int j = jw0 + l32;
  const int jc = min(j, T - 1);
  const float scale_log2 = scale * kLog2e;

  h16x8 kf[D / 16], vf[D / 16];
#pragma unroll
  for (int ds = 0; ds < D / 16; ds++) {
    kf[ds] = *reinterpret_cast<const h16x8*>(base + (size_t)jc * ld + H + hd * D + ds * 16 + hh * 8);
    vf[ds] = *reinterpret_cast<const h16x8*>(base + (size_t)jc * ld + 2 * H + hd * D + ds * 16 + hh * 8);
  }
  f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
  for (int t = 0; t < D / 32; t++) { dk[t] = zero16(); dv[t] = zero16(); }

  const int nq = (T + 63) / 64;
  const int ib0 = causal ? j0 / 64 : 0;
  // Q and dO tiles arrive through loads that write LDS (rows past the end of the sequence read as zero and are
  // masked below); the 2 x 64 row statistics of a tile go through a register
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const i32x4 rq = make_rsrc(base + hd * D, (size_t)(T - 1) * ld * sizeof(h16_t) + D * sizeof(h16_t));
  const i32x4 ro = make_rsrc(dobase + hd * D, (size_t)(T - 1) * H * sizeof(h16_t) + D * sizeof(h16_t));
  int voffq[IO::NI], voffo[IO::NI];
#pragma unroll
  for (int q = 0; q < IO::NI; q++) { voffq[q] = IO::dma_voff(q, wv, lane, ld); voffo[q] = IO::dma_voff(q, wv, lane, (size_t)H); }
  const unsigned lds_q = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
  const unsigned lds_o = lds_q + 2 * 64 * D * (unsigned)sizeof(h16_t);
  constexpr unsigned TILE_B = 64 * D * sizeof(h16_t);
  float rstat = 0.f;
  auto load_stats = [&](int i0) {
    if (threadIdx.x < 64) rstat = lbase[min(i0 + (int)threadIdx.x, T - 1)] * kLog2e;
    else if (threadIdx.x < 128) rstat = sbase[min(i0 + (int)threadIdx.x - 64, T - 1)];
  };
  auto store_stats = [&](int st) {
    if (threadIdx.x < 64) Ls[st * 64 + threadIdx.x] = rstat;
    else if (threadIdx.x < 128) Ss[st * 64 + threadIdx.x - 64] = rstat;
  };
  if (ib0 < nq) {
    IO::dma_tile(rq, voffq, (int)((size_t)ib0 * 64 * ld * sizeof(h16_t)), lds_q, wv);
    IO::dma_tile(ro, voffo, (int)((size_t)ib0 * 64 * H * sizeof(h16_t)), lds_o, wv);
    load_stats(ib0 * 64);
    store_stats(0);
  }
  wait_vmcnt<0>();
  __syncthreads();
  for (int ib = ib0; ib < nq; ib++) {
    const int cur = (ib - ib0) & 1, i0 = ib * 64;
    if (ib + 1 < nq) {
      IO::dma_tile(rq, voffq, (int)((size_t)(i0 + 64) * ld * sizeof(h16_t)), lds_q + (cur ^ 1) * TILE_B, wv);
      IO::dma_tile(ro, voffo, (int)((size_t)(i0 + 64) * H * sizeof(h16_t)), lds_o + (cur ^ 1) * TILE_B, wv);
      load_stats(i0 + 64);
    }
    const h16_t* Qt = Qs + cur * 64 * D;
    const h16_t* Ot = Os + cur * 64 * D;
    if (!(causal && i0 + 63 < jw0)) {               // wave-uniform: some query of the tile sees these keys
      f32x16 st[2] = {zero16(), zero16()}, dp[2] = {zero16(), zero16()};
      // Fragments are requested eight at a time, one group AHEAD of the MFMAs that use them (this kernel runs one
      // wave per SIMD, so nothing else hides the LDS latency): group g covers query half g / GD and head-dimension
      // chunks (g % GD) * 4 .. + 3.
      constexpr int GD = D / 64, NG1 = 2 * GD;
      h16x8 qa[2][4], oa[2][4];
      auto load1 = [&](int g, h16x8 (&q4)[4], h16x8 (&o4)[4]) {
        const int it = g / GD, d0 = (g % GD) * 4;
#pragma unroll
        for (int ds = 0; ds < 4; ds++) {
          q4[ds] = IO::frag(Qt, it * 32 + l32, (d0 + ds) * 2 + hh);
          o4[ds] = IO::frag(Ot, it * 32 + l32, (d0 + ds) * 2 + hh);
        }
      };
      load1(0, qa[0], oa[0]);
#pragma unroll
      for (int g = 0; g < NG1; g++) {
        if (g + 1 < NG1) load1(g + 1, qa[(g + 1) & 1], oa[(g + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
        const int it = g / GD, d0 = (g % GD) * 4;
#pragma unroll
        for (int ds = 0; ds < 4; ds++) {
          st[it] = KFKB_MFMA_H16(qa[g & 1][ds], kf[d0 + ds], st[it]);
          dp[it] = KFKB_MFMA_H16(oa[g & 1][ds], vf[d0 + ds], dp[it]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (i0 + 63 >= T || jw0 + 31 >= T || (causal && jw0 + 31 > i0)) {
#pragma unroll
        for (int it = 0; it < 2; it++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int i = i0 + it * 32 + acc_row(r, hh);
            if (i >= T || j >= T || (causal && j > i)) st[it][r] = -INFINITY;
          }
      }
#pragma unroll
      for (int it = 0; it < 2; it++)
#pragma unroll
        for (int q = 0; q < 4; q++) {                // four consecutive query rows per register quad
          const int il = it * 32 + q * 8 + hh * 4;
          const float4 l4 = *reinterpret_cast<const float4*>(Ls + cur * 64 + il);
          const float4 s4 = *reinterpret_cast<const float4*>(Ss + cur * 64 + il);
          const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, sv[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const float p = exp2_raw(fmaf(st[it][q * 4 + e], scale_log2, -lv[e]));
            st[it][q * 4 + e] = p;
            dp[it][q * 4 + e] = p * (dp[it][q * 4 + e] - sv[e]);
          }
        }
      // second half: groups of sixteen streamed rows, their transposed fragments again one group ahead
      h16x8 ot[2][D / 32], qt[2][D / 32];
      auto load3 = [&](int g, h16x8 (&o4)[D / 32], h16x8 (&q4)[D / 32]) {
        const int it = g >> 1, t16 = g & 1;
#pragma unroll
        for (int t = 0; t < D / 32; t++) {
          o4[t] = IO::frag_tr(Ot, it * 32 + t16 * 16 + tr_row, t * 32 + tr_col);
          q4[t] = IO::frag_tr(Qt, it * 32 + t16 * 16 + tr_row, t * 32 + tr_col);
        }
      };
      load3(0, ot[0], qt[0]);
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const int it = g >> 1, t16 = g & 1;
        if (g + 1 < 4) load3(g + 1, ot[(g + 1) & 1], qt[(g + 1) & 1]);
        const h16x8 pb = pack8(st[it], t16 * 8);
        const h16x8 dsb = pack8(dp[it], t16 * 8);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < D / 32; t++) {
          dv[t] = KFKB_MFMA_H16(ot[g & 1][t], pb, dv[t]);
          dk[t] = KFKB_MFMA_H16(qt[g & 1][t], dsb, dk[t]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (ib + 1 < nq) store_stats(cur ^ 1);
    wait_vmcnt<0>();
    __syncthreads();
  }
  if (j < T) {
    h16_t* krow = dqkv + ((size_t)bi * T + j) * ld + H + hd * D;
    h16_t* vrow = dqkv + ((size_t)bi * T + j) * ld + 2 * H + hd * D;
#pragma unroll
    for (int t = 0; t < D / 32; t++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        h16x4 a, b;
#pragma unroll
        for (int e = 0; e < 4; e++) { a[e] = (h16_t)(dk[t][q * 4 + e] * scale); b[e] = (h16_t)dv[t][q * 4 + e]; }
        *reinterpret_cast<h16x4*>(krow + t * 32 + q * 8 + hh * 4) = a;
        *reinterpret_cast<h16x4*>(vrow + t * 32 + q * 8 + hh * 4) = b;
      }
  }
}

// ------------------------------------------------------------------------------------------------

template <typename K>
static hipError_t set_smem(K kern, size_t bytes, bool& done) {
  if (done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) done = true;
  return e;
}

// two blocks per CU, all of an XCD's blocks resident at once (8 XCDs of 32 CUs)?
template <typename K>
static int pair_blocks(K kern, size_t smem, int gx, int gy, int causal) {
  if (!causal || gy % 8 != 0 || gx * (gy / 8) != 64 || 32 % gx != 0) return 0;
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 256, smem) != hipSuccess) return 0;
  return per_cu >= 2 ? 1 : 0;
}

template <int D>
static hipError_t fwd_d(const h16_t* qkv, h16_t* o, float* lse, int b, int T, int H, int heads, int causal, hipStream_t s) {
  static bool attr = false;
  const size_t smem = (size_t)4 * 64 * D * sizeof(h16_t);
  hipError_t e = set_smem(attn_fwd_h16_kernel<D>, smem, attr);
  if (e != hipSuccess) return e;
  const float scale_log2 = kLog2e / sqrtf((float)D);
  const double pairs = (double)b * heads * T * T * (causal ? 0.5 : 1.0);
  klaunch(attn_fwd_h16_kernel<D>, dim3((T + 127) / 128, b * heads), dim3(256), smem, s, PK_ATTN_FWD + D / 128, 4.0 * pairs * D,
          qkv, o, lse, T, H, heads, causal, scale_log2, pair_blocks(attn_fwd_h16_kernel<D>, smem, (T + 127) / 128, b * heads, causal));
  return hipGetLastError();
}

template <int D>
static hipError_t bwd_d(const h16_t* qkv, const h16_t* o, const h16_t* d_o, const float* lse, float* dsum, h16_t* dqkv,
                        int b, int T, int H, int heads, int causal, hipStream_t s) {
  static bool attr1 = false, attr2 = false;
  const size_t smem1 = (size_t)4 * 64 * D * sizeof(h16_t);
  const size_t smem2 = smem1 + 4 * 64 * sizeof(float);
  hipError_t e = set_smem(attn_bwd_dq_h16_kernel<D>, smem1, attr1);
  if (e != hipSuccess) return e;
  e = set_smem(attn_bwd_dkv_h16_kernel<D>, smem2, attr2);
  if (e != hipSuccess) return e;
  const float scale = 1.0f / sqrtf((float)D);
  const dim3 grid((T + 127) / 128, b * heads);
  const double pairs = (double)b * heads * T * T * (causal ? 0.5 : 1.0);
  klaunch(attn_bwd_dq_h16_kernel<D>, grid, dim3(256), smem1, s, PK_ATTN_DQ + D / 128, 6.0 * pairs * D, qkv, o, d_o, lse, dsum, dqkv,
          T, H, heads, causal, scale, pair_blocks(attn_bwd_dq_h16_kernel<D>, smem1, (int)grid.x, (int)grid.y, causal));
  klaunch(attn_bwd_dkv_h16_kernel<D>, grid, dim3(256), smem2, s, PK_ATTN_DKV + D / 128, 8.0 * pairs * D, qkv, d_o, lse,
          (const float*)dsum, dqkv, T, H, heads, causal, scale, pair_blocks(attn_bwd_dkv_h16_kernel<D>, smem2, (int)grid.x, (int)grid.y, causal));
  return hipGetLastError();
}

hipError_t launch_attention_fwd_h16(const h16_t* qkv, h16_t* o, float* lse, int b, int T, int H, int heads,
                                     int causal, hipStream_t s) {
  if (b <= 0 || T <= 0) return hipSuccess;
  if ((double)T * 3.0 * H * sizeof(h16_t) >= 2147483648.0) return hipErrorInvalidValue;   // 32-bit byte offsets inside a sample
  return (H / heads == 64) ? fwd_d<64>(qkv, o, lse, b, T, H, heads, causal, s)
                           : fwd_d<128>(qkv, o, lse, b, T, H, heads, causal, s);
}

hipError_t launch_attention_bwd_h16(const h16_t* qkv, const h16_t* o, const h16_t* d_o, const float* lse,
                                     float* dsum, h16_t* dqkv, int b, int T, int H, int heads, int causal,
                                     hipStream_t s) {
  if (b <= 0 || T <= 0) return hipSuccess;
  if ((double)T * 3.0 * H * sizeof(h16_t) >= 2147483648.0) return hipErrorInvalidValue;
  return (H / heads == 64) ? bwd_d<64>(qkv, o, d_o, lse, dsum, dqkv, b, T, H, heads, causal, s)
                           : bwd_d<128>(qkv, o, d_o, lse, dsum, dqkv, b, T, H, heads, causal, s);
}

#ifdef KFKB_H16_IS_F16
}  // namespace f16k
hipError_t launch_attention_fwd_f16(const void* qkv, void* o, float* lse, int b, int T, int H, int heads, int causal, hipStream_t s) {
  return f16k::launch_attention_fwd_h16((const f16_t*)qkv, (f16_t*)o, lse, b, T, H, heads, causal, s);
}
hipError_t launch_attention_bwd_f16(const void* qkv, const void* o, const void* d_o, const float* lse, float* dsum, void* dqkv,
                                    int b, int T, int H, int heads, int causal, hipStream_t s) {
  return f16k::launch_attention_bwd_h16((const f16_t*)qkv, (const f16_t*)o, (const f16_t*)d_o, lse, dsum, (f16_t*)dqkv, b, T, H, heads, causal, s);
}
#else
}  // namespace bf16k
hipError_t launch_attention_fwd_bf16(const void* qkv, void* o, float* lse, int b, int T, int H, int heads, int causal, hipStream_t s) {
  return bf16k::launch_attention_fwd_h16((const bf16_t*)qkv, (bf16_t*)o, lse, b, T, H, heads, causal, s);
}
hipError_t launch_attention_bwd_bf16(const void* qkv, const void* o, const void* d_o, const float* lse, float* dsum, void* dqkv,
                                     int b, int T, int H, int heads, int causal, hipStream_t s) {
  return bf16k::launch_attention_bwd_h16((const bf16_t*)qkv, (const bf16_t*)o, (const bf16_t*)d_o, lse, dsum, (bf16_t*)dqkv, b, T, H, heads, causal, s);
}
#endif

}  // namespace kfkb
