// 16-bit (bf16 or fp16 storage) GEMMs of the stage on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16 / _f16),
// fp32 accumulation.
//
//   NT:  C[M,N] = A[M,K] . B[N,K]^T     both operands contiguous along the reduction axis
//        (forward with the weight copy stored [out,in]; input gradients with the weights as given)
//   TN:  C[M,N] = A[K,M]^T . B[K,N]     both operands strided along the reduction axis, which is
//        the token axis (weight gradients: A = layer input, B = output gradient)
//
// One work-group = 256 threads = 2 x 2 waves computes a BM x BN tile (256 x 256 or 128 x 128) in 32-deep chunks.
// Four chunks live in LDS (a ring of four slots); they are filled by buffer loads that write straight into
// LDS (no registers, no LDS store instructions, out-of-range rows read as zero), requested three to four
// chunks ahead, one load instruction per group of MFMAs so that the loads of the four waves never queue up
// behind each other.  Measured on the MI355X: the matrix pipe alone (no loads, no LDS reads) takes 1035 clocks
// per chunk of a 256 x 256 tile, this loop about 1200; bursts of loads used to cost 1300 and more.
//
// NT chunks are stored [row][32] with the 16-byte piece index XOR-ed by ((row >> 2) & 3), TN chunks as they lie
// in memory, [reduction row][BM], piece index XOR 4 * (row & 3), and read with the LDS transpose read
// (ds_read_b64_tr_b16), which hands every lane four reduction-consecutive values of its column: both make
// the fragment reads bank-conflict free on the 64-bank LDS.
//
// The MFMA is issued with its operands swapped (A operand <- B tile, B operand <- A tile): the accumulator of
// lane l then holds, for output row m = l % 32, four consecutive output columns per register quad.  Finished
// values are rounded once and go through LDS, so that C is written in whole rows, 16 bytes per lane.
//
// Block index -> tile: consecutive block ids land on different XCDs (8 of them, each with its own
// L2), so block b works on tile (b % 8) * ceil(tiles/8) + b / 8: every XCD owns a contiguous run of
// the tile order, and that order walks groups of four tile-rows column by column.
#include "common.h"
#include "../../include/kfkb.h"
#include <algorithm>
#include <type_traits>

namespace kfkb {
// Built once per 16-bit storage type: this file as it is for bf16, through gemm_f16.hip (which defines
// KFKB_H16_IS_F16) for fp16.  Everything type-dependent lives in a namespace of its own, so the two builds share no
// symbol; the launchers the rest of the library calls are defined at the end of the file.
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
hipError_t launch_gemm_h16(const GemmArgs& g, hipStream_t s);
const char* gemm_h16_check(const GemmArgs& g);
bool wstep_groupable_h16(const WGrad* g, int n, int K, const WStepReduce* red);
hipError_t launch_wstep_h16(const WGrad* g, int n, int K, int nseg, hipStream_t s, const WStepReduce* red);

constexpr int BK = 64;             // slice depth of the register-staged TN kernel

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
__device__ __forceinline__ int linear_of_block(int total_tiles, int block = blockIdx.x) {
  const int per_xcd = (total_tiles + 7) / 8;
  return (block % 8) * per_xcd + block / 8;
}
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn, bool& valid) {
  const int t = linear_of_block(tiles_m * tiles_n);
  valid = t < tiles_m * tiles_n;
  tile_from_linear(t, tiles_m, tiles_n, tm, tn);
}

template <int EPI>
__device__ __forceinline__ void epilogue_quad(const f32x16& acc, int q, int m, int n, int N, const h16_t* __restrict__ bias,
                                              const h16_t* __restrict__ residual, h16_t* __restrict__ C,
                                              h16_t* __restrict__ C2, float* __restrict__ Cacc) {
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
    const h16x4 b = *reinterpret_cast<const h16x4*>(bias + n);
#pragma unroll
    for (int e = 0; e < 4; e++) v[e] += (float)b[e];
  }
  if (EPI == KFKB_EPI_BIAS_RES) {
    const h16x4 r = *reinterpret_cast<const h16x4*>(residual + o);
#pragma unroll
    for (int e = 0; e < 4; e++) v[e] += (float)r[e];
  }
  if (EPI == KFKB_EPI_GELU_BWD) {
    const h16x4 r = *reinterpret_cast<const h16x4*>(residual + o);
#pragma unroll
    for (int e = 0; e < 4; e++) v[e] *= gelu_grad_f((float)r[e]);
  }
  h16x4 out;
#pragma unroll
  for (int e = 0; e < 4; e++) out[e] = (h16_t)v[e];
  *reinterpret_cast<h16x4*>(C + o) = out;
  if (EPI == KFKB_EPI_BIAS_GELU) {
    h16x4 g;
#pragma unroll
    for (int e = 0; e < 4; e++) g[e] = (h16_t)gelu_f((float)out[e]);   // gelu of the stored (rounded) pre-activation
    *reinterpret_cast<h16x4*>(C2 + o) = g;
  }
}


constexpr int CK_ = 32;            // depth of a chunk
constexpr int RING = 4;            // chunks in LDS


// ------------------------------------------------------------------------------------------------
// The main loop shared by the NT and TN kernels.  LAYOUT owns the LDS rings, the DMA source offsets and the
// fragment reads; the loop owns the order of instructions.
//   One chunk = 32 reduction steps = two 16-deep k-steps; a k-step = TN groups of TM MFMAs.  Every group carries
//   one DMA instruction (dma0 during k-step 0, dma1 during k-step 1: the layout decides which piece of which later
//   chunk that is) and up to PER fragment reads of the next k-step.  A load that writes LDS keeps its wave from
//   issuing anything else for about 32 clocks (measured: one wave alone moves 31 bytes per clock), which is the
//   time one MFMA occupies the matrix pipe: in the 256 x 256 tiles every MFMA is therefore followed by exactly one
//   memory instruction, pinned there, and the pipe never waits for the issue port.
//   Between the k-steps every wave waits until at most WAIT_MID of its own loads are in flight (the layout's
//   issue order makes that "chunk kc+1 has landed") and all waves meet: after that chunk kc+1 is complete in LDS
//   and the ring slots that only chunk kc's first k-step still needed may be overwritten.
//   The position pc of a chunk inside the layout's period (the least common multiple of its ring lengths) is a
//   compile-time constant, so every LDS offset is an immediate.
// ------------------------------------------------------------------------------------------------
template <int TM, int TN, typename L>
__device__ __forceinline__ void main_loop(L& lay, f32x16 (&acc)[TM][TN], int nk) {
  h16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  lay.prologue();
  wait_vmcnt<L::WAIT_PRO>();
  __syncthreads();
#pragma unroll
  for (int j = 0; j < TN; j++) fb0[j] = lay.rd_b(0, 0, j);
#pragma unroll
  for (int i = 0; i < TM; i++) fa0[i] = lay.rd_a(0, 0, i);

  auto step = [&](h16x8 (&fa)[TM], h16x8 (&fb)[TN], h16x8 (&na)[TM], h16x8 (&nb)[TN], int npc, int nks, auto&& dma) {
    constexpr int NR = TM + TN;
    constexpr int PER = (NR + TN - 2) / (TN - 1);      // reads per group so that the last group has none
    auto rd = [&](int r) {
      if (r == 0) nb[0] = lay.rd_b(npc, nks, 0);
      else if (r <= TM) na[r - 1] = lay.rd_a(npc, nks, r - 1);
      else nb[r - TM] = lay.rd_b(npc, nks, r - TM);
    };
#pragma unroll
    for (int j = 0; j < TN; j++) {
      if constexpr (PER + 1 <= TM) {
        // MFMA i is followed by exactly one memory instruction (the DMA after the first, fragment reads after
        // the next ones): each issues while that MFMA occupies the matrix pipe
#pragma unroll
        for (int i = 0; i < TM; i++) {
          acc[i][j] = KFKB_MFMA_H16(fb[j], fa[i], acc[i][j]);
          __builtin_amdgcn_sched_barrier(0);
          if (i == 0) dma(j);
          else { const int r = j * PER + (i - 1); if (i - 1 < PER && r < NR) rd(r); }
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
#pragma unroll
        for (int r = j * PER; r < (j + 1) * PER && r < NR; r++) rd(r);
        dma(j);
#pragma unroll
        for (int i = 0; i < TM; i++) acc[i][j] = KFKB_MFMA_H16(fb[j], fa[i], acc[i][j]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  auto chunk = [&](int kc, int pc) {
    step(fa0, fb0, fa1, fb1, pc, 1, [&](int j) { lay.dma0(j, kc, pc); });
    wait_vmcnt<L::WAIT_MID>();
    wait_lgkm0();
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    step(fa1, fb1, fa0, fb0, (pc + 1) % L::PERIOD, 0, [&](int j) { lay.dma1(j, kc, pc); });
  };
  for (int kc = 0; kc < nk; kc += L::PERIOD) {
#pragma unroll
    for (int pc = 0; pc < L::PERIOD; pc++) {
      if (kc + pc < nk) chunk(kc + pc, pc);
    }
  }
  wait_vmcnt<0>();
}

// NT operands: X[rows, K] row-major, both.  LDS chunk [rows][32]: 16-byte piece p of row r holds logical piece
// p ^ ((r >> 2) & 3): the 16 rows a fragment read touches per clock land on 16 different 16-byte bank groups.
// BT: the B operand is stored chunk-major, [K/32][N][32] (the stage's weight copies): a chunk of B rows is then one
// contiguous run, where row-major rows give every load half a cache line per row and make L2 serve each line twice.
template <int BM, int BN, bool BT>
struct NtLayout32 {
  static constexpr int TM = BM / 64, TN = BN / 64, A_SLOT = BM * CK_, B_SLOT = BN * CK_;
  static_assert(TM == TN, "one DMA instruction per MFMA group");
  static constexpr int PERIOD = RING, WAIT_PRO = 5 * TN, WAIT_MID = 4 * TN;
  static constexpr size_t LDS_BYTES = (size_t)RING * (A_SLOT + B_SLOT) * 2;
  i32x4 ra, rb; unsigned lds0; int wave, nk, sb; int voa[TN], vob[TN];
  const h16_t* fa_base[2]; const h16_t* fb_base[2];
  __device__ __forceinline__ void init(char* smem, const h16_t* A, const h16_t* B, int M, int N, int K, int m0, int n0, int lane, int wave_) {
    wave = wave_; nk = K / CK_; sb = BT ? N * CK_ * 2 : CK_ * 2;      // bytes from one chunk of B to the next
    ra = make_rsrc(A, (size_t)M * K * 2); rb = make_rsrc(B, (size_t)N * K * 2);
    lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
    const int lrow = lane >> 2, lpiece = (lane & 3) ^ ((lane >> 4) & 3);
#pragma unroll
    for (int i = 0; i < TN; i++) {
      voa[i] = ((m0 + (i * 4 + wave) * 16 + lrow) * K + lpiece * 8) * 2;
      vob[i] = ((n0 + (i * 4 + wave) * 16 + lrow) * (BT ? CK_ : K) + lpiece * 8) * 2;
    }
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);
    const int frow = lane & 31, fhalf = lane >> 5, fsw = (lane >> 2) & 3;
    const h16_t* As = reinterpret_cast<const h16_t*>(smem);
    const h16_t* Bs = As + RING * A_SLOT;
#pragma unroll
    for (int ks = 0; ks < 2; ks++) {
      fa_base[ks] = As + (wm0 + frow) * CK_ + (((ks * 2 + fhalf) ^ fsw) << 3);
      fb_base[ks] = Bs + (wn0 + frow) * CK_ + (((ks * 2 + fhalf) ^ fsw) << 3);
    }
  }
  __device__ __forceinline__ void dma_a(int i, int kc, int slot) { dma16b(ra, voa[i], min(kc, nk - 1) * (CK_ * 2), lds0 + (slot * A_SLOT + (i * 4 + wave) * 512) * 2); }
  __device__ __forceinline__ void dma_b(int i, int kc, int slot) { dma16b(rb, vob[i], min(kc, nk - 1) * sb, lds0 + (RING * A_SLOT + slot * B_SLOT + (i * 4 + wave) * 512) * 2); }
  // issue order: A then B of chunks 0..2, A of chunk 3; then per chunk kc: B of kc+3 (k-step 0), A of kc+4 (k-step 1)
  __device__ __forceinline__ void prologue() {
#pragma unroll
    for (int c = 0; c < RING; c++) {
#pragma unroll
      for (int i = 0; i < TN; i++) dma_a(i, c, c);
      if (c < RING - 1) {
#pragma unroll
        for (int i = 0; i < TN; i++) dma_b(i, c, c);
      }
    }
  }
  __device__ __forceinline__ void dma0(int j, int kc, int pc) { dma_b(j, kc + 3, (pc + 3) & 3); }
  __device__ __forceinline__ void dma1(int j, int kc, int pc) { dma_a(j, kc + 4, pc); }
  __device__ __forceinline__ h16x8 rd_a(int slot, int ks, int i) { return *reinterpret_cast<const h16x8*>(fa_base[ks] + slot * A_SLOT + i * 32 * CK_); }
  __device__ __forceinline__ h16x8 rd_b(int slot, int ks, int j) { return *reinterpret_cast<const h16x8*>(fb_base[ks] + slot * B_SLOT + j * 32 * CK_); }
};

// NT operands with a chunk-major B (the stage's weight copies) and K % 64 == 0: A is staged in slices of 64
// reduction steps, so that every DMA instruction reads eight whole 128-byte rows (a 32-deep chunk of a row-major
// operand is half a cache line per row, and L2 then serves every line twice).  A slice feeds two chunks; the A ring
// holds three slices, the B ring four chunks, together all 160 KiB of the CU for 256 x 256 tiles (half for
// 128 x 128).  Slice S+3 overwrites slice S, which is free once chunk 2S+1 has passed its middle barrier: its
// first half is issued in k-step 1 of chunk 2S+1, its second half in k-step 1 of chunk 2S+2, five and four
// chunks before its first read.  B of chunk kc+3 goes out in k-step 0 of chunk kc.  Loads retire in order, so
// "at most 4 TN in flight" at the middle of chunk kc means B of kc+1 and everything older (the A slice of kc+1
// among it) has landed.
// LDS slice [rows][64]: 16-byte piece p of row r holds logical piece p ^ ((r >> 1) & 7): the 16 rows a fragment
// read touches per clock land on 16 different 16-byte bank groups.
template <int BM, int BN>
struct NtLayout64 {
  static constexpr int TM = BM / 64, TN = BN / 64, A_SLICE = BM * 64, B_SLOT = BN * CK_, A_RING = 3;
  // Per chunk and wave: TN pieces of B (one per MFMA group of the first k-step) and TM pieces of A (on the first TM
  // groups of the second k-step): a tile may be narrower in M than in N, not the other way round.
  static_assert(TM <= TN, "the A pieces of a chunk ride on the first TM groups of its second k-step");
  static constexpr int PERIOD = 12, WAIT_PRO = 3 * TM + 2 * TN, WAIT_MID = 2 * TM + 2 * TN;
  static constexpr size_t LDS_BYTES = (size_t)(A_RING * A_SLICE + RING * B_SLOT) * 2;
  i32x4 ra, rb; unsigned lds0; int wave, nk, ns, sb; int voa[2 * TM], vob[TN];
  const h16_t* fa_base[4]; const h16_t* fb_base[2];
  __device__ __forceinline__ void init(char* smem, const h16_t* A, const h16_t* B, int M, int N, int K, int m0, int n0, int lane, int wave_) {
    wave = wave_; nk = K / CK_; ns = K / 64; sb = N * CK_ * 2;       // bytes from one chunk of B to the next
    ra = make_rsrc(A, (size_t)M * K * 2); rb = make_rsrc(B, (size_t)N * K * 2);
    lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
    // A: instruction g = i * 4 + wave covers rows 8 g .. 8 g + 7, lane l row l / 8, physical piece l % 8
    const int arow = lane >> 3, apiece = (lane & 7) ^ (((wave & 1) << 2) | (lane >> 4));
#pragma unroll
    for (int i = 0; i < 2 * TM; i++) voa[i] = ((m0 + (i * 4 + wave) * 8 + arow) * K + apiece * 8) * 2;
    const int brow = lane >> 2, bpiece = (lane & 3) ^ ((lane >> 4) & 3);
#pragma unroll
    for (int i = 0; i < TN; i++) vob[i] = ((n0 + (i * 4 + wave) * 16 + brow) * CK_ + bpiece * 8) * 2;
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);
    const int frow = lane & 31, fhalf = lane >> 5, fsw_a = (lane >> 1) & 7, fsw_b = (lane >> 2) & 3;
    const h16_t* As = reinterpret_cast<const h16_t*>(smem);
    const h16_t* Bs = As + A_RING * A_SLICE;
#pragma unroll
    for (int q = 0; q < 4; q++) fa_base[q] = As + (wm0 + frow) * 64 + (((q * 2 + fhalf) ^ fsw_a) << 3);   // q = 2 (chunk & 1) + k-step
#pragma unroll
    for (int ks = 0; ks < 2; ks++) fb_base[ks] = Bs + (wn0 + frow) * CK_ + (((ks * 2 + fhalf) ^ fsw_b) << 3);
  }
  __device__ __forceinline__ void dma_a(int instr, int slice, int slot) {
    dma16b(ra, voa[instr], min(slice, ns - 1) * 128, lds0 + (slot * A_SLICE + (instr * 4 + wave) * 512) * 2);
  }
  __device__ __forceinline__ void dma_b(int i, int kc, int slot) {
    dma16b(rb, vob[i], min(kc, nk - 1) * sb, lds0 + (A_RING * A_SLICE + slot * B_SLOT + (i * 4 + wave) * 512) * 2);
  }
  // The order keeps the loop's invariant from the first chunk on: behind B of chunk c+1 come exactly two halves
  // of A slices and B of chunks c+2 and c+3 when chunk c reaches its middle.
  __device__ __forceinline__ void prologue() {
#pragma unroll
    for (int i = 0; i < 2 * TM; i++) dma_a(i, 0, 0);
#pragma unroll
    for (int i = 0; i < TN; i++) dma_b(i, 0, 0);
#pragma unroll
    for (int i = 0; i < TM; i++) dma_a(i, 1, 1);
#pragma unroll
    for (int i = 0; i < TN; i++) dma_b(i, 1, 1);
#pragma unroll
    for (int i = 0; i < TM; i++) dma_a(TM + i, 1, 1);
#pragma unroll
    for (int i = 0; i < TN; i++) dma_b(i, 2, 2);
#pragma unroll
    for (int i = 0; i < TM; i++) dma_a(i, 2, 2);
  }
  __device__ __forceinline__ void dma0(int j, int kc, int pc) { dma_b(j, kc + 3, (pc + 3) & 3); }
  __device__ __forceinline__ void dma1(int j, int kc, int pc) {
    if (j >= TM) return;
    if (pc & 1) dma_a(j, (kc >> 1) + 3, (pc >> 1) % 3);
    else dma_a(TM + j, (kc >> 1) + 2, ((pc >> 1) + 2) % 3);
  }
  __device__ __forceinline__ h16x8 rd_a(int pc, int ks, int i) {
    return *reinterpret_cast<const h16x8*>(fa_base[(pc & 1) * 2 + ks] + ((pc >> 1) % 3) * A_SLICE + i * 32 * 64);
  }
  __device__ __forceinline__ h16x8 rd_b(int pc, int ks, int j) { return *reinterpret_cast<const h16x8*>(fb_base[ks] + (pc & 3) * B_SLOT + j * 32 * CK_); }
};

// TN operands: X[K, cols] row-major, both (K = reduction).  LDS chunk [32 reduction rows][cols] as in memory, the
// 16-byte piece index XOR 4 * (row & 3); fragments come out of LDS transpose reads (ds_read_b64_tr_b16), two per
// fragment: each hands a lane four reduction-consecutive values of its column.
template <int BM, int BN>
struct TnLayout {
  static constexpr int TM = BM / 64, TN = BN / 64, A_SLOT = BM * CK_, B_SLOT = BN * CK_;
  static_assert(TM == TN, "one DMA instruction per MFMA group");
  static constexpr int PERIOD = RING, WAIT_PRO = 5 * TN, WAIT_MID = 4 * TN;
  static constexpr size_t LDS_BYTES = (size_t)RING * (A_SLOT + B_SLOT) * 2;
  static constexpr int CA = BM / 8, CB = BN / 8;           // 16-byte pieces per row
  static constexpr int RA = 64 / CA, RB = 64 / CB;         // rows one DMA instruction (1 KiB) covers
  i32x4 ra, rb; unsigned lds0; int wave, nk, sa, sb; int voa[TN], vob[TN];
  const h16_t* fa_base[TM]; const h16_t* fb_base[TN];
  __device__ __forceinline__ void init(char* smem, const h16_t* A, const h16_t* B, int M, int N, int K, int m0, int n0, int lane, int wave_) {
    wave = wave_; nk = K / CK_;
    ra = make_rsrc(A, (size_t)K * M * 2); rb = make_rsrc(B, (size_t)K * N * 2);
    sa = CK_ * M * 2; sb = CK_ * N * 2;                    // bytes per chunk step
    lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
#pragma unroll
    for (int i = 0; i < TN; i++) {
      const int rowa = (i * 4 + wave) * RA + lane / CA, pa = lane % CA;
      voa[i] = (rowa * M + m0 + (pa ^ (4 * (rowa & 3))) * 8) * 2;
      const int rowb = (i * 4 + wave) * RB + lane / CB, pb = lane % CB;
      vob[i] = (rowb * N + n0 + (pb ^ (4 * (rowb & 3))) * 8) * 2;
    }
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);
    const int g16 = lane >> 4, j16 = lane & 15;
    const int tr_row = (g16 >> 1) * 8 + (j16 >> 2), tr_col = (g16 & 1) * 16 + (j16 & 3) * 4;
    const int sw = 4 * (tr_row & 3);
    const h16_t* As = reinterpret_cast<const h16_t*>(smem);
    const h16_t* Bs = As + RING * A_SLOT;
#pragma unroll
    for (int i = 0; i < TM; i++) {
      const int col = wm0 + i * 32 + tr_col;
      fa_base[i] = As + tr_row * BM + (((col >> 3) ^ sw) << 3) + (col & 7);
    }
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int col = wn0 + j * 32 + tr_col;
      fb_base[j] = Bs + tr_row * BN + (((col >> 3) ^ sw) << 3) + (col & 7);
    }
  }
  __device__ __forceinline__ void dma_a(int i, int kc, int slot) { dma16b(ra, voa[i], min(kc, nk - 1) * sa, lds0 + (slot * A_SLOT + (i * 4 + wave) * 512) * 2); }
  __device__ __forceinline__ void dma_b(int i, int kc, int slot) { dma16b(rb, vob[i], min(kc, nk - 1) * sb, lds0 + (RING * A_SLOT + slot * B_SLOT + (i * 4 + wave) * 512) * 2); }
  __device__ __forceinline__ void prologue() {
#pragma unroll
    for (int c = 0; c < RING; c++) {
#pragma unroll
      for (int i = 0; i < TN; i++) dma_a(i, c, c);
      if (c < RING - 1) {
#pragma unroll
        for (int i = 0; i < TN; i++) dma_b(i, c, c);
      }
    }
  }
  __device__ __forceinline__ void dma0(int j, int kc, int pc) { dma_b(j, kc + 3, (pc + 3) & 3); }
  __device__ __forceinline__ void dma1(int j, int kc, int pc) { dma_a(j, kc + 4, pc); }
  static __device__ __forceinline__ h16x8 tr_pair(const h16_t* p, int second_offset) {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + second_offset));
    union { struct { s16x4 a, b; } s; h16x8 v; } u;
    u.s.a = lo; u.s.b = hi;
    return u.v;
  }
  __device__ __forceinline__ h16x8 rd_a(int slot, int ks, int i) { return tr_pair(fa_base[i] + slot * A_SLOT + ks * 16 * BM, 4 * BM); }
  __device__ __forceinline__ h16x8 rd_b(int slot, int ks, int j) { return tr_pair(fb_base[j] + slot * B_SLOT + ks * 16 * BN, 4 * BN); }
};

// The staged epilogues read the 256 accumulator registers of the large tiles with v_accvgpr_read_b32 in inline
// assembly, where the compiler's hazard recogniser does not see an accumulator read: the wait states an MFMA result
// needs before a vector instruction may read it (at most 18 for the 16-pass forms) are spent here, once, after the
// last MFMA of the main loop.
__device__ __forceinline__ void mfma_results_settled() { asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory"); }

// ---- epilogues ---------------------------------------------------------------------------------
// Accumulator of lane l, register 4 q + e: row (l % 32) of the 32 x 32 tile, column q * 8 + (l / 32) * 4 + e.
// The finished values (bias, residual or GELU derivative applied in fp32, rounded once) go through LDS so
// that every row is written with 16 bytes per lane, whole rows at a time; BIAS_GELU takes the GELU of the
// rounded pre-activation on the way out.
template <int BM, int BN> constexpr size_t epilogue_lds_bytes() { return (size_t)4 * (BM / 2) * (BN + 16); }
template <int BM, int BN, int EPI>
__device__ __forceinline__ void epilogue_staged(f32x16 (&acc)[BM / 64][BN / 64], char* smem, int M, int N, int m0, int n0, int lane, int wave,
                                                const h16_t* __restrict__ bias, const h16_t* __restrict__ residual,
                                                h16_t* __restrict__ C, h16_t* __restrict__ C2) {
  constexpr int TM = BM / 64, TN = BN / 64, WR = BM / 2, WC = BN / 2;
  constexpr int RS = WC * 2 + 16;                                 // row stride in bytes
  const int wm0 = (wave >> 1) * WR, wn0 = (wave & 1) * WC;
  const int frow = lane & 31, fhalf = lane >> 5;
  constexpr bool HAS_BIAS = EPI == KFKB_EPI_BIAS || EPI == KFKB_EPI_BIAS_GELU || EPI == KFKB_EPI_BIAS_RES;
  constexpr bool HAS_RES = EPI == KFKB_EPI_BIAS_RES || EPI == KFKB_EPI_GELU_BWD;
  constexpr int LPR = WC / 8, RPI = 64 / LPR;                     // lanes per row (16 bytes each), rows per instruction
  const int er = lane / LPR, ec = lane % LPR;
  // The residual of the wave's whole quadrant is requested at once, before the barrier (the fragment registers of
  // the main loop are free by now, and the memory latency is paid once), in the shape of the final store: 16 bytes
  // per lane along the rows, so that an instruction touches 8 cache lines and not 32.  It reaches the accumulator
  // layout through the wave's staging rows: every lane later reads exactly the 8 bytes it then overwrites with its
  // result, and a wave's LDS accesses execute in order.
  constexpr int NLD = WR / RPI;
  h16x8 rres[HAS_RES ? NLD : 1];
  if constexpr (HAS_RES) {
#pragma unroll
    for (int t = 0; t < NLD; t++) {
      const int m = min(m0 + wm0 + t * RPI + er, M - 1);
      rres[t] = *reinterpret_cast<const h16x8*>(residual + (size_t)m * N + n0 + wn0 + ec * 8);
    }
  }
  h16x4 bb[HAS_BIAS ? TN : 1][4];                                 // the lane's bias values, the same for every row block
  if constexpr (HAS_BIAS) {
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int q = 0; q < 4; q++) bb[j][q] = *reinterpret_cast<const h16x4*>(bias + n0 + wn0 + j * 32 + q * 8 + fhalf * 4);
  }
  __syncthreads();                                                // every wave is done with the ring
  if constexpr (TM * TN == 16) mfma_results_settled();
  char* ew = smem + wave * (WR * RS);
  if constexpr (HAS_RES) {
#pragma unroll
    for (int t = 0; t < NLD; t++) *reinterpret_cast<h16x8*>(ew + (t * RPI + er) * RS + ec * 16) = rres[t];
  }
#pragma unroll
  for (int i = 0; i < TM; i++) {
    __builtin_amdgcn_sched_barrier(0);                            // one 32-row block at a time
    h16x4 rr[TN][4];
    if constexpr (HAS_RES) {
#pragma unroll
      for (int j = 0; j < TN; j++)
#pragma unroll
        for (int q = 0; q < 4; q++)
          rr[j][q] = *reinterpret_cast<const h16x4*>(ew + (i * 32 + frow) * RS + (j * 32 + q * 8 + fhalf * 4) * 2);
    }
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        float v[4];
        if constexpr (TM * TN == 16) {
          // 256 accumulator registers sit in the AGPR half of the file; reading them here, one by one, keeps the
          // compiler from copying whole tiles into vector registers ahead of time (which spilled the residual)
#pragma unroll
          for (int e = 0; e < 4; e++) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v[e]) : "a"(acc[i][j][q * 4 + e]));
        } else {
#pragma unroll
          for (int e = 0; e < 4; e++) v[e] = acc[i][j][q * 4 + e];
        }
        if constexpr (HAS_BIAS) {
#pragma unroll
          for (int e = 0; e < 4; e++) v[e] += (float)bb[j][q][e];
        }
        if constexpr (EPI == KFKB_EPI_BIAS_RES) {
#pragma unroll
          for (int e = 0; e < 4; e++) v[e] += (float)rr[j][q][e];
        }
        if constexpr (EPI == KFKB_EPI_GELU_BWD) {
#pragma unroll
          for (int e = 0; e < 4; e++) v[e] *= gelu_grad_f((float)rr[j][q][e]);
        }
        h16x4 o;
#pragma unroll
        for (int e = 0; e < 4; e++) o[e] = (h16_t)v[e];
        *reinterpret_cast<h16x4*>(ew + (i * 32 + frow) * RS + (j * 32 + q * 8 + fhalf * 4) * 2) = o;
      }
  }
  wait_lgkm0();
#pragma unroll
  for (int r0 = 0; r0 < WR; r0 += RPI) {
    const int r = r0 + er, m = m0 + wm0 + r;
    const h16x8 v = *reinterpret_cast<const h16x8*>(ew + r * RS + ec * 16);
    if (m < M) {
      const size_t o = (size_t)m * N + n0 + wn0 + ec * 8;
      *reinterpret_cast<h16x8*>(C + o) = v;
      if constexpr (EPI == KFKB_EPI_BIAS_GELU) {
        h16x8 gl;
#pragma unroll
        for (int e = 0; e < 8; e++) gl[e] = (h16_t)gelu_f((float)v[e]);
        *reinterpret_cast<h16x8*>(C2 + o) = gl;
      }
    }
  }
}

// Cacc += acc for a whole tile (fp32, the gradient accumulators).  The accumulator layout would touch 32 rows with
// 32 bytes each per instruction; through LDS, 32 rows at a time, the wave reads and writes whole rows instead
// (1 KiB per instruction in 8 full cache lines).  The old values of two 32-row blocks are in flight at any time,
// the first two requested before the barrier that ends the main loop.  Sum order per element: old + acc, as in
// epilogue_quad.  Needs 4 * 32 * (BN * 2 + 16) bytes of LDS (less than the ring) and M, N multiples of the tile.
template <int BM, int BN>
__device__ __forceinline__ void epilogue_accum_staged(f32x16 (&acc)[BM / 64][BN / 64], char* smem, float* __restrict__ Cacc, int N,
                                                      int m0, int n0, int lane, int wave) {
  constexpr int TM = BM / 64, TN = BN / 64, WR = BM / 2, WC = BN / 2;
  static_assert(TM >= 2, "two 32-row blocks are requested ahead");
  constexpr int RS = WC * 4 + 16;                                 // row stride in bytes
  constexpr int LPR = WC / 4, RPI = 64 / LPR, NI = 32 / RPI;      // lanes per row, rows per instruction, instructions per block
  const int wm0 = (wave >> 1) * WR, wn0 = (wave & 1) * WC;
  const int frow = lane & 31, fhalf = lane >> 5;
  const int er = lane / LPR, ec = lane % LPR;
  float* cbase = Cacc + (size_t)(m0 + wm0 + er) * N + n0 + wn0 + ec * 4;
  float4 cin[2][NI];
  auto request = [&](int i, int slot) {
#pragma unroll
    for (int t = 0; t < NI; t++) cin[slot][t] = *reinterpret_cast<const float4*>(cbase + (size_t)(i * 32 + t * RPI) * N);
  };
  request(0, 0);
  request(1, 1);
  __syncthreads();                                                // every wave is done with the ring
  if constexpr (TM * TN == 16) mfma_results_settled();
  char* ew = smem + wave * (32 * RS);
#pragma unroll
  for (int i = 0; i < TM; i++) {
    __builtin_amdgcn_sched_barrier(0);                            // one 32-row block at a time
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        float v[4];
        if constexpr (TM * TN == 16) {                            // see epilogue_staged
#pragma unroll
          for (int e = 0; e < 4; e++) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v[e]) : "a"(acc[i][j][q * 4 + e]));
        } else {
#pragma unroll
          for (int e = 0; e < 4; e++) v[e] = acc[i][j][q * 4 + e];
        }
        *reinterpret_cast<float4*>(ew + frow * RS + (j * 32 + q * 8 + fhalf * 4) * 4) = make_float4(v[0], v[1], v[2], v[3]);
      }
    // a wave's LDS accesses execute in order: these reads see the block just written, the next block's writes
    // come after them
#pragma unroll
    for (int t = 0; t < NI; t++) {
      const float4 a = *reinterpret_cast<const float4*>(ew + (t * RPI + er) * RS + ec * 16);
      float4 c = cin[i & 1][t];
      c.x += a.x; c.y += a.y; c.z += a.z; c.w += a.w;
      *reinterpret_cast<float4*>(cbase + (size_t)(i * 32 + t * RPI) * N) = c;
    }
    if (i + 2 < TM) request(i + 2, i & 1);
  }
}

// The W step's tiles start from the gradient accumulator itself: acc <- Cacc tile, the matrix instructions add the
// products of every token on top in token order, the tile is stored once.  However many micro-batches one launch
// covers, every element sees the same sequence of fp32 additions (storing and re-loading an fp32 value changes
// nothing), so the gradients do not depend on how the W steps were batched.
// Both directions go through LDS, 32 rows at a time (the wave's own staging rows, whole rows per instruction).
// acc <- Cacc tile.  Every wave brings its own quadrant in, 32 rows at a time, with loads that write LDS directly
// (no staging registers: the accumulators alone fill half the register file), two 32-row blocks in flight, and reads
// each block back in accumulator layout.  A staged row is WC floats, its 16-byte pieces XOR-ed with (row & 15):
// an accumulator-layout read touches one piece column of 16 rows per clock, which then lie in 16 different banks.
template <int BM, int BN>
__device__ __forceinline__ void load_accum_dma(f32x16 (&acc)[BM / 64][BN / 64], char* smem, const float* __restrict__ Cacc, int N,
                                               int m0, int n0, int lane, int wave) {
  constexpr int TM = BM / 64, TN = BN / 64, WR = BM / 2, WC = BN / 2;
  constexpr int ROWB = WC * 4;                                    // bytes of a staged row
  constexpr int LPR = ROWB / 16, RPI = 64 / LPR, NI = 32 / RPI;   // lanes per row, rows per load instruction, instructions per block
  constexpr int BLKB = 32 * ROWB;                                 // bytes of a 32-row block
  static_assert((size_t)2 * 4 * BLKB <= (size_t)RING * (BM + BN) * CK_ * 2, "two blocks per wave fit the ring's LDS");
  static_assert(LPR >= 16, "the swizzle flips the low four bits of the piece index");
  const int wm0 = (wave >> 1) * WR, wn0 = (wave & 1) * WC;
  const int frow = lane & 31, fhalf = lane >> 5;
  const i32x4 rc = make_rsrc(Cacc + (size_t)(m0 + wm0) * N + n0 + wn0, (size_t)WR * N * 4);
  const unsigned lds_w = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem + wave * (2 * BLKB);
  int voff[NI];
#pragma unroll
  for (int g = 0; g < NI; g++) {
    const int row = g * RPI + lane / LPR, piece = (lane % LPR) ^ (row & 15);
    voff[g] = (row * N + piece * 4) * 4;
  }
  auto issue = [&](int blk, int slot) {
#pragma unroll
    for (int g = 0; g < NI; g++) dma16b(rc, voff[g], blk * 32 * N * 4, lds_w + slot * BLKB + g * 1024);
  };
  issue(0, 0);
  issue(1, 1);
#pragma unroll
  for (int i = 0; i < TM; i++) {
    if (i + 1 < TM) wait_vmcnt<NI>(); else wait_vmcnt<0>();       // loads retire in order: block i has landed
    asm volatile("" ::: "memory");
    const char* eb = smem + wave * (2 * BLKB) + (i & 1) * BLKB;
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const float4 v = *reinterpret_cast<const float4*>(eb + frow * ROWB + (((j * 8 + q * 2 + fhalf) ^ (frow & 15)) << 4));
        acc[i][j][q * 4 + 0] = v.x; acc[i][j][q * 4 + 1] = v.y; acc[i][j][q * 4 + 2] = v.z; acc[i][j][q * 4 + 3] = v.w;
      }
    wait_lgkm0();                                                 // read out before the slot is filled again
    asm volatile("" ::: "memory");
    if (i + 2 < TM) issue(i + 2, i & 1);
  }
  __syncthreads();                                                // the staging blocks become ring slots again
}

template <int BM, int BN>
__device__ __forceinline__ void store_accum_staged(f32x16 (&acc)[BM / 64][BN / 64], char* smem, float* __restrict__ Cacc, int N,
                                                   int m0, int n0, int lane, int wave) {
  constexpr int TM = BM / 64, TN = BN / 64, WR = BM / 2, WC = BN / 2;
  constexpr int RS = WC * 4 + 16;
  constexpr int LPR = WC / 4, RPI = 64 / LPR, NI = 32 / RPI;
  const int wm0 = (wave >> 1) * WR, wn0 = (wave & 1) * WC;
  const int frow = lane & 31, fhalf = lane >> 5;
  const int er = lane / LPR, ec = lane % LPR;
  float* cbase = Cacc + (size_t)(m0 + wm0 + er) * N + n0 + wn0 + ec * 4;
  __syncthreads();                                                // every wave is done with the ring
  if constexpr (TM * TN == 16) mfma_results_settled();
  char* ew = smem + wave * (32 * RS);
#pragma unroll
  for (int i = 0; i < TM; i++) {
    __builtin_amdgcn_sched_barrier(0);                            // one 32-row block at a time
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        float v[4];
        if constexpr (TM * TN == 16) {                            // see epilogue_staged
#pragma unroll
          for (int e = 0; e < 4; e++) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v[e]) : "a"(acc[i][j][q * 4 + e]));
        } else {
#pragma unroll
          for (int e = 0; e < 4; e++) v[e] = acc[i][j][q * 4 + e];
        }
        *reinterpret_cast<float4*>(ew + frow * RS + (j * 32 + q * 8 + fhalf * 4) * 4) = make_float4(v[0], v[1], v[2], v[3]);
      }
#pragma unroll
    for (int t = 0; t < NI; t++) {
      const float4 a = *reinterpret_cast<const float4*>(ew + (t * RPI + er) * RS + ec * 16);
      *reinterpret_cast<float4*>(cbase + (size_t)(i * 32 + t * RPI) * N) = a;
    }
  }
}

template <int BM, int BN, int EPI, bool BT>
__global__ void __launch_bounds__(256) gemm_h16_nt_kernel(int M, int N, int K, const h16_t* __restrict__ A, const h16_t* __restrict__ B,
                                                 const h16_t* __restrict__ bias, const h16_t* __restrict__ residual,
                                                 h16_t* __restrict__ C, h16_t* __restrict__ C2, float* __restrict__ Cacc,
                                                 int tiles_m, int tiles_n) {
  constexpr int TM = BM / 64, TN = BN / 64;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int tm, tn; bool valid;
  tile_of_block(tiles_m, tiles_n, tm, tn, valid);
  if (!valid) return;
  const int m0 = tm * BM, n0 = tn * BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  typename std::conditional<BT, NtLayout64<BM, BN>, NtLayout32<BM, BN, false>>::type lay;
  lay.init(smem, A, B, M, N, K, m0, n0, lane, wave);
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;
  main_loop<TM, TN>(lay, acc, K / CK_);
  if constexpr (EPI == KFKB_EPI_ACCUM) {
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2), frow = lane & 31, fhalf = lane >> 5;
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
  } else {
    epilogue_staged<BM, BN, EPI>(acc, smem, M, N, m0, n0, lane, wave, bias, residual, C, C2);
  }
}

// C[M,N] (+)= A[K,M]^T . B[K,N]; EPI NONE (bf16 C) or ACCUM (fp32 Cacc +=)
template <int BM, int BN, int EPI>
__device__ __forceinline__ void tn_tile(int M, int N, int K, const h16_t* __restrict__ A, const h16_t* __restrict__ B,
                                        h16_t* __restrict__ C, float* __restrict__ Cacc, int tm, int tn, char* smem) {
  constexpr int TM = BM / 64, TN = BN / 64;
  const int m0 = tm * BM, n0 = tn * BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  TnLayout<BM, BN> lay;
  lay.init(smem, A, B, M, N, K, m0, n0, lane, wave);
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;
  main_loop<TM, TN>(lay, acc, K / CK_);
  if constexpr (EPI == KFKB_EPI_ACCUM) {
    epilogue_accum_staged<BM, BN>(acc, smem, Cacc, N, m0, n0, lane, wave);
  } else {
    epilogue_staged<BM, BN, KFKB_EPI_NONE>(acc, smem, M, N, m0, n0, lane, wave, nullptr, nullptr, C, nullptr);
  }
}


template <int BM, int BN, int EPI>
__global__ void __launch_bounds__(256) gemm_h16_tn_kernel(int M, int N, int K, const h16_t* __restrict__ A,
                                                           const h16_t* __restrict__ B, h16_t* __restrict__ C,
                                                           float* __restrict__ Cacc, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int tm, tn; bool valid;
  tile_of_block(tiles_m, tiles_n, tm, tn, valid);
  if (!valid) return;
  tn_tile<BM, BN, EPI>(M, N, K, A, B, C, Cacc, tm, tn, smem);
}

// Several weight-gradient products that share the reduction length K (the token axis) in one launch:
// a backward pass of one block has four of them, each too small to fill the chip on its own.
// Every product covers `nseg` segments of the token axis (one per micro-batch of the W step's window), each with
// operands of its own: Cacc[M,N] += sum_s A_s[K,M]^T . B_s[K,N], K tokens per segment.
struct TnProblem { int M, N, tiles_m, tiles_n, first_tile; float* Cacc; const h16_t* A[kWSeg]; const h16_t* B[kWSeg]; };
struct TnGroup { int count, K, total_tiles, nseg; TnProblem p[4]; };

// The small reductions of the same step, done by extra workgroups of the same launch, on the CUs the tiles leave
// idle (192 tiles of 256 x 256 on 256 CUs for a GPT-2-medium block), instead of by launches of their own:
//   column sums over the token axis of up to four bf16 matrices dy[rows, width] (the bias gradients), and
//   the finishing pass of up to two LayerNorm-parameter reductions: sums over the partial rows
//   partial[parts][2][width] (fp32) that the LayerNorm backward kernels left behind.
// Work items are strips of 64 columns, dealt round-robin to the reduce workgroups; one workgroup owns a strip from
// the first row to the last and adds in a fixed order, so the sums do not depend on timing or on the launch shape.
struct RedColsum { const h16_t* dy[kWSeg]; float* out; int width, first_item; };
struct RedLnFinal { const float* partial[kWSeg]; float* out0; float* out1; int parts, width, first_item; };
struct ReduceGroup { int n_colsum, n_ln, rows, total_items, nseg; RedColsum c[4]; RedLnFinal ln[2]; };

__device__ __forceinline__ void reduce_colsum_strip(const h16_t* dy, float* out, int width, int strip, int rows, float* red) {
  const int cl = threadIdx.x & 7, rl = threadIdx.x >> 3;              // 8 lanes x 16 bytes = one 128-byte row piece
  const h16_t* src = dy + strip * 64 + cl * 8;
  const size_t w = width;
  float a[8];
#pragma unroll
  for (int e = 0; e < 8; e++) a[e] = 0.f;
  int r = rl;
  for (; r + 32 * 15 < rows; r += 32 * 16) {                          // sixteen loads in flight per lane
    h16x8 v[16];
#pragma unroll
    for (int u = 0; u < 16; u++) v[u] = *reinterpret_cast<const h16x8*>(src + (size_t)(r + 32 * u) * w);
#pragma unroll
    for (int u = 0; u < 16; u++)
#pragma unroll
      for (int e = 0; e < 8; e++) a[e] += (float)v[u][e];
  }
  for (; r < rows; r += 32) {
    const h16x8 v = *reinterpret_cast<const h16x8*>(src + (size_t)r * w);
#pragma unroll
    for (int e = 0; e < 8; e++) a[e] += (float)v[e];
  }
#pragma unroll
  for (int e = 0; e < 8; e++) red[rl * 65 + cl * 8 + e] = a[e];
  __syncthreads();
  if (threadIdx.x < 64) {
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 32; j++) t += red[j * 65 + threadIdx.x];
    out[strip * 64 + threadIdx.x] += t;
  }
  __syncthreads();
}

__device__ __forceinline__ void reduce_ln_strip(const float* partial, float* out0, float* out1, int parts, int width, int strip, float* red) {
  const int c4 = threadIdx.x & 15, pl = threadIdx.x >> 4;             // 16 lanes x float4 = 64 columns, 16 part lanes
  const size_t w = width;
  const float* src = partial + strip * 64 + c4 * 4;
  float4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
  int p = pl;
  for (; p + 16 * 3 < parts; p += 16 * 4) {
    float4 v0[4], v1[4];
#pragma unroll
    for (int u = 0; u < 4; u++) {
      v0[u] = *reinterpret_cast<const float4*>(src + (size_t)(p + 16 * u) * 2 * w);
      v1[u] = *reinterpret_cast<const float4*>(src + (size_t)(p + 16 * u) * 2 * w + w);
    }
#pragma unroll
    for (int u = 0; u < 4; u++) {
      s0.x += v0[u].x; s0.y += v0[u].y; s0.z += v0[u].z; s0.w += v0[u].w;
      s1.x += v1[u].x; s1.y += v1[u].y; s1.z += v1[u].z; s1.w += v1[u].w;
    }
  }
  for (; p < parts; p += 16) {
    const float4 v0 = *reinterpret_cast<const float4*>(src + (size_t)p * 2 * w);
    const float4 v1 = *reinterpret_cast<const float4*>(src + (size_t)p * 2 * w + w);
    s0.x += v0.x; s0.y += v0.y; s0.z += v0.z; s0.w += v0.w;
    s1.x += v1.x; s1.y += v1.y; s1.z += v1.z; s1.w += v1.w;
  }
  float* r0 = red + pl * 65 + c4 * 4;
  float* r1 = red + 16 * 65 + pl * 65 + c4 * 4;
  r0[0] = s0.x; r0[1] = s0.y; r0[2] = s0.z; r0[3] = s0.w;
  r1[0] = s1.x; r1[1] = s1.y; r1[2] = s1.z; r1[3] = s1.w;
  __syncthreads();
  if (threadIdx.x < 128) {
    const int half = threadIdx.x >> 6, c = threadIdx.x & 63;
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 16; j++) t += red[half * 16 * 65 + j * 65 + c];
    float* out = half ? out1 : out0;
    out[strip * 64 + c] += t;
  }
  __syncthreads();
}

// The kernel's by-value arguments, read in place: indexing a copy of them with a run-time index (problem, segment)
// would put the copy into scratch memory; through the kernel-argument segment they are scalar loads.
typedef const __attribute__((address_space(4))) TnGroup* tn_group_args;
typedef const __attribute__((address_space(4))) ReduceGroup* reduce_group_args;

__device__ __forceinline__ void reduce_role(reduce_group_args rg, int rb, int nrb, char* smem) {
  float* red = reinterpret_cast<float*>(smem);                        // 32 x 65 floats
  const int total = rg->total_items, nseg = rg->nseg, rows = rg->rows, n_colsum = rg->n_colsum, n_ln = rg->n_ln;
  for (int item = rb; item < total; item += nrb) {
    // items are numbered LayerNorm strips first, then column-sum strips
    int kind = 0, q = 0;                                              // 0: LayerNorm finishing pass q, 1: column sum q
    for (int c = n_colsum - 1; c >= 0 && kind == 0; c--)
      if (item >= rg->c[c].first_item) { kind = 1; q = c; }
    if (kind == 0)
      for (int c = n_ln - 1; c >= 0; c--)
        if (item >= rg->ln[c].first_item) { q = c; break; }
    // a strip's segments (micro-batches) are summed one after the other and added in that order: the bits of one
    // launch per micro-batch
    if (kind == 1) {
      float* out = rg->c[q].out; const int width = rg->c[q].width, strip = item - rg->c[q].first_item;
      for (int seg = 0; seg < nseg; seg++) reduce_colsum_strip(rg->c[q].dy[seg], out, width, strip, rows, red);
    } else {
      float* out0 = rg->ln[q].out0; float* out1 = rg->ln[q].out1;
      const int parts = rg->ln[q].parts, width = rg->ln[q].width, strip = item - rg->ln[q].first_item;
      for (int seg = 0; seg < nseg; seg++) reduce_ln_strip(rg->ln[q].partial[seg], out0, out1, parts, width, strip, red);
    }
  }
}

// TnLayout for a token axis made of several segments (micro-batches) with operands of their own: the ring runs on
// across segment boundaries.  Two cursors, one per operand, name the chunk the next load instructions fetch
// (segment, chunk inside it); a cursor steps once per chunk, after the chunk's last instruction, and takes the next
// segment's base pointer from the kernel arguments when it crosses a boundary.  Past the end it stays on the last
// chunk (those loads land in slots nobody reads any more).
template <int BM, int BN>
struct TnLayoutSeg : TnLayout<BM, BN> {
  using Base = TnLayout<BM, BN>;
  using Base::TM; using Base::TN;
  tn_group_args grp; int prob, nseg, nks, M_, N_, K_;
  int seg_a, ka, seg_b, kb;
  __device__ __forceinline__ void init_seg(char* smem, tn_group_args g_, int prob_, int M, int N, int K, int nseg_, int m0, int n0, int lane, int wave_) {
    grp = g_; prob = prob_; nseg = nseg_; nks = K / CK_; M_ = M; N_ = N; K_ = K;
    Base::init(smem, grp->p[prob].A[0], grp->p[prob].B[0], M, N, K, m0, n0, lane, wave_);
    seg_a = ka = seg_b = kb = 0;
  }
  __device__ __forceinline__ void step_a() {
    if (ka + 1 < nks) { ka++; return; }
    if (seg_a + 1 < nseg) { seg_a++; ka = 0; this->ra = make_rsrc(grp->p[prob].A[seg_a], (size_t)K_ * M_ * 2); }
  }
  __device__ __forceinline__ void step_b() {
    if (kb + 1 < nks) { kb++; return; }
    if (seg_b + 1 < nseg) { seg_b++; kb = 0; this->rb = make_rsrc(grp->p[prob].B[seg_b], (size_t)K_ * N_ * 2); }
  }
  __device__ __forceinline__ void dma_a(int i, int slot) { dma16b(this->ra, this->voa[i], ka * this->sa, this->lds0 + (slot * Base::A_SLOT + (i * 4 + this->wave) * 512) * 2); }
  __device__ __forceinline__ void dma_b(int i, int slot) { dma16b(this->rb, this->vob[i], kb * this->sb, this->lds0 + (RING * Base::A_SLOT + slot * Base::B_SLOT + (i * 4 + this->wave) * 512) * 2); }
  __device__ __forceinline__ void prologue() {
#pragma unroll
    for (int c = 0; c < RING; c++) {
#pragma unroll
      for (int i = 0; i < TN; i++) dma_a(i, c);
      step_a();
      if (c < RING - 1) {
#pragma unroll
        for (int i = 0; i < TN; i++) dma_b(i, c);
        step_b();
      }
    }
  }
  __device__ __forceinline__ void dma0(int j, int kc, int pc) { dma_b(j, (pc + 3) & 3); if (j == TN - 1) step_b(); }
  __device__ __forceinline__ void dma1(int j, int kc, int pc) { dma_a(j, pc); if (j == TN - 1) step_a(); }
};

template <int BM, int BN>
__global__ void __launch_bounds__(256) gemm_h16_tn_grouped_kernel(TnGroup grp_arg, ReduceGroup rg_arg, int reduce_blocks) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  static_assert(sizeof(TnGroup) % 8 == 0 && alignof(ReduceGroup) == 8, "the second argument follows the first without padding");
  const __attribute__((address_space(4))) char* kargs = (const __attribute__((address_space(4))) char*)__builtin_amdgcn_kernarg_segment_ptr();
  tn_group_args grp = (tn_group_args)kargs;
  reduce_group_args rg = (reduce_group_args)(kargs + sizeof(TnGroup));
  // The first blocks of the grid (a multiple of 8, so the tiles keep their XCDs) reduce: they are on their CUs from
  // the start and finish in the shadow of the tiles, also when the tiles need several rounds.
  if ((int)blockIdx.x < reduce_blocks) {
    reduce_role(rg, blockIdx.x, reduce_blocks, smem);
    return;
  }
  const int total_tiles = grp->total_tiles, count = grp->count, K = grp->K, nseg = grp->nseg;
  const int t = linear_of_block(total_tiles, blockIdx.x - reduce_blocks);
  if (t >= total_tiles) return;
  int i = 0;
  for (int q = 1; q < count; q++) if (t >= grp->p[q].first_tile) i = q;
  const int M = grp->p[i].M, N = grp->p[i].N;
  float* Cacc = grp->p[i].Cacc;
  int tm, tn;
  tile_from_linear(t - grp->p[i].first_tile, grp->p[i].tiles_m, grp->p[i].tiles_n, tm, tn);
  constexpr int TM = BM / 64, TN = BN / 64;
  const int m0 = tm * BM, n0 = tn * BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  f32x16 acc[TM][TN];
  load_accum_dma<BM, BN>(acc, smem, Cacc, N, m0, n0, lane, wave);
  TnLayoutSeg<BM, BN> lay;
  lay.init_seg(smem, grp, i, M, N, K, nseg, m0, n0, lane, wave);
  main_loop<TM, TN>(lay, acc, nseg * (K / CK_));                  // one token axis, segment after segment
  store_accum_staged<BM, BN>(acc, smem, Cacc, N, m0, n0, lane, wave);
  (void)grp_arg; (void)rg_arg;
}

// ------------------------------------------------------------------------------------------------
// TN kernel, register-staged variant: accepts a ragged reduction length K (zero-fills the tail).
// Tiles are stored [reduction row][BM + 32].
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ h16x8 lds_tr_frag(const h16_t* p, int row_stride) {
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * row_stride));
  union { struct { s16x4 a, b; } s; h16x8 v; } u;
  u.s.a = lo; u.s.b = hi;
  return u.v;
}

template <int BM, int BN, int EPI>
__global__ void __launch_bounds__(256) gemm_h16_tn_staged_kernel(int M, int N, int K, const h16_t* __restrict__ A,
                                                           const h16_t* __restrict__ B, h16_t* __restrict__ C,
                                                           float* __restrict__ Cacc, int tiles_m, int tiles_n) {
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int SA = BM + 32, SB = BN + 32;          // LDS row strides (elements): +64 bytes per row
  constexpr int CA = BM / 8, CB = BN / 8;            // 16-byte chunks per tile row
  constexpr int LA = BM / 32, LB = BN / 32;          // chunks per thread per slice
  extern __shared__ __attribute__((aligned(16))) char smem[];
  h16_t* As = reinterpret_cast<h16_t*>(smem);                       // [2][64][SA]
  h16_t* Bs = As + 2 * BK * SA;                                      // [2][64][SB]

  int tm, tn; bool valid;
  tile_of_block(tiles_m, tiles_n, tm, tn, valid);
  if (!valid) return;
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);

  h16x8 ra[LA], rb[LB];
  auto load_global = [&](int kt) {
#pragma unroll
    for (int i = 0; i < LA; i++) {
      const int c = tid % CA, r = tid / CA + (256 / CA) * i;
      const int k = kt * BK + r;
      h16x8 z;
#pragma unroll
      for (int e = 0; e < 8; e++) z[e] = (h16_t)0.f;
      ra[i] = (k < K) ? *reinterpret_cast<const h16x8*>(A + (size_t)k * M + m0 + c * 8) : z;
    }
#pragma unroll
    for (int i = 0; i < LB; i++) {
      const int c = tid % CB, r = tid / CB + (256 / CB) * i;
      const int k = kt * BK + r;
      h16x8 z;
#pragma unroll
      for (int e = 0; e < 8; e++) z[e] = (h16_t)0.f;
      rb[i] = (k < K) ? *reinterpret_cast<const h16x8*>(B + (size_t)k * N + n0 + c * 8) : z;
    }
  };
  auto store_lds = [&](int st) {
#pragma unroll
    for (int i = 0; i < LA; i++) {
      const int c = tid % CA, r = tid / CA + (256 / CA) * i;
      *reinterpret_cast<h16x8*>(As + (st * BK + r) * SA + c * 8) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < LB; i++) {
      const int c = tid % CB, r = tid / CB + (256 / CB) * i;
      *reinterpret_cast<h16x8*>(Bs + (st * BK + r) * SB + c * 8) = rb[i];
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
      h16x8 fa[TM], fb[TN];
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
          acc[i][j] = KFKB_MFMA_H16(fb[j], fa[i], acc[i][j]);
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
const char* gemm_h16_check(const GemmArgs& g) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return "16-bit GEMM: empty shape";
  if (g.kind == KFKB_GEMM_NT) {
    if (g.N % 128 != 0) return "16-bit NT GEMM needs N % 128 == 0";
    if (g.K % 32 != 0) return "16-bit NT GEMM needs K % 32 == 0";
    if (g.b_tiled && g.K % 64 != 0) return "16-bit NT GEMM with a chunk-major B needs K % 64 == 0";
  } else if (g.kind == KFKB_GEMM_TN) {
    if (g.M % 128 != 0 || g.N % 128 != 0) return "16-bit TN GEMM needs M % 128 == 0 and N % 128 == 0";
    if (g.epilogue != KFKB_EPI_ACCUM && g.epilogue != KFKB_EPI_NONE) return "16-bit TN GEMM supports epilogues NONE and ACCUM";
  } else {
    return "16-bit GEMM supports the NT and TN forms";
  }
  // the kernels address their operands with 32-bit byte offsets
  if ((double)g.M * g.K * 2 >= 4294967296.0 || (double)g.N * g.K * 2 >= 4294967296.0) return "16-bit GEMM: an operand of 4 GiB or more";
  return nullptr;
}

template <int BM, int BN> constexpr size_t tile_lds_bytes() {
  return std::max((size_t)RING * (BM + BN) * CK_ * sizeof(h16_t), epilogue_lds_bytes<BM, BN>());
}
template <int BM, int BN> constexpr size_t tile64_lds_bytes() { return std::max(NtLayout64<BM, BN>::LDS_BYTES, epilogue_lds_bytes<BM, BN>()); }

template <int BM, int BN, int EPI, bool BT>
static hipError_t launch_nt_bt(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = g.N / BN;
  const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
  constexpr size_t smem = BT ? tile64_lds_bytes<BM, BN>() : tile_lds_bytes<BM, BN>();
  auto kern = gemm_h16_nt_kernel<BM, BN, EPI, BT>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  klaunch(kern, dim3(grid), dim3(256), smem, s, PK_GEMM_NT + (BM != BN ? 400 : BM == 256 ? 100 : 0) + EPI, 2.0 * g.M * g.N * g.K, g.M, g.N, g.K,
          (const h16_t*)g.A, (const h16_t*)g.B, (const h16_t*)g.bias, (const h16_t*)g.residual, (h16_t*)g.C,
          (h16_t*)g.C2, g.Cacc, tiles_m, tiles_n);
  return hipGetLastError();
}
template <int BM, int BN, int EPI>
static hipError_t launch_nt(const GemmArgs& g, hipStream_t s) {
  return g.b_tiled ? launch_nt_bt<BM, BN, EPI, true>(g, s) : launch_nt_bt<BM, BN, EPI, false>(g, s);
}

template <int BM, int BN, int EPI>
static hipError_t launch_tn_staged(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = g.M / BM, tiles_n = g.N / BN;
  const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
  const size_t smem = (size_t)2 * BK * (BM + 32 + BN + 32) * sizeof(h16_t);
  auto kern = gemm_h16_tn_staged_kernel<BM, BN, EPI>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  klaunch(kern, dim3(grid), dim3(256), smem, s, PK_GEMM_TN + 200 + (BM == 256 ? 100 : 0) + EPI, 2.0 * g.M * g.N * g.K, g.M, g.N, g.K,
          (const h16_t*)g.A, (const h16_t*)g.B, (h16_t*)g.C, g.Cacc, tiles_m, tiles_n);
  return hipGetLastError();
}

template <int BM, int BN, int EPI>
static hipError_t launch_tn(const GemmArgs& g, hipStream_t s) {
  if (g.K % CK_ != 0) return launch_tn_staged<BM, BN, EPI>(g, s);
  const int tiles_m = g.M / BM, tiles_n = g.N / BN;
  const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
  constexpr size_t smem = tile_lds_bytes<BM, BN>();
  auto kern = gemm_h16_tn_kernel<BM, BN, EPI>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  klaunch(kern, dim3(grid), dim3(256), smem, s, PK_GEMM_TN + (BM == 256 ? 100 : 0) + EPI, 2.0 * g.M * g.N * g.K, g.M, g.N, g.K,
          (const h16_t*)g.A, (const h16_t*)g.B, (h16_t*)g.C, g.Cacc, tiles_m, tiles_n);
  return hipGetLastError();
}

template <int BM, int BN>
static hipError_t launch_group(const TnGroup& grp, const ReduceGroup& rg, double flops, hipStream_t s) {
  const int gemm_blocks = ((grp.total_tiles + 7) / 8) * 8;
  int reduce_blocks = 0;
  if (rg.total_items > 0) {
    // as many as the tiles leave CU slots idle in their last round; where that is few (the tiles fill their rounds)
    // 128 of them take the first round's slots for a while instead
    constexpr size_t lds_cu = 160 * 1024;
    const int slots = 256 * (int)(lds_cu / tile_lds_bytes<BM, BN>());
    const int idle = (slots - gemm_blocks % slots) % slots;
    reduce_blocks = (idle >= 48 ? std::min(idle, 128) : 128) / 8 * 8;
    reduce_blocks = std::min(reduce_blocks, (rg.total_items + 7) / 8 * 8);
  }
  constexpr size_t smem = tile_lds_bytes<BM, BN>();
  auto kern = gemm_h16_tn_grouped_kernel<BM, BN>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  klaunch(kern, dim3(gemm_blocks + reduce_blocks), dim3(256), smem, s, PK_GEMM_TN + (BM == 256 ? 301 : 300), flops, grp, rg, reduce_blocks);
  return hipGetLastError();
}

// fewest 256 x 256 tiles a launch must have before they are preferred over 128 x 128 tiles
static long big_tile_min() { return g_big_tile_min; }

// Can these weight gradients (and, if given, the reductions of the same W step) go into one grouped launch?
bool wstep_groupable_h16(const WGrad* g, int n, int K, const WStepReduce* red) {
  if (n <= 0 || n > 4 || K <= 0 || K % CK_ != 0) return false;
  for (int i = 0; i < n; i++) {
    if (g[i].M <= 0 || g[i].N <= 0 || g[i].M % 128 != 0 || g[i].N % 128 != 0) return false;
    // the kernels address their operands with 32-bit byte offsets
    if ((double)g[i].M * K * 2 >= 4294967296.0 || (double)g[i].N * K * 2 >= 4294967296.0) return false;
  }
  if (red != nullptr) {
    if (red->rows != K || red->n_colsum > 4 || red->n_ln > 2) return false;
    for (int i = 0; i < red->n_colsum; i++) if (red->width[i] <= 0 || red->width[i] % 64 != 0) return false;
    for (int i = 0; i < red->n_ln; i++) if (red->ln_width[i] <= 0 || red->ln_width[i] % 64 != 0 || red->ln_parts[i] <= 0) return false;
  }
  return true;
}

hipError_t launch_wstep_h16(const WGrad* g, int n, int K, int nseg, hipStream_t s, const WStepReduce* red) {
  if (nseg < 1 || nseg > kWSeg || !wstep_groupable_h16(g, n, K, red)) return hipErrorInvalidValue;
  // 256 x 256 tiles when every problem divides into them and the group still gives most CUs a tile
  long big_tiles = 0;
  bool big = true;
  for (int i = 0; i < n; i++) {
    big = big && g[i].M % 256 == 0 && g[i].N % 256 == 0;
    big_tiles += (long)(g[i].M / 256) * (g[i].N / 256);
  }
  big = big && big_tiles >= big_tile_min();
  const int BT = big ? 256 : 128;
  TnGroup grp{};
  grp.count = n; grp.K = K; grp.nseg = nseg;
  double flops = 0;
  for (int i = 0; i < n; i++) {
    TnProblem& p = grp.p[i];
    p.M = g[i].M; p.N = g[i].N; p.tiles_m = g[i].M / BT; p.tiles_n = g[i].N / BT; p.first_tile = grp.total_tiles;
    p.Cacc = g[i].Cacc;
    for (int sg = 0; sg < nseg; sg++) { p.A[sg] = (const h16_t*)g[i].A[sg]; p.B[sg] = (const h16_t*)g[i].B[sg]; }
    grp.total_tiles += p.tiles_m * p.tiles_n;
    flops += 2.0 * g[i].M * g[i].N * K * nseg;
  }
  // the reductions ride along (strips of 64 columns)
  ReduceGroup rg{};
  if (red != nullptr) {
    rg.n_colsum = red->n_colsum; rg.n_ln = red->n_ln; rg.rows = red->rows; rg.nseg = nseg;
    for (int i = 0; i < red->n_ln; i++) {
      rg.ln[i] = RedLnFinal{{}, red->ln_out0[i], red->ln_out1[i], red->ln_parts[i], red->ln_width[i], rg.total_items};
      for (int sg = 0; sg < nseg; sg++) rg.ln[i].partial[sg] = red->ln_partial[i][sg];
      rg.total_items += red->ln_width[i] / 64;
    }
    for (int i = 0; i < red->n_colsum; i++) {
      rg.c[i] = RedColsum{{}, red->out[i], red->width[i], rg.total_items};
      for (int sg = 0; sg < nseg; sg++) rg.c[i].dy[sg] = (const h16_t*)red->dy[i][sg];
      rg.total_items += red->width[i] / 64;
    }
  }
  if (big) return launch_group<256, 256>(grp, rg, flops, s);
  return launch_group<128, 128>(grp, rg, flops, s);
}

// Large tiles when they still give most CUs a tile; small tiles otherwise.
static bool use_big_tiles(int M, int N, bool m_must_divide) {
  if (N % 256 != 0) return false;
  if (m_must_divide && M % 256 != 0) return false;
  const long tiles = (long)((M + 255) / 256) * (N / 256);
  return tiles >= big_tile_min();
}

// Tile shape of an NT product.  256 x 256 tiles where they give most CUs a tile (use_big_tiles).  Otherwise, for a
// chunk-major B, 128 x 256 tiles where they use the CUs better than 128 x 128 tiles would: a shape is rated by the
// share of CU slots its tiles fill over whole rounds of 256, times what a tile of that shape reaches of a
// 256 x 256 tile's rate (g_mid_tile_rate / 100 for 128 x 256, 0.84 for 128 x 128; measured 1430 - 1480, 1300 - 1330 and
// 1210 - 1260 TFLOP/s on products that fill their rounds: 1, 0.9, 0.84).
static double round_fill(long tiles) { return (double)tiles / (double)(((tiles + 255) / 256) * 256); }
static int nt_tile_shape(const GemmArgs& g) {                     // 2: 256 x 256, 1: 128 x 256, 0: 128 x 128
  const bool mid_ok = g.b_tiled && g.N % 256 == 0 && g.K % 64 == 0 && g_mid_tile_mode != 0;
  if (mid_ok && g_mid_tile_mode == 2) return 1;
  const bool big_ok = use_big_tiles(g.M, g.N, false);
  if (!mid_ok) return big_ok ? 2 : 0;
  const long tm = (g.M + 127) / 128;
  const double big = round_fill((long)((g.M + 255) / 256) * (g.N / 256));
  const double mid = round_fill(tm * (g.N / 256)) * g_mid_tile_rate / 100.0;
  const double small = round_fill(tm * (g.N / 128)) * 0.84;
  if (big_ok) return big >= mid ? 2 : 1;       // 128 x 128 tiles only where 256 x 256 would leave a quarter of the CUs idle
  return mid > small ? 1 : 0;
}

template <int EPI>
static hipError_t launch_nt_epi(const GemmArgs& g, hipStream_t s) {
  const int shape = nt_tile_shape(g);
  if (shape == 2) return launch_nt<256, 256, EPI>(g, s);
  if (shape == 1) return launch_nt_bt<128, 256, EPI, true>(g, s);
  return launch_nt<128, 128, EPI>(g, s);
}

hipError_t launch_gemm_h16(const GemmArgs& g, hipStream_t s) {
  if (gemm_h16_check(g) != nullptr) return hipErrorInvalidValue;
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

#ifdef KFKB_H16_IS_F16
}  // namespace f16k
hipError_t launch_gemm_f16(const GemmArgs& g, hipStream_t s) { return f16k::launch_gemm_h16(g, s); }
hipError_t launch_wstep_f16(const WGrad* g, int n, int K, int nseg, hipStream_t s, const WStepReduce* red) {
  return f16k::launch_wstep_h16(g, n, K, nseg, s, red);
}
#else
}  // namespace bf16k
hipError_t launch_gemm_bf16(const GemmArgs& g, hipStream_t s) { return bf16k::launch_gemm_h16(g, s); }
hipError_t launch_wstep_bf16(const WGrad* g, int n, int K, int nseg, hipStream_t s, const WStepReduce* red) {
  return bf16k::launch_wstep_h16(g, n, K, nseg, s, red);
}
bool wstep_groupable(const WGrad* g, int n, int K, const WStepReduce* red) { return bf16k::wstep_groupable_h16(g, n, K, red); }
const char* gemm_bf16_check(const GemmArgs& g) { return bf16k::gemm_h16_check(g); }
#endif

}  // namespace kfkb
