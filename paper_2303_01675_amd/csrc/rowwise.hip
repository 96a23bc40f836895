// Bandwidth-bound kernels of the stage: LayerNorm forward / backward, GELU backward, column sums
// (bias and LayerNorm parameter gradients), fills, transposes and the transfer-delay kernel.
// All statistics and sums are fp32; storage type T is float or bf16.  wave64 throughout.
#include "common.h"
#include <algorithm>

namespace kfkb {

// ------------------------------------------------------------------------------------------------
// LayerNorm forward.  A row is shared by WPR waves of a 256-thread block (1, 2 or 4; the block holds 4 / WPR rows)
// and lives in registers between the passes: lane l of the row's wave w owns the 8-element chunks
// (i * WPR + w) * 64 + l, i < NCH  (H % 8 == 0, H <= 512 * NCH * WPR).  Wide rows are split over waves so that a
// lane holds a few chunks only: many waves fit a CU and enough loads are in flight to keep HBM busy; the waves of
// a row meet in LDS, partial sums added in wave order.
// ------------------------------------------------------------------------------------------------
template <int WPR>
__device__ __forceinline__ float row_sum(float v, float* red, int wave, int lane) {
  v = wave_sum(v);
  if constexpr (WPR == 1) return v;
  if (lane == 0) red[wave] = v;
  __syncthreads();
  const int w0 = wave / WPR * WPR;
  float t = red[w0];
#pragma unroll
  for (int j = 1; j < WPR; j++) t += red[w0 + j];
  return t;
}

template <typename T, int NCH, int WPR>
__global__ void __launch_bounds__(256) ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                     const T* __restrict__ beta, T* __restrict__ y,
                                                     float* __restrict__ mean, float* __restrict__ rstd,
                                                     int rows, int H, float eps) {
  __shared__ float red[2][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = min(blockIdx.x * (4 / WPR) + wave / WPR, rows - 1);      // waves past the end redo the last row
  const bool owner = blockIdx.x * (4 / WPR) + wave / WPR < rows;
  if (WPR == 1 && !owner) return;
  const int wr = wave % WPR;
  const int nchunks = H >> 3;
  const T* xr = x + (size_t)row * H;
  float v[NCH][8];
  Raw8<T> graw[NCH], braw[NCH];                               // requested with the row: they arrive under the two reductions
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; i++) {
    const int c = (i * WPR + wr) * 64 + lane;
    if (c < nchunks) {
      Vec8<T>::load(xr + c * 8, v[i]);
      graw[i] = Vec8<T>::load_raw(gamma + c * 8);
      braw[i] = Vec8<T>::load_raw(beta + c * 8);
#pragma unroll
      for (int e = 0; e < 8; e++) s += v[i][e];
    }
  }
  const float mu = row_sum<WPR>(s, red[0], wave, lane) / (float)H;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; i++) {
    const int c = (i * WPR + wr) * 64 + lane;
    if (c < nchunks) {
#pragma unroll
      for (int e = 0; e < 8; e++) { const float d = v[i][e] - mu; q += d * d; }
    }
  }
  const float rs = 1.0f / sqrtf(row_sum<WPR>(q, red[1], wave, lane) / (float)H + eps);
  if (!owner) return;
  if (lane == 0 && wr == 0) { mean[row] = mu; rstd[row] = rs; }
  T* yr = y + (size_t)row * H;
#pragma unroll
  for (int i = 0; i < NCH; i++) {
    const int c = (i * WPR + wr) * 64 + lane;
    if (c < nchunks) {
      float g[8], b[8], o[8];
      Vec8<T>::unpack(graw[i], g);
      Vec8<T>::unpack(braw[i], b);
#pragma unroll
      for (int e = 0; e < 8; e++) o[e] = (v[i][e] - mu) * rs * g[e] + b[e];
      Vec8<T>::store(yr + c * 8, o);
    }
  }
}

// LayerNorm backward, input gradient:  g = dy*gamma;  dx = rstd (g - mean(g) - xhat mean(g xhat)) [+ dres]
// Rows are shared by WPR waves as in the forward kernel.
template <typename T, int NCH, int WPR>
__global__ void __launch_bounds__(256) ln_bwd_dx_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                        const float* __restrict__ mean, const float* __restrict__ rstd,
                                                        const T* __restrict__ gamma, const T* __restrict__ dres,
                                                        T* __restrict__ dx, int rows, int H) {
  __shared__ float red[2][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = min(blockIdx.x * (4 / WPR) + wave / WPR, rows - 1);
  const bool owner = blockIdx.x * (4 / WPR) + wave / WPR < rows;
  if (WPR == 1 && !owner) return;
  const int wr = wave % WPR;
  const int nchunks = H >> 3;
  const float mu = mean[row], rs = rstd[row];
  const T* xr = x + (size_t)row * H;
  const T* dyr = dy + (size_t)row * H;
  const T* rr = dres != nullptr ? dres + (size_t)row * H : xr;          // no residual: x again (in bounds, unused)
  Raw8<T> xraw[NCH], graw[NCH], mraw[NCH], rraw[NCH];
#pragma unroll
  for (int i = 0; i < NCH; i++) {                                        // every load of the row in flight at once
    const int c = min((i * WPR + wr) * 64 + lane, nchunks - 1);
    xraw[i] = Vec8<T>::load_raw(xr + c * 8);
    graw[i] = Vec8<T>::load_raw(dyr + c * 8);
    mraw[i] = Vec8<T>::load_raw(gamma + c * 8);
    rraw[i] = Vec8<T>::load_raw(rr + c * 8);
  }
  float xh[NCH][8], g[NCH][8];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; i++) {
    const int c = (i * WPR + wr) * 64 + lane;
    if (c < nchunks) {
      float gm[8];
      Vec8<T>::unpack(xraw[i], xh[i]);
      Vec8<T>::unpack(graw[i], g[i]);
      Vec8<T>::unpack(mraw[i], gm);
#pragma unroll
      for (int e = 0; e < 8; e++) {
        xh[i][e] = (xh[i][e] - mu) * rs;
        g[i][e] *= gm[e];
        s1 += g[i][e];
        s2 += g[i][e] * xh[i][e];
      }
    }
  }
  const float m1 = row_sum<WPR>(s1, red[0], wave, lane) / (float)H;
  const float m2 = row_sum<WPR>(s2, red[1], wave, lane) / (float)H;
  if (!owner) return;
  T* dxr = dx + (size_t)row * H;
#pragma unroll
  for (int i = 0; i < NCH; i++) {
    const int c = (i * WPR + wr) * 64 + lane;
    if (c < nchunks) {
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; e++) o[e] = rs * (g[i][e] - m1 - xh[i][e] * m2);
      if (dres != nullptr) {
        float r[8];
        Vec8<T>::unpack(rraw[i], r);
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] += r[e];
      }
      Vec8<T>::store(dxr + c * 8, o);
    }
  }
}

// LayerNorm backward with the parameter-gradient partial sums folded in (rows short enough to keep the
// per-lane column sums in registers; used for H <= 1024).  A block owns a run of rows, wave w takes every fourth of
// them; a lane always holds the same columns, so it adds dy and dy * xhat of its rows into registers, the
// four waves meet in LDS in fixed order and the block writes one partial row [2][H] for the finishing pass.
template <typename T, int NCH>
__global__ void __launch_bounds__(256) ln_bwd_fused_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                           const float* __restrict__ mean, const float* __restrict__ rstd,
                                                           const T* __restrict__ gamma, const T* __restrict__ dres,
                                                           T* __restrict__ dx, float* __restrict__ partial, int rows, int H,
                                                           int rows_per_block) {
  extern __shared__ float lnred[];                    // [2][4][H]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nchunks = H >> 3;
  const int r0 = blockIdx.x * rows_per_block;
  const int r1 = min(rows, r0 + rows_per_block);
  float sb[NCH][8], sg[NCH][8], gm[NCH][8];
#pragma unroll
  for (int i = 0; i < NCH; i++) {
    const int c = lane + 64 * i;
#pragma unroll
    for (int e = 0; e < 8; e++) { sb[i][e] = 0.f; sg[i][e] = 0.f; gm[i][e] = 0.f; }
    if (c < nchunks) Vec8<T>::load(gamma + c * 8, gm[i]);
  }
  // The loads of a wave's next row are in flight while it works on the current one (and the residual gradient
  // comes in with the row, not after the row sums): a wave has only a few rows, one after the other, and
  // every wait for memory it cannot overlap is time the whole kernel waits.
  struct RowIn { Raw8<T> x[NCH], g[NCH], r[NCH]; float mu, rs; };
  // every lane issues the same number of loads whatever its columns and whether or not there is a residual
  // gradient (lanes past the end re-read the last chunk, no residual re-reads x; neither value is used): the
  // compiler can then count the loads in flight and wait for the current row's only
  const T* rsrc = dres != nullptr ? dres : x;
  auto fetch = [&](int row, RowIn& in) {
    in.mu = mean[row]; in.rs = rstd[row];
#pragma unroll
    for (int i = 0; i < NCH; i++) {
      const size_t off = (size_t)row * H + min(lane + 64 * i, nchunks - 1) * 8;
      in.x[i] = Vec8<T>::load_raw(x + off);
      in.g[i] = Vec8<T>::load_raw(dy + off);
      in.r[i] = Vec8<T>::load_raw(rsrc + off);
    }
  };
  RowIn cur, nxt;
  if (r0 + wave < r1) fetch(r0 + wave, cur);
  for (int row = r0 + wave; row < r1; row += 4) {
    const bool more = row + 4 < r1;
    fetch(more ? row + 4 : row, nxt);               // the last turn re-reads its own row (in bounds, unused)
    const float mu = cur.mu, rs = cur.rs;
    float xh[NCH][8], g[NCH][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; i++) {
      const int c = lane + 64 * i;
      if (c < nchunks) {
        Vec8<T>::unpack(cur.x[i], xh[i]);
        Vec8<T>::unpack(cur.g[i], g[i]);
#pragma unroll
        for (int e = 0; e < 8; e++) {
          xh[i][e] = (xh[i][e] - mu) * rs;
          sb[i][e] += g[i][e];
          sg[i][e] += g[i][e] * xh[i][e];
          g[i][e] *= gm[i][e];
          s1 += g[i][e];
          s2 += g[i][e] * xh[i][e];
        }
      }
    }
    const float m1 = wave_sum(s1) / (float)H;
    const float m2 = wave_sum(s2) / (float)H;
    T* dxr = dx + (size_t)row * H;
#pragma unroll
    for (int i = 0; i < NCH; i++) {
      const int c = lane + 64 * i;
      if (c < nchunks) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = rs * (g[i][e] - m1 - xh[i][e] * m2);
        if (dres != nullptr) {
          float r[8];
          Vec8<T>::unpack(cur.r[i], r);
#pragma unroll
          for (int e = 0; e < 8; e++) o[e] += r[e];
        }
        Vec8<T>::store(dxr + c * 8, o);
      }
    }
    if (more) cur = nxt;
  }
#pragma unroll
  for (int i = 0; i < NCH; i++) {
    const int c = lane + 64 * i;
    if (c < nchunks) {
#pragma unroll
      for (int e = 0; e < 8; e++) {
        lnred[(0 * 4 + wave) * H + c * 8 + e] = sb[i][e];
        lnred[(1 * 4 + wave) * H + c * 8 + e] = sg[i][e];
      }
    }
  }
  __syncthreads();
  float* p = partial + (size_t)blockIdx.x * 2 * H;
  for (int c = threadIdx.x; c < 2 * H; c += 256) {
    const int slot = c / H, col = c - slot * H;
    p[c] = ((lnred[(slot * 4 + 0) * H + col] + lnred[(slot * 4 + 1) * H + col]) + lnred[(slot * 4 + 2) * H + col]) +
           lnred[(slot * 4 + 3) * H + col];
  }
}

// ------------------------------------------------------------------------------------------------
// Column sums in two deterministic passes.
//   pass 1: block (colblock, part) sums rows [part*rpp, (part+1)*rpp) of 256 columns; a thread owns
//           8 adjacent columns and every 8th row; the 8 row-lanes meet in LDS in fixed order.
//           XHAT = true additionally sums dy * (x - mean) * rstd   (LayerNorm gamma gradient).
//           partial layout: [part][2][width]  (slot 0: sum dy, slot 1: sum dy*xhat)
//   pass 2: one thread per column adds the parts in ascending order into the fp32 gradient.
// ------------------------------------------------------------------------------------------------
template <typename T, bool XHAT>
__global__ void __launch_bounds__(256) colsum_partial_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                             const float* __restrict__ mean,
                                                             const float* __restrict__ rstd,
                                                             float* __restrict__ partial, int rows, int width,
                                                             int rows_per_part) {
  __shared__ float red[2][8][256 + 8];
  const int cg = threadIdx.x & 31, rl = threadIdx.x >> 5;
  const int col = blockIdx.x * 256 + cg * 8;
  const int part = blockIdx.y;
  const int r0 = part * rows_per_part;
  const int r1 = min(rows, r0 + rows_per_part);
  float a[8], b[8];
#pragma unroll
  for (int e = 0; e < 8; e++) { a[e] = 0.f; b[e] = 0.f; }
  if (col < width) {
    for (int r = r0 + rl; r < r1; r += 8) {
      float d[8];
      Vec8<T>::load(dy + (size_t)r * width + col, d);
#pragma unroll
      for (int e = 0; e < 8; e++) a[e] += d[e];
      if (XHAT) {
        float xv[8];
        Vec8<T>::load(x + (size_t)r * width + col, xv);
        const float mu = mean[r], rs = rstd[r];
#pragma unroll
        for (int e = 0; e < 8; e++) b[e] += d[e] * ((xv[e] - mu) * rs);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; e++) { red[0][rl][cg * 8 + e] = a[e]; red[1][rl][cg * 8 + e] = b[e]; }
  __syncthreads();
  const int c = threadIdx.x;
  if (blockIdx.x * 256 + c < width) {
    float sa = 0.f, sb = 0.f;
#pragma unroll
    for (int j = 0; j < 8; j++) { sa += red[0][j][c]; sb += red[1][j][c]; }
    float* p = partial + (size_t)part * 2 * width;
    p[blockIdx.x * 256 + c] = sa;
    if (XHAT) p[width + blockIdx.x * 256 + c] = sb;
  }
}

// 32 columns per block; 8 threads share a column, each adds every 8th part in ascending order, and the
// eight partial sums meet in LDS in fixed order: the result does not depend on timing.
__global__ void __launch_bounds__(256) colsum_final_kernel(const float* __restrict__ partial, int parts, int width,
                                                           float* __restrict__ out0, float* __restrict__ out1) {
  __shared__ float red[2][8][32];
  const int cl = threadIdx.x & 31, pl = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + cl;
  float s0 = 0.f, s1 = 0.f;
  if (c < width) {
    // four loads in flight per accumulator, added in ascending part order
    int p = pl;
    for (; p + 24 < parts; p += 32) {
      const float* q = partial + (size_t)p * 2 * width + c;
      const float a0 = q[0], a1 = q[(size_t)16 * width], a2 = q[(size_t)32 * width], a3 = q[(size_t)48 * width];
      s0 = (((s0 + a0) + a1) + a2) + a3;
      if (out1 != nullptr) {
        const float b0 = q[width], b1 = q[(size_t)17 * width], b2 = q[(size_t)33 * width], b3 = q[(size_t)49 * width];
        s1 = (((s1 + b0) + b1) + b2) + b3;
      }
    }
    for (; p < parts; p += 8) {
      s0 += partial[(size_t)p * 2 * width + c];
      if (out1 != nullptr) s1 += partial[(size_t)p * 2 * width + width + c];
    }
  }
  red[0][pl][cl] = s0; red[1][pl][cl] = s1;
  __syncthreads();
  if (pl == 0 && c < width) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int j = 0; j < 8; j++) { a += red[0][j][cl]; b += red[1][j][cl]; }
    out0[c] += a;
    if (out1 != nullptr) out1[c] += b;
  }
}

static inline int reduce_parts(int rows) { return std::max(1, std::min(64, (rows + 31) / 32)); }

// out_sum == nullptr: only the partial sums are written (the finishing pass is issued separately)
template <typename T, bool XHAT>
static hipError_t colsum_launch(const T* dy, const T* x, const float* mean, const float* rstd, float* out_sum,
                                float* out_xhat, float* scratch, int rows, int width, hipStream_t s) {
  const int parts = reduce_parts(rows);
  const int rpp = (rows + parts - 1) / parts;
  dim3 grid((width + 255) / 256, parts);
  const double bytes = (double)rows * width * sizeof(T) * (XHAT ? 2 : 1);
  klaunch(colsum_partial_kernel<T, XHAT>, grid, dim3(256), 0, s, (XHAT ? PK_COLSUM_XHAT : PK_COLSUM) + (int)sizeof(T), bytes, dy, x,
          mean, rstd, scratch, rows, width, rpp);
  if (out_sum != nullptr)
    klaunch(colsum_final_kernel, dim3((width + 31) / 32), dim3(256), 0, s, PK_COLSUM_FINAL, (double)parts * width * 4 * (XHAT ? 2 : 1),
            scratch, parts, width, out_sum, XHAT ? out_xhat : (float*)nullptr);
  return hipGetLastError();
}

// Up to four column sums over the same rows in one pair of launches (the four bias gradients of a block).
struct ColsumProblem { const void* dy; float* out; int width, first_block, col_off; };
struct ColsumGroup { int count, rows, rows_per_part, total_width; ColsumProblem p[4]; };

template <typename T>
__global__ void __launch_bounds__(256) colsum_group_partial_kernel(ColsumGroup g, float* __restrict__ partial) {
  __shared__ float red[8][256 + 8];
  int pi = 0;
#pragma unroll
  for (int q = 1; q < 4; q++) if (q < g.count && (int)blockIdx.x >= g.p[q].first_block) pi = q;
  const ColsumProblem pr = g.p[pi];
  const T* dy = (const T*)pr.dy;
  const int cg = threadIdx.x & 31, rl = threadIdx.x >> 5;
  const int cb = (blockIdx.x - pr.first_block) * 256;
  const int col = cb + cg * 8;
  const int part = blockIdx.y;
  const int r0 = part * g.rows_per_part;
  const int r1 = min(g.rows, r0 + g.rows_per_part);
  float a[8];
#pragma unroll
  for (int e = 0; e < 8; e++) a[e] = 0.f;
  if (col < pr.width) {
    for (int r = r0 + rl; r < r1; r += 8) {
      float d[8];
      Vec8<T>::load(dy + (size_t)r * pr.width + col, d);
#pragma unroll
      for (int e = 0; e < 8; e++) a[e] += d[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; e++) red[rl][cg * 8 + e] = a[e];
  __syncthreads();
  const int c = threadIdx.x;
  if (cb + c < pr.width) {
    float sa = 0.f;
#pragma unroll
    for (int j = 0; j < 8; j++) sa += red[j][c];
    partial[(size_t)part * g.total_width + pr.col_off + cb + c] = sa;
  }
}

__global__ void __launch_bounds__(256) colsum_group_final_kernel(ColsumGroup g, const float* __restrict__ partial, int parts) {
  __shared__ float red[8][32];
  const int cl = threadIdx.x & 31, pl = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + cl;
  float s0 = 0.f;
  if (c < g.total_width)
    for (int p = pl; p < parts; p += 8) s0 += partial[(size_t)p * g.total_width + c];
  red[pl][cl] = s0;
  __syncthreads();
  if (pl == 0 && c < g.total_width) {
    float a = 0.f;
#pragma unroll
    for (int j = 0; j < 8; j++) a += red[j][cl];
    int pi = 0;
#pragma unroll
    for (int q = 1; q < 4; q++) if (q < g.count && c >= g.p[q].col_off) pi = q;
    g.p[pi].out[c - g.p[pi].col_off] += a;
  }
}

hipError_t launch_colsum_group(int dt, int n, const void* const* dy, float* const* out, const int* widths, float* scratch,
                               int rows, hipStream_t s) {
  if (rows <= 0 || n <= 0) return hipSuccess;
  if (n > 4) return hipErrorInvalidValue;
  ColsumGroup g{};
  g.count = n; g.rows = rows;
  const int parts = reduce_parts(rows);
  g.rows_per_part = (rows + parts - 1) / parts;
  int blocks = 0;
  double bytes = 0;
  for (int i = 0; i < n; i++) {
    g.p[i] = ColsumProblem{dy[i], out[i], widths[i], blocks, g.total_width};
    blocks += (widths[i] + 255) / 256;
    g.total_width += widths[i];
    bytes += (double)rows * widths[i] * dt_bytes(dt);
  }
  if (dt == DT_BF16)
    klaunch(colsum_group_partial_kernel<bf16_t>, dim3(blocks, parts), dim3(256), 0, s, PK_COLSUM + 10, bytes, g, scratch);
  else if (dt == DT_F16)
    klaunch(colsum_group_partial_kernel<f16_t>, dim3(blocks, parts), dim3(256), 0, s, PK_COLSUM + 10, bytes, g, scratch);
  else
    klaunch(colsum_group_partial_kernel<float>, dim3(blocks, parts), dim3(256), 0, s, PK_COLSUM + 12, bytes, g, scratch);
  klaunch(colsum_group_final_kernel, dim3((g.total_width + 31) / 32), dim3(256), 0, s, PK_COLSUM_FINAL + 1,
          (double)parts * g.total_width * 4, g, (const float*)scratch, parts);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) gelu_bwd_kernel(const T* __restrict__ dg, const T* __restrict__ u,
                                                       T* __restrict__ du, size_t nvec) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < nvec; i += stride) {
    float a[8], b[8], o[8];
    Vec8<T>::load(dg + i * 8, a);
    Vec8<T>::load(u + i * 8, b);
#pragma unroll
    for (int e = 0; e < 8; e++) o[e] = a[e] * gelu_grad_f(b[e]);
    Vec8<T>::store(du + i * 8, o);
  }
}

// g = gelu(u) of the stored pre-activation, as the fc1 epilogues form it (recomputation in the backward pass)
template <typename T>
__global__ void __launch_bounds__(256) gelu_fwd_kernel(const T* __restrict__ u, T* __restrict__ g, size_t nvec) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < nvec; i += stride) {
    float a[8], o[8];
    Vec8<T>::load(u + i * 8, a);
#pragma unroll
    for (int e = 0; e < 8; e++) o[e] = gelu_f(a[e]);
    Vec8<T>::store(g + i * 8, o);
  }
}

__global__ void __launch_bounds__(256) fill_zero_kernel(float* __restrict__ p, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t n4 = n >> 2;
  float4* p4 = reinterpret_cast<float4*>(p);
  for (size_t j = i; j < n4; j += stride) p4[j] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (size_t j = (n4 << 2) + i; j < n; j += stride) p[j] = 0.f;
}

template <typename U>
__global__ void __launch_bounds__(256) transpose_kernel(const U* __restrict__ in, U* __restrict__ out, int rows, int cols) {
  __shared__ U tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
#pragma unroll
  for (int j = 0; j < 32; j += 8) {
    const int r = r0 + ty + j, c = c0 + tx;
    if (r < rows && c < cols) tile[ty + j][tx] = in[(size_t)r * cols + c];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 32; j += 8) {
    const int c = c0 + ty + j, r = r0 + tx;
    if (r < rows && c < cols) out[(size_t)c * rows + r] = tile[tx][ty + j];
  }
}

// Weight operand of the NT GEMMs in chunk-major form: dst[kc][n][kk] = B[n][32 kc + kk], B[N][K] being the operand
// as the GEMM sees it.  TRANSPOSED: the source holds B^T, src[K][N] (a forward product reads W[in,out] as B = W^T);
// otherwise src[N][K] (an input-gradient product reads W[in,out] as it is).  A 32-deep chunk of consecutive
// rows is then one contiguous run of memory, whole cache lines for every load of the GEMM.
template <bool TRANSPOSED>
__global__ void __launch_bounds__(256) tile_weights_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, int N, int K) {
  __shared__ uint16_t tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
  const int n0 = blockIdx.x * 32, kc = blockIdx.y;
#pragma unroll
  for (int j = 0; j < 32; j += 8) {
    if (TRANSPOSED) {                 // read src[32 kc + (ty + j)][n0 + tx]
      const int k = kc * 32 + ty + j, n = n0 + tx;
      tile[ty + j][tx] = (k < K && n < N) ? src[(size_t)k * N + n] : (uint16_t)0;     // tile[kk][nn]
    } else {                          // read src[n0 + (ty + j)][32 kc + tx]
      const int n = n0 + ty + j, k = kc * 32 + tx;
      tile[tx][ty + j] = (k < K && n < N) ? src[(size_t)n * K + k] : (uint16_t)0;     // tile[kk][nn]
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 32; j += 8) {
    const int n = n0 + ty + j;
    if (n < N) dst[((size_t)kc * N + n) * 32 + tx] = tile[tx][ty + j];
  }
}

// Returns after `ticks` ticks of the 100 MHz device wall clock.  One wave; it sleeps between polls
// and always terminates because the clock is monotonic and `ticks` is bounded by the host.
__global__ void delay_kernel(long long ticks) {
  const long long t0 = wall_clock64();
  while (wall_clock64() - t0 < ticks) __builtin_amdgcn_s_sleep(32);
}

// Device -> pinned host copy of a boundary tensor (the "send" of an output), 16 bytes per lane and step.  The
// destination is written once and never read here: stores go past the caches.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) send_copy_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
    const u32x4_t v = __builtin_nontemporal_load(src + i);
    __builtin_nontemporal_store(v, dst + i);
  }
}

// The device wall clock, for a delay that counts from an event on another stream: the producer's stream stamps
// the clock when it is done, the transfer's stream waits until `ticks` after that stamp.  The wait also ends
// `ticks` after its own start, so it is bounded whatever the stamp holds.
__global__ void clock_stamp_kernel(long long* stamp) {
  if (threadIdx.x == 0) *stamp = wall_clock64();
}
__global__ void delay_since_kernel(const long long* stamp, long long ticks) {
  const long long since = *stamp, me = wall_clock64();
  long long now = me;
  while (now - since < ticks && now - me < ticks) { __builtin_amdgcn_s_sleep(32); now = wall_clock64(); }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
static inline int nch_for(int H) { const int n = (H + 511) / 512; return n <= 1 ? 1 : n <= 2 ? 2 : n <= 4 ? 4 : n <= 8 ? 8 : 16; }

// How a row is dealt to the lanes of the forward and dx kernels: WPR waves per row, NCH chunks of 8 per lane,
// 512 * NCH * WPR >= H.  At most 4 chunks per lane: wide rows go over more waves, not into more registers.
struct RowShape { int nch, wpr, code; };
static inline RowShape row_shape(int H) {
  const int per_wave = (H + 511) / 512;                        // chunks per lane if one wave took the row
  int wpr = per_wave <= 2 ? 1 : per_wave <= 4 ? 2 : 4;
  int nch = (per_wave + wpr - 1) / wpr;
  nch = nch <= 1 ? 1 : nch <= 2 ? 2 : 4;
  const int wcode = wpr == 1 ? 0 : wpr == 2 ? 1 : 2, ncode = nch == 1 ? 0 : nch == 2 ? 1 : 2;
  return RowShape{nch, wpr, wcode * 20 + ncode * 4};
}

#define KFKB_ROW_SWITCH(RS, ...)                                                                       \
  switch ((RS).wpr * 8 + (RS).nch) {                                                                   \
    case 1 * 8 + 1: { constexpr int WPR = 1, NCH = 1; __VA_ARGS__; break; }                            \
    case 1 * 8 + 2: { constexpr int WPR = 1, NCH = 2; __VA_ARGS__; break; }                            \
    case 2 * 8 + 2: { constexpr int WPR = 2, NCH = 2; __VA_ARGS__; break; }                            \
    case 4 * 8 + 2: { constexpr int WPR = 4, NCH = 2; __VA_ARGS__; break; }                            \
    default: { constexpr int WPR = 4, NCH = 4; __VA_ARGS__; break; }                                   \
  }

template <typename T>
static hipError_t ln_fwd_t(const T* x, const T* g, const T* b, T* y, float* mean, float* rstd, int rows, int H,
                           float eps, hipStream_t s) {
  const RowShape rs = row_shape(H);
  const int rpb = 4 / rs.wpr;
  const dim3 grid((rows + rpb - 1) / rpb);
  const double bytes = 2.0 * rows * H * sizeof(T);
  KFKB_ROW_SWITCH(rs, klaunch(ln_fwd_kernel<T, NCH, WPR>, grid, dim3(256), 0, s, PK_LN_FWD + rs.code + (int)sizeof(T) / 4, bytes, x, g, b, y, mean, rstd, rows, H, eps));
  return hipGetLastError();
}

hipError_t launch_ln_fwd(int dt, const void* x, const void* gamma, const void* beta, void* y, float* mean,
                         float* rstd, int rows, int H, float eps, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dt == DT_BF16)
    return ln_fwd_t<bf16_t>((const bf16_t*)x, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)y, mean, rstd, rows, H, eps, s);
  if (dt == DT_F16)
    return ln_fwd_t<f16_t>((const f16_t*)x, (const f16_t*)gamma, (const f16_t*)beta, (f16_t*)y, mean, rstd, rows, H, eps, s);
  return ln_fwd_t<float>((const float*)x, (const float*)gamma, (const float*)beta, (float*)y, mean, rstd, rows, H, eps, s);
}

template <typename T, int NCH>
static hipError_t ln_bwd_fused_launch(const T* dy, const T* x, const float* mean, const float* rstd, const T* gamma,
                                      const T* dres, T* dx, float* dgamma, float* dbeta, float* scratch, int rows, int H,
                                      hipStream_t s) {
  const int rpb = std::max(8, ((rows + 511) / 512 + 3) / 4 * 4);   // at most 512 partial rows
  const int parts = (rows + rpb - 1) / rpb;
  const double bytes = (dres ? 4.0 : 3.0) * rows * H * sizeof(T);
  klaunch(ln_bwd_fused_kernel<T, NCH>, dim3(parts), dim3(256), (size_t)8 * H * sizeof(float), s,
          PK_LN_BWD_DX + 80 + NCH * 4 + (int)sizeof(T) / 4, bytes, dy, x, mean, rstd, gamma, dres, dx, scratch, rows, H, rpb);
  if (dgamma != nullptr)
    klaunch(colsum_final_kernel, dim3((H + 31) / 32), dim3(256), 0, s, PK_COLSUM_FINAL, (double)parts * H * 8, (const float*)scratch,
            parts, H, dbeta, dgamma);
  return hipGetLastError();
}

template <typename T>
static hipError_t ln_bwd_t(const T* dy, const T* x, const float* mean, const float* rstd, const T* gamma,
                           const T* dres, T* dx, float* dgamma, float* dbeta, float* scratch, int rows, int H,
                           hipStream_t s) {
  const int nch = nch_for(H);
  // Rows of up to 1024 values: dx and the partial parameter sums in one pass (fewer launches; the pass is short either
  // way).  Longer rows: the dx kernel, which gives every CU many rows at a time, then the partial sums (measured at
  // 4096 rows of 2048: 26 us fused, 19 us in two launches; 1.3B-class stage 272.5 -> 269.0 ms per iteration; at 1024
  // the two launches were slower, 44.1 -> 44.6 ms on the GPT-2-medium-shaped stage).
  if (nch == 1) return ln_bwd_fused_launch<T, 1>(dy, x, mean, rstd, gamma, dres, dx, dgamma, dbeta, scratch, rows, H, s);
  if (nch == 2) return ln_bwd_fused_launch<T, 2>(dy, x, mean, rstd, gamma, dres, dx, dgamma, dbeta, scratch, rows, H, s);
  const RowShape rs = row_shape(H);
  const int rpb = 4 / rs.wpr;
  const dim3 grid((rows + rpb - 1) / rpb);
  const double bytes = (dres ? 4.0 : 3.0) * rows * H * sizeof(T);
  KFKB_ROW_SWITCH(rs, klaunch(ln_bwd_dx_kernel<T, NCH, WPR>, grid, dim3(256), 0, s, PK_LN_BWD_DX + rs.code + (int)sizeof(T) / 4, bytes, dy, x, mean, rstd, gamma, dres, dx, rows, H));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return colsum_launch<T, true>(dy, x, mean, rstd, dgamma != nullptr ? dbeta : (float*)nullptr, dgamma, scratch, rows, H, s);
}

hipError_t launch_ln_bwd(int dt, const void* dy, const void* x, const float* mean, const float* rstd,
                         const void* gamma, const void* dres, void* dx, float* dgamma, float* dbeta,
                         float* scratch, int rows, int H, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dt == DT_BF16)
    return ln_bwd_t<bf16_t>((const bf16_t*)dy, (const bf16_t*)x, mean, rstd, (const bf16_t*)gamma, (const bf16_t*)dres,
                            (bf16_t*)dx, dgamma, dbeta, scratch, rows, H, s);
  if (dt == DT_F16)
    return ln_bwd_t<f16_t>((const f16_t*)dy, (const f16_t*)x, mean, rstd, (const f16_t*)gamma, (const f16_t*)dres,
                           (f16_t*)dx, dgamma, dbeta, scratch, rows, H, s);
  return ln_bwd_t<float>((const float*)dy, (const float*)x, mean, rstd, (const float*)gamma, (const float*)dres,
                         (float*)dx, dgamma, dbeta, scratch, rows, H, s);
}

// The finishing pass of launch_ln_bwd called with dgamma == nullptr: adds the partial sums it left in `scratch`
// into dgamma / dbeta.  rows and H must be those of that call (they fix the number of partial rows).
int ln_bwd_partial_rows(int rows, int H) {
  if (nch_for(H) <= 2) {
    const int rpb = std::max(8, ((rows + 511) / 512 + 3) / 4 * 4);
    return (rows + rpb - 1) / rpb;
  }
  return reduce_parts(rows);
}

hipError_t launch_ln_bwd_final(const float* scratch, int rows, int H, float* dgamma, float* dbeta, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  const int parts = ln_bwd_partial_rows(rows, H);
  klaunch(colsum_final_kernel, dim3((H + 31) / 32), dim3(256), 0, s, PK_COLSUM_FINAL, (double)parts * H * 8, scratch, parts, H,
          dbeta, dgamma);
  return hipGetLastError();
}

size_t colsum_scratch_floats(int rows, int N) { return rows <= 0 ? 0 : (size_t)reduce_parts(rows) * 2 * N; }

hipError_t launch_colsum_accum(int dt, const void* dy, float* out, float* scratch, int rows, int N, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dt == DT_BF16)
    return colsum_launch<bf16_t, false>((const bf16_t*)dy, nullptr, nullptr, nullptr, out, nullptr, scratch, rows, N, s);
  if (dt == DT_F16)
    return colsum_launch<f16_t, false>((const f16_t*)dy, nullptr, nullptr, nullptr, out, nullptr, scratch, rows, N, s);
  return colsum_launch<float, false>((const float*)dy, nullptr, nullptr, nullptr, out, nullptr, scratch, rows, N, s);
}

hipError_t launch_gelu_bwd(int dt, const void* dg, const void* u, void* du, size_t n, hipStream_t s) {
  const size_t nvec = n / 8;
  if (nvec == 0) return hipSuccess;
  const int grid = (int)std::min<size_t>((nvec + 255) / 256, 8192);
  if (dt == DT_BF16)
    klaunch(gelu_bwd_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, PK_GELU_BWD + 2, 3.0 * n * 2, (const bf16_t*)dg, (const bf16_t*)u, (bf16_t*)du, nvec);
  else if (dt == DT_F16)
    klaunch(gelu_bwd_kernel<f16_t>, dim3(grid), dim3(256), 0, s, PK_GELU_BWD + 2, 3.0 * n * 2, (const f16_t*)dg, (const f16_t*)u, (f16_t*)du, nvec);
  else
    klaunch(gelu_bwd_kernel<float>, dim3(grid), dim3(256), 0, s, PK_GELU_BWD + 4, 3.0 * n * 4, (const float*)dg, (const float*)u, (float*)du, nvec);
  return hipGetLastError();
}

hipError_t launch_gelu_fwd(int dt, const void* u, void* g, size_t n, hipStream_t s) {
  const size_t nvec = n / 8;
  if (nvec == 0) return hipSuccess;
  const int grid = (int)std::min<size_t>((nvec + 255) / 256, 8192);
  if (dt == DT_BF16)
    klaunch(gelu_fwd_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, PK_GELU_BWD + 12, 2.0 * n * 2, (const bf16_t*)u, (bf16_t*)g, nvec);
  else if (dt == DT_F16)
    klaunch(gelu_fwd_kernel<f16_t>, dim3(grid), dim3(256), 0, s, PK_GELU_BWD + 12, 2.0 * n * 2, (const f16_t*)u, (f16_t*)g, nvec);
  else
    klaunch(gelu_fwd_kernel<float>, dim3(grid), dim3(256), 0, s, PK_GELU_BWD + 14, 2.0 * n * 4, (const float*)u, (float*)g, nvec);
  return hipGetLastError();
}

hipError_t launch_fill_zero(float* p, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const int grid = (int)std::min<size_t>((n / 4 + 255) / 256 + 1, 4096);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, s, p, n);
  return hipGetLastError();
}

hipError_t launch_transpose(int dt, const void* in, void* out, int rows, int cols, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  const dim3 grid((cols + 31) / 32, (rows + 31) / 32);
  if (dt_is16(dt))
    hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, s, (const uint16_t*)in, (uint16_t*)out, rows, cols);
  else
    hipLaunchKernelGGL(transpose_kernel<uint32_t>, grid, dim3(256), 0, s, (const uint32_t*)in, (uint32_t*)out, rows, cols);
  return hipGetLastError();
}

hipError_t launch_tile_weights(const void* src, void* dst, int N, int K, bool transposed, hipStream_t s) {
  if (N <= 0 || K <= 0) return hipSuccess;
  const dim3 grid((N + 31) / 32, (K + 31) / 32);
  if (transposed) hipLaunchKernelGGL(tile_weights_kernel<true>, grid, dim3(256), 0, s, (const uint16_t*)src, (uint16_t*)dst, N, K);
  else hipLaunchKernelGGL(tile_weights_kernel<false>, grid, dim3(256), 0, s, (const uint16_t*)src, (uint16_t*)dst, N, K);
  return hipGetLastError();
}

hipError_t launch_delay(int64_t ns, hipStream_t s) {
  if (ns <= 0) return hipSuccess;
  if (ns > 2000000000LL) ns = 2000000000LL;                   // never spin longer than two seconds
  hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, s, (long long)(ns / 10));
  return hipGetLastError();
}

hipError_t launch_send_copy(void* dst_device_view_of_host, const void* src, size_t bytes, int blocks, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  if ((bytes & 15) != 0 || (((uintptr_t)dst_device_view_of_host | (uintptr_t)src) & 15) != 0 || blocks < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(send_copy_kernel, dim3(blocks), dim3(256), 0, s, (const u32x4_t*)src, (u32x4_t*)dst_device_view_of_host, bytes / 16);
  return hipGetLastError();
}

hipError_t launch_clock_stamp(long long* stamp, hipStream_t s) {
  hipLaunchKernelGGL(clock_stamp_kernel, dim3(1), dim3(64), 0, s, stamp);
  return hipGetLastError();
}

hipError_t launch_delay_since(const long long* stamp, int64_t ns, hipStream_t s) {
  if (ns <= 0) return hipSuccess;
  if (ns > 2000000000LL) ns = 2000000000LL;
  hipLaunchKernelGGL(delay_since_kernel, dim3(1), dim3(64), 0, s, stamp, (long long)(ns / 10));
  return hipGetLastError();
}

}  // namespace kfkb
