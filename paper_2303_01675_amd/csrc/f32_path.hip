// fp32 kernels of the stage: a register-tiled GEMM over arbitrary strides (covers forward,
// input-gradient and weight-gradient forms with every epilogue) and row-at-a-time attention
// forward / backward.  This is the exact-arithmetic path used for small stages and for
// checking; the bf16 path has its own MFMA kernels.  Any shape is accepted (bounds-checked).
#include "common.h"
#include "../../include/kfkb.h"

namespace kfkb {

// ------------------------------------------------------------------------------------------------
// C[M,N] (+)= sum_k A(m,k) B(k,n);  A(m,k) = A[m*a_m + k*a_k],  B(k,n) = B[k*b_k + n*b_n].
// 64x64 tile per block, 16-deep slices through LDS, 4x4 outputs per thread.
// ------------------------------------------------------------------------------------------------
template <int EPI>
__global__ void __launch_bounds__(256) gemm_f32_kernel(int M, int N, int K, const float* __restrict__ A, long a_m, long a_k,
                                                       const float* __restrict__ B, long b_k, long b_n,
                                                       const float* __restrict__ bias, const float* __restrict__ residual,
                                                       float* __restrict__ C, float* __restrict__ C2,
                                                       float* __restrict__ Cacc) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int t = 0; t < 4; t++) {
      const int idx = threadIdx.x + t * 256;           // 1024 elements per operand slice
      {
        // A slice: let the faster-varying thread index follow the operand's unit stride
        const int mm = (a_k == 1) ? idx / 16 : idx % 64;
        const int kk = (a_k == 1) ? idx % 16 : idx / 64;
        const int m = m0 + mm, k = k0 + kk;
        As[kk][mm] = (m < M && k < K) ? A[m * a_m + k * a_k] : 0.f;
      }
      {
        const int nn = (b_k == 1) ? idx / 16 : idx % 64;
        const int kk = (b_k == 1) ? idx % 16 : idx / 64;
        const int n = n0 + nn, k = k0 + kk;
        Bs[kk][nn] = (n < N && k < K) ? B[k * b_k + n * b_n] : 0.f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; kk++) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; i++) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; j++) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      const size_t o = (size_t)m * N + n;
      float v = acc[i][j];
      if (EPI == KFKB_EPI_NONE) C[o] = v;
      if (EPI == KFKB_EPI_BIAS) C[o] = v + bias[n];
      if (EPI == KFKB_EPI_BIAS_GELU) { v += bias[n]; C[o] = v; C2[o] = gelu_f(v); }
      if (EPI == KFKB_EPI_BIAS_RES) C[o] = v + bias[n] + residual[o];
      if (EPI == KFKB_EPI_ACCUM) Cacc[o] += v;
      if (EPI == KFKB_EPI_GELU_BWD) C[o] = v * gelu_grad_f(residual[o]);
    }
  }
}

hipError_t launch_gemm_f32(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  long a_m, a_k, b_k, b_n;
  switch (g.kind) {
    case KFKB_GEMM_NN: a_m = g.K; a_k = 1; b_k = g.N; b_n = 1; break;
    case KFKB_GEMM_NT: a_m = g.K; a_k = 1; b_k = 1; b_n = g.K; break;
    default: /* TN */ a_m = 1; a_k = g.M; b_k = g.N; b_n = 1; break;
  }
  const dim3 grid((g.N + 63) / 64, (g.M + 63) / 64);
  const float* A = (const float*)g.A; const float* B = (const float*)g.B;
  const float* bias = (const float*)g.bias; const float* res = (const float*)g.residual;
  float* C = (float*)g.C; float* C2 = (float*)g.C2;
#define KFKB_LAUNCH_F32(E) klaunch(gemm_f32_kernel<E>, grid, dim3(256), 0, s, PK_GEMM_F32 + E, 2.0 * g.M * g.N * g.K, g.M, g.N, g.K, A, a_m, a_k, B, b_k, b_n, bias, res, C, C2, g.Cacc)
  switch (g.epilogue) {
    case KFKB_EPI_NONE: KFKB_LAUNCH_F32(KFKB_EPI_NONE); break;
    case KFKB_EPI_BIAS: KFKB_LAUNCH_F32(KFKB_EPI_BIAS); break;
    case KFKB_EPI_BIAS_GELU: KFKB_LAUNCH_F32(KFKB_EPI_BIAS_GELU); break;
    case KFKB_EPI_BIAS_RES: KFKB_LAUNCH_F32(KFKB_EPI_BIAS_RES); break;
    case KFKB_EPI_ACCUM: KFKB_LAUNCH_F32(KFKB_EPI_ACCUM); break;
    default: KFKB_LAUNCH_F32(KFKB_EPI_GELU_BWD); break;
  }
#undef KFKB_LAUNCH_F32
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Attention, fp32, one wave per (sample, head, row).  qkv is [b*T, 3H]; q of head h sits at columns
// h*d.., k at H + h*d.., v at 2H + h*d...  Scores of the row are kept in LDS (T floats).
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) attn_fwd_f32_kernel(const float* __restrict__ qkv, float* __restrict__ o,
                                                          float* __restrict__ lse, int T, int H, int heads, int d,
                                                          int causal, float scale) {
  extern __shared__ float sc[];                       // T scores, then d query values
  float* qs = sc + T;
  const int lane = threadIdx.x;
  const int i = blockIdx.x, hd = blockIdx.y, bi = blockIdx.z;
  const size_t ld = 3 * (size_t)H;
  const float* base = qkv + (size_t)bi * T * ld;
  const float* qrow = base + (size_t)i * ld + hd * d;
  for (int t = lane; t < d; t += 64) qs[t] = qrow[t];
  __syncthreads();
  const int last = causal ? i : T - 1;
  float mx = -INFINITY;
  for (int j = lane; j <= last; j += 64) {
    const float* krow = base + (size_t)j * ld + H + hd * d;
    float s = 0.f;
    for (int t = 0; t < d; t++) s += qs[t] * krow[t];
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j <= last; j += 64) { const float e = __expf(sc[j] - mx); sc[j] = e; sum += e; }
  sum = wave_sum(sum);
  __syncthreads();
  const float inv = 1.0f / sum;
  for (int t = lane; t < d; t += 64) {
    float acc = 0.f;
    for (int j = 0; j <= last; j++) acc += sc[j] * base[(size_t)j * ld + 2 * H + hd * d + t];
    o[((size_t)bi * T + i) * H + hd * d + t] = acc * inv;
  }
  if (lane == 0) lse[((size_t)bi * heads + hd) * T + i] = mx + __logf(sum);
}

// dsum[b, head, i] = sum_t do[i, t] * o[i, t]  (the row term of the softmax backward)
template <typename T>
__global__ void __launch_bounds__(256) attn_dsum_kernel(const T* __restrict__ o, const T* __restrict__ d_o,
                                                        float* __restrict__ dsum, int Tlen, int H, int heads, int d,
                                                        int total) {
  const int w = blockIdx.x * 4 + (threadIdx.x >> 6);       // one wave per (b, head, i)
  if (w >= total) return;
  const int lane = threadIdx.x & 63;
  const int i = w % Tlen, hd = (w / Tlen) % heads, bi = w / (Tlen * heads);
  const size_t off = ((size_t)bi * Tlen + i) * H + hd * d;
  float s = 0.f;
  for (int t = lane; t < d; t += 64) s += to_f<T>(o[off + t]) * to_f<T>(d_o[off + t]);
  s = wave_sum(s);
  if (lane == 0) dsum[w] = s;
}
template __global__ void attn_dsum_kernel<float>(const float*, const float*, float*, int, int, int, int, int);
template __global__ void attn_dsum_kernel<bf16_t>(const bf16_t*, const bf16_t*, float*, int, int, int, int, int);

hipError_t launch_attn_dsum(int dt, const void* o, const void* d_o, float* dsum, int b, int T, int H, int heads, hipStream_t s) {
  const int total = b * heads * T;
  if (total <= 0) return hipSuccess;
  if (dt == DT_BF16)
    klaunch(attn_dsum_kernel<bf16_t>, dim3((total + 3) / 4), dim3(256), 0, s, PK_ATTN_DSUM + 2, 2.0 * b * T * H * 2, (const bf16_t*)o, (const bf16_t*)d_o, dsum, T, H, heads, H / heads, total);
  else
    hipLaunchKernelGGL(attn_dsum_kernel<float>, dim3((total + 3) / 4), dim3(256), 0, s, (const float*)o, (const float*)d_o, dsum, T, H, heads, H / heads, total);
  return hipGetLastError();
}

// dq of one query row:  p_j = exp(s_j - lse); ds_j = p_j (do.v_j - dsum); dq = scale * sum_j ds_j k_j
__global__ void __launch_bounds__(64) attn_bwd_dq_f32_kernel(const float* __restrict__ qkv, const float* __restrict__ d_o,
                                                             const float* __restrict__ lse, const float* __restrict__ dsum,
                                                             float* __restrict__ dqkv, int T, int H, int heads, int d,
                                                             int causal, float scale) {
  extern __shared__ float sc[];                       // T ds values, d query values, d do values
  float* qs = sc + T;
  float* dos = qs + d;
  const int lane = threadIdx.x;
  const int i = blockIdx.x, hd = blockIdx.y, bi = blockIdx.z;
  const size_t ld = 3 * (size_t)H;
  const float* base = qkv + (size_t)bi * T * ld;
  for (int t = lane; t < d; t += 64) {
    qs[t] = base[(size_t)i * ld + hd * d + t];
    dos[t] = d_o[((size_t)bi * T + i) * H + hd * d + t];
  }
  __syncthreads();
  const size_t st = ((size_t)bi * heads + hd) * T + i;
  const float l = lse[st], ds0 = dsum[st];
  const int last = causal ? i : T - 1;
  for (int j = lane; j <= last; j += 64) {
    const float* krow = base + (size_t)j * ld + H + hd * d;
    const float* vrow = base + (size_t)j * ld + 2 * H + hd * d;
    float s = 0.f, dp = 0.f;
    for (int t = 0; t < d; t++) { s += qs[t] * krow[t]; dp += dos[t] * vrow[t]; }
    const float p = __expf(s * scale - l);
    sc[j] = p * (dp - ds0);
  }
  __syncthreads();
  for (int t = lane; t < d; t += 64) {
    float acc = 0.f;
    for (int j = 0; j <= last; j++) acc += sc[j] * base[(size_t)j * ld + H + hd * d + t];
    dqkv[((size_t)bi * T + i) * ld + hd * d + t] = acc * scale;
  }
}

// dk, dv of one key row j:  dv = sum_i p_ij do_i ;  dk = scale * sum_i ds_ij q_i   (i >= j if causal)
__global__ void __launch_bounds__(64) attn_bwd_dkv_f32_kernel(const float* __restrict__ qkv, const float* __restrict__ d_o,
                                                              const float* __restrict__ lse, const float* __restrict__ dsum,
                                                              float* __restrict__ dqkv, int T, int H, int heads, int d,
                                                              int causal, float scale) {
  extern __shared__ float sc[];                       // T p values, T ds values, d key values, d value values
  float* dsv = sc + T;
  float* ks = dsv + T;
  float* vs = ks + d;
  const int lane = threadIdx.x;
  const int j = blockIdx.x, hd = blockIdx.y, bi = blockIdx.z;
  const size_t ld = 3 * (size_t)H;
  const float* base = qkv + (size_t)bi * T * ld;
  for (int t = lane; t < d; t += 64) {
    ks[t] = base[(size_t)j * ld + H + hd * d + t];
    vs[t] = base[(size_t)j * ld + 2 * H + hd * d + t];
  }
  __syncthreads();
  const int first = causal ? j : 0;
  const size_t st = ((size_t)bi * heads + hd) * T;
  for (int i = first + lane; i < T; i += 64) {
    const float* qrow = base + (size_t)i * ld + hd * d;
    const float* dorow = d_o + ((size_t)bi * T + i) * H + hd * d;
    float s = 0.f, dp = 0.f;
    for (int t = 0; t < d; t++) { s += qrow[t] * ks[t]; dp += dorow[t] * vs[t]; }
    const float p = __expf(s * scale - lse[st + i]);
    sc[i] = p;
    dsv[i] = p * (dp - dsum[st + i]);
  }
  __syncthreads();
  for (int t = lane; t < d; t += 64) {
    float adv = 0.f, adk = 0.f;
    for (int i = first; i < T; i++) {
      adv += sc[i] * d_o[((size_t)bi * T + i) * H + hd * d + t];
      adk += dsv[i] * base[(size_t)i * ld + hd * d + t];
    }
    dqkv[((size_t)bi * T + j) * ld + H + hd * d + t] = adk * scale;
    dqkv[((size_t)bi * T + j) * ld + 2 * H + hd * d + t] = adv;
  }
}

hipError_t launch_attention_fwd_f32(const float* qkv, float* o, float* lse, int b, int T, int H, int heads,
                                    int causal, hipStream_t s) {
  if (b <= 0 || T <= 0) return hipSuccess;
  const int d = H / heads;
  const float scale = 1.0f / sqrtf((float)d);
  hipLaunchKernelGGL(attn_fwd_f32_kernel, dim3(T, heads, b), dim3(64), (T + d) * sizeof(float), s, qkv, o, lse, T, H, heads, d, causal, scale);
  return hipGetLastError();
}

hipError_t launch_attention_bwd_f32(const float* qkv, const float* o, const float* d_o, const float* lse,
                                    float* dsum, float* dqkv, int b, int T, int H, int heads, int causal,
                                    hipStream_t s) {
  if (b <= 0 || T <= 0) return hipSuccess;
  const int d = H / heads;
  const float scale = 1.0f / sqrtf((float)d);
  hipError_t e = launch_attn_dsum(DT_F32, o, d_o, dsum, b, T, H, heads, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_bwd_dq_f32_kernel, dim3(T, heads, b), dim3(64), (T + 2 * d) * sizeof(float), s, qkv, d_o, lse, dsum, dqkv, T, H, heads, d, causal, scale);
  hipLaunchKernelGGL(attn_bwd_dkv_f32_kernel, dim3(T, heads, b), dim3(64), (2 * T + 2 * d) * sizeof(float), s, qkv, d_o, lse, dsum, dqkv, T, H, heads, d, causal, scale);
  return hipGetLastError();
}

}  // namespace kfkb
