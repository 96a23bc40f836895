// Internal helpers shared by the HIP translation units of libkfkb (not part of the C boundary).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

namespace kfkb {

typedef __bf16 bf16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16_t;
typedef f16_t f16x8 __attribute__((ext_vector_type(8)));
typedef f16_t f16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// ---- bf16 <-> fp32 (round to nearest even on the way down) -----------------------------------
__device__ __forceinline__ float bf2f(bf16_t v) { return (float)v; }
__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)f; }

template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v) { return (float)v; }
template <> __device__ __forceinline__ float to_f<f16_t>(f16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return (bf16_t)v; }
template <> __device__ __forceinline__ f16_t from_f<f16_t>(float v) { return (f16_t)v; }

// 8 consecutive elements of T <-> 8 floats, vector loads (16 B for bf16, 2 x 16 B for fp32).
// eight values as they come from memory: loaded now, converted where they are first used (a load whose
// result is converted at once cannot be kept in flight across other work)
template <typename T> struct Raw8;
template <> struct Raw8<float> { float4 a, b; };
template <> struct Raw8<bf16_t> { bf16x8 v; };
template <> struct Raw8<f16_t> { f16x8 v; };
template <typename T> struct Vec8;
template <> struct Vec8<float> {
  static __device__ __forceinline__ Raw8<float> load_raw(const float* p) {
    Raw8<float> r; r.a = *reinterpret_cast<const float4*>(p); r.b = *reinterpret_cast<const float4*>(p + 4); return r;
  }
  static __device__ __forceinline__ void unpack(const Raw8<float>& r, float (&v)[8]) {
    v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w; v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
  }
  static __device__ __forceinline__ void load(const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
};
template <> struct Vec8<bf16_t> {
  static __device__ __forceinline__ Raw8<bf16_t> load_raw(const bf16_t* p) {
    Raw8<bf16_t> r; r.v = *reinterpret_cast<const bf16x8*>(p); return r;
  }
  static __device__ __forceinline__ void unpack(const Raw8<bf16_t>& r, float (&v)[8]) {
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = (float)r.v[i];
  }
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = (float)a[i];
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    bf16x8 a;
#pragma unroll
    for (int i = 0; i < 8; i++) a[i] = (bf16_t)v[i];
    *reinterpret_cast<bf16x8*>(p) = a;
  }
};
template <> struct Vec8<f16_t> {
  static __device__ __forceinline__ Raw8<f16_t> load_raw(const f16_t* p) {
    Raw8<f16_t> r; r.v = *reinterpret_cast<const f16x8*>(p); return r;
  }
  static __device__ __forceinline__ void unpack(const Raw8<f16_t>& r, float (&v)[8]) {
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = (float)r.v[i];
  }
  static __device__ __forceinline__ void load(const f16_t* p, float (&v)[8]) {
    const f16x8 a = *reinterpret_cast<const f16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = (float)a[i];
  }
  static __device__ __forceinline__ void store(f16_t* p, const float (&v)[8]) {
    f16x8 a;
#pragma unroll
    for (int i = 0; i < 8; i++) a[i] = (f16_t)v[i];
    *reinterpret_cast<f16x8*>(p) = a;
  }
};

// ---- wave64 reductions --------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- loads that write LDS directly ---------------------------------------------------------------
// buffer_load_dwordx4 ... lds: lane l of the wave moves 16 bytes from (resource base + voff + soff) to LDS byte address
// lds_addr + 16 l; bytes past the resource's size read as zero.  Issued through inline assembly so that the compiler
// does not serialise every later LDS read behind them; the caller counts them with wait_vmcnt before the barrier
// that publishes the data.
typedef int i32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void dma16b(i32x4 rsrc, int voff, int soff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "m0");
}
__device__ __forceinline__ i32x4 make_rsrc(const void* p, size_t bytes) {
  const unsigned long long a = (unsigned long long)p;
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(a & 0xffffffffu));
  r[1] = __builtin_amdgcn_readfirstlane((int)(a >> 32));
  r[2] = __builtin_amdgcn_readfirstlane((int)(bytes > 0xFFFFFFFFull ? 0xFFFFFFFFull : bytes));
  r[3] = 0x00020000;
  return r;
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0070 | 0x0F00);
}
__device__ __forceinline__ void wait_lgkm0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// ---- GELU, tanh form: 0.5 u (1 + tanh(z)), z = c0 (u + c1 u^3) ---------------------------------
// With s = 1 / (1 + exp(-2 z)): 0.5 (1 + tanh z) = s and 1 - tanh^2 z = 4 s (1 - s), hence
//   gelu(u) = u s,   gelu'(u) = s + u s (1 - s) 2 z'(u),   2 z' = 2 c0 (1 + 3 c1 u^2).
// exp(-2 z) is taken as exp2 of a polynomial in u; its overflow to +inf gives s = 0, its underflow s = 1.
__device__ __forceinline__ float gelu_sigmoid_f(float u) {
  constexpr float k0 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;   // -2 c0 log2(e)
  constexpr float k1 = k0 * 0.044715f;
  const float e = __builtin_amdgcn_exp2f(u * (k0 + k1 * u * u));
  return __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ __forceinline__ float gelu_f(float u) { return u * gelu_sigmoid_f(u); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  constexpr float d0 = 2.0f * 0.7978845608028654f, d1 = d0 * 3.0f * 0.044715f;
  const float s = gelu_sigmoid_f(u);
  return s + u * s * (1.0f - s) * (d0 + d1 * u * u);
}

// ---- optional per-kernel timing -------------------------------------------------------------------
// When collection is on, a launch goes through hipExtLaunchKernelGGL with a start and a stop event,
// which carry the kernel's own begin / end timestamps; otherwise it is a plain launch.
// `work` is the launch's algorithmic work: flops for the matrix-core kernels, bytes for the
// bandwidth-bound ones.  Keys name kernel instantiations (see prof_key_name in engine.hip).
enum ProfClass { PK_GEMM_NT = 1000, PK_GEMM_TN = 2000, PK_ATTN_FWD = 3000, PK_ATTN_DQ = 3100, PK_ATTN_DKV = 3200,
                 PK_ATTN_DSUM = 3300, PK_LN_FWD = 4000, PK_LN_BWD_DX = 4100, PK_COLSUM = 4200, PK_COLSUM_XHAT = 4300,
                 PK_COLSUM_FINAL = 4400, PK_GELU_BWD = 4500, PK_GEMM_F32 = 5000, PK_ATTN_F32 = 5100 };
bool prof_acquire(int key, double work, hipEvent_t* e0, hipEvent_t* e1);
// records the calling thread's error message (what kfkb_last_error returns) and hands `code` back
int set_error(int code, const char* fmt, ...);

template <typename... KArgs, typename... Args>
inline void klaunch(void (*kern)(KArgs...), dim3 grid, dim3 block, size_t smem, hipStream_t s, int key, double work,
                    Args... args) {
  hipEvent_t e0, e1;
  if (prof_acquire(key, work, &e0, &e1)) hipExtLaunchKernelGGL(kern, grid, block, (unsigned)smem, s, e0, e1, 0, (KArgs)args...);
  else hipLaunchKernelGGL(kern, grid, block, (unsigned)smem, s, (KArgs)args...);
}

// ---- launch-side declarations (definitions in the .hip files) ----------------------------------
enum { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2 };
static inline size_t dt_bytes(int dt) { return dt == DT_F32 ? 4 : 2; }
static inline bool dt_is16(int dt) { return dt != DT_F32; }

// Rows of partial column sums that the two-stage column reductions write before their
// finishing pass (fixed, so results do not depend on the launch).
constexpr int kReduceParts = 256;

hipError_t launch_ln_fwd(int dt, const void* x, const void* gamma, const void* beta, void* y, float* mean,
                         float* rstd, int rows, int H, float eps, hipStream_t s);
hipError_t launch_ln_bwd(int dt, const void* dy, const void* x, const float* mean, const float* rstd,
                         const void* gamma, const void* dres, void* dx, float* dgamma, float* dbeta,
                         float* scratch, int rows, int H, hipStream_t s);
// dgamma == nullptr: dx and the partial sums only; launch_ln_bwd_final adds them into dgamma / dbeta later
hipError_t launch_ln_bwd_final(const float* scratch, int rows, int H, float* dgamma, float* dbeta, hipStream_t s);
hipError_t launch_colsum_accum(int dt, const void* dy, float* out, float* scratch, int rows, int N, hipStream_t s);
hipError_t launch_colsum_group(int dt, int n, const void* const* dy, float* const* out, const int* widths, float* scratch,
                               int rows, hipStream_t s);   // up to 4 column sums over the same rows
hipError_t launch_gelu_bwd(int dt, const void* dg, const void* u, void* du, size_t n, hipStream_t s);
hipError_t launch_gelu_fwd(int dt, const void* u, void* g, size_t n, hipStream_t s);   // g = gelu(u), n % 8 == 0
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t s);
hipError_t launch_transpose(int dt, const void* in, void* out, int rows, int cols, hipStream_t s);
// bf16 weight operand B[N][K] of an NT GEMM -> chunk-major [K/32][N][32]; transposed: src holds B^T as [K][N]
hipError_t launch_tile_weights(const void* src, void* dst, int N, int K, bool transposed, hipStream_t s);
hipError_t launch_delay(int64_t ns, hipStream_t s);
hipError_t launch_send_copy(void* dst_device_view_of_host, const void* src, size_t bytes, int blocks, hipStream_t s);
// one device clock reading into *stamp, and a wait until `ns` after that reading (at most `ns` from its own start,
// whatever the stamp holds; at most two seconds)
hipError_t launch_clock_stamp(long long* stamp, hipStream_t s);
hipError_t launch_delay_since(const long long* stamp, int64_t ns, hipStream_t s);

struct GemmArgs {
  int kind, epilogue, M, N, K;
  const void *A, *B, *bias, *residual;
  void *C, *C2;
  float* Cacc;
  bool b_tiled = false;      // NT only: B is stored chunk-major, [K/32][N][32] (see launch_tile_weights)
};
hipError_t launch_gemm_f32(const GemmArgs& g, hipStream_t s);
// 16-bit storage (bf16 or fp16, the same kernels built once per type): NT and TN only
hipError_t launch_gemm_bf16(const GemmArgs& g, hipStream_t s);
hipError_t launch_gemm_f16(const GemmArgs& g, hipStream_t s);
static inline hipError_t launch_gemm_16(int dt, const GemmArgs& g, hipStream_t s) {
  return dt == DT_F16 ? launch_gemm_f16(g, s) : launch_gemm_bf16(g, s);
}
// A W step: every accumulation into the gradients of one block, for a window of up to kWSeg micro-batches
// (segments), in one launch.  Weight gradients: G[M,N] (fp32) += sum over segments A_s[K,M]^T . B_s[K,N], K = tokens
// per micro-batch; the tile starts from G and the products of every token are added on top in token order, so the
// result does not depend on how many micro-batches a launch covers.  The small reductions ride along in the same
// launch: column sums over the token axis of up to four 16-bit matrices dy_s[rows, width] (out[c] += sum_r dy_s[r][c],
// one segment after the other) and the finishing pass of up to two LayerNorm backward reductions (partial rows left
// by launch_ln_bwd called with dgamma == nullptr; ln_parts = ln_bwd_partial_rows(rows, width); out0 += the first
// half of every partial row, out1 += the second).
constexpr int kWSeg = 8;
struct WGrad { int M, N; float* Cacc; const void* A[kWSeg]; const void* B[kWSeg]; };
struct WStepReduce {
  int rows, n_colsum, n_ln;
  const void* dy[4][kWSeg]; float* out[4]; int width[4];
  const float* ln_partial[2][kWSeg]; float* ln_out0[2]; float* ln_out1[2]; int ln_parts[2]; int ln_width[2];
};
// shapes one grouped launch takes: M, N multiples of 128, K a multiple of 32, reduction widths multiples of 64
bool wstep_groupable(const WGrad* g, int n, int K, const WStepReduce* red);
hipError_t launch_wstep_bf16(const WGrad* g, int n, int K, int nseg, hipStream_t s, const WStepReduce* red);
hipError_t launch_wstep_f16(const WGrad* g, int n, int K, int nseg, hipStream_t s, const WStepReduce* red);
static inline hipError_t launch_wstep_16(int dt, const WGrad* g, int n, int K, int nseg, hipStream_t s, const WStepReduce* red) {
  return dt == DT_F16 ? launch_wstep_f16(g, n, K, nseg, s, red) : launch_wstep_bf16(g, n, K, nseg, s, red);
}
int ln_bwd_partial_rows(int rows, int H);        // partial rows launch_ln_bwd leaves in its scratch
size_t colsum_scratch_floats(int rows, int N);   // floats of `scratch` that launch_colsum_accum writes and reads
// fewest 256 x 256 tiles a product must divide into before they are preferred over 128 x 128 tiles
// (kfkb_set_big_tile_min)
extern int g_big_tile_min;
extern int g_mid_tile_mode;      // 128 x 256 tiles for NT products with a chunk-major B: 0 never, 1 where they rate best, 2 wherever they fit
extern int g_mid_tile_rate;      // what such a tile reaches of a 256 x 256 tile's rate, in percent
const char* gemm_bf16_check(const GemmArgs& g);                  // NULL if the shape is supported (either 16-bit type)

hipError_t launch_attention_fwd_f32(const float* qkv, float* o, float* lse, int b, int T, int H, int heads,
                                    int causal, hipStream_t s);
hipError_t launch_attention_bwd_f32(const float* qkv, const float* o, const float* d_o, const float* lse,
                                    float* dsum, float* dqkv, int b, int T, int H, int heads, int causal,
                                    hipStream_t s);
// 16-bit storage: `dt` is DT_BF16 or DT_F16
hipError_t launch_attention_fwd_bf16(const void* qkv, void* o, float* lse, int b, int T, int H, int heads, int causal, hipStream_t s);
hipError_t launch_attention_bwd_bf16(const void* qkv, const void* o, const void* d_o, const float* lse, float* dsum, void* dqkv,
                                     int b, int T, int H, int heads, int causal, hipStream_t s);
hipError_t launch_attention_fwd_f16(const void* qkv, void* o, float* lse, int b, int T, int H, int heads, int causal, hipStream_t s);
hipError_t launch_attention_bwd_f16(const void* qkv, const void* o, const void* d_o, const float* lse, float* dsum, void* dqkv,
                                    int b, int T, int H, int heads, int causal, hipStream_t s);
static inline hipError_t launch_attention_fwd_16(int dt, const void* qkv, void* o, float* lse, int b, int T, int H, int heads,
                                                 int causal, hipStream_t s) {
  return dt == DT_F16 ? launch_attention_fwd_f16(qkv, o, lse, b, T, H, heads, causal, s)
                      : launch_attention_fwd_bf16(qkv, o, lse, b, T, H, heads, causal, s);
}
static inline hipError_t launch_attention_bwd_16(int dt, const void* qkv, const void* o, const void* d_o, const float* lse,
                                                 float* dsum, void* dqkv, int b, int T, int H, int heads, int causal, hipStream_t s) {
  return dt == DT_F16 ? launch_attention_bwd_f16(qkv, o, d_o, lse, dsum, dqkv, b, T, H, heads, causal, s)
                      : launch_attention_bwd_bf16(qkv, o, d_o, lse, dsum, dqkv, b, T, H, heads, causal, s);
}

}  // namespace kfkb
