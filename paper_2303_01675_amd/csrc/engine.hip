// Host side of libkfkb: the process-global stage, the kFkB planner, the transfer engine and the
// C entry points declared in include/kfkb.h.  Every arithmetic step runs in the HIP kernels of the
// other translation units; this file only sequences them on three HIP streams.
#include "common.h"
#include "../../include/kfkb.h"

#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <thread>
#include <vector>

using namespace kfkb;

// ---- per-kernel timing (see common.h) -------------------------------------------------------------
namespace {
struct ProfRec { int key; double work; hipEvent_t e0, e1; };
bool g_prof_on = false;
std::vector<ProfRec> g_prof_recs;
std::vector<hipEvent_t> g_prof_pool;      // events created so far, reused run after run
size_t g_prof_next = 0;

int g_prof_dt = DT_BF16;      // storage type of the stage whose kernels are being timed (names say bf16 or f16)

void prof_key_name_bf16(int key, char* out, size_t cap, int* bound);
void prof_key_name(int key, char* out, size_t cap, int* bound) {
  prof_key_name_bf16(key, out, cap, bound);
  if (g_prof_dt != DT_F16) return;
  for (char* p = strstr(out, "bf16"); p != nullptr; p = strstr(p, "bf16")) memmove(p, p + 1, strlen(p));   // "bf16" -> "f16"
}

void prof_key_name_bf16(int key, char* out, size_t cap, int* bound) {
  static const char* epi[] = {"none", "bias", "bias_gelu", "bias_res", "accum", "gelu_bwd"};
  *bound = 1;
  if (key >= PK_GEMM_NT && key < PK_ATTN_FWD) {
    const bool tn = key >= PK_GEMM_TN;
    const int r = key - (tn ? PK_GEMM_TN : PK_GEMM_NT);
    *bound = 0;
    if (tn && (r == 300 || r == 301)) { snprintf(out, cap, "gemm_bf16_tn_grouped_kernel<%d,%d>", r == 301 ? 256 : 128, r == 301 ? 256 : 128); return; }
    if (!tn && r >= 400) { snprintf(out, cap, "gemm_bf16_nt_kernel<128,256,%s>", epi[r - 400]); return; }
    const bool staged = r >= 200;
    const int tile = (r % 200) >= 100 ? 256 : 128;
    snprintf(out, cap, "gemm_bf16_%s_kernel<%d,%d,%s>", tn ? (staged ? "tn_staged" : "tn") : "nt", tile, tile, epi[r % 100]);
  } else if (key >= PK_ATTN_FWD && key < PK_ATTN_DSUM) {
    const int cls = (key - PK_ATTN_FWD) / 100;
    *bound = 0;
    snprintf(out, cap, "%s<%d>", cls == 0 ? "attn_fwd_bf16_kernel" : cls == 1 ? "attn_bwd_dq_bf16_kernel" : "attn_bwd_dkv_bf16_kernel", (key - PK_ATTN_FWD) % 100 ? 128 : 64);
  } else if (key >= PK_ATTN_DSUM && key < PK_LN_FWD) snprintf(out, cap, "attn_dsum_kernel");
  // forward and dx kernels: key = class + 20 log2(waves per row) + 4 log2(chunks per lane) + (float ? 1 : 0)
  else if (key >= PK_LN_FWD && key < PK_LN_BWD_DX) snprintf(out, cap, "ln_fwd_kernel<%s,%d,%d>", (key & 3) == 1 ? "float" : "bf16", 1 << ((key - PK_LN_FWD) % 20 / 4), 1 << ((key - PK_LN_FWD) / 20));
  else if (key >= PK_LN_BWD_DX && key < PK_LN_BWD_DX + 80) snprintf(out, cap, "ln_bwd_dx_kernel<%s,%d,%d>", (key & 3) == 1 ? "float" : "bf16", 1 << ((key - PK_LN_BWD_DX) % 20 / 4), 1 << ((key - PK_LN_BWD_DX) / 20));
  else if (key >= PK_LN_BWD_DX + 80 && key < PK_COLSUM) snprintf(out, cap, "ln_bwd_fused_kernel<%s,%d>", (key & 3) == 1 ? "float" : "bf16", (key - PK_LN_BWD_DX - 80) / 4);
  else if (key == PK_COLSUM + 10 || key == PK_COLSUM + 12) snprintf(out, cap, "colsum_group_partial_kernel<%s>", key == PK_COLSUM + 12 ? "float" : "bf16");
  else if (key == PK_COLSUM_FINAL + 1) snprintf(out, cap, "colsum_group_final_kernel");
  else if (key >= PK_COLSUM && key < PK_COLSUM_XHAT) snprintf(out, cap, "colsum_partial_kernel<%s,false>", key - PK_COLSUM == 4 ? "float" : "bf16");
  else if (key >= PK_COLSUM_XHAT && key < PK_COLSUM_FINAL) snprintf(out, cap, "colsum_partial_kernel<%s,true>", key - PK_COLSUM_XHAT == 4 ? "float" : "bf16");
  else if (key == PK_COLSUM_FINAL) snprintf(out, cap, "colsum_final_kernel");
  else if (key >= PK_GELU_BWD + 10 && key < PK_GEMM_F32) snprintf(out, cap, "gelu_fwd_kernel<%s>", key - PK_GELU_BWD == 14 ? "float" : "bf16");
  else if (key >= PK_GELU_BWD && key < PK_GEMM_F32) snprintf(out, cap, "gelu_bwd_kernel<%s>", key - PK_GELU_BWD == 4 ? "float" : "bf16");
  else if (key >= PK_GEMM_F32 && key < PK_ATTN_F32) { *bound = 2; snprintf(out, cap, "gemm_f32_kernel<%s>", epi[key - PK_GEMM_F32]); }
  else snprintf(out, cap, "kernel_%d", key);
}
}  // namespace

namespace kfkb {
int g_big_tile_min = 192;
int g_mid_tile_mode = 1;
int g_mid_tile_rate = 90;
bool prof_acquire(int key, double work, hipEvent_t* e0, hipEvent_t* e1) {
  if (!g_prof_on) return false;
  while (g_prof_pool.size() < g_prof_next + 2) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return false;
    g_prof_pool.push_back(e);
  }
  *e0 = g_prof_pool[g_prof_next++];
  *e1 = g_prof_pool[g_prof_next++];
  g_prof_recs.push_back(ProfRec{key, work, *e0, *e1});
  return true;
}
}  // namespace kfkb

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

}  // namespace

namespace kfkb {
int set_error(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
}  // namespace kfkb

namespace {

#define HIPCHK(expr)                                                                                   \
  do {                                                                                                 \
    hipError_t e_ = (expr);                                                                            \
    if (e_ != hipSuccess) return fail(KFKB_E_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));      \
  } while (0)

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// ---- planning (host only) ----------------------------------------------------------------------
// Group-level state machine: fill w forward groups, then alternate one forward group with the oldest
// pending backward group, then drain.  Inside a group micro-batches ascend.
int build_order(int k, int M, int w, std::vector<kfkb_op_t>& out) {
  out.clear();
  const int G = (M + k - 1) / k;
  w = std::min(w, G);
  int fg = 0, bg = 0;
  auto emit = [&](int op, int g) {
    for (int mb = g * k; mb < std::min(M, (g + 1) * k); mb++) out.push_back(kfkb_op_t{op, mb, 0.0, 0.0});
  };
  while (bg < G) {
    if (fg < G && fg - bg < w) {
      emit(KFKB_OP_F, fg++);
    } else if (fg < G) {
      emit(KFKB_OP_F, fg++);
      emit(KFKB_OP_B, bg++);
    } else {
      emit(KFKB_OP_B, bg++);
    }
  }
  return (int)out.size();
}

int peak_live_of(const std::vector<kfkb_op_t>& order) {
  int live = 0, peak = 0;
  for (const auto& o : order) {
    live += o.op == KFKB_OP_F ? 1 : -1;
    peak = std::max(peak, live);
  }
  return peak;
}

// Receive list of a plan: the order the receive stream is fed in (it is FIFO, so this fixes which transfer waits
// behind which).  Two orders:
//   consumption order   the plan's own op order: the upstream gradients of a schedule unit come before the inputs of
//                       the next forward unit, which then arrive while the unit's backwards run.  With k >= 2 this is
//                       the better one under delay: a backward unit never waits behind k input transfers, and the
//                       inputs are still early (measured: very wide stage, 15 ms per transfer, k = 8: 2.36 s against
//                       2.96 s per iteration).
//   inputs ahead        every forward unit moved ahead of the backward unit before it (the upstream neighbour sends
//                       one schedule unit ahead).  With k = 1 a unit is one micro-batch, and the next input then
//                       arrives while the current forward runs and its output travels, so that on two compute lanes
//                       F(mb+1) can run beside B(mb).
// mode: 0 consumption order, 1 inputs ahead, 2 (default) inputs ahead exactly for k = 1.
int g_inputs_ahead_mode = 2;
bool inputs_ahead_for(int k) { return g_inputs_ahead_mode == 2 ? k == 1 : g_inputs_ahead_mode != 0; }

void build_receive_plan(const std::vector<kfkb_op_t>& order, int k, std::vector<kfkb_op_t>& plan) {
  if (!inputs_ahead_for(k)) { plan = order; return; }
  std::vector<std::vector<kfkb_op_t>> units;
  for (const auto& o : order) {
    if (!units.empty() && units.back().back().op == o.op) units.back().push_back(o);
    else units.push_back({o});
  }
  for (size_t i = 0; i + 1 < units.size();) {
    if (units[i][0].op == KFKB_OP_B && units[i + 1][0].op == KFKB_OP_F) {
      std::swap(units[i], units[i + 1]);
      i += 2;
    } else {
      i += 1;
    }
  }
  plan.clear();
  for (const auto& u : units) plan.insert(plan.end(), u.begin(), u.end());
}

// ---- the stage ---------------------------------------------------------------------------------
struct BlockParams {          // element offsets inside one block's parameter run
  size_t ln1_g, ln1_b, w_qkv, b_qkv, w_o, b_o, ln2_g, ln2_b, w_1, b_1, w_2, b_2, total;
};

struct MbState {
  int x_slot = -1, dy_slot = -1, stash = -1, y_buf = -1, dx_buf = -1;
  bool x_issued = false, dy_issued = false, fwd_begun = false, fwd_done = false, bwd_begun = false, bwd_done = false;
};

struct Pool {                 // device buffers handed round between transfers and compute
  std::vector<char*> buf;
  std::vector<hipEvent_t> release;   // event after which the buffer may be overwritten (or null)
  std::vector<int> free_list;
  // all buffers free again; release events are kept, so work of an earlier iteration that still reads
  // or sends a buffer is waited for before the buffer is overwritten
  void reset() { free_list.clear(); for (int i = (int)buf.size() - 1; i >= 0; i--) free_list.push_back(i); }
  int take() { if (free_list.empty()) return -1; int s = free_list.back(); free_list.pop_back(); return s; }
  void give(int s, hipEvent_t ev) { release[s] = ev; free_list.insert(free_list.begin(), s); }
};

struct Stage {
  bool inited = false, bound = false;
  kfkb_config_t cfg{};
  int dt = 0, L = 0, H = 0, heads = 0, d = 0, T = 0, b = 0, F = 0, m = 0, Mmax = 0;
  size_t n = 0, esz = 4;
  BlockParams po{};
  const char* weights = nullptr;
  float* grad = nullptr;
  const char* h_in = nullptr; const char* h_up = nullptr; char* h_out = nullptr; char* h_ingrad = nullptr;
  char* d_out = nullptr; char* d_ingrad = nullptr;           // the device's view of the two pinned output arrays (null: none)
  int send_blocks = 8;                                        // > 0: sends go through the library's copy kernel with that many workgroups
  // workspace carve-up
  char* ws = nullptr; size_t ws_bytes = 0; int k_bound = 0; int n_stash = 0;
  char* wt = nullptr;                        // bf16 only: weight matrices stored [out, in]
  std::vector<char*> stash; std::vector<int> stash_free;
  Pool xs, dys, ys, dxs;
  size_t stash_block_bytes = 0, stash_bytes = 0;
  // Compute lanes.  Ops are admitted in schedule order; up to `lanes` of them are in flight, each on its lane's
  // stream, and their blocks are enqueued in turn, so that independent micro-batches fill each other's idle
  // phases (launch gaps, memory-bound epilogues and row kernels, partly filled last rounds of tiles).
  // The weight and bias gradients of a block (its "W step") go to the OTHER lane's stream when
  // wgrad_overlap is set, and run beside the op's own chain of input gradients.
  // Per-lane backward scratch: t_n0 (dc, d_o, da in turn); dx1, du, dqkv and the LayerNorm partial sums alternate
  // between two buffers and the block input gradient rotates over three, so that the W step of a block can still
  // read them while the next block's chain runs (the chain waits for it two blocks later).
  static constexpr int kRing = 8;
  struct Lane {
    hipStream_t s = nullptr;
    char* t_n0 = nullptr; char* t_dx1[2] = {nullptr, nullptr}; char* t_dxr[3] = {nullptr, nullptr, nullptr};
    char* t_mf[2] = {nullptr, nullptr}; char* t_3n[2] = {nullptr, nullptr};
    float* dsum = nullptr; float* red_ln[2][2] = {{nullptr, nullptr}, {nullptr, nullptr}}; float* red_w[2] = {nullptr, nullptr};
    // recompute only: forward temporaries (a, c, g) and the backward's recomputed copies, two of each like du
    char* f_a = nullptr; char* f_c = nullptr; char* f_g = nullptr;
    char* r_a[2] = {nullptr, nullptr}; char* r_c[2] = {nullptr, nullptr}; char* r_g[2] = {nullptr, nullptr};
    hipEvent_t ev_chain[kRing] = {}, ev_wdone[kRing] = {};   // per block of a backward pass, reused round-robin
    bool w_elsewhere[kRing] = {};                            // that block's W step ran on the other lane's stream
    uint64_t seq = 0;                                        // blocks of backward passes issued on this lane
    hipEvent_t ev_tail = nullptr;
  };
  Lane lane[2];
  // W-step windows (16-bit stages whose shapes take the grouped launch): the backwards of one schedule unit run
  // back to back, so the gradient accumulation of a block is done ONCE for up to kWSeg of them: their operands are
  // kept in a pool [window position][block] and the W step of block l is launched when the last of them has passed
  // block l.  The fp32 gradients are then read and written once per window instead of once per micro-batch, and
  // the matrix pipes work through a k times longer token axis per tile.  The result is the same bit for bit
  // whatever the window (see launch_wstep_16).  Activation slots and input slots of a window's micro-batches go
  // back to their pools when its last W step has been enqueued.  Not with activation recomputation: the recomputed
  // LayerNorm and GELU outputs would have to be kept for the whole window, which is the memory that mode is there to
  // save; every backward then accumulates by itself.
  struct WOps { char *du = nullptr, *dqkv = nullptr, *dx1 = nullptr, *dx = nullptr; float* ln[2] = {nullptr, nullptr}; };
  struct Deferred { int stash, x_slot, dy_slot; };
  bool wstep_grouped = false;                                // the stage's W steps take the grouped launch
  int wwin_cap = 1;                                          // window positions the bound workspace holds
  int wwin_max = kWSeg;                                      // stage_set_wstep_window
  std::vector<WOps> wpool;                                   // [position * L + block]
  std::vector<hipEvent_t> ev_wops;                           // [position * L + block]: that chain has written its operands
  std::vector<int> w_arrived;                                // per block: chains of the open window enqueued so far
  std::vector<Deferred> w_deferred;                          // slots of the open window's finished micro-batches
  bool w_open = false;                                       // a window has been opened and its last W step is not enqueued yet
  int w_size = 0, w_mbs[kWSeg] = {};                         // the open window: its micro-batches in backward order
  hipEvent_t ev_wlast = nullptr;                             // the most recent W step (they are chained, so: all of them)
  int lanes = 2;
  bool wgrad_overlap = true;
  // cfg.recompute: the LayerNorm outputs a, c and the GELU output g are not stashed; a forward keeps them in
  // per-lane temporaries, a backward forms them again from x, x1 and u (same kernels, same bits)
  bool recompute = false;
  bool fuse_w_reductions = true;   // false (stage_set_fused_w_reductions): the W step's small reductions as launches of their own
  hipStream_t ss = nullptr, sr = nullptr;
  std::vector<hipEvent_t> ev_g;                            // per block: last accumulation into its gradients
  std::vector<char> ev_g_set;
  hipEvent_t ev_zero = nullptr;
  hipEvent_t last_done = nullptr;                          // end of the most recent backward op, W steps included
  std::vector<hipEvent_t> ev_w;                            // per micro-batch: its last W step is done
  std::vector<hipEvent_t> stash_release;                   // per activation slot: last reader (or null)
  std::vector<hipEvent_t> ev_x, ev_dy, ev_f0, ev_f1, ev_b0, ev_b1, ev_ys, ev_dxs;
  std::vector<hipEvent_t> ev_t0[4];                        // start of the transfer of each direction and micro-batch
  bool adaptive_pending = false;                           // an iteration of run_kFkB_adaptive has not been observed yet
  hipEvent_t ev_epoch = nullptr, ev_run_end = nullptr;
  bool epoch_valid = false, run_timed = false;
  std::vector<int64_t> dl_x, dl_dy, dl_y, dl_dx;
  std::vector<MbState> mb;
  struct LogEntry { int op, mb; };
  std::vector<LogEntry> log;
  int last_k = 0;
};

Stage g;
kfkb_config_t g_cfg_pending{};
bool g_cfg_set = false;

size_t stash_block_bytes_of(const Stage& s) {
  // a, qkv(3), o, x1, c, y : 8 n ; u, g : 2 m F ; LN statistics 4 m floats ; lse b*heads*T floats
  // with recomputation a, c and g are not kept: 6 n and m F
  const size_t elems = s.recompute ? 6 * s.n + (size_t)s.m * s.F : 8 * s.n + 2 * (size_t)s.m * s.F;
  return align_up(elems * s.esz) + align_up((4 * (size_t)s.m + (size_t)s.b * s.heads * s.T) * 4);
}

int warmup_for(const Stage& s, int k, int M) {
  const int S = std::max(1, s.cfg.num_stages);
  const int G = (M + k - 1) / k;
  return std::min(std::max(0, S - 1 - s.cfg.stage_index), G);
}

int peak_live_for(const Stage& s, int k, int M) {
  return std::min((warmup_for(s, k, M) + 1) * k, M);
}

// scratch of the column reductions, in floats: bias gradients of a block side by side (64 parts x 2 slots x
// (F + 5 H)); LayerNorm parameter gradients (at most 512 parts x 2 slots x H), kept for the deferred finishing pass
size_t red_w_floats(const Stage& s) { return (size_t)128 * (s.F + 5 * (size_t)s.H); }
size_t red_ln_floats(const Stage& s) { return (size_t)1024 * s.H; }

struct LaneCarve { size_t tn, tmf, t3n, dsum, red_ln, red_w, rec, total; };
LaneCarve lane_carve(const Stage& s) {
  LaneCarve c{};
  const size_t act = align_up(s.n * s.esz);
  size_t off = 0;
  c.tn = off; off += 6 * act;
  c.tmf = off; off += 2 * align_up((size_t)s.m * s.F * s.esz);
  c.t3n = off; off += 2 * align_up(3 * s.n * s.esz);
  c.dsum = off; off += align_up((size_t)s.b * s.heads * s.T * 4);
  c.red_ln = off; off += 4 * align_up(red_ln_floats(s) * 4);
  c.red_w = off; off += 2 * align_up(red_w_floats(s) * 4);
  c.rec = off;
  if (s.recompute) off += 3 * (2 * act + align_up((size_t)s.m * s.F * s.esz));      // forward temporaries + two backward sets
  c.total = off;
  return c;
}

struct Carve { size_t wt, stash, xs, dys, ys, dxs, lanes, wpool, total; int n_stash, n_x, n_io, wwin; };

// bytes of one (window position, block) entry of the W-step operand pool
struct WOpsCarve { size_t du, dqkv, dx1, dx, ln, total; };
WOpsCarve wops_carve(const Stage& s) {
  WOpsCarve c{};
  const size_t act = align_up(s.n * s.esz);
  size_t off = 0;
  c.du = off; off += align_up((size_t)s.m * s.F * s.esz);
  c.dqkv = off; off += align_up(3 * s.n * s.esz);
  c.dx1 = off; off += act;
  c.dx = off; off += act;
  c.ln = off; off += 2 * align_up(red_ln_floats(s) * 4);
  c.total = off;
  return c;
}

Carve carve_for(const Stage& s, int k_max) {
  Carve c{};
  const int live = peak_live_for(s, k_max, s.Mmax);
  c.n_stash = live; c.n_x = std::min(live + k_max, std::max(s.Mmax, 1)) ; c.n_io = std::min(2 * k_max, std::max(s.Mmax, 1));
  const size_t act = align_up(s.n * s.esz);
  size_t off = 0;
  c.wt = off;
  if (dt_is16(s.dt)) off += align_up((size_t)2 * s.L * ((size_t)4 * s.H * s.H + 2 * (size_t)s.H * s.F) * 2);
  c.stash = off; off += (size_t)c.n_stash * s.L * stash_block_bytes_of(s);
  c.xs = off; off += (size_t)c.n_x * act;
  c.dys = off; off += (size_t)c.n_io * act;
  c.ys = off; off += (size_t)c.n_io * act;
  c.dxs = off; off += (size_t)c.n_io * act;
  c.lanes = off; off += 2 * lane_carve(s).total;
  c.wwin = (s.wstep_grouped && !s.recompute && k_max >= 2) ? std::min(k_max, kWSeg) : 1;
  c.wpool = off;
  if (c.wwin >= 2) off += (size_t)c.wwin * s.L * wops_carve(s).total;
  c.total = off;
  return c;
}

inline const char* wptr(const Stage& s, int l, size_t off) { return s.weights + ((size_t)l * s.po.total + off) * s.esz; }
inline float* gptr(const Stage& s, int l, size_t off) { return s.grad + (size_t)l * s.po.total + off; }

// pointers into one (slot, block) of the stash
struct StashView { char *a, *qkv, *o, *x1, *c, *y, *u, *gact; float *mean1, *rstd1, *mean2, *rstd2, *lse; };
StashView view(const Stage& s, int slot, int l) {
  char* p = s.stash[slot] + (size_t)l * s.stash_block_bytes;
  const size_t nb = s.n * s.esz, fb = (size_t)s.m * s.F * s.esz;
  StashView v;
  float* st;
  if (s.recompute) {                                   // a, c, gact: the caller's temporaries
    v.a = nullptr; v.c = nullptr; v.gact = nullptr;
    v.qkv = p; v.o = p + 3 * nb; v.x1 = p + 4 * nb; v.y = p + 5 * nb; v.u = p + 6 * nb;
    st = reinterpret_cast<float*>(p + align_up(6 * nb + fb));
  } else {
    v.a = p; v.qkv = p + nb; v.o = p + 4 * nb; v.x1 = p + 5 * nb; v.c = p + 6 * nb; v.y = p + 7 * nb;
    v.u = p + 8 * nb; v.gact = p + 8 * nb + fb;
    st = reinterpret_cast<float*>(p + align_up(8 * nb + 2 * fb));
  }
  v.mean1 = st; v.rstd1 = st + s.m; v.mean2 = st + 2 * s.m; v.rstd2 = st + 3 * s.m; v.lse = st + 4 * (size_t)s.m;
  return v;
}

// chunk-major copies of the weight matrices of block l (bf16), as the B operand of the NT GEMMs:
// forward products read W^T (B[N = out][K = in]), input-gradient products read W (B[N = in][K = out])
struct WtView { const char *qkv, *o, *w1, *w2, *qkv_d, *o_d, *w1_d, *w2_d; };
WtView wt_view(const Stage& s, int l) {
  const size_t H = s.H, F = s.F;
  const size_t per = (3 * H * H + H * H + 2 * H * F) * 2;
  const char* p = s.wt + (size_t)l * 2 * per;
  const char* d = p + per;
  return WtView{p, p + 3 * H * H * 2, p + 4 * H * H * 2, p + (4 * H * H + H * F) * 2,
                d, d + 3 * H * H * 2, d + 4 * H * H * 2, d + (4 * H * H + H * F) * 2};
}

int gemm(const Stage& s, hipStream_t st, int kind, int epi, int M, int N, int K, const void* A, const void* B, const void* bias,
         const void* res, void* C, void* C2, float* Cacc, bool b_tiled = false) {
  GemmArgs a{kind, epi, M, N, K, A, B, bias, res, C, C2, Cacc};
  a.b_tiled = b_tiled;
  if (dt_is16(s.dt)) {
    const char* why = gemm_bf16_check(a);
    if (why) return fail(KFKB_E_ARG, "%s (M=%d N=%d K=%d)", why, M, N, K);
    HIPCHK(launch_gemm_16(s.dt, a, st));
  } else {
    HIPCHK(launch_gemm_f32(a, st));
  }
  return 0;
}

// forward linear map y = x W + b (+ epilogue): fp32 reads W [in,out] as given, bf16 reads the [out,in] copy
int linear_fwd(const Stage& s, hipStream_t st, int epi, int in, int out, const void* x, const void* W, const void* Wt, const void* bias,
               const void* res, void* y, void* y2) {
  if (dt_is16(s.dt)) return gemm(s, st, KFKB_GEMM_NT, epi, s.m, out, in, x, Wt, bias, res, y, y2, nullptr, true);
  return gemm(s, st, KFKB_GEMM_NN, epi, s.m, out, in, x, W, bias, res, y, y2, nullptr);
}

int refresh_weights() {
  if (!dt_is16(g.dt)) return 0;
  hipStream_t st = g.lane[0].s;
  for (int l = 0; l < g.L; l++) {
    WtView w = wt_view(g, l);
    // W is stored [in, out]: forward B = W^T has N = out, K = in; input-gradient B = W has N = in, K = out
    HIPCHK(launch_tile_weights(wptr(g, l, g.po.w_qkv), (void*)w.qkv, 3 * g.H, g.H, true, st));
    HIPCHK(launch_tile_weights(wptr(g, l, g.po.w_o), (void*)w.o, g.H, g.H, true, st));
    HIPCHK(launch_tile_weights(wptr(g, l, g.po.w_1), (void*)w.w1, g.F, g.H, true, st));
    HIPCHK(launch_tile_weights(wptr(g, l, g.po.w_2), (void*)w.w2, g.H, g.F, true, st));
    HIPCHK(launch_tile_weights(wptr(g, l, g.po.w_qkv), (void*)w.qkv_d, g.H, 3 * g.H, false, st));
    HIPCHK(launch_tile_weights(wptr(g, l, g.po.w_o), (void*)w.o_d, g.H, g.H, false, st));
    HIPCHK(launch_tile_weights(wptr(g, l, g.po.w_1), (void*)w.w1_d, g.H, g.F, false, st));
    HIPCHK(launch_tile_weights(wptr(g, l, g.po.w_2), (void*)w.w2_d, g.F, g.H, false, st));
  }
  return 0;
}

int attention_fwd(const Stage& s, hipStream_t st, const void* qkv, void* o, float* lse) {
  if (dt_is16(s.dt)) HIPCHK(launch_attention_fwd_16(s.dt, qkv, o, lse, s.b, s.T, s.H, s.heads, s.cfg.causal, st));
  else HIPCHK(launch_attention_fwd_f32((const float*)qkv, (float*)o, lse, s.b, s.T, s.H, s.heads, s.cfg.causal, st));
  return 0;
}
int attention_bwd(const Stage& s, hipStream_t st, const void* qkv, const void* o, const void* d_o, const float* lse, float* dsum, void* dqkv) {
  if (dt_is16(s.dt))
    HIPCHK(launch_attention_bwd_16(s.dt, qkv, o, d_o, lse, dsum, dqkv, s.b, s.T, s.H, s.heads, s.cfg.causal, st));
  else
    HIPCHK(launch_attention_bwd_f32((const float*)qkv, (const float*)o, (const float*)d_o, lse, dsum, (float*)dqkv, s.b, s.T, s.H, s.heads, s.cfg.causal, st));
  return 0;
}

#define TRY(expr) do { int rc_ = (expr); if (rc_ != 0) return rc_; } while (0)

// ---- the stage computation, one block at a time ------------------------------------------------
// An op in flight: forward (blocks 0 .. L-1) or backward (blocks L-1 .. 0) of one micro-batch on one lane.
struct ActiveOp {
  int op = 0, mb = 0, lane = 0, next = 0, left = 0;
  bool other_busy = false;        // the other lane has an op in flight (set by whoever enqueues the blocks)
  hipStream_t w_stream = nullptr; // where W steps of this op went, if not to the op's own stream
  int out_buf = -1;               // Y buffer (forward) or dX buffer (backward)
  const char* cur = nullptr;      // forward: input of the next block; backward: output gradient of the next block
  // an op over blocks [first, ...) of a stage that has been cut into virtual stages: where the input of block
  // `first` lies and where the gradient with respect to it goes (null: the stage's own rule)
  int first = 0;
  const char* x_first = nullptr;
  char* dx_first = nullptr;
  // backward op that belongs to a W-step window of wsize >= 2 micro-batches, at position wpos (0: none)
  int wpos = 0, wsize = 0;
};

int forward_block(ActiveOp& a) {
  const Stage& s = g;
  const MbState& st = s.mb[a.mb];
  hipStream_t q = s.lane[a.lane].s;
  const int l = a.next;
  StashView v = view(s, st.stash, l);
  WtView w = dt_is16(s.dt) ? wt_view(s, l) : WtView{};
  const char* x = a.cur;
  char* y = (l == s.L - 1) ? s.ys.buf[a.out_buf] : v.y;
  if (s.recompute) { const Stage::Lane& ln = s.lane[a.lane]; v.a = ln.f_a; v.c = ln.f_c; v.gact = ln.f_g; }
  HIPCHK(launch_ln_fwd(s.dt, x, wptr(s, l, s.po.ln1_g), wptr(s, l, s.po.ln1_b), v.a, v.mean1, v.rstd1, s.m, s.H, s.cfg.ln_eps, q));
  TRY(linear_fwd(s, q, KFKB_EPI_BIAS, s.H, 3 * s.H, v.a, wptr(s, l, s.po.w_qkv), w.qkv, wptr(s, l, s.po.b_qkv), nullptr, v.qkv, nullptr));
  TRY(attention_fwd(s, q, v.qkv, v.o, v.lse));
  TRY(linear_fwd(s, q, KFKB_EPI_BIAS_RES, s.H, s.H, v.o, wptr(s, l, s.po.w_o), w.o, wptr(s, l, s.po.b_o), x, v.x1, nullptr));
  HIPCHK(launch_ln_fwd(s.dt, v.x1, wptr(s, l, s.po.ln2_g), wptr(s, l, s.po.ln2_b), v.c, v.mean2, v.rstd2, s.m, s.H, s.cfg.ln_eps, q));
  TRY(linear_fwd(s, q, KFKB_EPI_BIAS_GELU, s.H, s.F, v.c, wptr(s, l, s.po.w_1), w.w1, wptr(s, l, s.po.b_1), nullptr, v.u, v.gact));
  TRY(linear_fwd(s, q, KFKB_EPI_BIAS_RES, s.F, s.H, v.gact, wptr(s, l, s.po.w_2), w.w2, wptr(s, l, s.po.b_2), v.x1, y, nullptr));
  a.cur = y;
  a.next++; a.left--;
  return 0;
}

// The W step of block l for `nseg` micro-batches (their operands in ops[0 .. nseg-1], in backward order) on stream
// qw: weight gradients, bias column sums and the LayerNorm-parameter finishing pass.  Grouped stages do it in one
// launch; otherwise (fp32, shapes the grouped launch does not take) one micro-batch at a time with the plain kernels.
struct WOperands { const void *a, *c, *o, *gact, *dqkv, *du, *dx1, *dy; const float* ln1; const float* ln2; float* red_w; };

int launch_w_step(Stage& s, int l, const WOperands* ops, int nseg, hipStream_t qw) {
  const int widths[4] = {3 * s.H, s.F, s.H, s.H};
  float* bias_out[4] = {gptr(s, l, s.po.b_qkv), gptr(s, l, s.po.b_1), gptr(s, l, s.po.b_2), gptr(s, l, s.po.b_o)};
  if (s.wstep_grouped) {
    WGrad wg[4] = {};
    // order of the group: qkv, fc1, fc2, proj (as the chain produces their operands last to first)
    const int wm[4] = {s.H, s.H, s.F, s.H}, wn[4] = {3 * s.H, s.F, s.H, s.H};
    float* wacc[4] = {gptr(s, l, s.po.w_qkv), gptr(s, l, s.po.w_1), gptr(s, l, s.po.w_2), gptr(s, l, s.po.w_o)};
    WStepReduce red{};
    red.rows = s.m; red.n_colsum = 4; red.n_ln = 2;
    for (int i = 0; i < 4; i++) { wg[i].M = wm[i]; wg[i].N = wn[i]; wg[i].Cacc = wacc[i]; red.out[i] = bias_out[i]; red.width[i] = widths[i]; }
    for (int sg = 0; sg < nseg; sg++) {
      const WOperands& o = ops[sg];
      wg[0].A[sg] = o.a; wg[0].B[sg] = o.dqkv;
      wg[1].A[sg] = o.c; wg[1].B[sg] = o.du;
      wg[2].A[sg] = o.gact; wg[2].B[sg] = o.dy;
      wg[3].A[sg] = o.o; wg[3].B[sg] = o.dx1;
      red.dy[0][sg] = o.dqkv; red.dy[1][sg] = o.du; red.dy[2][sg] = o.dy; red.dy[3][sg] = o.dx1;
      red.ln_partial[0][sg] = o.ln2; red.ln_partial[1][sg] = o.ln1;     // partial rows: [sum dy | sum dy * xhat] -> beta, gamma
    }
    red.ln_out0[0] = gptr(s, l, s.po.ln2_b); red.ln_out1[0] = gptr(s, l, s.po.ln2_g);
    red.ln_out0[1] = gptr(s, l, s.po.ln1_b); red.ln_out1[1] = gptr(s, l, s.po.ln1_g);
    red.ln_parts[0] = red.ln_parts[1] = ln_bwd_partial_rows(s.m, s.H);
    red.ln_width[0] = red.ln_width[1] = s.H;
    HIPCHK(launch_wstep_16(s.dt, wg, 4, s.m, nseg, qw, s.fuse_w_reductions ? &red : nullptr));
    if (!s.fuse_w_reductions) {
      for (int sg = 0; sg < nseg; sg++) {                          // the same sums, one micro-batch after the other
        const WOperands& o = ops[sg];
        const void* srcs[4] = {o.dqkv, o.du, o.dy, o.dx1};
        HIPCHK(launch_ln_bwd_final(o.ln2, s.m, s.H, gptr(s, l, s.po.ln2_g), gptr(s, l, s.po.ln2_b), qw));
        HIPCHK(launch_ln_bwd_final(o.ln1, s.m, s.H, gptr(s, l, s.po.ln1_g), gptr(s, l, s.po.ln1_b), qw));
        HIPCHK(launch_colsum_group(s.dt, 4, srcs, bias_out, widths, o.red_w, s.m, qw));
      }
    }
    return 0;
  }
  for (int sg = 0; sg < nseg; sg++) {
    const WOperands& o = ops[sg];
    const GemmArgs wg[4] = {
        GemmArgs{KFKB_GEMM_TN, KFKB_EPI_ACCUM, s.H, 3 * s.H, s.m, o.a, o.dqkv, nullptr, nullptr, nullptr, nullptr, gptr(s, l, s.po.w_qkv)},
        GemmArgs{KFKB_GEMM_TN, KFKB_EPI_ACCUM, s.H, s.F, s.m, o.c, o.du, nullptr, nullptr, nullptr, nullptr, gptr(s, l, s.po.w_1)},
        GemmArgs{KFKB_GEMM_TN, KFKB_EPI_ACCUM, s.F, s.H, s.m, o.gact, o.dy, nullptr, nullptr, nullptr, nullptr, gptr(s, l, s.po.w_2)},
        GemmArgs{KFKB_GEMM_TN, KFKB_EPI_ACCUM, s.H, s.H, s.m, o.o, o.dx1, nullptr, nullptr, nullptr, nullptr, gptr(s, l, s.po.w_o)}};
    for (int i = 0; i < 4; i++) {
      if (dt_is16(s.dt)) {
        const char* why = gemm_bf16_check(wg[i]);
        if (why) return fail(KFKB_E_ARG, "%s (M=%d N=%d K=%d)", why, wg[i].M, wg[i].N, wg[i].K);
        HIPCHK(launch_gemm_16(s.dt, wg[i], qw));
      } else {
        HIPCHK(launch_gemm_f32(wg[i], qw));
      }
    }
    const void* srcs[4] = {o.dqkv, o.du, o.dy, o.dx1};
    HIPCHK(launch_ln_bwd_final(o.ln2, s.m, s.H, gptr(s, l, s.po.ln2_g), gptr(s, l, s.po.ln2_b), qw));
    HIPCHK(launch_ln_bwd_final(o.ln1, s.m, s.H, gptr(s, l, s.po.ln1_g), gptr(s, l, s.po.ln1_b), qw));
    HIPCHK(launch_colsum_group(s.dt, 4, srcs, bias_out, widths, o.red_w, s.m, qw));
  }
  return 0;
}

int backward_block(ActiveOp& a) {
  Stage& s = g;
  const MbState& st = s.mb[a.mb];
  Stage::Lane& ln = s.lane[a.lane];
  hipStream_t q = ln.s;
  const int l = a.next;
  const bool windowed = a.wsize >= 2;
  const uint64_t seq = ln.seq++;
  const int par = (int)(seq & 1), ring = (int)(seq % Stage::kRing);
  // where this block's W-step operands go: the window's pool entry, or the lane's alternating buffers
  Stage::WOps* wp = windowed ? &s.wpool[(size_t)a.wpos * s.L + l] : nullptr;
  char* du = windowed ? wp->du : ln.t_mf[par];
  char* dqkv = windowed ? wp->dqkv : ln.t_3n[par];
  char* dx1 = windowed ? wp->dx1 : ln.t_dx1[par];
  float* red_ln2 = windowed ? wp->ln[1] : ln.red_ln[par][1];
  float* red_ln1 = windowed ? wp->ln[0] : ln.red_ln[par][0];
  char* dc = ln.t_n0;
  char* d_o = ln.t_n0;           // dc is dead once dx1 exists
  char* da = ln.t_n0;            // d_o is dead once dqkv exists
  const char* dy = a.cur;
  StashView v = view(s, st.stash, l);
  const bool bt = dt_is16(s.dt);                        // 16-bit input-gradient products read the chunk-major copies
  WtView w = bt ? wt_view(s, l) : WtView{};
  const char* x = (l == 0) ? s.xs.buf[st.x_slot] : (a.x_first != nullptr && l == a.first) ? a.x_first : view(s, st.stash, l - 1).y;
  char* dx = (l == 0) ? s.dxs.buf[a.out_buf] : (a.dx_first != nullptr && l == a.first) ? a.dx_first : windowed ? wp->dx : ln.t_dxr[seq % 3];
  // where the W step of this block goes: the other lane's stream, beside this chain, when that lane has nothing
  // of its own to do; behind the chain otherwise (the other lane's op then fills the chip beside it).  A window's
  // W step follows the chain of whichever of its micro-batches passes the block last.
  hipStream_t qw = (windowed || !s.wgrad_overlap) ? q : !a.other_busy ? s.lane[1 - a.lane].s : q;
  // the buffers about to be overwritten were last read by the W step of two blocks ago
  if (!windowed && seq >= 2 && ln.w_elsewhere[(seq - 2) % Stage::kRing]) HIPCHK(hipStreamWaitEvent(q, ln.ev_wdone[(seq - 2) % Stage::kRing], 0));
  if (s.recompute) {
    // what the forward did not keep: LayerNorm outputs from the kept inputs (the statistics come out as they were),
    // GELU output from the kept pre-activation
    v.a = ln.r_a[par]; v.c = ln.r_c[par]; v.gact = ln.r_g[par];        // (no windows with recomputation)
    HIPCHK(launch_ln_fwd(s.dt, x, wptr(s, l, s.po.ln1_g), wptr(s, l, s.po.ln1_b), v.a, v.mean1, v.rstd1, s.m, s.H, s.cfg.ln_eps, q));
    HIPCHK(launch_ln_fwd(s.dt, v.x1, wptr(s, l, s.po.ln2_g), wptr(s, l, s.po.ln2_b), v.c, v.mean2, v.rstd2, s.m, s.H, s.cfg.ln_eps, q));
    HIPCHK(launch_gelu_fwd(s.dt, v.u, v.gact, (size_t)s.m * s.F, q));
  }
  // y = x1 + g W2 + b2
  TRY(gemm(s, q, KFKB_GEMM_NT, KFKB_EPI_GELU_BWD, s.m, s.F, s.H, dy, bt ? w.w2_d : wptr(s, l, s.po.w_2), nullptr, v.u, du, nullptr, nullptr, bt));
  // u = c W1 + b1
  TRY(gemm(s, q, KFKB_GEMM_NT, KFKB_EPI_NONE, s.m, s.H, s.F, du, bt ? w.w1_d : wptr(s, l, s.po.w_1), nullptr, nullptr, dc, nullptr, nullptr, bt));
  // c = LN2(x1), plus the residual path; the parameter gradients are finished in the W step
  HIPCHK(launch_ln_bwd(s.dt, dc, v.x1, v.mean2, v.rstd2, wptr(s, l, s.po.ln2_g), dy, dx1, nullptr, nullptr, red_ln2, s.m, s.H, q));
  // x1 = x + o Wo + bo
  TRY(gemm(s, q, KFKB_GEMM_NT, KFKB_EPI_NONE, s.m, s.H, s.H, dx1, bt ? w.o_d : wptr(s, l, s.po.w_o), nullptr, nullptr, d_o, nullptr, nullptr, bt));
  // o = attention(qkv)
  TRY(attention_bwd(s, q, v.qkv, v.o, d_o, v.lse, ln.dsum, dqkv));
  // qkv = a Wqkv + bqkv
  TRY(gemm(s, q, KFKB_GEMM_NT, KFKB_EPI_NONE, s.m, s.H, 3 * s.H, dqkv, bt ? w.qkv_d : wptr(s, l, s.po.w_qkv), nullptr, nullptr, da, nullptr, nullptr, bt));
  // a = LN1(x), plus the residual path
  HIPCHK(launch_ln_bwd(s.dt, da, x, v.mean1, v.rstd1, wptr(s, l, s.po.ln1_g), dx1, dx, nullptr, nullptr, red_ln1, s.m, s.H, q));

  // ---- W step: every accumulation into the gradients of block l, in micro-batch order -----------------
  if (windowed) {
    HIPCHK(hipEventRecord(s.ev_wops[(size_t)a.wpos * s.L + l], q));
    if (++s.w_arrived[l] == s.w_size) {                   // the window's last chain through this block: its W step
      for (int p = 0; p < s.w_size; p++)
        if (p != a.wpos) HIPCHK(hipStreamWaitEvent(q, s.ev_wops[(size_t)p * s.L + l], 0));
      if (s.ev_wlast != nullptr) HIPCHK(hipStreamWaitEvent(q, s.ev_wlast, 0));   // W steps follow one another
      WOperands ops[kWSeg];
      for (int p = 0; p < s.w_size; p++) {
        const MbState& mp = s.mb[s.w_mbs[p]];
        StashView vp = view(s, mp.stash, l);
        const Stage::WOps& o = s.wpool[(size_t)p * s.L + l];
        const char* dyp = (l == s.L - 1) ? s.dys.buf[mp.dy_slot] : s.wpool[(size_t)p * s.L + l + 1].dx;
        ops[p] = WOperands{vp.a, vp.c, vp.o, vp.gact, o.dqkv, o.du, o.dx1, dyp, o.ln[0], o.ln[1], ln.red_w[par]};
      }
      TRY(launch_w_step(s, l, ops, s.w_size, q));
      HIPCHK(hipEventRecord(s.ev_g[l], q));
      s.ev_g_set[l] = 1;
      s.ev_wlast = s.ev_g[l];
      s.w_arrived[l] = 0;
    }
    a.cur = dx;
    a.next--; a.left--;
    return 0;
  }
  if (qw != q) {
    HIPCHK(hipEventRecord(ln.ev_chain[ring], q));
    HIPCHK(hipStreamWaitEvent(qw, ln.ev_chain[ring], 0));
  }
  if (s.ev_g_set[l]) HIPCHK(hipStreamWaitEvent(qw, s.ev_g[l], 0));     // the previous micro-batch's W step of this block
  const WOperands ops{v.a, v.c, v.o, v.gact, dqkv, du, dx1, dy, red_ln1, red_ln2, ln.red_w[par]};
  TRY(launch_w_step(s, l, &ops, 1, qw));
  HIPCHK(hipEventRecord(s.ev_g[l], qw));
  s.ev_g_set[l] = 1;
  s.ev_wlast = s.ev_g[l];
  ln.w_elsewhere[ring] = qw != q;
  if (qw != q) { HIPCHK(hipEventRecord(ln.ev_wdone[ring], qw)); a.w_stream = qw; }
  a.cur = dx;
  a.next--; a.left--;
  return 0;
}

// ---- transfers ---------------------------------------------------------------------------------
// Receive X_mb (op F) or dY_mb (op B) into a free slot.  Returns 0 issued, 1 not possible yet.
int issue_recv(int op, int mbi) {
  MbState& st = g.mb[mbi];
  const size_t bytes = g.n * g.esz;
  if (op == KFKB_OP_F) {
    if (st.x_issued) return 0;
    const int slot = g.xs.take();
    if (slot < 0) return 1;
    if (g.xs.release[slot]) HIPCHK(hipStreamWaitEvent(g.sr, g.xs.release[slot], 0));
    HIPCHK(hipEventRecord(g.ev_t0[0][mbi], g.sr));
    HIPCHK(launch_delay(g.dl_x[mbi], g.sr));
    HIPCHK(hipMemcpyAsync(g.xs.buf[slot], g.h_in + (size_t)mbi * bytes, bytes, hipMemcpyHostToDevice, g.sr));
    HIPCHK(hipEventRecord(g.ev_x[mbi], g.sr));
    st.x_slot = slot; st.x_issued = true;
    return 0;
  }
  if (st.dy_issued) return 0;
  if (!st.fwd_done) return 1;                        // the neighbour echoes: dY_mb follows the arrival of Y_mb
  const int slot = g.dys.take();
  if (slot < 0) return 1;
  if (g.dys.release[slot]) HIPCHK(hipStreamWaitEvent(g.sr, g.dys.release[slot], 0));
  HIPCHK(hipStreamWaitEvent(g.sr, g.ev_ys[mbi], 0));
  HIPCHK(hipEventRecord(g.ev_t0[1][mbi], g.sr));
  HIPCHK(launch_delay(g.dl_dy[mbi], g.sr));
  HIPCHK(hipMemcpyAsync(g.dys.buf[slot], g.h_up + (size_t)mbi * bytes, bytes, hipMemcpyHostToDevice, g.sr));
  HIPCHK(hipEventRecord(g.ev_dy[mbi], g.sr));
  st.dy_slot = slot; st.dy_issued = true;
  return 0;
}

// The copy of a send: the library's own kernel writing the pinned array through its device view, or the runtime's
// device-to-host copy.  The kernel is the default: when iterations are enqueued back to back for more than about
// three seconds the runtime's copies of 64 MiB go from 1.2 ms to 5.3 ms each for long stretches (measured on the
// very wide stage: 2517 against 2385 ms per iteration over 20 iterations), the kernel's stay at 1.2 ms; eight
// workgroups keep PCIe busy and take little from the matrix kernels running beside them.
int send_copy(char* h_dst, char* d_dst, const char* src, size_t bytes) {
  if (g.send_blocks > 0 && d_dst != nullptr && (bytes & 15) == 0) {
    HIPCHK(launch_send_copy(d_dst, src, bytes, g.send_blocks, g.ss));
  } else {
    HIPCHK(hipMemcpyAsync(h_dst, src, bytes, hipMemcpyDeviceToHost, g.ss));
  }
  return 0;
}

int begin_log_epoch() {
  HIPCHK(hipEventRecord(g.ev_epoch, g.lane[0].s));
  HIPCHK(hipStreamWaitEvent(g.lane[1].s, g.ev_epoch, 0));
  g.epoch_valid = true;
  g.log.clear();
  return 0;
}

// Admission of F(mb) on a lane: takes the micro-batch's activation slot and output buffer, orders the lane's
// stream after the arrival of X_mb and after the last readers of what it is about to overwrite.
// Returns 0 admitted, 1 no slot free yet (only when wait_ok), < 0 error.
int begin_forward(int mbi, int lane, bool wait_ok, ActiveOp& a) {
  MbState& st = g.mb[mbi];
  if (st.fwd_done && !st.bwd_done) return fail(KFKB_E_STATE, "forward of micro-batch %d while it is live", mbi);
  if (st.fwd_done || st.fwd_begun) return fail(KFKB_E_STATE, "forward of micro-batch %d issued twice in this iteration", mbi);
  if (g.stash_free.empty() || g.ys.free_list.empty()) {
    if (wait_ok) return 1;
    if (g.stash_free.empty()) return fail(KFKB_E_STATE, "no free activation slot for micro-batch %d (peak live = %d)", mbi, g.n_stash);
    return fail(KFKB_E_STATE, "no free output buffer for micro-batch %d", mbi);
  }
  if (!st.x_issued) {
    int rc = issue_recv(KFKB_OP_F, mbi);
    if (rc < 0) return rc;
    if (rc == 1) return wait_ok ? 1 : fail(KFKB_E_STATE, "no free input slot for micro-batch %d", mbi);
  }
  const int ybuf = g.ys.take();
  st.stash = g.stash_free.back(); g.stash_free.pop_back();
  st.y_buf = ybuf;
  st.fwd_begun = true;
  if (!g.epoch_valid) TRY(begin_log_epoch());
  hipStream_t q = g.lane[lane].s;
  HIPCHK(hipStreamWaitEvent(q, g.ev_x[mbi], 0));
  if (g.ys.release[ybuf]) HIPCHK(hipStreamWaitEvent(q, g.ys.release[ybuf], 0));
  if (g.stash_release[st.stash]) {                   // the slot's last owner may still be read on another stream
    HIPCHK(hipStreamWaitEvent(q, g.stash_release[st.stash], 0));
    g.stash_release[st.stash] = nullptr;
  }
  HIPCHK(hipEventRecord(g.ev_f0[mbi], q));
  g.log.push_back({KFKB_OP_F, mbi});
  a = ActiveOp{};
  a.op = KFKB_OP_F; a.mb = mbi; a.lane = lane; a.next = 0; a.left = g.L; a.out_buf = ybuf; a.cur = g.xs.buf[st.x_slot];
  return 0;
}

int end_forward(ActiveOp& a) {
  const int mbi = a.mb;
  MbState& st = g.mb[mbi];
  hipStream_t q = g.lane[a.lane].s;
  HIPCHK(hipEventRecord(g.ev_f1[mbi], q));
  // send Y_mb as soon as the forward has delivered it
  const size_t bytes = g.n * g.esz;
  HIPCHK(hipStreamWaitEvent(g.ss, g.ev_f1[mbi], 0));
  HIPCHK(hipEventRecord(g.ev_t0[2][mbi], g.ss));
  HIPCHK(launch_delay(g.dl_y[mbi], g.ss));
  TRY(send_copy(g.h_out + (size_t)mbi * bytes, g.d_out ? g.d_out + (size_t)mbi * bytes : nullptr, g.ys.buf[a.out_buf], bytes));
  HIPCHK(hipEventRecord(g.ev_ys[mbi], g.ss));
  g.ys.give(a.out_buf, g.ev_ys[mbi]);
  st.fwd_done = true;
  return 0;
}

// wpos / wsize: position and size of the op's W-step window (wsize < 2: the op accumulates its gradients itself)
int begin_backward(int mbi, int lane, bool wait_ok, ActiveOp& a, int wpos = 0, int wsize = 0) {
  MbState& st = g.mb[mbi];
  // a window opens with its first micro-batch, once the previous one has enqueued all its W steps
  if (wsize >= 2 && wpos == 0 && g.w_open) return wait_ok ? 1 : fail(KFKB_E_STATE, "backward of micro-batch %d: the previous W-step window is still open", mbi);
  if (st.bwd_done || st.bwd_begun) return fail(KFKB_E_STATE, "backward of micro-batch %d without a live forward", mbi);
  if (!st.fwd_done) {
    if (wait_ok && st.fwd_begun) return 1;            // its forward is still being enqueued
    return fail(KFKB_E_STATE, "backward of micro-batch %d without a live forward", mbi);
  }
  if (g.dxs.free_list.empty()) return wait_ok ? 1 : fail(KFKB_E_STATE, "no free input-gradient buffer for micro-batch %d", mbi);
  if (!st.dy_issued) {
    int rc = issue_recv(KFKB_OP_B, mbi);
    if (rc < 0) return rc;
    if (rc == 1) return wait_ok ? 1 : fail(KFKB_E_STATE, "no free gradient slot for micro-batch %d", mbi);
  }
  const int dxbuf = g.dxs.take();
  st.bwd_begun = true;
  hipStream_t q = g.lane[lane].s;
  if (wsize >= 2) {
    if (wpos == 0) { g.w_open = true; g.w_size = wsize; std::fill(g.w_arrived.begin(), g.w_arrived.end(), 0); g.w_deferred.clear(); }
    g.w_mbs[wpos] = mbi;
    // the pool entries were last read by the W steps of the previous window (chained: the last one stands for all)
    if (g.ev_wlast != nullptr) HIPCHK(hipStreamWaitEvent(q, g.ev_wlast, 0));
  }
  HIPCHK(hipStreamWaitEvent(q, g.ev_dy[mbi], 0));
  HIPCHK(hipStreamWaitEvent(q, g.ev_f1[mbi], 0));    // the forward may have run on the other lane
  if (g.dxs.release[dxbuf]) HIPCHK(hipStreamWaitEvent(q, g.dxs.release[dxbuf], 0));
  HIPCHK(hipEventRecord(g.ev_b0[mbi], q));
  g.log.push_back({KFKB_OP_B, mbi});
  a = ActiveOp{};
  a.op = KFKB_OP_B; a.mb = mbi; a.lane = lane; a.next = g.L - 1; a.left = g.L; a.out_buf = dxbuf; a.cur = g.dys.buf[st.dy_slot];
  a.wpos = wpos; a.wsize = wsize;
  return 0;
}

// The open window's last W step (block 0) has just been enqueued on stream q of lane `lane`: everything its
// micro-batches held may be reused once that step is done.
int close_window_on(hipStream_t q) {
  const int last = g.w_mbs[g.w_size - 1];
  HIPCHK(hipEventRecord(g.ev_w[last], q));
  for (const auto& d : g.w_deferred) {
    g.stash_release[d.stash] = g.ev_w[last];
    g.stash_free.push_back(d.stash);
    g.xs.give(d.x_slot, g.ev_w[last]);
    g.dys.give(d.dy_slot, g.ev_w[last]);
  }
  g.w_deferred.clear();
  for (int p = 0; p < g.w_size; p++) { MbState& m = g.mb[g.w_mbs[p]]; m.stash = m.x_slot = m.dy_slot = -1; }
  g.w_open = false;
  g.last_done = g.ev_w[last];
  return 0;
}

int end_backward(ActiveOp& a) {
  const int mbi = a.mb;
  MbState& st = g.mb[mbi];
  hipStream_t q = g.lane[a.lane].s;
  HIPCHK(hipEventRecord(g.ev_b1[mbi], q));           // dX_mb is complete
  // after ev_done nothing reads the micro-batch's activations or dY any more
  hipEvent_t ev_done = g.ev_b1[mbi];
  if (a.w_stream != nullptr) {
    hipStream_t qw = a.w_stream;
    HIPCHK(hipStreamWaitEvent(qw, g.ev_b1[mbi], 0));
    HIPCHK(hipEventRecord(g.ev_w[mbi], qw));
    ev_done = g.ev_w[mbi];
  }
  const size_t bytes = g.n * g.esz;
  HIPCHK(hipStreamWaitEvent(g.ss, g.ev_b1[mbi], 0));
  HIPCHK(hipEventRecord(g.ev_t0[3][mbi], g.ss));
  HIPCHK(launch_delay(g.dl_dx[mbi], g.ss));
  TRY(send_copy(g.h_ingrad + (size_t)mbi * bytes, g.d_ingrad ? g.d_ingrad + (size_t)mbi * bytes : nullptr, g.dxs.buf[a.out_buf], bytes));
  HIPCHK(hipEventRecord(g.ev_dxs[mbi], g.ss));
  g.dxs.give(a.out_buf, g.ev_dxs[mbi]);
  if (a.wsize >= 2) {
    // the window's W steps still read this micro-batch's activations and gradients: its slots go back when the
    // last of them has been enqueued (by the window's last micro-batch, which ends after all the others)
    g.w_deferred.push_back(Stage::Deferred{st.stash, st.x_slot, st.dy_slot});
    st.bwd_done = true;
    if (a.wpos == a.wsize - 1) TRY(close_window_on(q));
    return 0;
  }
  // early release: the micro-batch's activations and its input slots return to their pools
  g.stash_release[st.stash] = ev_done;
  g.stash_free.push_back(st.stash);
  g.xs.give(st.x_slot, ev_done);
  g.dys.give(st.dy_slot, ev_done);
  st.stash = st.x_slot = st.dy_slot = -1;
  st.bwd_done = true;
  g.last_done = ev_done;
  return 0;
}

// one op from start to end on lane 0 (the single-op entry points)
int run_single(int op, int mbi) {
  ActiveOp a;
  TRY(op == KFKB_OP_F ? begin_forward(mbi, 0, false, a) : begin_backward(mbi, 0, false, a));
  while (a.left > 0) TRY(op == KFKB_OP_F ? forward_block(a) : backward_block(a));
  return op == KFKB_OP_F ? end_forward(a) : end_backward(a);
}

// orders stream q after everything enqueued so far on the other compute streams
int join_compute_streams(hipStream_t q) {
  for (int i = 0; i < 2; i++) {
    if (g.lane[i].s == q) continue;
    HIPCHK(hipEventRecord(g.lane[i].ev_tail, g.lane[i].s));
    HIPCHK(hipStreamWaitEvent(q, g.lane[i].ev_tail, 0));
  }
  return 0;
}

int live_count() {
  int live = 0;
  for (const auto& m : g.mb) live += (m.fwd_done && !m.bwd_done) ? 1 : 0;
  return live;
}

void reset_iteration_state() {
  for (auto& m : g.mb) m = MbState{};
  g.xs.reset(); g.dys.reset(); g.ys.reset(); g.dxs.reset();
  g.stash_free.clear();
  for (int i = g.n_stash - 1; i >= 0; i--) g.stash_free.push_back(i);
}

// The four streams of the stage, chosen once per process.  HIP multiplexes streams onto a few hardware queues
// (four per process by default) and two streams on one queue run one after the other, so eight streams are
// created and four that demonstrably run side by side are kept: pairs of 200 us delay kernels are timed.
// Order of the result: lane 0, send, receive, lane 1 (if fewer than four independent streams exist, the later
// entries share).  The streams live until the process ends.
hipStream_t g_stream_pick[4] = {nullptr, nullptr, nullptr, nullptr};
bool g_streams_picked = false;

int pick_streams() {
  if (g_streams_picked) return 0;
  constexpr int P = 8;
  hipStream_t pool[P];
  for (int i = 0; i < P; i++) HIPCHK(hipStreamCreateWithFlags(&pool[i], hipStreamNonBlocking));
  for (int rep = 0; rep < 2; rep++) {
    for (int i = 0; i < P; i++) HIPCHK(launch_delay(2000, pool[i]));
    for (int i = 0; i < P; i++) HIPCHK(hipStreamSynchronize(pool[i]));
  }
  bool together[P][P] = {};
  for (int i = 0; i < P; i++)
    for (int j = i + 1; j < P; j++) {
      const auto t0 = std::chrono::steady_clock::now();
      HIPCHK(launch_delay(200000, pool[i]));
      HIPCHK(launch_delay(200000, pool[j]));
      HIPCHK(hipStreamSynchronize(pool[i]));
      HIPCHK(hipStreamSynchronize(pool[j]));
      const double us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
      together[i][j] = together[j][i] = us < 330.0;
    }
  int chosen[4], n = 0;
  for (int i = 0; i < P && n < 4; i++) {
    bool ok = true;
    for (int c = 0; c < n; c++) ok = ok && together[chosen[c]][i];
    if (ok) chosen[n++] = i;
  }
  for (int i = 0; n < 4 && i < P; i++) {              // not enough independent ones: take what is left
    bool used = false;
    for (int c = 0; c < n; c++) used = used || chosen[c] == i;
    if (!used) chosen[n++] = i;
  }
  for (int c = 0; c < 4; c++) g_stream_pick[c] = pool[chosen[c]];
  for (int i = 0; i < P; i++) {
    bool used = false;
    for (int c = 0; c < 4; c++) used = used || chosen[c] == i;
    if (!used) hipStreamDestroy(pool[i]);
  }
  g_streams_picked = true;
  return 0;
}


// ---- cost model and tuner (host only) --------------------------------------------------------------
// Discrete-event run of the engine's own transfer rules with constant op and transfer times.
double predict_iteration(int k, int M, int w, double tf, double tb, const double (&tc)[4], int x_slots, int dy_slots) {
  std::vector<kfkb_op_t> order, plan;
  build_order(k, M, w, order);
  build_receive_plan(order, k, plan);
  const int live = peak_live_of(order);
  constexpr double kBusy = -1.0;
  std::vector<double> pool[2];
  pool[0].assign(x_slots > 0 ? x_slots : live + k, 0.0);
  pool[1].assign(dy_slots > 0 ? dy_slots : 2 * k, 0.0);
  std::vector<double> arrive[2], sent_y(M, -1.0);
  std::vector<int> slot[2];
  for (int d = 0; d < 2; d++) { arrive[d].assign(M, -1.0); slot[d].assign(M, -1); }
  double t_recv = 0.0, t_send = 0.0, t_comp = 0.0;
  size_t rp = 0;
  auto receives = [&]() {
    while (rp < plan.size()) {
      const int d = plan[rp].op == KFKB_OP_F ? 0 : 1, mb = plan[rp].mb;
      if (d == 1 && sent_y[mb] < 0.0) return;          // the echo: dY follows the arrival of Y
      int best = -1;
      for (size_t i = 0; i < pool[d].size(); i++)
        if (pool[d][i] != kBusy && (best < 0 || pool[d][i] < pool[d][best])) best = (int)i;
      if (best < 0) return;
      double begin = std::max(t_recv, pool[d][best]);
      if (d == 1) begin = std::max(begin, sent_y[mb]);
      pool[d][best] = kBusy;
      t_recv = begin + tc[d];
      arrive[d][mb] = t_recv;
      slot[d][mb] = best;
      rp++;
    }
  };
  for (const auto& op : order) {
    receives();
    const int d = op.op == KFKB_OP_F ? 0 : 1;
    if (arrive[d][op.mb] < 0.0) return -1.0;            // the receive plan cannot feed this op
    t_comp = std::max(t_comp, arrive[d][op.mb]) + (d == 0 ? tf : tb);
    t_send = std::max(t_send, t_comp) + tc[2 + d];
    if (d == 0) {
      sent_y[op.mb] = t_send;
    } else {
      pool[0][slot[0][op.mb]] = t_comp;
      pool[1][slot[1][op.mb]] = t_comp;
    }
  }
  return std::max(t_comp, std::max(t_send, t_recv));
}

struct TunerState {
  int window = 4, interval = 4;
  std::vector<int> candidates{1};
  std::vector<double> tf, tb;                         // per candidate; < 0: not profiled
  std::vector<double> samples[4];                     // last `window` samples per direction
  std::vector<double> estimates;
  long iterations = 0;
  int k = 1;
  double mean(int d) const {
    if (samples[d].empty()) return 0.0;
    double s = 0.0;
    for (double v : samples[d]) s += v;
    return s / (double)samples[d].size();
  }
};
TunerState g_tuner;

int make_events(std::vector<hipEvent_t>& v, int n) {
  v.resize(n);
  for (auto& e : v) HIPCHK(hipEventCreate(&e));
  return 0;
}

// ---- S virtual stages on the one GPU (the multi-stage pipeline, rehearsed on one device) ---------------------
// The stage's L blocks are cut into S consecutive virtual stages of L / S blocks; virtual stage v follows its own
// kFkB plan with w = min(S-1-v, G) warm-up groups, forwards a micro-batch after stage v-1 has and backwards it
// after stage v+1 has.  Activations cross a boundary as a delayed device-to-device copy on the send stream,
// gradients on the receive stream; a delay counts from the moment the producer finished (a device clock stamp),
// so delays of different boundaries overlap as they would on separate links while copies stay FIFO per stream.
// The one GPU issues the ops of all stages in list-schedule order: every stage imagined on a device of its own,
// forward 1 time unit, backward 2, transfers free; the op that would start earliest goes next, ties to the later
// stage.  Micro-batch mb keeps activation slot mb for the whole iteration (the workspace must hold M slots).
struct PipeEntry { int stage, op, mb; };

int pipeline_list_schedule(int S, int k, int M, std::vector<PipeEntry>& out) {
  std::vector<std::vector<kfkb_op_t>> orders(S);
  const int G = (M + k - 1) / k;
  for (int v = 0; v < S; v++) build_order(k, M, std::min(S - 1 - v, G), orders[v]);
  std::vector<size_t> nxt(S, 0);
  std::vector<long long> clock(S, 0);
  std::vector<long long> fdone((size_t)S * M, -1), bdone((size_t)S * M, -1);
  out.clear();
  const size_t total = (size_t)2 * M * S;
  while (out.size() < total) {
    int best_v = -1; long long best_start = 0;
    for (int v = 0; v < S; v++) {
      if (nxt[v] >= orders[v].size()) continue;
      const kfkb_op_t& o = orders[v][nxt[v]];
      long long ready = 0;
      if (o.op == KFKB_OP_F) {
        if (v > 0) { const long long d = fdone[(size_t)(v - 1) * M + o.mb]; if (d < 0) continue; ready = d; }
      } else {
        const long long d = fdone[(size_t)v * M + o.mb];
        if (d < 0) continue;
        ready = d;
        if (v < S - 1) { const long long e = bdone[(size_t)(v + 1) * M + o.mb]; if (e < 0) continue; ready = std::max(ready, e); }
      }
      const long long start = std::max(clock[v], ready);
      if (best_v < 0 || start < best_start || (start == best_start && v > best_v)) { best_v = v; best_start = start; }
    }
    if (best_v < 0) return fail(KFKB_E_STATE, "pipeline plans dead-lock (S=%d k=%d M=%d)", S, k, M);
    const kfkb_op_t& o = orders[best_v][nxt[best_v]++];
    const long long fin = best_start + (o.op == KFKB_OP_F ? 1 : 2);
    clock[best_v] = fin;
    (o.op == KFKB_OP_F ? fdone : bdone)[(size_t)best_v * M + o.mb] = fin;
    out.push_back(PipeEntry{best_v, o.op, o.mb});
  }
  return 0;
}

struct PipeSim {
  bool bound = false;
  int S = 0, M = 0;
  char* wire = nullptr;                       // [3][S-1][M] boundary tensors: forward copy, gradient as produced, gradient copy
  long long* stamps = nullptr;                // [2][S-1][M] device clock when the producer finished
  std::vector<hipEvent_t> ev_f0, ev_f1, ev_b0, ev_b1, ev_w, ev_tf, ev_tb;
  std::vector<int64_t> dl_f, dl_b;            // [S-1][M]
  std::vector<PipeEntry> log;
  hipEvent_t ev_join[4] = {};
  size_t act() const { return align_up(g.n * g.esz); }
  char* tensor(int which, int boundary, int mb) const { return wire + (((size_t)which * (S - 1) + boundary) * M + mb) * act(); }
  long long* stamp(int which, int boundary, int mb) const { return stamps + ((size_t)which * (S - 1) + boundary) * M + mb; }
};
PipeSim gp;

// Drops the pipeline binding.  Its events may still be named as "last reader" of a pooled buffer: everything is
// waited for first and those references are cleared, so nothing keeps a handle to a destroyed event.
void pipeline_release() {
  if (gp.bound && g.inited) {
    for (hipStream_t q : {g.lane[0].s, g.lane[1].s, g.sr, g.ss}) (void)hipStreamSynchronize(q);
    for (Pool* p : {&g.xs, &g.dys, &g.ys, &g.dxs}) std::fill(p->release.begin(), p->release.end(), nullptr);
    std::fill(g.stash_release.begin(), g.stash_release.end(), nullptr);
    g.last_done = nullptr;
  }
  for (auto* v : {&gp.ev_f0, &gp.ev_f1, &gp.ev_b0, &gp.ev_b1, &gp.ev_w, &gp.ev_tf, &gp.ev_tb})
    for (auto e : *v) (void)hipEventDestroy(e);
  for (auto e : gp.ev_join) if (e) (void)hipEventDestroy(e);
  gp = PipeSim{};
}

int pipe_begin_forward(int v, int mbi, int lane, ActiveOp& a) {
  MbState& st = g.mb[mbi];
  const int S = gp.S, M = gp.M, Ls = g.L / S;
  hipStream_t q = g.lane[lane].s;
  int ybuf = -1;
  if (v == S - 1 && g.ys.free_list.empty()) return 1;
  if (v == 0) {
    if (!st.x_issued) {
      const int rc = issue_recv(KFKB_OP_F, mbi);
      if (rc != 0) return rc;
    }
    HIPCHK(hipStreamWaitEvent(q, g.ev_x[mbi], 0));
  } else {
    HIPCHK(hipStreamWaitEvent(q, gp.ev_tf[(size_t)(v - 1) * M + mbi], 0));
  }
  if (v == S - 1) {
    ybuf = g.ys.take();
    if (g.ys.release[ybuf]) HIPCHK(hipStreamWaitEvent(q, g.ys.release[ybuf], 0));
  }
  HIPCHK(hipEventRecord(gp.ev_f0[(size_t)v * M + mbi], q));
  gp.log.push_back(PipeEntry{v, KFKB_OP_F, mbi});
  a = ActiveOp{};
  a.op = KFKB_OP_F; a.mb = mbi; a.lane = lane; a.next = v * Ls; a.left = Ls; a.out_buf = ybuf; a.first = v * Ls;
  a.cur = v == 0 ? g.xs.buf[st.x_slot] : gp.tensor(0, v - 1, mbi);
  return 0;
}

int pipe_end_forward(ActiveOp& a, int v) {
  const int mbi = a.mb, S = gp.S, M = gp.M, Ls = g.L / S;
  MbState& st = g.mb[mbi];
  hipStream_t q = g.lane[a.lane].s;
  const size_t bytes = g.n * g.esz;
  if (v == S - 1) {
    HIPCHK(hipEventRecord(gp.ev_f1[(size_t)v * M + mbi], q));
    HIPCHK(hipStreamWaitEvent(g.ss, gp.ev_f1[(size_t)v * M + mbi], 0));
    HIPCHK(hipEventRecord(g.ev_t0[2][mbi], g.ss));
    HIPCHK(launch_delay(g.dl_y[mbi], g.ss));
    TRY(send_copy(g.h_out + (size_t)mbi * bytes, g.d_out ? g.d_out + (size_t)mbi * bytes : nullptr, g.ys.buf[a.out_buf], bytes));
    HIPCHK(hipEventRecord(g.ev_ys[mbi], g.ss));
    g.ys.give(a.out_buf, g.ev_ys[mbi]);
    st.fwd_done = true;
    return 0;
  }
  HIPCHK(launch_clock_stamp(gp.stamp(0, v, mbi), q));
  HIPCHK(hipEventRecord(gp.ev_f1[(size_t)v * M + mbi], q));
  HIPCHK(hipStreamWaitEvent(g.ss, gp.ev_f1[(size_t)v * M + mbi], 0));
  HIPCHK(launch_delay_since(gp.stamp(0, v, mbi), gp.dl_f[(size_t)v * M + mbi], g.ss));
  HIPCHK(hipMemcpyAsync(gp.tensor(0, v, mbi), view(g, st.stash, (v + 1) * Ls - 1).y, bytes, hipMemcpyDeviceToDevice, g.ss));
  HIPCHK(hipEventRecord(gp.ev_tf[(size_t)v * M + mbi], g.ss));
  return 0;
}

int pipe_begin_backward(int v, int mbi, int lane, ActiveOp& a) {
  MbState& st = g.mb[mbi];
  const int S = gp.S, M = gp.M, Ls = g.L / S;
  hipStream_t q = g.lane[lane].s;
  if (v == 0 && g.dxs.free_list.empty()) return 1;
  if (v == S - 1) {
    if (!st.dy_issued) {
      const int rc = issue_recv(KFKB_OP_B, mbi);
      if (rc != 0) return rc;
    }
    HIPCHK(hipStreamWaitEvent(q, g.ev_dy[mbi], 0));
  } else {
    HIPCHK(hipStreamWaitEvent(q, gp.ev_tb[(size_t)v * M + mbi], 0));
  }
  HIPCHK(hipStreamWaitEvent(q, gp.ev_f1[(size_t)v * M + mbi], 0));      // its forward may have run on the other lane
  int dxbuf = -1;
  if (v == 0) {
    dxbuf = g.dxs.take();
    if (g.dxs.release[dxbuf]) HIPCHK(hipStreamWaitEvent(q, g.dxs.release[dxbuf], 0));
  }
  HIPCHK(hipEventRecord(gp.ev_b0[(size_t)v * M + mbi], q));
  gp.log.push_back(PipeEntry{v, KFKB_OP_B, mbi});
  a = ActiveOp{};
  a.op = KFKB_OP_B; a.mb = mbi; a.lane = lane; a.next = (v + 1) * Ls - 1; a.left = Ls; a.out_buf = dxbuf; a.first = v * Ls;
  a.cur = v == S - 1 ? g.dys.buf[st.dy_slot] : gp.tensor(2, v, mbi);
  if (v > 0) { a.x_first = gp.tensor(0, v - 1, mbi); a.dx_first = gp.tensor(1, v - 1, mbi); }
  return 0;
}

int pipe_end_backward(ActiveOp& a, int v) {
  const int mbi = a.mb, S = gp.S, M = gp.M;
  MbState& st = g.mb[mbi];
  hipStream_t q = g.lane[a.lane].s;
  const size_t bytes = g.n * g.esz;
  if (v > 0) HIPCHK(launch_clock_stamp(gp.stamp(1, v - 1, mbi), q));
  hipEvent_t ev_b1 = gp.ev_b1[(size_t)v * M + mbi];
  HIPCHK(hipEventRecord(ev_b1, q));
  hipEvent_t ev_done = ev_b1;                          // after it nothing of this op reads its operands any more
  if (a.w_stream != nullptr) {
    HIPCHK(hipStreamWaitEvent(a.w_stream, ev_b1, 0));
    HIPCHK(hipEventRecord(gp.ev_w[(size_t)v * M + mbi], a.w_stream));
    ev_done = gp.ev_w[(size_t)v * M + mbi];
  }
  if (v == S - 1) { g.dys.give(st.dy_slot, ev_done); st.dy_slot = -1; }
  if (v == 0) {
    HIPCHK(hipStreamWaitEvent(g.ss, ev_b1, 0));
    HIPCHK(hipEventRecord(g.ev_t0[3][mbi], g.ss));
    HIPCHK(launch_delay(g.dl_dx[mbi], g.ss));
    TRY(send_copy(g.h_ingrad + (size_t)mbi * bytes, g.d_ingrad ? g.d_ingrad + (size_t)mbi * bytes : nullptr, g.dxs.buf[a.out_buf], bytes));
    HIPCHK(hipEventRecord(g.ev_dxs[mbi], g.ss));
    g.dxs.give(a.out_buf, g.ev_dxs[mbi]);
    g.xs.give(st.x_slot, ev_done);
    st.x_slot = -1;
    st.bwd_done = true;
  } else {
    HIPCHK(hipStreamWaitEvent(g.sr, ev_b1, 0));
    HIPCHK(launch_delay_since(gp.stamp(1, v - 1, mbi), gp.dl_b[(size_t)(v - 1) * M + mbi], g.sr));
    HIPCHK(hipMemcpyAsync(gp.tensor(2, v - 1, mbi), gp.tensor(1, v - 1, mbi), bytes, hipMemcpyDeviceToDevice, g.sr));
    HIPCHK(hipEventRecord(gp.ev_tb[(size_t)(v - 1) * M + mbi], g.sr));
  }
  g.last_done = ev_done;
  return 0;
}
}  // namespace

// =================================================================================================
extern "C" {

const char* kfkb_last_error(void) { return g_err.c_str(); }

int kfkb_schedule(int k, int num_microbatches, int warmup_groups, kfkb_op_t* out, int cap) {
  if (k < 1 || num_microbatches < 1 || k > num_microbatches || warmup_groups < 0)
    return fail(KFKB_E_ARG, "kfkb_schedule needs 1 <= k <= M and w >= 0 (k=%d M=%d w=%d)", k, num_microbatches, warmup_groups);
  if (out == nullptr || cap < 2 * num_microbatches) return fail(KFKB_E_ARG, "kfkb_schedule: output too small");
  std::vector<kfkb_op_t> order;
  const int n = build_order(k, num_microbatches, warmup_groups, order);
  std::copy(order.begin(), order.end(), out);
  return n;
}

int kfkb_peak_live(int k, int num_microbatches, int warmup_groups) {
  if (k < 1 || num_microbatches < 1 || k > num_microbatches || warmup_groups < 0)
    return fail(KFKB_E_ARG, "kfkb_peak_live needs 1 <= k <= M and w >= 0");
  std::vector<kfkb_op_t> order;
  build_order(k, num_microbatches, warmup_groups, order);
  return peak_live_of(order);
}

size_t kfkb_activation_bytes_per_microbatch_ex(int layers, int micro_batch, int seq, int hidden, int heads, int mlp_width,
                                               int elem_bytes, int recompute) {
  const size_t m = (size_t)micro_batch * seq, n = m * hidden;
  const size_t elems = recompute ? 6 * n + m * mlp_width : 8 * n + 2 * m * mlp_width;
  return (size_t)layers * (elems * elem_bytes + (4 * m + (size_t)micro_batch * heads * seq) * 4);
}

size_t kfkb_activation_bytes_per_microbatch(int layers, int micro_batch, int seq, int hidden, int heads, int mlp_width,
                                            int elem_bytes) {
  return kfkb_activation_bytes_per_microbatch_ex(layers, micro_batch, seq, hidden, heads, mlp_width, elem_bytes, 0);
}

int stage_config(const kfkb_config_t* cfg) {
  if (cfg == nullptr) return fail(KFKB_E_ARG, "stage_config: null config");
  if (g.inited) return fail(KFKB_E_STATE, "stage_config after stage_init");
  g_cfg_pending = *cfg;
  g_cfg_set = true;
  return 0;
}

int stage_init(const void* weights, int layers, int hidden, int heads, int seq) {
  if (g.inited) return fail(KFKB_E_STATE, "a stage already exists; call stage_destroy first");
  kfkb_config_t c{};
  if (g_cfg_set) c = g_cfg_pending;
  if (c.micro_batch == 0) c.micro_batch = 1;
  if (c.mlp_ratio == 0) c.mlp_ratio = 4;
  if (c.ln_eps == 0.f) c.ln_eps = 1e-5f;
  if (c.num_stages == 0) c.num_stages = 1;
  if (c.max_microbatches == 0) c.max_microbatches = 1;
  if (weights == nullptr) return fail(KFKB_E_ARG, "stage_init: null weights");
  if (layers < 1 || hidden < 1 || heads < 1 || seq < 1 || c.micro_batch < 1 || c.mlp_ratio < 1 || c.max_microbatches < 1)
    return fail(KFKB_E_ARG, "stage_init: sizes must be positive");
  if (c.dtype != KFKB_F32 && c.dtype != KFKB_BF16 && c.dtype != KFKB_F16) return fail(KFKB_E_ARG, "stage_init: unknown dtype %d", c.dtype);
  if (c.stage_index < 0 || c.stage_index >= c.num_stages) return fail(KFKB_E_ARG, "stage_init: stage_index outside [0, num_stages)");
  if (hidden % heads != 0) return fail(KFKB_E_ARG, "stage_init: hidden %d not divisible by heads %d", hidden, heads);
  const int d = hidden / heads;
  if (c.dtype != KFKB_F32) {
    if (hidden % 128 != 0) return fail(KFKB_E_ARG, "stage_init: 16-bit storage needs hidden %% 128 == 0 (got %d)", hidden);
    if (d != 64 && d != 128) return fail(KFKB_E_ARG, "stage_init: 16-bit storage needs head size 64 or 128 (got %d)", d);
    if ((double)seq * 3.0 * hidden * 2.0 >= 2147483648.0)
      return fail(KFKB_E_ARG, "stage_init: seq * 3 * hidden * 2 bytes must stay below 2 GiB for 16-bit storage (seq = %d, hidden = %d)", seq, hidden);
  } else {
    if (hidden % 8 != 0) return fail(KFKB_E_ARG, "stage_init: fp32 needs hidden %% 8 == 0 (got %d)", hidden);
    if (d > 128) return fail(KFKB_E_ARG, "stage_init: fp32 needs head size <= 128 (got %d)", d);
    if (seq > 4096) return fail(KFKB_E_ARG, "stage_init: fp32 path supports seq <= 4096");
  }
  if (hidden > 8192) return fail(KFKB_E_ARG, "stage_init: hidden > 8192 is not supported");
  Stage s;
  s.cfg = c; s.dt = c.dtype; s.L = layers; s.H = hidden; s.heads = heads; s.d = d; s.T = seq; s.b = c.micro_batch;
  s.F = c.mlp_ratio * hidden; s.m = s.b * s.T; s.n = (size_t)s.m * s.H; s.esz = dt_bytes(s.dt); s.Mmax = c.max_microbatches;
  s.recompute = c.recompute != 0;
  g_prof_dt = s.dt;
  if (s.recompute && ((size_t)s.m * s.F) % 8 != 0) return fail(KFKB_E_ARG, "stage_init: recomputation needs tokens * mlp width %% 8 == 0");
  const size_t H = hidden, F = s.F;
  BlockParams& p = s.po;
  size_t o = 0;
  p.ln1_g = o; o += H; p.ln1_b = o; o += H; p.w_qkv = o; o += H * 3 * H; p.b_qkv = o; o += 3 * H;
  p.w_o = o; o += H * H; p.b_o = o; o += H; p.ln2_g = o; o += H; p.ln2_b = o; o += H;
  p.w_1 = o; o += H * F; p.b_1 = o; o += F; p.w_2 = o; o += F * H; p.b_2 = o; o += H; p.total = o;
  s.weights = (const char*)weights;
  if (dt_is16(s.dt)) {
    WGrad wg[4] = {};
    const int wm[4] = {s.H, s.H, s.F, s.H}, wn[4] = {3 * s.H, s.F, s.H, s.H};
    for (int i = 0; i < 4; i++) { wg[i].M = wm[i]; wg[i].N = wn[i]; }
    WStepReduce red{};
    red.rows = s.m; red.n_colsum = 4; red.n_ln = 2;
    const int widths[4] = {3 * s.H, s.F, s.H, s.H};
    for (int i = 0; i < 4; i++) red.width[i] = widths[i];
    red.ln_width[0] = red.ln_width[1] = s.H;
    red.ln_parts[0] = red.ln_parts[1] = ln_bwd_partial_rows(s.m, s.H);
    s.wstep_grouped = wstep_groupable(wg, 4, s.m, &red);
  }
  s.stash_block_bytes = stash_block_bytes_of(s);
  s.mb.assign(s.Mmax, MbState{});
  s.dl_x.assign(s.Mmax, 0); s.dl_dy.assign(s.Mmax, 0); s.dl_y.assign(s.Mmax, 0); s.dl_dx.assign(s.Mmax, 0);
  g = s;
  TRY(pick_streams());
  g.lane[0].s = g_stream_pick[0]; g.ss = g_stream_pick[1]; g.sr = g_stream_pick[2]; g.lane[1].s = g_stream_pick[3];
  for (auto& ln : g.lane) {
    for (int i = 0; i < Stage::kRing; i++) { HIPCHK(hipEventCreate(&ln.ev_chain[i])); HIPCHK(hipEventCreate(&ln.ev_wdone[i])); }
    HIPCHK(hipEventCreate(&ln.ev_tail));
  }
  TRY(make_events(g.ev_w, g.Mmax));
  TRY(make_events(g.ev_g, g.L));
  g.ev_g_set.assign(g.L, 0);
  HIPCHK(hipEventCreate(&g.ev_zero));
  TRY(make_events(g.ev_x, g.Mmax)); TRY(make_events(g.ev_dy, g.Mmax));
  TRY(make_events(g.ev_f0, g.Mmax)); TRY(make_events(g.ev_f1, g.Mmax));
  TRY(make_events(g.ev_b0, g.Mmax)); TRY(make_events(g.ev_b1, g.Mmax));
  TRY(make_events(g.ev_ys, g.Mmax)); TRY(make_events(g.ev_dxs, g.Mmax));
  for (auto& v : g.ev_t0) TRY(make_events(v, g.Mmax));
  HIPCHK(hipEventCreate(&g.ev_epoch));
  HIPCHK(hipEventCreate(&g.ev_run_end));
  // How much of the chip one op's kernels fill decides how ops are best run.  A block whose matrix products are a
  // few hundred GFLOP leaves gaps (launch latency, partly filled rounds of tiles, memory-bound row kernels) that a
  // second micro-batch in flight and W steps beside the chain fill: two lanes.  From about 2 TFLOP per block
  // forward on, every kernel runs many rounds of tiles on all CUs, kernels of two streams only take each other's
  // CUs and cache, and one op at a time with its W steps behind its chain is faster (measured, two lanes against
  // one, ms per iteration: hidden 2048 with 4096 tokens, 0.41 TFLOP, 268 / 290; hidden 4096 with 2048 tokens,
  // 0.82 TFLOP, 308 / 313; hidden 8192 with 4096 tokens, 6.6 TFLOP, 1156 / 1090 for 32 micro-batches).
  // stage_set_compute_lanes / stage_set_wgrad_stream override.
  const bool big_ops = 24.0 * (double)g.m * (double)g.H * (double)g.H >= 2.0e12;
  g.lanes = big_ops ? 1 : 2;
  g.wgrad_overlap = !big_ops;
  g.inited = true;
  return 0;
}

size_t stage_param_count(void) { return g.inited ? (size_t)g.L * g.po.total : 0; }

size_t stage_activation_bytes(int k, int num_microbatches) {
  if (!g.inited || k < 1 || num_microbatches < 1 || k > num_microbatches) return 0;
  return (size_t)peak_live_for(g, k, num_microbatches) *
         kfkb_activation_bytes_per_microbatch_ex(g.L, g.b, g.T, g.H, g.heads, g.F, (int)g.esz, g.recompute ? 1 : 0);
}

size_t stage_workspace_bytes(int k_max) {
  if (!g.inited || k_max < 1) return 0;
  return carve_for(g, std::min(k_max, g.Mmax)).total;
}

int stage_bind(void* workspace, size_t workspace_bytes, float* grad_accum, const void* host_inputs,
               const void* host_upstream_grads, void* host_outputs, void* host_input_grads) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_bind before stage_init");
  if (!workspace || !grad_accum || !host_inputs || !host_upstream_grads || !host_outputs || !host_input_grads)
    return fail(KFKB_E_ARG, "stage_bind: null pointer");
  if (((uintptr_t)workspace & 255) != 0) return fail(KFKB_E_ARG, "stage_bind: workspace must be 256-byte aligned");
  int kb = 0;
  for (int k = 1; k <= g.Mmax; k++) {
    if (carve_for(g, k).total <= workspace_bytes) kb = k; else break;
  }
  if (kb == 0) return fail(KFKB_E_MEMLIMIT, "stage_bind: workspace of %zu bytes is smaller than stage_workspace_bytes(1) = %zu", workspace_bytes, carve_for(g, 1).total);
  if (g.bound && live_count() != 0) return fail(KFKB_E_STATE, "stage_bind while micro-batches are live");
  const Carve c = carve_for(g, kb);
  g.ws = (char*)workspace; g.ws_bytes = workspace_bytes; g.k_bound = kb; g.n_stash = c.n_stash;
  g.grad = grad_accum;
  g.h_in = (const char*)host_inputs; g.h_up = (const char*)host_upstream_grads;
  g.h_out = (char*)host_outputs; g.h_ingrad = (char*)host_input_grads;
  {                                                   // pinned arrays have a device view; anything else is copied by the runtime
    void* dv = nullptr;
    g.d_out = hipHostGetDevicePointer(&dv, host_outputs, 0) == hipSuccess ? (char*)dv : nullptr;
    dv = nullptr;
    g.d_ingrad = hipHostGetDevicePointer(&dv, host_input_grads, 0) == hipSuccess ? (char*)dv : nullptr;
    (void)hipGetLastError();
  }
  const size_t act = align_up(g.n * g.esz);
  g.wt = g.ws + c.wt;
  g.stash.resize(c.n_stash);
  for (int i = 0; i < c.n_stash; i++) g.stash[i] = g.ws + c.stash + (size_t)i * g.L * g.stash_block_bytes;
  auto fill_pool = [&](Pool& p, size_t off, int cnt) {
    p.buf.resize(cnt); p.release.assign(cnt, nullptr);
    for (int i = 0; i < cnt; i++) p.buf[i] = g.ws + off + (size_t)i * act;
  };
  fill_pool(g.xs, c.xs, c.n_x); fill_pool(g.dys, c.dys, c.n_io); fill_pool(g.ys, c.ys, c.n_io); fill_pool(g.dxs, c.dxs, c.n_io);
  const LaneCarve lc = lane_carve(g);
  for (int i = 0; i < 2; i++) {
    Stage::Lane& ln = g.lane[i];
    char* base = g.ws + c.lanes + (size_t)i * lc.total;
    ln.t_n0 = base + lc.tn;
    for (int j = 0; j < 2; j++) ln.t_dx1[j] = base + lc.tn + (size_t)(1 + j) * act;
    for (int j = 0; j < 3; j++) ln.t_dxr[j] = base + lc.tn + (size_t)(3 + j) * act;
    for (int j = 0; j < 2; j++) {
      ln.t_mf[j] = base + lc.tmf + (size_t)j * align_up((size_t)g.m * g.F * g.esz);
      ln.t_3n[j] = base + lc.t3n + (size_t)j * align_up(3 * g.n * g.esz);
    }
    ln.dsum = reinterpret_cast<float*>(base + lc.dsum);
    for (int j = 0; j < 4; j++) ln.red_ln[j >> 1][j & 1] = reinterpret_cast<float*>(base + lc.red_ln + (size_t)j * align_up(red_ln_floats(g) * 4));
    for (int j = 0; j < 2; j++) ln.red_w[j] = reinterpret_cast<float*>(base + lc.red_w + (size_t)j * align_up(red_w_floats(g) * 4));
    if (g.recompute) {
      const size_t set = 2 * act + align_up((size_t)g.m * g.F * g.esz);
      char* r = base + lc.rec;
      ln.f_a = r; ln.f_c = r + act; ln.f_g = r + 2 * act;
      for (int j = 0; j < 2; j++) { char* q = r + (size_t)(1 + j) * set; ln.r_a[j] = q; ln.r_c[j] = q + act; ln.r_g[j] = q + 2 * act; }
    }
  }
  g.wwin_cap = c.wwin;
  g.wpool.clear();
  for (auto e : g.ev_wops) (void)hipEventDestroy(e);
  g.ev_wops.clear();
  if (c.wwin >= 2) {
    const WOpsCarve wc = wops_carve(g);
    g.wpool.resize((size_t)c.wwin * g.L);
    for (size_t i = 0; i < g.wpool.size(); i++) {
      char* base = g.ws + c.wpool + i * wc.total;
      Stage::WOps& w = g.wpool[i];
      w.du = base + wc.du; w.dqkv = base + wc.dqkv; w.dx1 = base + wc.dx1; w.dx = base + wc.dx;
      w.ln[0] = reinterpret_cast<float*>(base + wc.ln);
      w.ln[1] = reinterpret_cast<float*>(base + wc.ln + align_up(red_ln_floats(g) * 4));
    }
    TRY(make_events(g.ev_wops, (int)g.wpool.size()));
  }
  g.w_arrived.assign(g.L, 0);
  g.w_deferred.clear();
  g.w_open = false; g.w_size = 0; g.ev_wlast = nullptr;
  g.stash_release.assign(c.n_stash, nullptr);
  reset_iteration_state();
  g.epoch_valid = false; g.run_timed = false; g.log.clear();
  pipeline_release();                                 // a pipeline binding refers to the previous workspace
  g.bound = true;
  TRY(refresh_weights());
  HIPCHK(hipStreamSynchronize(g.lane[0].s));
  return 0;
}

int stage_set_delays(const int64_t* recv_input_ns, const int64_t* recv_upstream_grad_ns, const int64_t* send_output_ns,
                     const int64_t* send_input_grad_ns) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_set_delays before stage_init");
  auto set = [&](std::vector<int64_t>& v, const int64_t* src) {
    for (int i = 0; i < g.Mmax; i++) v[i] = src ? std::max<int64_t>(0, src[i]) : 0;
  };
  set(g.dl_x, recv_input_ns); set(g.dl_dy, recv_upstream_grad_ns); set(g.dl_y, send_output_ns); set(g.dl_dx, send_input_grad_ns);
  return 0;
}

int stage_refresh_weights(void) {
  if (!g.bound) return fail(KFKB_E_STATE, "stage_refresh_weights before stage_bind");
  return refresh_weights();
}

int stage_forward(int mb) {
  if (!g.bound) return fail(KFKB_E_STATE, "stage_forward before stage_bind");
  if (mb < 0 || mb >= g.Mmax) return fail(KFKB_E_ARG, "stage_forward: micro-batch %d outside [0, %d)", mb, g.Mmax);
  if (g.mb[mb].fwd_done && g.mb[mb].bwd_done) g.mb[mb] = MbState{};     // a finished micro-batch may run again
  g.run_timed = false;
  return run_single(KFKB_OP_F, mb);
}

int stage_backward(int mb) {
  if (!g.bound) return fail(KFKB_E_STATE, "stage_backward before stage_bind");
  if (mb < 0 || mb >= g.Mmax) return fail(KFKB_E_ARG, "stage_backward: micro-batch %d outside [0, %d)", mb, g.Mmax);
  g.run_timed = false;
  return run_single(KFKB_OP_B, mb);
}

int run_kFkB(int k, int num_microbatches, size_t mem_limit) {
  if (!g.bound) return fail(KFKB_E_STATE, "run_kFkB before stage_bind");
  const int M = num_microbatches;
  if (M < 1 || M > g.Mmax) return fail(KFKB_E_ARG, "run_kFkB: num_microbatches %d outside [1, %d]", M, g.Mmax);
  if (k > M) return fail(KFKB_E_ARG, "run_kFkB: k = %d exceeds the number of micro-batches %d", k, M);
  if (live_count() != 0) return fail(KFKB_E_STATE, "run_kFkB while micro-batches are live");
  auto fits = [&](int kk, bool& over_limit) {
    over_limit = mem_limit != 0 && stage_activation_bytes(kk, M) > mem_limit;
    return !over_limit && kk <= g.k_bound && peak_live_for(g, kk, M) <= g.n_stash;
  };
  bool over = false;
  if (k <= 0) {                                       // largest admissible group size dividing M
    int best = 0;
    for (int kk = 1; kk <= M; kk++) {
      bool o2;
      if (M % kk == 0 && fits(kk, o2)) best = kk;
    }
    if (best == 0) return fail(KFKB_E_MEMLIMIT, "run_kFkB: no group size fits mem_limit = %zu bytes and the bound workspace", mem_limit);
    k = best;
  } else if (!fits(k, over)) {
    if (over) return fail(KFKB_E_MEMLIMIT, "run_kFkB: plan k=%d needs %zu activation bytes, limit is %zu", k, stage_activation_bytes(k, M), mem_limit);
    return fail(KFKB_E_MEMLIMIT, "run_kFkB: plan k=%d needs a workspace of stage_workspace_bytes(%d) = %zu bytes, %zu bound", k, k, stage_workspace_bytes(k), g.ws_bytes);
  }
  std::vector<kfkb_op_t> order, plan;
  build_order(k, M, warmup_for(g, k, M), order);
  build_receive_plan(order, k, plan);
  reset_iteration_state();
  g.last_k = k;
  TRY(begin_log_epoch());
  HIPCHK(hipStreamWaitEvent(g.ss, g.ev_epoch, 0));
  HIPCHK(hipStreamWaitEvent(g.sr, g.ev_epoch, 0));
  // Ops are admitted in schedule order, as many as there are lanes at a time and only while an activation
  // slot is free (the plan's peak of live micro-batches is never exceeded: k = 1 on the last stage runs one op
  // at a time); the blocks of the ops in flight are enqueued in turn.
  // W-step windows: the backwards of a schedule unit, in runs of at most `wcap`; a run of one accumulates by itself
  const int wcap = g.wstep_grouped ? std::min(g.wwin_cap, g.wwin_max) : 1;
  std::vector<int> wpos(order.size(), 0), wsize(order.size(), 0);
  if (wcap >= 2) {
    for (size_t i = 0; i < order.size();) {
      if (order[i].op != KFKB_OP_B) { i++; continue; }
      size_t j = i;
      while (j < order.size() && order[j].op == KFKB_OP_B) j++;          // the unit [i, j)
      for (size_t b0 = i; b0 < j; b0 += wcap) {
        const int n = (int)std::min<size_t>(wcap, j - b0);
        for (int p2 = 0; p2 < n; p2++) { wpos[b0 + p2] = p2; wsize[b0 + p2] = n; }
      }
      i = j;
    }
  }
  g.w_open = false;
  size_t rp = 0, next = 0;
  std::vector<ActiveOp> act;
  while (next < order.size() || !act.empty()) {
    while (rp < plan.size()) {                        // receives run ahead as far as slots and the echo allow
      const int rc = issue_recv(plan[rp].op, plan[rp].mb);
      if (rc < 0) return rc;
      if (rc == 1) break;
      rp++;
    }
    while (next < order.size() && (int)act.size() < g.lanes) {
      int lane = 0;
      for (const auto& a : act) if (a.lane == lane) lane = 1 - lane;
      ActiveOp a;
      const bool wait_ok = !act.empty();
      const int rc = order[next].op == KFKB_OP_F ? begin_forward(order[next].mb, lane, wait_ok, a)
                                                 : begin_backward(order[next].mb, lane, wait_ok, a, wpos[next], wsize[next]);
      if (rc < 0) return rc;
      if (rc == 1) break;                             // needs something an op in flight still holds
      act.push_back(a);
      next++;
    }
    for (size_t i = 0; i < act.size();) {
      ActiveOp& a = act[i];
      a.other_busy = act.size() > 1;
      TRY(a.op == KFKB_OP_F ? forward_block(a) : backward_block(a));
      if (a.left == 0) {
        TRY(a.op == KFKB_OP_F ? end_forward(a) : end_backward(a));
        act.erase(act.begin() + i);
      } else {
        i++;
      }
    }
  }
  // the run ends when the last transfer has landed and both lanes have drained
  hipStream_t q0 = g.lane[0].s;
  HIPCHK(hipStreamWaitEvent(q0, g.ev_dxs[order.back().mb], 0));
  TRY(join_compute_streams(q0));
  HIPCHK(hipEventRecord(g.ev_run_end, q0));
  g.run_timed = true;
  return 0;
}


int kfkb_enumerate_candidates(int global_batch, size_t mem_limit, size_t bytes_per_sample, int num_stages,
                              int stage_index, int k_max, int* out_k, int* out_b, int cap) {
  if (global_batch < 1 || num_stages < 1 || stage_index < 0 || stage_index >= num_stages || k_max < 0 || cap < 0 ||
      (cap > 0 && (out_k == nullptr || out_b == nullptr)))
    return fail(KFKB_E_ARG, "kfkb_enumerate_candidates: bad argument");
  int n = 0;
  for (int k = 1; k <= global_batch && (k_max == 0 || k <= k_max); k++) {
    int best = 0;
    for (int b = global_batch; b >= 1 && best == 0; b--) {
      if (global_batch % b != 0) continue;
      const int M = global_batch / b;
      if (M < k) continue;
      const int G = (M + k - 1) / k;
      const int w = std::min(num_stages - 1 - stage_index, G);
      const size_t live = (size_t)std::min((w + 1) * k, M);
      // live * b * bytes_per_sample <= mem_limit without overflow
      if (bytes_per_sample == 0 || live * (size_t)b <= mem_limit / bytes_per_sample) best = b;
    }
    if (best == 0) break;
    if (n < cap) { out_k[n] = k; out_b[n] = best; }
    n++;
  }
  return std::min(n, cap);
}

double kfkb_predict_iteration_ms(int k, int num_microbatches, int warmup_groups, double t_fwd, double t_bwd,
                                 double t_recv_x, double t_recv_dy, double t_send_y, double t_send_dx,
                                 int x_slots, int dy_slots) {
  const int M = num_microbatches;
  if (M < 1 || k < 1 || k > M || warmup_groups < 0 || t_fwd < 0 || t_bwd < 0 || t_recv_x < 0 || t_recv_dy < 0 ||
      t_send_y < 0 || t_send_dx < 0 || x_slots < 0 || dy_slots < 0)
    return (double)fail(KFKB_E_ARG, "kfkb_predict_iteration_ms: need 1 <= k <= M, w >= 0 and non-negative times");
  const double tc[4] = {t_recv_x, t_recv_dy, t_send_y, t_send_dx};
  const double t = predict_iteration(k, M, warmup_groups, t_fwd, t_bwd, tc, x_slots, dy_slots);
  if (t < 0.0) return (double)fail(KFKB_E_STATE, "kfkb_predict_iteration_ms: the slot pools cannot feed plan k=%d", k);
  return t;
}

int kfkb_tuner_config(int window, int interval, const int* candidates, int num_candidates) {
  if (window < 1 || interval < 1 || candidates == nullptr || num_candidates < 1 || num_candidates > 8)
    return fail(KFKB_E_ARG, "kfkb_tuner_config: window, interval >= 1 and 1..8 candidates");
  std::vector<int> c(candidates, candidates + num_candidates);
  std::sort(c.begin(), c.end());
  if (c.front() < 1 || std::adjacent_find(c.begin(), c.end()) != c.end())
    return fail(KFKB_E_ARG, "kfkb_tuner_config: candidates must be distinct and positive");
  g_tuner = TunerState{};
  g_tuner.window = window; g_tuner.interval = interval; g_tuner.candidates = c;
  g_tuner.tf.assign(c.size(), -1.0); g_tuner.tb.assign(c.size(), -1.0);
  g_tuner.estimates.assign(c.size(), -1.0);
  g_tuner.k = c.front();
  return 0;
}

int kfkb_tuner_set_compute_profile(int k, double t_fwd, double t_bwd) {
  if (t_fwd < 0 || t_bwd < 0) return fail(KFKB_E_ARG, "kfkb_tuner_set_compute_profile: negative time");
  for (size_t i = 0; i < g_tuner.candidates.size(); i++)
    if (g_tuner.candidates[i] == k) { g_tuner.tf[i] = t_fwd; g_tuner.tb[i] = t_bwd; return 0; }
  return fail(KFKB_E_ARG, "kfkb_tuner_set_compute_profile: k = %d is not a candidate", k);
}

int kfkb_tuner_push_sample(double t_recv_x, double t_recv_dy, double t_send_y, double t_send_dx) {
  const double v[4] = {t_recv_x, t_recv_dy, t_send_y, t_send_dx};
  for (int d = 0; d < 4; d++) {
    if (v[d] < 0) return fail(KFKB_E_ARG, "kfkb_tuner_push_sample: negative time");
    g_tuner.samples[d].push_back(v[d]);
    if ((int)g_tuner.samples[d].size() > g_tuner.window) g_tuner.samples[d].erase(g_tuner.samples[d].begin());
  }
  g_tuner.iterations++;
  return 0;
}

int kfkb_tuner_next_k(int num_microbatches, int warmup_groups, size_t mem_limit, size_t bytes_per_microbatch,
                      double* estimates, int cap) {
  const int M = num_microbatches;
  if (M < 1 || warmup_groups < 0) return fail(KFKB_E_ARG, "kfkb_tuner_next_k: need M >= 1 and w >= 0");
  TunerState& t = g_tuner;
  if (t.iterations > 0 && t.iterations % t.interval == 0) {
    const double tc[4] = {t.mean(0), t.mean(1), t.mean(2), t.mean(3)};
    int best = -1;
    for (size_t i = 0; i < t.candidates.size(); i++) {
      const int k = t.candidates[i];
      t.estimates[i] = -1.0;
      if (k > M || t.tf[i] < 0.0) continue;
      const int G = (M + k - 1) / k;
      const size_t live = (size_t)std::min((std::min(warmup_groups, G) + 1) * k, M);
      if (mem_limit != 0 && live * bytes_per_microbatch > mem_limit) continue;
      t.estimates[i] = predict_iteration(k, M, warmup_groups, t.tf[i], t.tb[i], tc, 0, 0);
      if (t.estimates[i] >= 0.0 && (best < 0 || t.estimates[i] < t.estimates[best])) best = (int)i;
    }
    if (best < 0) return fail(KFKB_E_MEMLIMIT, "kfkb_tuner_next_k: no admissible candidate");
    t.k = t.candidates[best];
  }
  if (estimates != nullptr)
    for (int i = 0; i < cap && i < (int)t.estimates.size(); i++) estimates[i] = t.estimates[i];
  return t.k;
}

int stage_get_transfer_ms(int direction, double* out, int cap) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_get_transfer_ms before stage_init");
  if (direction < 0 || direction > 3 || (out == nullptr && cap > 0)) return fail(KFKB_E_ARG, "stage_get_transfer_ms: direction 0..3");
  const std::vector<hipEvent_t>* t1[4] = {&g.ev_x, &g.ev_dy, &g.ev_ys, &g.ev_dxs};
  int n = 0;
  for (int mb = 0; mb < g.Mmax && n < cap; mb++) {
    const MbState& st = g.mb[mb];
    const bool done = direction == 0 ? st.x_issued : direction == 1 ? st.dy_issued : direction == 2 ? st.fwd_done : st.bwd_done;
    if (!done) break;
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, g.ev_t0[direction][mb], (*t1[direction])[mb]));
    out[n++] = (double)ms;
  }
  return n;
}

// mean transfer time per direction of the last iteration -> the tuner's windows
static int tuner_observe_last() {
  TRY(stage_sync());
  double mean[4];
  std::vector<double> buf(g.Mmax);
  for (int d = 0; d < 4; d++) {
    const int n = stage_get_transfer_ms(d, buf.data(), g.Mmax);
    if (n < 0) return n;
    if (n == 0) return fail(KFKB_E_STATE, "tuner: the last iteration has no transfers to observe");
    double s = 0.0;
    for (int i = 0; i < n; i++) s += buf[i];
    mean[d] = s / n;
  }
  return kfkb_tuner_push_sample(mean[0], mean[1], mean[2], mean[3]);
}

int stage_tuner_calibrate(int num_microbatches, int repeats) {
  if (!g.bound) return fail(KFKB_E_STATE, "stage_tuner_calibrate before stage_bind");
  const int M = num_microbatches;
  if (M < 1 || M > g.Mmax || repeats < 1) return fail(KFKB_E_ARG, "stage_tuner_calibrate: need 1 <= M <= %d and repeats >= 1", g.Mmax);
  if (live_count() != 0) return fail(KFKB_E_STATE, "stage_tuner_calibrate while micro-batches are live");
  const auto dx = g.dl_x, ddy = g.dl_dy, dy = g.dl_y, ddx = g.dl_dx;
  auto restore = [&]() { g.dl_x = dx; g.dl_dy = ddy; g.dl_y = dy; g.dl_dx = ddx; };
  for (auto* v : {&g.dl_x, &g.dl_dy, &g.dl_y, &g.dl_dx}) std::fill(v->begin(), v->end(), 0);
  std::vector<kfkb_op_t> log(2 * (size_t)M);
  for (size_t i = 0; i < g_tuner.candidates.size(); i++) {
    const int k = g_tuner.candidates[i];
    if (k > M || k > g.k_bound) continue;
    double sf = 0.0, sb = 0.0, total = 0.0;
    int rc = run_kFkB(k, M, 0);                       // warm-up of this plan
    if (rc == 0) rc = stage_sync();
    for (int r = 0; rc == 0 && r < repeats; r++) {
      rc = run_kFkB(k, M, 0);
      if (rc == 0) rc = stage_sync();
      if (rc != 0) break;
      const int n = stage_get_order(log.data(), (int)log.size());
      if (n < 0) { rc = n; break; }
      for (int j = 0; j < n; j++) (log[j].op == KFKB_OP_F ? sf : sb) += log[j].t_end_ms - log[j].t_start_ms;
      total += stage_last_run_ms();
    }
    if (rc != 0) { restore(); return rc; }
    const double tf = sf / ((double)repeats * M), tb = sb / ((double)repeats * M);
    // ops of two lanes overlap: scale the op times so that M of each add up to the measured iteration
    const double scale = (tf + tb) > 0.0 ? (total / repeats) / (M * (tf + tb)) : 1.0;
    g_tuner.tf[i] = tf * scale; g_tuner.tb[i] = tb * scale;
  }
  restore();
  g.adaptive_pending = false;
  return 0;
}

int run_kFkB_adaptive(int num_microbatches, size_t mem_limit) {
  if (!g.bound) return fail(KFKB_E_STATE, "run_kFkB_adaptive before stage_bind");
  if (g.adaptive_pending) TRY(tuner_observe_last());
  const int w = 0;                                    // evaluated with each plan's own warm-up depth below
  (void)w;
  const size_t per_mb = kfkb_activation_bytes_per_microbatch_ex(g.L, g.b, g.T, g.H, g.heads, g.F, (int)g.esz, g.recompute ? 1 : 0);
  const int S = std::max(1, g.cfg.num_stages);
  const int k = kfkb_tuner_next_k(num_microbatches, std::max(0, S - 1 - g.cfg.stage_index), mem_limit, per_mb, nullptr, 0);
  if (k < 0) return k;
  TRY(run_kFkB(k, num_microbatches, mem_limit));
  g.adaptive_pending = true;
  return k;
}


int kfkb_pipeline_schedule(int num_stages, int k, int num_microbatches, kfkb_pipe_op_t* out, int cap) {
  const int S = num_stages, M = num_microbatches;
  if (S < 1 || M < 1 || k < 1 || k > M) return fail(KFKB_E_ARG, "kfkb_pipeline_schedule: need S >= 1 and 1 <= k <= M (S=%d k=%d M=%d)", S, k, M);
  if ((long long)2 * S * M > cap || out == nullptr) return fail(KFKB_E_ARG, "kfkb_pipeline_schedule: out holds %d ops, %lld needed", cap, (long long)2 * S * M);
  std::vector<PipeEntry> sched;
  TRY(pipeline_list_schedule(S, k, M, sched));
  for (size_t i = 0; i < sched.size(); i++) out[i] = kfkb_pipe_op_t{sched[i].stage, sched[i].op, sched[i].mb, 0.0, 0.0};
  return (int)sched.size();
}

size_t stage_pipeline_bytes(int num_stages, int num_microbatches) {
  if (!g.inited || num_stages < 1 || num_microbatches < 1) return 0;
  const size_t cells = (size_t)(num_stages - 1) * num_microbatches;
  return 3 * cells * align_up(g.n * g.esz) + align_up(2 * cells * sizeof(long long)) + 256;
}

int stage_pipeline_bind(void* buffer, size_t bytes, int num_stages, int num_microbatches) {
  const int S = num_stages, M = num_microbatches;
  if (!g.bound) return fail(KFKB_E_STATE, "stage_pipeline_bind before stage_bind");
  if (S < 1 || M < 1 || M > g.Mmax) return fail(KFKB_E_ARG, "stage_pipeline_bind: need S >= 1 and 1 <= M <= %d (S=%d M=%d)", g.Mmax, S, M);
  if (g.L % S != 0) return fail(KFKB_E_ARG, "stage_pipeline_bind: %d blocks do not divide into %d stages", g.L, S);
  if (g.n_stash < M) return fail(KFKB_E_MEMLIMIT, "stage_pipeline_bind: the bound workspace holds %d activation slots, %d micro-batches need one each", g.n_stash, M);
  if (S > 1 && (buffer == nullptr || ((uintptr_t)buffer & 255) != 0)) return fail(KFKB_E_ARG, "stage_pipeline_bind: buffer must be non-null and 256-byte aligned");
  if (bytes < stage_pipeline_bytes(S, M)) return fail(KFKB_E_MEMLIMIT, "stage_pipeline_bind: %zu bytes given, stage_pipeline_bytes(%d, %d) = %zu", bytes, S, M, stage_pipeline_bytes(S, M));
  if (live_count() != 0) return fail(KFKB_E_STATE, "stage_pipeline_bind while micro-batches are live");
  TRY(stage_sync());
  pipeline_release();
  gp.S = S; gp.M = M;
  const size_t cells = (size_t)(S - 1) * M;
  gp.wire = (char*)buffer;
  gp.stamps = reinterpret_cast<long long*>(gp.wire + 3 * cells * align_up(g.n * g.esz));
  TRY(make_events(gp.ev_f0, S * M)); TRY(make_events(gp.ev_f1, S * M));
  TRY(make_events(gp.ev_b0, S * M)); TRY(make_events(gp.ev_b1, S * M)); TRY(make_events(gp.ev_w, S * M));
  TRY(make_events(gp.ev_tf, (int)cells)); TRY(make_events(gp.ev_tb, (int)cells));
  for (auto& e : gp.ev_join) HIPCHK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
  gp.dl_f.assign(cells, 0); gp.dl_b.assign(cells, 0);
  gp.bound = true;
  return 0;
}

int stage_set_pipeline_delays(const int64_t* forward_ns, const int64_t* backward_ns) {
  if (!gp.bound) return fail(KFKB_E_STATE, "stage_set_pipeline_delays before stage_pipeline_bind");
  for (size_t i = 0; i < gp.dl_f.size(); i++) {
    gp.dl_f[i] = forward_ns ? std::max<int64_t>(0, forward_ns[i]) : 0;
    gp.dl_b[i] = backward_ns ? std::max<int64_t>(0, backward_ns[i]) : 0;
  }
  return 0;
}

int run_pipeline_kFkB(int k) {
  if (!gp.bound || !g.bound) return fail(KFKB_E_STATE, "run_pipeline_kFkB before stage_pipeline_bind");
  const int S = gp.S, M = gp.M;
  if (k < 1 || k > M) return fail(KFKB_E_ARG, "run_pipeline_kFkB: need 1 <= k <= M (k=%d M=%d)", k, M);
  if (live_count() != 0) return fail(KFKB_E_STATE, "run_pipeline_kFkB while micro-batches are live");
  std::vector<PipeEntry> sched;
  TRY(pipeline_list_schedule(S, k, M, sched));
  // nothing of an earlier iteration may still be running: every stream waits for every other
  hipStream_t all[4] = {g.lane[0].s, g.lane[1].s, g.ss, g.sr};
  for (int i = 0; i < 4; i++) HIPCHK(hipEventRecord(gp.ev_join[i], all[i]));
  for (int i = 0; i < 4; i++)
    for (int j = 0; j < 4; j++) if (i != j) HIPCHK(hipStreamWaitEvent(all[i], gp.ev_join[j], 0));
  reset_iteration_state();
  g.stash_free.clear();                                  // micro-batch mb owns activation slot mb
  for (int mbi = 0; mbi < M; mbi++) { g.mb[mbi].stash = mbi; g.stash_release[mbi] = nullptr; }
  g.last_k = k;
  TRY(begin_log_epoch());
  HIPCHK(hipStreamWaitEvent(g.ss, g.ev_epoch, 0));
  HIPCHK(hipStreamWaitEvent(g.sr, g.ev_epoch, 0));
  gp.log.clear();
  std::vector<char> f_ended((size_t)S * M, 0), b_ended((size_t)S * M, 0);
  struct Act { ActiveOp a; int stage; };
  std::vector<Act> act;
  size_t next = 0;
  while (next < sched.size() || !act.empty()) {
    while (next < sched.size() && (int)act.size() < g.lanes) {
      const PipeEntry e = sched[next];
      const size_t me = (size_t)e.stage * M + e.mb;
      bool ready;
      if (e.op == KFKB_OP_F) ready = e.stage == 0 || f_ended[me - M];
      else ready = f_ended[me] && (e.stage == S - 1 || b_ended[me + M]);
      if (!ready) break;                                // its producer is still being enqueued
      int lane = 0;
      for (const auto& x : act) if (x.a.lane == lane) lane = 1 - lane;
      Act n; n.stage = e.stage;
      const int rc = e.op == KFKB_OP_F ? pipe_begin_forward(e.stage, e.mb, lane, n.a) : pipe_begin_backward(e.stage, e.mb, lane, n.a);
      if (rc < 0) return rc;
      if (rc == 1) break;                               // a buffer an op in flight still holds
      act.push_back(n);
      next++;
    }
    if (act.empty()) return fail(KFKB_E_STATE, "run_pipeline_kFkB: op %zu of the schedule cannot start (stage %d, micro-batch %d)", next, sched[next].stage, sched[next].mb);
    for (size_t i = 0; i < act.size();) {
      ActiveOp& a = act[i].a;
      a.other_busy = act.size() > 1;
      TRY(a.op == KFKB_OP_F ? forward_block(a) : backward_block(a));
      if (a.left == 0) {
        TRY(a.op == KFKB_OP_F ? pipe_end_forward(a, act[i].stage) : pipe_end_backward(a, act[i].stage));
        (a.op == KFKB_OP_F ? f_ended : b_ended)[(size_t)act[i].stage * M + a.mb] = 1;
        act.erase(act.begin() + i);
      } else {
        i++;
      }
    }
  }
  hipStream_t q0 = g.lane[0].s;
  HIPCHK(hipStreamWaitEvent(q0, g.ev_dxs[sched.back().mb], 0));
  TRY(join_compute_streams(q0));
  HIPCHK(hipEventRecord(g.ev_run_end, q0));
  g.run_timed = true;
  // whoever takes an activation slot next (a single-stage run on the same binding) waits for the end of this run
  for (int mbi = 0; mbi < M; mbi++) { g.stash_release[mbi] = g.ev_run_end; g.mb[mbi].stash = -1; }
  return 0;
}

int stage_get_pipeline_order(kfkb_pipe_op_t* out, int cap) {
  if (!gp.bound) return fail(KFKB_E_STATE, "stage_get_pipeline_order before stage_pipeline_bind");
  if (out == nullptr && cap > 0) return fail(KFKB_E_ARG, "stage_get_pipeline_order: null output");
  const int n = std::min<int>(cap, (int)gp.log.size());
  for (int i = 0; i < n; i++) {
    const PipeEntry& e = gp.log[i];
    const size_t c = (size_t)e.stage * gp.M + e.mb;
    float t0 = 0.f, t1 = 0.f;
    HIPCHK(hipEventElapsedTime(&t0, g.ev_epoch, e.op == KFKB_OP_F ? gp.ev_f0[c] : gp.ev_b0[c]));
    HIPCHK(hipEventElapsedTime(&t1, g.ev_epoch, e.op == KFKB_OP_F ? gp.ev_f1[c] : gp.ev_b1[c]));
    out[i] = kfkb_pipe_op_t{e.stage, e.op, e.mb, (double)t0, (double)t1};
  }
  return n;
}

int stage_last_k(void) { return g.last_k; }

int stage_side_streams_overlap(void) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_side_streams_overlap before stage_init");
  for (hipStream_t q : {g.lane[0].s, g.lane[1].s, g.ss, g.sr}) HIPCHK(hipStreamSynchronize(q));
  for (int rep = 0; rep < 2; rep++) {                 // first round warms the launch path up
    const auto t0 = std::chrono::steady_clock::now();
    for (hipStream_t s : {g.lane[0].s, g.ss, g.sr}) HIPCHK(launch_delay(rep == 0 ? 1000 : 1000000, s));
    for (hipStream_t s : {g.lane[0].s, g.ss, g.sr}) HIPCHK(hipStreamSynchronize(s));
    const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    if (rep == 1) return ms < 1.8 ? 1 : 0;
  }
  return 0;
}

int stage_zero_grads(void) {
  if (!g.bound) return fail(KFKB_E_STATE, "stage_zero_grads before stage_bind");
  hipStream_t q0 = g.lane[0].s;
  TRY(join_compute_streams(q0));                                        // accumulation may still be in flight there
  HIPCHK(launch_fill_zero(g.grad, (size_t)g.L * g.po.total, q0));
  HIPCHK(hipEventRecord(g.ev_zero, q0));
  HIPCHK(hipStreamWaitEvent(g.lane[1].s, g.ev_zero, 0));
  std::fill(g.ev_g_set.begin(), g.ev_g_set.end(), 0);
  return 0;
}

int stage_set_wgrad_stream(int enable) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_set_wgrad_stream before stage_init");
  if (g.bound && live_count() != 0) return fail(KFKB_E_STATE, "stage_set_wgrad_stream while micro-batches are live");
  for (int i = 0; i < 2; i++) HIPCHK(hipStreamSynchronize(g.lane[i].s));
  const int prev = g.wgrad_overlap ? 1 : 0;
  g.wgrad_overlap = enable != 0;
  return prev;
}

int stage_set_fused_w_reductions(int enable) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_set_fused_w_reductions before stage_init");
  if (g.bound && live_count() != 0) return fail(KFKB_E_STATE, "stage_set_fused_w_reductions while micro-batches are live");
  for (int i = 0; i < 2; i++) HIPCHK(hipStreamSynchronize(g.lane[i].s));
  const int prev = g.fuse_w_reductions ? 1 : 0;
  g.fuse_w_reductions = enable != 0;
  return prev;
}

int stage_set_wstep_window(int max_microbatches) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_set_wstep_window before stage_init");
  if (max_microbatches < 1) return fail(KFKB_E_ARG, "stage_set_wstep_window: need a window of at least 1 micro-batch (got %d)", max_microbatches);
  if (g.bound && live_count() != 0) return fail(KFKB_E_STATE, "stage_set_wstep_window while micro-batches are live");
  const int prev = g.wwin_max;
  g.wwin_max = std::min(max_microbatches, kWSeg);
  return prev;
}

int stage_set_send_copy_blocks(int blocks) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_set_send_copy_blocks before stage_init");
  if (blocks < 0 || blocks > 4096) return fail(KFKB_E_ARG, "stage_set_send_copy_blocks: 0 (the runtime's copy) or 1 .. 4096 workgroups (got %d)", blocks);
  const int prev = g.send_blocks;
  g.send_blocks = blocks;
  return prev;
}

int kfkb_set_inputs_ahead(int mode) {
  if (mode < 0 || mode > 2) return fail(KFKB_E_ARG, "kfkb_set_inputs_ahead: mode is 0, 1 or 2 (by k) (got %d)", mode);
  const int prev = g_inputs_ahead_mode;
  g_inputs_ahead_mode = mode;
  return prev;
}

int kfkb_set_mid_tiles(int mode, int rate_percent) {
  if (mode < 0 || mode > 2 || rate_percent < 1 || rate_percent > 100)
    return fail(KFKB_E_ARG, "kfkb_set_mid_tiles: mode 0 .. 2 and rate 1 .. 100 percent (got %d, %d)", mode, rate_percent);
  const int prev = kfkb::g_mid_tile_mode;
  kfkb::g_mid_tile_mode = mode;
  kfkb::g_mid_tile_rate = rate_percent;
  return prev;
}

int kfkb_set_big_tile_min(int tiles) {
  if (tiles < 1) return fail(KFKB_E_ARG, "kfkb_set_big_tile_min: need tiles >= 1 (got %d)", tiles);
  const int prev = kfkb::g_big_tile_min;
  kfkb::g_big_tile_min = tiles;
  return prev;
}

int stage_set_compute_lanes(int lanes) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_set_compute_lanes before stage_init");
  if (lanes != 1 && lanes != 2) return fail(KFKB_E_ARG, "stage_set_compute_lanes: 1 or 2 lanes (got %d)", lanes);
  if (g.bound && live_count() != 0) return fail(KFKB_E_STATE, "stage_set_compute_lanes while micro-batches are live");
  for (int i = 0; i < 2; i++) HIPCHK(hipStreamSynchronize(g.lane[i].s));
  const int prev = g.lanes;
  g.lanes = lanes;
  return prev;
}

int stage_sync(void) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_sync before stage_init");
  for (int i = 0; i < 2; i++) HIPCHK(hipStreamSynchronize(g.lane[i].s));
  HIPCHK(hipStreamSynchronize(g.sr));
  HIPCHK(hipStreamSynchronize(g.ss));
  return 0;
}

int stage_sync_timeout(double seconds) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_sync_timeout before stage_init");
  const auto t0 = std::chrono::steady_clock::now();
  for (;;) {
    bool done = true;
    for (hipStream_t s : {g.lane[0].s, g.lane[1].s, g.sr, g.ss}) {
      hipError_t e = hipStreamQuery(s);
      if (e == hipErrorNotReady) done = false;
      else if (e != hipSuccess) return fail(KFKB_E_HIP, "hipStreamQuery failed: %s", hipGetErrorString(e));
    }
    if (done) return 0;
    if (std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > seconds)
      return fail(KFKB_E_TIMEOUT, "stage_sync_timeout: work still pending after %.3f s", seconds);
    std::this_thread::sleep_for(std::chrono::microseconds(200));
  }
}

int stage_get_order(kfkb_op_t* out, int cap) {
  if (!g.inited) return fail(KFKB_E_STATE, "stage_get_order before stage_init");
  if (out == nullptr && cap > 0) return fail(KFKB_E_ARG, "stage_get_order: null output");
  const int n = std::min<int>(cap, (int)g.log.size());
  for (int i = 0; i < n; i++) {
    const auto& e = g.log[i];
    float t0 = 0.f, t1 = 0.f;
    hipEvent_t a = e.op == KFKB_OP_F ? g.ev_f0[e.mb] : g.ev_b0[e.mb];
    hipEvent_t b = e.op == KFKB_OP_F ? g.ev_f1[e.mb] : g.ev_b1[e.mb];
    HIPCHK(hipEventElapsedTime(&t0, g.ev_epoch, a));
    HIPCHK(hipEventElapsedTime(&t1, g.ev_epoch, b));
    out[i] = kfkb_op_t{e.op, e.mb, (double)t0, (double)t1};
  }
  return n;
}

double stage_last_run_ms(void) {
  if (!g.inited || !g.run_timed) return -1.0;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, g.ev_epoch, g.ev_run_end) != hipSuccess) return -1.0;
  return (double)ms;
}

int stage_destroy(void) {
  if (!g.inited) return 0;
  for (hipStream_t q : {g.lane[0].s, g.lane[1].s, g.sr, g.ss}) hipStreamSynchronize(q);
  pipeline_release();
  for (auto* v : {&g.ev_x, &g.ev_dy, &g.ev_f0, &g.ev_f1, &g.ev_b0, &g.ev_b1, &g.ev_ys, &g.ev_dxs, &g.ev_w, &g.ev_g, &g.ev_t0[0], &g.ev_t0[1], &g.ev_t0[2], &g.ev_t0[3]})
    for (auto e : *v) hipEventDestroy(e);
  for (auto& ln : g.lane) {
    for (int i = 0; i < Stage::kRing; i++) { hipEventDestroy(ln.ev_chain[i]); hipEventDestroy(ln.ev_wdone[i]); }
    hipEventDestroy(ln.ev_tail);
  }
  for (auto e : g.ev_wops) hipEventDestroy(e);
  hipEventDestroy(g.ev_epoch); hipEventDestroy(g.ev_run_end); hipEventDestroy(g.ev_zero);
  g = Stage{};
  g_cfg_set = false;
  return 0;
}

// ---- per-kernel timing ----------------------------------------------------------------------------
int kfkb_profile(int enable) {
  g_prof_on = enable != 0;
  if (g_prof_on) { g_prof_recs.clear(); g_prof_next = 0; }
  return 0;
}

int kfkb_profile_report(kfkb_kernel_stat_t* out, int cap) {
  if (out == nullptr && cap > 0) return fail(KFKB_E_ARG, "kfkb_profile_report: null output");
  std::vector<int> keys;
  std::vector<kfkb_kernel_stat_t> st;
  for (const auto& r : g_prof_recs) {
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, r.e0, r.e1));
    size_t i = 0;
    for (; i < keys.size(); i++) if (keys[i] == r.key) break;
    if (i == keys.size()) {
      keys.push_back(r.key);
      kfkb_kernel_stat_t z{};
      prof_key_name(r.key, z.name, sizeof z.name, &z.bound);
      st.push_back(z);
    }
    st[i].launches += 1; st[i].total_ms += ms; st[i].work += r.work;
  }
  const int n = std::min<int>(cap, (int)st.size());
  for (int i = 0; i < n; i++) out[i] = st[i];
  return n;
}

// ---- per-kernel entry points --------------------------------------------------------------------
#define CHECK_DT(dt) if ((dt) != KFKB_F32 && (dt) != KFKB_BF16 && (dt) != KFKB_F16) return fail(KFKB_E_ARG, "unknown dtype %d", (dt))

int kfkb_op_gemm(int dtype, int kind, int epilogue, int M, int N, int K, const void* A, const void* B, const void* bias,
                 const void* residual, void* C, void* C2, float* Cacc, void* stream) {
  CHECK_DT(dtype);
  if (kind < KFKB_GEMM_NN || kind > KFKB_GEMM_TN || epilogue < KFKB_EPI_NONE || epilogue > KFKB_EPI_GELU_BWD)
    return fail(KFKB_E_ARG, "kfkb_op_gemm: bad kind or epilogue");
  if (M < 0 || N < 0 || K < 0 || !A || !B) return fail(KFKB_E_ARG, "kfkb_op_gemm: bad shape or null operand");
  const bool need_bias = epilogue == KFKB_EPI_BIAS || epilogue == KFKB_EPI_BIAS_GELU || epilogue == KFKB_EPI_BIAS_RES;
  const bool need_res = epilogue == KFKB_EPI_BIAS_RES || epilogue == KFKB_EPI_GELU_BWD;
  if ((need_bias && !bias) || (need_res && !residual) || (epilogue == KFKB_EPI_BIAS_GELU && !C2) ||
      (epilogue == KFKB_EPI_ACCUM ? !Cacc : !C))
    return fail(KFKB_E_ARG, "kfkb_op_gemm: epilogue %d misses an operand", epilogue);
  if (M == 0 || N == 0) return 0;
  GemmArgs a{kind, epilogue, M, N, K, A, B, bias, residual, C, C2, Cacc};
  if (dtype != KFKB_F32) {
    const char* why = gemm_bf16_check(a);
    if (why) return fail(KFKB_E_ARG, "%s (M=%d N=%d K=%d)", why, M, N, K);
    HIPCHK(launch_gemm_16(dtype, a, (hipStream_t)stream));
  } else {
    HIPCHK(launch_gemm_f32(a, (hipStream_t)stream));
  }
  return 0;
}

int kfkb_op_tile_weights(const void* src, void* dst, int N, int K, int transposed, void* stream) {
  if (!src || !dst || N <= 0 || K <= 0 || N % 8 != 0 || K % 32 != 0)
    return fail(KFKB_E_ARG, "kfkb_op_tile_weights: need N %% 8 == 0, K %% 32 == 0 and non-null pointers (N=%d K=%d)", N, K);
  HIPCHK(launch_tile_weights(src, dst, N, K, transposed != 0, (hipStream_t)stream));
  return 0;
}

int kfkb_op_gemm_nt_tiled(int epilogue, int M, int N, int K, const void* A, const void* Bt, const void* bias,
                          const void* residual, void* C, void* C2, float* Cacc, void* stream) {
  if (epilogue < KFKB_EPI_NONE || epilogue > KFKB_EPI_GELU_BWD) return fail(KFKB_E_ARG, "kfkb_op_gemm_nt_tiled: bad epilogue");
  if (M < 0 || N < 0 || K < 0 || !A || !Bt) return fail(KFKB_E_ARG, "kfkb_op_gemm_nt_tiled: bad shape or null operand");
  const bool need_bias = epilogue == KFKB_EPI_BIAS || epilogue == KFKB_EPI_BIAS_GELU || epilogue == KFKB_EPI_BIAS_RES;
  const bool need_res = epilogue == KFKB_EPI_BIAS_RES || epilogue == KFKB_EPI_GELU_BWD;
  if ((need_bias && !bias) || (need_res && !residual) || (epilogue == KFKB_EPI_BIAS_GELU && !C2) ||
      (epilogue == KFKB_EPI_ACCUM ? !Cacc : !C))
    return fail(KFKB_E_ARG, "kfkb_op_gemm_nt_tiled: epilogue %d misses an operand", epilogue);
  if (M == 0 || N == 0) return 0;
  GemmArgs a{KFKB_GEMM_NT, epilogue, M, N, K, A, Bt, bias, residual, C, C2, Cacc};
  a.b_tiled = true;
  const char* why = gemm_bf16_check(a);
  if (why) return fail(KFKB_E_ARG, "%s (M=%d N=%d K=%d)", why, M, N, K);
  HIPCHK(launch_gemm_bf16(a, (hipStream_t)stream));
  return 0;
}

static int check_rows(const char* who, int dtype, int rows, int H) {
  if (rows < 0 || H < 8 || H % 8 != 0 || H > 8192 * 4) return fail(KFKB_E_ARG, "%s: need rows >= 0 and width %% 8 == 0 (rows=%d width=%d)", who, rows, H);
  (void)dtype;
  return 0;
}

int kfkb_op_layernorm_fwd(int dtype, const void* x, const void* gamma, const void* beta, void* y, float* mean, float* rstd,
                          int rows, int H, float eps, void* stream) {
  CHECK_DT(dtype);
  TRY(check_rows("kfkb_op_layernorm_fwd", dtype, rows, H));
  if (H > 8192) return fail(KFKB_E_ARG, "kfkb_op_layernorm_fwd: H > 8192");
  if (rows == 0) return 0;
  if (!x || !gamma || !beta || !y || !mean || !rstd) return fail(KFKB_E_ARG, "kfkb_op_layernorm_fwd: null pointer");
  HIPCHK(launch_ln_fwd(dtype, x, gamma, beta, y, mean, rstd, rows, H, eps, (hipStream_t)stream));
  return 0;
}

int kfkb_op_layernorm_bwd(int dtype, const void* dy, const void* x, const float* mean, const float* rstd, const void* gamma,
                          const void* dres, void* dx, float* dgamma, float* dbeta, float* scratch, int rows, int H,
                          void* stream) {
  CHECK_DT(dtype);
  TRY(check_rows("kfkb_op_layernorm_bwd", dtype, rows, H));
  if (H > 8192) return fail(KFKB_E_ARG, "kfkb_op_layernorm_bwd: H > 8192");
  if (rows == 0) return 0;
  if (!dy || !x || !mean || !rstd || !gamma || !dx || !dgamma || !dbeta || !scratch) return fail(KFKB_E_ARG, "kfkb_op_layernorm_bwd: null pointer");
  HIPCHK(launch_ln_bwd(dtype, dy, x, mean, rstd, gamma, dres, dx, dgamma, dbeta, scratch, rows, H, (hipStream_t)stream));
  return 0;
}

int kfkb_op_colsum_accum(int dtype, const void* dy, float* out, float* scratch, int rows, int N, void* stream) {
  CHECK_DT(dtype);
  TRY(check_rows("kfkb_op_colsum_accum", dtype, rows, N));
  if (rows == 0) return 0;
  if (!dy || !out || !scratch) return fail(KFKB_E_ARG, "kfkb_op_colsum_accum: null pointer");
  HIPCHK(launch_colsum_accum(dtype, dy, out, scratch, rows, N, (hipStream_t)stream));
  return 0;
}

size_t kfkb_op_reduce_scratch_floats(int width) { return width > 0 ? (size_t)1024 * width : 0; }

int kfkb_op_gelu_bwd(int dtype, const void* dg, const void* u, void* du, size_t n, void* stream) {
  CHECK_DT(dtype);
  if (n % 8 != 0) return fail(KFKB_E_ARG, "kfkb_op_gelu_bwd: element count must be a multiple of 8");
  if (n && (!dg || !u || !du)) return fail(KFKB_E_ARG, "kfkb_op_gelu_bwd: null pointer");
  HIPCHK(launch_gelu_bwd(dtype, dg, u, du, n, (hipStream_t)stream));
  return 0;
}

static int check_attn(const char* who, int dtype, int b, int T, int H, int heads) {
  if (b < 0 || T < 0 || H < 1 || heads < 1 || H % heads != 0) return fail(KFKB_E_ARG, "%s: bad shape", who);
  const int d = H / heads;
  if (dtype != KFKB_F32 && d != 64 && d != 128) return fail(KFKB_E_ARG, "%s: 16-bit storage needs head size 64 or 128 (got %d)", who, d);
  if (dtype == KFKB_F32 && (d > 128 || T > 4096)) return fail(KFKB_E_ARG, "%s: fp32 needs head size <= 128 and T <= 4096", who);
  // the 16-bit kernels address the rows of one sample's qkv with 32-bit byte offsets
  if (dtype != KFKB_F32 && (double)T * 3.0 * H * 2.0 >= 2147483648.0)
    return fail(KFKB_E_ARG, "%s: T * 3 * H * 2 bytes must stay below 2 GiB for 16-bit storage (T = %d, H = %d)", who, T, H);
  return 0;
}

int kfkb_op_attention_fwd(int dtype, const void* qkv, void* o, float* lse, int b, int T, int H, int heads, int causal,
                          void* stream) {
  CHECK_DT(dtype);
  TRY(check_attn("kfkb_op_attention_fwd", dtype, b, T, H, heads));
  if (b == 0 || T == 0) return 0;
  if (!qkv || !o || !lse) return fail(KFKB_E_ARG, "kfkb_op_attention_fwd: null pointer");
  if (dtype != KFKB_F32) HIPCHK(launch_attention_fwd_16(dtype, qkv, o, lse, b, T, H, heads, causal, (hipStream_t)stream));
  else HIPCHK(launch_attention_fwd_f32((const float*)qkv, (float*)o, lse, b, T, H, heads, causal, (hipStream_t)stream));
  return 0;
}

int kfkb_op_attention_bwd(int dtype, const void* qkv, const void* o, const void* d_o, const float* lse, float* dsum,
                          void* dqkv, int b, int T, int H, int heads, int causal, void* stream) {
  CHECK_DT(dtype);
  TRY(check_attn("kfkb_op_attention_bwd", dtype, b, T, H, heads));
  if (b == 0 || T == 0) return 0;
  if (!qkv || !o || !d_o || !lse || !dsum || !dqkv) return fail(KFKB_E_ARG, "kfkb_op_attention_bwd: null pointer");
  if (dtype != KFKB_F32)
    HIPCHK(launch_attention_bwd_16(dtype, qkv, o, d_o, lse, dsum, dqkv, b, T, H, heads, causal, (hipStream_t)stream));
  else
    HIPCHK(launch_attention_bwd_f32((const float*)qkv, (const float*)o, (const float*)d_o, lse, dsum, (float*)dqkv, b, T, H, heads, causal, (hipStream_t)stream));
  return 0;
}

int kfkb_op_transpose(int dtype, const void* in, void* out, int rows, int cols, void* stream) {
  CHECK_DT(dtype);
  if (rows < 0 || cols < 0) return fail(KFKB_E_ARG, "kfkb_op_transpose: negative size");
  if (rows == 0 || cols == 0) return 0;
  if (!in || !out) return fail(KFKB_E_ARG, "kfkb_op_transpose: null pointer");
  HIPCHK(launch_transpose(dtype, in, out, rows, cols, (hipStream_t)stream));
  return 0;
}

int kfkb_op_delay(int64_t ns, void* stream) {
  if (ns < 0) return fail(KFKB_E_ARG, "kfkb_op_delay: negative delay");
  HIPCHK(launch_delay(ns, (hipStream_t)stream));
  return 0;
}

}  // extern "C"
