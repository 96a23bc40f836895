"""ctypes binding of libkfkb.so: the same names as the C boundary, argument marshalling only."""
import ctypes as C
import os

import numpy as np
import torch

__all__ = [
    "KfkbError", "load_library", "library_path", "F32", "BF16", "F16", "OP_F", "OP_B",
    "GEMM_NN", "GEMM_NT", "GEMM_TN", "EPI_NONE", "EPI_BIAS", "EPI_BIAS_GELU", "EPI_BIAS_RES", "EPI_ACCUM",
    "EPI_GELU_BWD", "PARAM_ORDER", "param_shapes", "param_offsets", "pack_weights", "unpack_params",
    "kfkb_schedule", "kfkb_peak_live", "kfkb_activation_bytes_per_microbatch",
    "kfkb_enumerate_candidates", "kfkb_predict_iteration_ms", "kfkb_tuner_config", "kfkb_tuner_set_compute_profile", "kfkb_tuner_push_sample", "kfkb_tuner_next_k",
    "stage_get_transfer_ms", "stage_tuner_calibrate", "run_kFkB_adaptive",
    "kfkb_pipeline_schedule", "stage_pipeline_bytes", "stage_pipeline_bind", "stage_set_pipeline_delays",
    "run_pipeline_kFkB", "stage_get_pipeline_order",
    "stage_config", "stage_init", "stage_param_count", "stage_activation_bytes", "stage_workspace_bytes",
    "stage_bind", "stage_set_delays", "stage_refresh_weights", "stage_forward", "stage_backward", "run_kFkB",
    "stage_last_k", "stage_side_streams_overlap", "stage_zero_grads", "stage_set_wgrad_stream", "stage_set_compute_lanes", "stage_set_fused_w_reductions", "kfkb_set_big_tile_min", "kfkb_set_mid_tiles", "stage_set_wstep_window", "kfkb_set_inputs_ahead", "stage_set_send_copy_blocks", "stage_sync", "stage_sync_timeout", "stage_destroy", "stage_get_order",
    "stage_last_run_ms", "StageBuffers", "kfkb_profile", "kfkb_profile_report",
    "kfkb_op_gemm", "kfkb_op_tile_weights", "kfkb_op_gemm_nt_tiled", "kfkb_op_layernorm_fwd", "kfkb_op_layernorm_bwd", "kfkb_op_colsum_accum",
    "kfkb_op_colsum_accum_static",
    "kfkb_op_reduce_scratch_floats", "kfkb_op_gelu_bwd", "kfkb_op_attention_fwd", "kfkb_op_attention_bwd",
    "kfkb_op_transpose", "kfkb_op_delay",
]

F32, BF16, F16 = 0, 1, 2
OP_F, OP_B = 0, 1
GEMM_NN, GEMM_NT, GEMM_TN = 0, 1, 2
EPI_NONE, EPI_BIAS, EPI_BIAS_GELU, EPI_BIAS_RES, EPI_ACCUM, EPI_GELU_BWD = range(6)

PARAM_ORDER = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


class KfkbError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("kfkb error %d: %s" % (code, message))
        self.code = code


class _Config(C.Structure):
    _fields_ = [("dtype", C.c_int), ("micro_batch", C.c_int), ("mlp_ratio", C.c_int), ("causal", C.c_int),
                ("ln_eps", C.c_float), ("num_stages", C.c_int), ("stage_index", C.c_int),
                ("max_microbatches", C.c_int), ("recompute", C.c_int)]


class _KernelStat(C.Structure):
    _fields_ = [("name", C.c_char * 80), ("bound", C.c_int), ("launches", C.c_longlong), ("total_ms", C.c_double),
                ("work", C.c_double)]


class _Op(C.Structure):
    _fields_ = [("op", C.c_int), ("mb", C.c_int), ("t_start_ms", C.c_double), ("t_end_ms", C.c_double)]


class _PipeOp(C.Structure):
    _fields_ = [("stage", C.c_int), ("op", C.c_int), ("mb", C.c_int), ("t_start_ms", C.c_double), ("t_end_ms", C.c_double)]


_LIB = None


def library_path():
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkfkb.so")


def load_library():
    """Loads libkfkb.so built in-tree.  There is no fallback: without the library nothing runs."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError("libkfkb.so is not built: run `python -m paper_2303_01675_amd.build` "
                           "(or __graft_entry__.build()) first; expected at " + path)
    lib = C.CDLL(path)
    vp, i, sz, fp, i64p = C.c_void_p, C.c_int, C.c_size_t, C.POINTER(C.c_float), C.POINTER(C.c_int64)
    sigs = {
        "kfkb_last_error": (C.c_char_p, []),
        "kfkb_schedule": (i, [i, i, i, C.POINTER(_Op), i]),
        "kfkb_peak_live": (i, [i, i, i]),
        "kfkb_activation_bytes_per_microbatch": (sz, [i, i, i, i, i, i, i]),
        "kfkb_activation_bytes_per_microbatch_ex": (sz, [i, i, i, i, i, i, i, i]),
        "kfkb_enumerate_candidates": (i, [i, sz, sz, i, i, i, C.POINTER(C.c_int), C.POINTER(C.c_int), i]),
        "kfkb_predict_iteration_ms": (C.c_double, [i, i, i] + [C.c_double] * 6 + [i, i]),
        "kfkb_tuner_config": (i, [i, i, C.POINTER(C.c_int), i]),
        "kfkb_tuner_set_compute_profile": (i, [i, C.c_double, C.c_double]),
        "kfkb_tuner_push_sample": (i, [C.c_double] * 4),
        "kfkb_tuner_next_k": (i, [i, i, sz, sz, C.POINTER(C.c_double), i]),
        "stage_get_transfer_ms": (i, [i, C.POINTER(C.c_double), i]),
        "stage_tuner_calibrate": (i, [i, i]),
        "run_kFkB_adaptive": (i, [i, sz]),
        "stage_config": (i, [C.POINTER(_Config)]),
        "stage_init": (i, [vp, i, i, i, i]),
        "stage_param_count": (sz, []),
        "stage_activation_bytes": (sz, [i, i]),
        "stage_workspace_bytes": (sz, [i]),
        "stage_bind": (i, [vp, sz, vp, vp, vp, vp, vp]),
        "stage_set_delays": (i, [i64p, i64p, i64p, i64p]),
        "stage_refresh_weights": (i, []),
        "stage_forward": (i, [i]),
        "stage_backward": (i, [i]),
        "run_kFkB": (i, [i, i, sz]),
        "stage_last_k": (i, []),
        "stage_side_streams_overlap": (i, []),
        "stage_zero_grads": (i, []),
        "stage_set_wgrad_stream": (i, [i]),
        "stage_set_compute_lanes": (i, [i]),
        "stage_set_fused_w_reductions": (i, [i]),
        "kfkb_set_big_tile_min": (i, [i]),
        "stage_set_wstep_window": (i, [i]),
        "kfkb_set_inputs_ahead": (i, [i]),
        "kfkb_set_mid_tiles": (i, [i, i]),
        "stage_set_send_copy_blocks": (i, [i]),
        "stage_sync": (i, []),
        "stage_sync_timeout": (i, [C.c_double]),
        "stage_destroy": (i, []),
        "stage_get_order": (i, [C.POINTER(_Op), i]),
        "kfkb_pipeline_schedule": (i, [i, i, i, C.POINTER(_PipeOp), i]),
        "stage_pipeline_bytes": (sz, [i, i]),
        "stage_pipeline_bind": (i, [vp, sz, i, i]),
        "stage_set_pipeline_delays": (i, [C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
        "run_pipeline_kFkB": (i, [i]),
        "stage_get_pipeline_order": (i, [C.POINTER(_PipeOp), i]),
        "stage_last_run_ms": (C.c_double, []),
        "kfkb_profile": (i, [i]),
        "kfkb_profile_report": (i, [C.POINTER(_KernelStat), i]),
        "kfkb_op_gemm": (i, [i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, vp]),
        "kfkb_op_tile_weights": (i, [vp, vp, i, i, i, vp]),
        "kfkb_op_gemm_nt_tiled": (i, [i, i, i, i, vp, vp, vp, vp, vp, vp, vp, vp]),
        "kfkb_op_layernorm_fwd": (i, [i, vp, vp, vp, vp, vp, vp, i, i, C.c_float, vp]),
        "kfkb_op_layernorm_bwd": (i, [i, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, vp]),
        "kfkb_op_colsum_accum": (i, [i, vp, vp, vp, i, i, vp]),
        "kfkb_op_colsum_accum_static": (i, [i, vp, vp, i, i, vp]),
        "kfkb_op_reduce_scratch_floats": (sz, [i]),
        "kfkb_op_gelu_bwd": (i, [i, vp, vp, vp, sz, vp]),
        "kfkb_op_attention_fwd": (i, [i, vp, vp, vp, i, i, i, i, i, vp]),
        "kfkb_op_attention_bwd": (i, [i, vp, vp, vp, vp, vp, vp, i, i, i, i, i, vp]),
        "kfkb_op_transpose": (i, [i, vp, vp, i, i, vp]),
        "kfkb_op_delay": (i, [C.c_int64, vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _LIB = lib
    return lib


def _check(rc):
    if rc < 0:
        raise KfkbError(rc, load_library().kfkb_last_error().decode())
    return rc


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        return t.data_ptr()
    return int(t)


def _stream(stream):
    if stream is None:
        return None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


# ---- parameter layout (the flat buffer the C boundary documents) ---------------------------------

def param_shapes(H, F):
    return {"ln1_g": (H,), "ln1_b": (H,), "w_qkv": (H, 3 * H), "b_qkv": (3 * H,), "w_o": (H, H), "b_o": (H,),
            "ln2_g": (H,), "ln2_b": (H,), "w_1": (H, F), "b_1": (F,), "w_2": (F, H), "b_2": (H,)}


def param_offsets(H, F):
    """name -> (offset, shape) inside one block's run, and the run's length."""
    off, out = 0, {}
    for name in PARAM_ORDER:
        shp = param_shapes(H, F)[name]
        out[name] = (off, shp)
        off += int(np.prod(shp))
    return out, off


def pack_weights(blocks, dtype, device="cuda"):
    """blocks: list of dicts of numpy arrays (PARAM_ORDER keys) -> one flat device tensor."""
    flat = np.concatenate([np.asarray(b[n], dtype=np.float32).reshape(-1) for b in blocks for n in PARAM_ORDER])
    t = torch.from_numpy(flat)
    if dtype == BF16:
        t = t.to(torch.bfloat16)
    elif dtype == F16:
        t = t.to(torch.float16)
    return t.to(device)


def unpack_params(flat, L, H, F):
    """flat tensor / array in the boundary layout -> list of dicts of float64 numpy arrays."""
    a = flat.detach().float().cpu().numpy().astype(np.float64) if isinstance(flat, torch.Tensor) else np.asarray(flat, dtype=np.float64)
    offs, per = param_offsets(H, F)
    out = []
    for l in range(L):
        blk = {}
        for name, (o, shp) in offs.items():
            blk[name] = a[l * per + o: l * per + o + int(np.prod(shp))].reshape(shp)
        out.append(blk)
    return out


# ---- host-only planning -------------------------------------------------------------------------------

def kfkb_schedule(k, num_microbatches, warmup_groups=0):
    lib = load_library()
    cap = 2 * max(num_microbatches, 1)
    buf = (_Op * cap)()
    n = _check(lib.kfkb_schedule(k, num_microbatches, warmup_groups, buf, cap))
    return [("F" if buf[j].op == OP_F else "B", buf[j].mb) for j in range(n)]


def kfkb_peak_live(k, num_microbatches, warmup_groups=0):
    return _check(load_library().kfkb_peak_live(k, num_microbatches, warmup_groups))


def kfkb_activation_bytes_per_microbatch(layers, micro_batch, seq, hidden, heads, mlp_width, elem_bytes, recompute=0):
    return load_library().kfkb_activation_bytes_per_microbatch_ex(layers, micro_batch, seq, hidden, heads, mlp_width, elem_bytes,
                                                                  int(recompute))


# ---- the stage -----------------------------------------------------------------------------------------

def kfkb_enumerate_candidates(global_batch, mem_limit, bytes_per_sample, num_stages=1, stage_index=0, k_max=0, cap=4096):
    ks, bs = (C.c_int * cap)(), (C.c_int * cap)()
    n = _check(load_library().kfkb_enumerate_candidates(global_batch, mem_limit, bytes_per_sample, num_stages, stage_index,
                                                        k_max, ks, bs, cap))
    return [(ks[j], bs[j]) for j in range(n)]


def kfkb_predict_iteration_ms(k, num_microbatches, warmup_groups, t_fwd, t_bwd, t_recv_x, t_recv_dy, t_send_y, t_send_dx,
                              x_slots=0, dy_slots=0):
    t = load_library().kfkb_predict_iteration_ms(k, num_microbatches, warmup_groups, t_fwd, t_bwd, t_recv_x, t_recv_dy,
                                                 t_send_y, t_send_dx, x_slots, dy_slots)
    if t < 0:
        _check(int(t))
    return t


def kfkb_tuner_config(window, interval, candidates):
    arr = (C.c_int * len(candidates))(*candidates)
    return _check(load_library().kfkb_tuner_config(window, interval, arr, len(candidates)))


def kfkb_tuner_set_compute_profile(k, t_fwd, t_bwd):
    return _check(load_library().kfkb_tuner_set_compute_profile(k, t_fwd, t_bwd))


def kfkb_tuner_push_sample(t_recv_x, t_recv_dy, t_send_y, t_send_dx):
    return _check(load_library().kfkb_tuner_push_sample(t_recv_x, t_recv_dy, t_send_y, t_send_dx))


def kfkb_tuner_next_k(num_microbatches, warmup_groups=0, mem_limit=0, bytes_per_microbatch=0, num_candidates=8):
    """(k, [estimate of every candidate at the last evaluation, -1 where skipped])"""
    est = (C.c_double * num_candidates)(*([-1.0] * num_candidates))
    k = _check(load_library().kfkb_tuner_next_k(num_microbatches, warmup_groups, mem_limit, bytes_per_microbatch, est, num_candidates))
    return k, list(est)


def stage_get_transfer_ms(direction, cap=4096):
    buf = (C.c_double * cap)()
    n = _check(load_library().stage_get_transfer_ms(direction, buf, cap))
    return [buf[j] for j in range(n)]


def stage_tuner_calibrate(num_microbatches, repeats=2):
    return _check(load_library().stage_tuner_calibrate(num_microbatches, repeats))


def run_kFkB_adaptive(num_microbatches, mem_limit=0):
    return _check(load_library().run_kFkB_adaptive(num_microbatches, mem_limit))


def stage_config(dtype=F32, micro_batch=1, mlp_ratio=4, causal=1, ln_eps=1e-5, num_stages=1, stage_index=0,
                 max_microbatches=1, recompute=0):
    cfg = _Config(dtype, micro_batch, mlp_ratio, causal, ln_eps, num_stages, stage_index, max_microbatches, int(recompute))
    return _check(load_library().stage_config(C.byref(cfg)))


def stage_init(weights, layers, hidden, heads, seq):
    return _check(load_library().stage_init(_ptr(weights), layers, hidden, heads, seq))


def stage_param_count():
    return load_library().stage_param_count()


def stage_activation_bytes(k, num_microbatches):
    return load_library().stage_activation_bytes(k, num_microbatches)


def stage_workspace_bytes(k_max):
    return load_library().stage_workspace_bytes(k_max)


def stage_bind(workspace, grad_accum, host_inputs, host_upstream_grads, host_outputs, host_input_grads):
    return _check(load_library().stage_bind(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _ptr(grad_accum), _ptr(host_inputs), _ptr(host_upstream_grads),
                                            _ptr(host_outputs), _ptr(host_input_grads)))


def stage_set_delays(recv_input_ns=None, recv_upstream_grad_ns=None, send_output_ns=None, send_input_grad_ns=None):
    keep = []

    def arr(a):
        if a is None:
            return None
        a = np.ascontiguousarray(a, dtype=np.int64)
        keep.append(a)
        return a.ctypes.data_as(C.POINTER(C.c_int64))
    return _check(load_library().stage_set_delays(arr(recv_input_ns), arr(recv_upstream_grad_ns),
                                                  arr(send_output_ns), arr(send_input_grad_ns)))


def stage_refresh_weights():
    return _check(load_library().stage_refresh_weights())


def stage_forward(mb):
    return _check(load_library().stage_forward(mb))


def stage_backward(mb):
    return _check(load_library().stage_backward(mb))


def run_kFkB(k, num_microbatches, mem_limit=0):
    return _check(load_library().run_kFkB(k, num_microbatches, int(mem_limit)))


def stage_last_k():
    return load_library().stage_last_k()


def stage_side_streams_overlap():
    return _check(load_library().stage_side_streams_overlap())


def stage_zero_grads():
    return _check(load_library().stage_zero_grads())


def stage_set_wgrad_stream(enable):
    return _check(load_library().stage_set_wgrad_stream(int(bool(enable))))


def stage_set_compute_lanes(lanes):
    return _check(load_library().stage_set_compute_lanes(int(lanes)))


def stage_set_fused_w_reductions(enable):
    return _check(load_library().stage_set_fused_w_reductions(int(bool(enable))))


def kfkb_set_big_tile_min(tiles):
    return _check(load_library().kfkb_set_big_tile_min(int(tiles)))


def stage_set_send_copy_blocks(blocks):
    return _check(load_library().stage_set_send_copy_blocks(int(blocks)))


def kfkb_set_mid_tiles(mode, rate_percent=90):
    return _check(load_library().kfkb_set_mid_tiles(int(mode), int(rate_percent)))


def kfkb_set_inputs_ahead(mode):
    return _check(load_library().kfkb_set_inputs_ahead(int(mode)))


def stage_set_wstep_window(max_microbatches):
    return _check(load_library().stage_set_wstep_window(int(max_microbatches)))


def stage_sync():
    return _check(load_library().stage_sync())


def stage_sync_timeout(seconds):
    return _check(load_library().stage_sync_timeout(float(seconds)))


def stage_destroy():
    return _check(load_library().stage_destroy())


def stage_get_order(cap=4096):
    buf = (_Op * cap)()
    n = _check(load_library().stage_get_order(buf, cap))
    return [("F" if buf[j].op == OP_F else "B", buf[j].mb, buf[j].t_start_ms, buf[j].t_end_ms) for j in range(n)]


def kfkb_pipeline_schedule(num_stages, k, num_microbatches):
    cap = 2 * max(num_stages, 1) * max(num_microbatches, 1)
    buf = (_PipeOp * cap)()
    n = _check(load_library().kfkb_pipeline_schedule(num_stages, k, num_microbatches, buf, cap))
    return [(buf[j].stage, "F" if buf[j].op == OP_F else "B", buf[j].mb) for j in range(n)]


def stage_pipeline_bytes(num_stages, num_microbatches):
    return load_library().stage_pipeline_bytes(num_stages, num_microbatches)


def stage_pipeline_bind(buffer, num_stages, num_microbatches):
    nbytes = buffer.numel() * buffer.element_size() if buffer is not None else 0
    return _check(load_library().stage_pipeline_bind(_ptr(buffer), nbytes, num_stages, num_microbatches))


def stage_set_pipeline_delays(forward_ns=None, backward_ns=None):
    keep = []

    def arr(a):
        if a is None:
            return None
        a = np.ascontiguousarray(a, dtype=np.int64)
        keep.append(a)
        return a.ctypes.data_as(C.POINTER(C.c_int64))
    return _check(load_library().stage_set_pipeline_delays(arr(forward_ns), arr(backward_ns)))


def run_pipeline_kFkB(k):
    return _check(load_library().run_pipeline_kFkB(k))


def stage_get_pipeline_order(cap=16384):
    buf = (_PipeOp * cap)()
    n = _check(load_library().stage_get_pipeline_order(buf, cap))
    return [(buf[j].stage, "F" if buf[j].op == OP_F else "B", buf[j].mb, buf[j].t_start_ms, buf[j].t_end_ms) for j in range(n)]


def stage_last_run_ms():
    return load_library().stage_last_run_ms()


def kfkb_profile(enable):
    return _check(load_library().kfkb_profile(1 if enable else 0))


def kfkb_profile_report(cap=256):
    """List of dicts: name, bound ('mfma' flops | 'hbm' bytes | 'alu' flops), launches, total_ms, work."""
    buf = (_KernelStat * cap)()
    n = _check(load_library().kfkb_profile_report(buf, cap))
    kinds = {0: "mfma", 1: "hbm", 2: "alu"}
    return [dict(name=buf[j].name.decode(), bound=kinds[buf[j].bound], launches=buf[j].launches,
                 total_ms=buf[j].total_ms, work=buf[j].work) for j in range(n)]


class StageBuffers:
    """Allocates, with PyTorch, every buffer the stage borrows, and binds them.  Marshalling only."""

    def __init__(self, blocks, dtype, heads, seq, micro_batch, max_microbatches, k_max, causal=1, mlp_ratio=4,
                 num_stages=1, stage_index=0, ln_eps=1e-5, recompute=0):
        self.dtype = dtype
        self.tdtype = torch.bfloat16 if dtype == BF16 else torch.float16 if dtype == F16 else torch.float32
        self.L = len(blocks)
        self.H = int(np.asarray(blocks[0]["ln1_g"]).shape[0])
        self.F = int(np.asarray(blocks[0]["b_1"]).shape[0])
        self.heads, self.T, self.b, self.M = heads, seq, micro_batch, max_microbatches
        assert self.F == mlp_ratio * self.H
        stage_destroy()
        stage_config(dtype=dtype, micro_batch=micro_batch, mlp_ratio=mlp_ratio, causal=causal, ln_eps=ln_eps,
                     num_stages=num_stages, stage_index=stage_index, max_microbatches=max_microbatches, recompute=recompute)
        self.weights = pack_weights(blocks, dtype)
        stage_init(self.weights, self.L, self.H, heads, seq)
        nbytes = stage_workspace_bytes(k_max)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.grads = torch.zeros(stage_param_count(), dtype=torch.float32, device="cuda")
        shape = (max_microbatches, micro_batch, seq, self.H)
        self.h_in = torch.zeros(shape, dtype=self.tdtype).pin_memory()
        self.h_up = torch.zeros(shape, dtype=self.tdtype).pin_memory()
        self.h_out = torch.zeros(shape, dtype=self.tdtype).pin_memory()
        self.h_ingrad = torch.zeros(shape, dtype=self.tdtype).pin_memory()
        torch.cuda.synchronize()
        stage_bind(self.workspace, self.grads, self.h_in, self.h_up, self.h_out, self.h_ingrad)

    def set_inputs(self, xs, dys):
        for mb, (x, dy) in enumerate(zip(xs, dys)):
            self.h_in[mb].copy_(torch.from_numpy(np.asarray(x, dtype=np.float32)).to(self.tdtype))
            self.h_up[mb].copy_(torch.from_numpy(np.asarray(dy, dtype=np.float32)).to(self.tdtype))

    def set_inputs_one(self, mb, x, dy):
        self.h_in[mb].copy_(torch.from_numpy(np.asarray(x, dtype=np.float32)).to(self.tdtype))
        self.h_up[mb].copy_(torch.from_numpy(np.asarray(dy, dtype=np.float32)).to(self.tdtype))

    def outputs(self, M=None):
        M = self.M if M is None else M
        return (self.h_out[:M].float().numpy().astype(np.float64), self.h_ingrad[:M].float().numpy().astype(np.float64))

    def gradients(self):
        return unpack_params(self.grads, self.L, self.H, self.F)

    def close(self):
        stage_destroy()


# ---- per-kernel entry points ----------------------------------------------------------------------------

def kfkb_op_gemm(dtype, kind, epilogue, M, N, K, A, B, bias=None, residual=None, Cout=None, C2=None, Cacc=None, stream=None):
    return _check(load_library().kfkb_op_gemm(dtype, kind, epilogue, M, N, K, _ptr(A), _ptr(B), _ptr(bias), _ptr(residual),
                                              _ptr(Cout), _ptr(C2), _ptr(Cacc), _stream(stream)))


def kfkb_op_tile_weights(src, dst, N, K, transposed, stream=None):
    return _check(load_library().kfkb_op_tile_weights(_ptr(src), _ptr(dst), N, K, int(bool(transposed)), _stream(stream)))


def kfkb_op_gemm_nt_tiled(epilogue, M, N, K, A, Bt, bias=None, residual=None, Cout=None, C2=None, Cacc=None, stream=None):
    return _check(load_library().kfkb_op_gemm_nt_tiled(epilogue, M, N, K, _ptr(A), _ptr(Bt), _ptr(bias), _ptr(residual),
                                                       _ptr(Cout), _ptr(C2), _ptr(Cacc), _stream(stream)))


def kfkb_op_layernorm_fwd(dtype, x, gamma, beta, y, mean, rstd, rows, H, eps, stream=None):
    return _check(load_library().kfkb_op_layernorm_fwd(dtype, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(mean),
                                                       _ptr(rstd), rows, H, eps, _stream(stream)))


def kfkb_op_layernorm_bwd(dtype, dy, x, mean, rstd, gamma, dres, dx, dgamma, dbeta, scratch, rows, H, stream=None):
    return _check(load_library().kfkb_op_layernorm_bwd(dtype, _ptr(dy), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gamma),
                                                       _ptr(dres), _ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(scratch),
                                                       rows, H, _stream(stream)))


def kfkb_op_colsum_accum(dtype, dy, out, scratch, rows, N, stream=None):
    return _check(load_library().kfkb_op_colsum_accum(dtype, _ptr(dy), _ptr(out), _ptr(scratch), rows, N, _stream(stream)))


def kfkb_op_colsum_accum_static(dtype, dy, out, rows, N, stream=None):
    return _check(load_library().kfkb_op_colsum_accum_static(dtype, _ptr(dy), _ptr(out), rows, N, _stream(stream)))


def kfkb_op_reduce_scratch_floats(width):
    return load_library().kfkb_op_reduce_scratch_floats(width)


def kfkb_op_gelu_bwd(dtype, dg, u, du, n, stream=None):
    return _check(load_library().kfkb_op_gelu_bwd(dtype, _ptr(dg), _ptr(u), _ptr(du), n, _stream(stream)))


def kfkb_op_attention_fwd(dtype, qkv, o, lse, b, T, H, heads, causal, stream=None):
    return _check(load_library().kfkb_op_attention_fwd(dtype, _ptr(qkv), _ptr(o), _ptr(lse), b, T, H, heads, causal,
                                                       _stream(stream)))


def kfkb_op_attention_bwd(dtype, qkv, o, d_o, lse, dsum, dqkv, b, T, H, heads, causal, stream=None):
    return _check(load_library().kfkb_op_attention_bwd(dtype, _ptr(qkv), _ptr(o), _ptr(d_o), _ptr(lse), _ptr(dsum),
                                                       _ptr(dqkv), b, T, H, heads, causal, _stream(stream)))


def kfkb_op_transpose(dtype, inp, out, rows, cols, stream=None):
    return _check(load_library().kfkb_op_transpose(dtype, _ptr(inp), _ptr(out), rows, cols, _stream(stream)))


def kfkb_op_delay(ns, stream=None):
    return _check(load_library().kfkb_op_delay(int(ns), _stream(stream)))
