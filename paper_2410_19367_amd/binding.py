"""ctypes binding of libbitpipe_stage.so: the same names as the C ABI, argument marshalling only.

Device buffers are passed as torch tensors (their data_ptr is used) or as integer addresses;
nothing here computes.  The library must have been built (paper_2410_19367_amd/build.py); there
is no fallback if it is missing.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbitpipe_stage.so")

BP_OK, BP_EINVAL, BP_ESHAPE, BP_ESTATE, BP_EDEP, BP_ENOMEM, BP_EHIP = 0, -1, -2, -3, -4, -5, -6
BP_F32, BP_BF16 = 0, 1
TENSOR_IDS = {n: i for i, n in enumerate(
    ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"))}
KERNEL_IDS = {n: i for i, n in enumerate(
    ("gemm", "attn_fwd", "attn_bwd", "ln_fwd", "ln_bwd", "gelu_fwd", "gelu_bwd", "colsum", "other"))}

# every symbol include/bitpipe_stage.h declares
EXPORTS = (
    "bp_stage_init", "bp_stage_init_ex", "bp_stage_stash_bytes", "bp_stage_held_bytes", "bp_stage_reset_peak_bytes", "bp_stage_destroy", "bp_stage_set_param",
    "bp_stage_get_grad", "bp_stage_zero_grad", "bp_stage_merge_directions", "bp_stage_wait_forward", "bp_stage_set_seqlens", "bp_stage_forward",
    "bp_stage_backward", "bp_stage_backward_dir", "bp_schedule_vmap", "bp_schedule_generate",
    "bp_schedule_validate", "bp_schedule_simulate", "bp_run_schedule", "bp_schedule_vmap_ex",
    "bp_schedule_generate_ex", "bp_schedule_validate_ex", "bp_schedule_simulate_ex", "bp_run_schedule_ex",
    "bp_schedule_hops", "bp_prof_enable",
    "bp_prof_get", "bp_prof_gemm_shapes", "bp_prof_gemm_get", "bp_op_gemm", "bp_op_wgrad_group", "bp_op_layernorm_fwd", "bp_op_layernorm_bwd",
    "bp_op_layernorm_bwd_static", "bp_static_scratch_floats",
    "bp_op_bias_gelu_fwd", "bp_op_bias_gelu_bwd", "bp_op_colsum_workspace",
    "bp_op_attention_fwd", "bp_op_attention_bwd", "bp_last_error", "bp_version",
)


class bp_opts(C.Structure):
    _fields_ = [("n_chunks", C.c_int), ("mlp", C.c_int), ("dtype", C.c_int),
                ("max_inflight", C.c_int), ("ln_eps", C.c_float), ("hip_stream", C.c_void_p),
                ("wgrad_group", C.c_int), ("stash_recompute", C.c_int), ("forward_ahead", C.c_int)]


class bp_layout(C.Structure):
    _fields_ = [("v", C.c_int), ("looping", C.c_int)]


class bp_op(C.Structure):
    _fields_ = [("kind", C.c_int8), ("dir", C.c_int8), ("vdev", C.c_int16),
                ("stage", C.c_int32), ("mb", C.c_int32)]


class BitPipeError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"[{code}] {msg}")
        self.code = code


_lib = None


def lib():
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: run `python paper_2410_19367_amd/build.py` first")
        l = C.CDLL(LIB_PATH)
        vp, ci, cf = C.c_void_p, C.c_int, C.c_float
        l.bp_stage_init.argtypes = [C.POINTER(vp), ci, ci, ci, ci, ci, ci]
        l.bp_stage_init_ex.argtypes = [C.POINTER(vp), ci, ci, ci, ci, ci, ci, C.POINTER(bp_opts)]
        l.bp_stage_stash_bytes.argtypes = [vp]
        l.bp_stage_stash_bytes.restype = C.c_size_t
        szp = C.POINTER(C.c_size_t)
        l.bp_stage_held_bytes.argtypes = [vp, szp, szp, szp, szp]
        l.bp_stage_reset_peak_bytes.argtypes = [vp]
        l.bp_stage_destroy.argtypes = [vp]
        l.bp_stage_set_param.argtypes = [vp, ci, ci, ci, vp, C.c_size_t]
        l.bp_stage_get_grad.argtypes = [vp, ci, ci, ci, vp, C.c_size_t]
        l.bp_stage_zero_grad.argtypes = [vp]
        l.bp_stage_merge_directions.argtypes = [vp]
        l.bp_stage_wait_forward.argtypes = [vp]
        l.bp_stage_set_seqlens.argtypes = [vp, ci, vp]
        l.bp_stage_forward.argtypes = [vp, ci, ci, vp, vp]
        l.bp_stage_backward.argtypes = [vp, ci, ci, vp, vp]
        l.bp_stage_backward_dir.argtypes = [vp, ci, ci, vp, vp, ci]
        l.bp_schedule_vmap.argtypes = [ci, ci, ci]
        l.bp_schedule_generate.argtypes = [ci, ci, ci, C.POINTER(bp_op), ci, C.POINTER(ci)]
        l.bp_schedule_validate.argtypes = [C.POINTER(bp_op), ci, ci, ci]
        l.bp_schedule_simulate.argtypes = [C.POINTER(bp_op), ci, ci, ci, ci, ci, C.POINTER(ci),
                                           C.POINTER(ci), C.POINTER(ci)]
        l.bp_run_schedule.argtypes = [vp, C.POINTER(bp_op), ci, ci, vp, vp, C.POINTER(cf)]
        lp = C.POINTER(bp_layout)
        l.bp_schedule_vmap_ex.argtypes = [lp, ci, ci, ci]
        l.bp_schedule_generate_ex.argtypes = [lp, ci, ci, ci, C.POINTER(bp_op), ci, C.POINTER(ci)]
        l.bp_schedule_validate_ex.argtypes = [lp, C.POINTER(bp_op), ci, ci, ci]
        l.bp_schedule_simulate_ex.argtypes = [lp, C.POINTER(bp_op), ci, ci, ci, ci, ci, C.POINTER(ci),
                                              C.POINTER(ci), C.POINTER(ci)]
        l.bp_run_schedule_ex.argtypes = [vp, lp, C.POINTER(bp_op), ci, ci, vp, vp, C.POINTER(cf)]
        l.bp_schedule_hops.argtypes = [lp, C.POINTER(bp_op), ci, ci, ci, C.POINTER(C.c_long), C.POINTER(C.c_long)]
        l.bp_prof_enable.argtypes = [vp, ci]
        l.bp_prof_get.argtypes = [vp, ci, C.POINTER(C.c_double), C.POINTER(C.c_longlong),
                                  C.POINTER(C.c_double), C.POINTER(C.c_double)]
        l.bp_prof_gemm_shapes.argtypes = [vp]
        l.bp_prof_gemm_get.argtypes = [vp, ci, C.POINTER(ci), C.POINTER(C.c_double), C.POINTER(C.c_longlong)]
        l.bp_op_gemm.argtypes = [ci, ci, ci, ci, ci, ci, vp, ci, vp, ci, vp, ci, vp, vp, ci, vp]
        l.bp_op_wgrad_group.argtypes = [ci, ci, ci, ci, ci, C.POINTER(vp), C.POINTER(vp), vp, ci, vp,
                                        C.c_size_t, vp]
        l.bp_op_layernorm_fwd.argtypes = [ci, ci, ci, vp, vp, vp, cf, vp, vp, vp, vp]
        l.bp_op_layernorm_bwd.argtypes = [ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        l.bp_op_layernorm_bwd_static.argtypes = [ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        l.bp_static_scratch_floats.restype = C.c_size_t
        l.bp_op_bias_gelu_fwd.argtypes = [ci, ci, ci, vp, vp, vp, vp]
        l.bp_op_bias_gelu_bwd.argtypes = [ci, ci, ci, vp, vp, vp, vp, vp, vp, vp]
        l.bp_op_colsum_workspace.argtypes = [ci, ci]
        l.bp_op_colsum_workspace.restype = C.c_size_t
        l.bp_op_attention_fwd.argtypes = [ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp]
        l.bp_op_attention_bwd.argtypes = [ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp]
        l.bp_last_error.restype = C.c_char_p
        l.bp_version.restype = C.c_char_p
        _lib = l
    return _lib


def _ptr(t):
    """Address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _check(rc):
    if rc != 0:
        raise BitPipeError(rc, bp_last_error())
    return rc


def bp_last_error() -> str:
    return lib().bp_last_error().decode()


def bp_version() -> str:
    return lib().bp_version().decode()


# ---------------------------------------------------------------- stage calls

def bp_stage_init(layers, hidden, heads, seq, microbatch, causal):
    h = C.c_void_p()
    _check(lib().bp_stage_init(C.byref(h), layers, hidden, heads, seq, microbatch, int(causal)))
    return h


def bp_stage_init_ex(layers, hidden, heads, seq, microbatch, causal, n_chunks=0, mlp=0,
                     dtype=BP_BF16, max_inflight=0, ln_eps=0.0, hip_stream=None, wgrad_group=0,
                     stash_recompute=0, forward_ahead=0):
    h = C.c_void_p()
    o = bp_opts(n_chunks, mlp, dtype, max_inflight, ln_eps, hip_stream, wgrad_group, stash_recompute,
                forward_ahead)
    _check(lib().bp_stage_init_ex(C.byref(h), layers, hidden, heads, seq, microbatch, int(causal),
                                  C.byref(o)))
    return h


def bp_stage_stash_bytes(st) -> int:
    return lib().bp_stage_stash_bytes(st)


def bp_stage_held_bytes(st) -> dict:
    a, b, c, d = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    _check(lib().bp_stage_held_bytes(st, C.byref(a), C.byref(b), C.byref(c), C.byref(d)))
    return dict(live_stash=a.value, group_stash=b.value, group_grads=c.value, peak_total=d.value)


def bp_stage_reset_peak_bytes(st):
    return _check(lib().bp_stage_reset_peak_bytes(st))


def bp_stage_destroy(st):
    return _check(lib().bp_stage_destroy(st))


def bp_stage_set_param(st, chunk, layer, tensor_id, host_f32: np.ndarray):
    a = np.ascontiguousarray(host_f32, dtype=np.float32)
    return _check(lib().bp_stage_set_param(st, chunk, layer, tensor_id, a.ctypes.data, a.size))


def bp_stage_get_grad(st, chunk, layer, tensor_id, shape) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _check(lib().bp_stage_get_grad(st, chunk, layer, tensor_id, out.ctypes.data, out.size))
    return out


def bp_stage_zero_grad(st):
    return _check(lib().bp_stage_zero_grad(st))


def bp_stage_merge_directions(st):
    return _check(lib().bp_stage_merge_directions(st))


def bp_stage_wait_forward(st):
    return _check(lib().bp_stage_wait_forward(st))


def bp_stage_set_seqlens(st, mb, lens):
    if lens is None:
        return _check(lib().bp_stage_set_seqlens(st, mb, None))
    a = np.ascontiguousarray(lens, dtype=np.int32)
    return _check(lib().bp_stage_set_seqlens(st, mb, a.ctypes.data))


def bp_stage_forward(st, chunk, mb, act_in, act_out):
    return _check(lib().bp_stage_forward(st, chunk, mb, _ptr(act_in), _ptr(act_out)))


def bp_stage_backward(st, chunk, mb, grad_out, grad_in):
    return _check(lib().bp_stage_backward(st, chunk, mb, _ptr(grad_out), _ptr(grad_in)))


def bp_stage_backward_dir(st, chunk, mb, grad_out, grad_in, direction):
    return _check(lib().bp_stage_backward_dir(st, chunk, mb, _ptr(grad_out), _ptr(grad_in), direction))


# ---------------------------------------------------------------- schedule calls (pure CPU)

def bp_schedule_vmap(direction, stage, D):
    return lib().bp_schedule_vmap(direction, stage, D)


def bp_schedule_generate(D, N, variant=0):
    """Returns a ctypes array of bp_op holding one iteration's serial order."""
    cap = 4 * max(D, 0) * max(N, 0) + 1
    arr = (bp_op * cap)()
    n = C.c_int(0)
    _check(lib().bp_schedule_generate(D, N, variant, arr, cap, C.byref(n)))
    return (bp_op * n.value)(*arr[:n.value])


def ops_to_tuples(order):
    """[(kind 'F'|'B', dir, vdev, stage, mb)] of a bp_op array."""
    return [("FB"[o.kind], o.dir, o.vdev, o.stage, o.mb) for o in order]


def ops_from_tuples(tuples):
    arr = (bp_op * len(tuples))()
    for i, (k, d, v, s, m) in enumerate(tuples):
        arr[i] = bp_op("FB".index(k) if isinstance(k, str) else k, d, v, s, m)
    return arr


def bp_schedule_validate(order, D, N):
    return _check(lib().bp_schedule_validate(order, len(order), D, N))


def bp_schedule_simulate(order, D, N, cost_f=1, cost_b=2):
    ms = C.c_int(0)
    idle = (C.c_int * D)()
    peak = (C.c_int * D)()
    _check(lib().bp_schedule_simulate(order, len(order), D, N, cost_f, cost_b, C.byref(ms), idle, peak))
    return ms.value, list(idle), list(peak)


def bp_run_schedule(st, order, D, inputs, targets) -> float:
    loss = C.c_float(0)
    _check(lib().bp_run_schedule(st, order, len(order), D, _ptr(inputs), _ptr(targets), C.byref(loss)))
    return loss.value


def bp_schedule_vmap_ex(layout, direction, stage, D):
    return lib().bp_schedule_vmap_ex(C.byref(layout), direction, stage, D)


def bp_schedule_generate_ex(layout, D, N, variant=0):
    cap = 2 * max(layout.v, 0) * max(D, 0) * max(N, 0) + 1
    arr = (bp_op * cap)()
    n = C.c_int(0)
    _check(lib().bp_schedule_generate_ex(C.byref(layout), D, N, variant, arr, cap, C.byref(n)))
    return (bp_op * n.value)(*arr[:n.value])


def bp_schedule_validate_ex(layout, order, D, N):
    return _check(lib().bp_schedule_validate_ex(C.byref(layout), order, len(order), D, N))


def bp_schedule_simulate_ex(layout, order, D, N, cost_f=1, cost_b=2):
    ms = C.c_int(0)
    idle = (C.c_int * D)()
    peak = (C.c_int * D)()
    _check(lib().bp_schedule_simulate_ex(C.byref(layout), order, len(order), D, N, cost_f, cost_b,
                                         C.byref(ms), idle, peak))
    return ms.value, list(idle), list(peak)


def bp_schedule_hops(layout, order, D, N):
    p2p, local = C.c_long(0), C.c_long(0)
    _check(lib().bp_schedule_hops(C.byref(layout), order, len(order), D, N, C.byref(p2p), C.byref(local)))
    return p2p.value, local.value


def bp_run_schedule_ex(st, layout, order, D, inputs, targets) -> float:
    loss = C.c_float(0)
    _check(lib().bp_run_schedule_ex(st, C.byref(layout), order, len(order), D, _ptr(inputs), _ptr(targets),
                                    C.byref(loss)))
    return loss.value


# ---------------------------------------------------------------- timing

def bp_prof_enable(st, on):
    return _check(lib().bp_prof_enable(st, int(on)))


def bp_prof_get(st, kernel_id):
    ms, n, fl, by = C.c_double(0), C.c_longlong(0), C.c_double(0), C.c_double(0)
    _check(lib().bp_prof_get(st, kernel_id, C.byref(ms), C.byref(n), C.byref(fl), C.byref(by)))
    return dict(ms=ms.value, launches=n.value, flops=fl.value, bytes=by.value)


def bp_prof_gemm_shapes(st):
    """List of dicts, one per distinct GEMM shape launched since timing was enabled."""
    n = lib().bp_prof_gemm_shapes(st)
    if n < 0:
        _check(n)
    out = []
    for i in range(n):
        dims = (C.c_int * 7)()
        ms, cnt = C.c_double(0), C.c_longlong(0)
        _check(lib().bp_prof_gemm_get(st, i, dims, C.byref(ms), C.byref(cnt)))
        M, N, K, a_t, b_t, nseg, epi = list(dims)
        out.append(dict(M=M, N=N, K=K, a_t=a_t, b_t=b_t, segments=nseg, epilogue=epi, ms=ms.value, launches=cnt.value))
    return out


# ---------------------------------------------------------------- single operations

def bp_op_gemm(dtype, a_t, b_t, M, N, K, A, lda, B, ldb, Cm, ldc, bias=None, residual=None,
               accumulate=0, stream=None):
    return _check(lib().bp_op_gemm(dtype, a_t, b_t, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(Cm), ldc,
                                   _ptr(bias), _ptr(residual), accumulate, stream))


def bp_op_wgrad_group(dtype, M, N, T, X, dY, dW, overwrite=0, workspace=None, workspace_elems=0, stream=None):
    n = len(X)
    xs = (C.c_void_p * n)(*[_ptr(x) for x in X])
    ys = (C.c_void_p * n)(*[_ptr(y) for y in dY])
    return _check(lib().bp_op_wgrad_group(dtype, M, N, T, n, xs, ys, _ptr(dW), overwrite, _ptr(workspace),
                                          workspace_elems, stream))


def bp_op_layernorm_fwd(dtype, T, H, x, gamma, beta, eps, out, mean, rstd, stream=None):
    return _check(lib().bp_op_layernorm_fwd(dtype, T, H, _ptr(x), _ptr(gamma), _ptr(beta), eps,
                                            _ptr(out), _ptr(mean), _ptr(rstd), stream))


def bp_op_layernorm_bwd(dtype, T, H, dout, x, mean, rstd, gamma, residual_grad, dx, dgamma, dbeta,
                        workspace, stream=None):
    return _check(lib().bp_op_layernorm_bwd(dtype, T, H, _ptr(dout), _ptr(x), _ptr(mean), _ptr(rstd),
                                            _ptr(gamma), _ptr(residual_grad), _ptr(dx), _ptr(dgamma),
                                            _ptr(dbeta), _ptr(workspace), stream))


def bp_op_layernorm_bwd_static(dtype, T, H, dout, x, mean, rstd, gamma, residual_grad, dx, dgamma, dbeta,
                               stream=None):
    return _check(lib().bp_op_layernorm_bwd_static(dtype, T, H, _ptr(dout), _ptr(x), _ptr(mean), _ptr(rstd),
                                                   _ptr(gamma), _ptr(residual_grad), _ptr(dx), _ptr(dgamma),
                                                   _ptr(dbeta), stream))


def bp_static_scratch_floats() -> int:
    return lib().bp_static_scratch_floats()


def bp_op_bias_gelu_fwd(dtype, T, F, u, bias, g, stream=None):
    return _check(lib().bp_op_bias_gelu_fwd(dtype, T, F, _ptr(u), _ptr(bias), _ptr(g), stream))


def bp_op_bias_gelu_bwd(dtype, T, F, dg, u, bias, du, dbias, workspace, stream=None):
    return _check(lib().bp_op_bias_gelu_bwd(dtype, T, F, _ptr(dg), _ptr(u), _ptr(bias), _ptr(du),
                                            _ptr(dbias), _ptr(workspace), stream))


def bp_op_colsum_workspace(T, N) -> int:
    return lib().bp_op_colsum_workspace(T, N)


def bp_op_attention_fwd(dtype, B, S, heads, head_dim, causal, lens, qkv, ctx, lse, stream=None):
    return _check(lib().bp_op_attention_fwd(dtype, B, S, heads, head_dim, int(causal), _ptr(lens),
                                            _ptr(qkv), _ptr(ctx), _ptr(lse), stream))


def bp_op_attention_bwd(dtype, B, S, heads, head_dim, causal, lens, qkv, ctx, lse, dctx, dqkv, delta,
                        stream=None):
    return _check(lib().bp_op_attention_bwd(dtype, B, S, heads, head_dim, int(causal), _ptr(lens),
                                            _ptr(qkv), _ptr(ctx), _ptr(lse), _ptr(dctx), _ptr(dqkv),
                                            _ptr(delta), stream))
