"""ctypes binding of libhanayo.so: same names as include/hanayo.h, marshalling only.

Device buffers are torch tensors (torch is used for device memory and streams
only); a tensor argument is passed as its data pointer.  Every call raises
HanayoError on a non-zero return code.  There is no fallback: if the library is
missing this module fails to import.
"""

import ctypes
import os

import numpy as np
# torch ships its own HIP runtime (libamdhip64.so.7).  It has to be in the process before
# libhanayo.so is loaded so that the loader binds the library to that same runtime: two HIP
# runtimes in one process cannot both open the GPU.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhanayo.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libhanayo.so is not built: run `python -m paper_2308_15762_amd.build`")
_lib = ctypes.CDLL(LIB_PATH)

OK, EINVAL, EBUFSIZE, ESTATE, EUNSUPPORTED, EHIP = 0, -1, -2, -3, -4, -5
F, B = 0, 1
PRE_LN, POST_LN = 0, 1
MASK_NONE, MASK_CAUSAL = 0, 1
FP32, BF16 = 0, 1
N_PARAMS = 12
PARAM_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")

TASK_DTYPE = np.dtype([("kind", np.uint8), ("chunk", np.uint8), ("rsvd", np.uint16),
                       ("mb", np.uint32), ("stage", np.uint32)])
assert TASK_DTYPE.itemsize == 12


class ChunkDesc(ctypes.Structure):
    _fields_ = [("n_blocks", ctypes.c_int), ("hidden", ctypes.c_int), ("heads", ctypes.c_int),
                ("ffn", ctypes.c_int), ("seq", ctypes.c_int), ("mb", ctypes.c_int),
                ("norm", ctypes.c_int), ("mask", ctypes.c_int), ("dtype", ctypes.c_int),
                ("ln_eps", ctypes.c_float)]


class EndsDesc(ctypes.Structure):
    _fields_ = [("vocab", ctypes.c_int), ("max_pos", ctypes.c_int), ("final_ln", ctypes.c_int)]


class EndsArgs(ctypes.Structure):
    _fields_ = [("desc", EndsDesc),
                ("wte", ctypes.c_void_p), ("d_wte", ctypes.c_void_p), ("wpe", ctypes.c_void_p), ("d_wpe", ctypes.c_void_p),
                ("head", ctypes.c_void_p), ("d_head", ctypes.c_void_p), ("lnf", ctypes.c_void_p), ("d_lnf", ctypes.c_void_p),
                ("tokens", ctypes.POINTER(ctypes.c_void_p)), ("labels", ctypes.POINTER(ctypes.c_void_p)),
                ("loss", ctypes.c_void_p), ("loss_grad", ctypes.POINTER(ctypes.c_void_p)),
                ("loss_scale", ctypes.c_float), ("workspace", ctypes.c_void_p)]


class ExecArgs(ctypes.Structure):
    _fields_ = [("desc", ctypes.POINTER(ChunkDesc)),
                ("P", ctypes.c_int), ("W", ctypes.c_int), ("M", ctypes.c_int), ("rank", ctypes.c_int),
                ("weights", ctypes.POINTER(ctypes.c_void_p)), ("grads", ctypes.POINTER(ctypes.c_void_p)),
                ("act_in", ctypes.POINTER(ctypes.c_void_p)), ("grad_in", ctypes.POINTER(ctypes.c_void_p)),
                ("act_out", ctypes.POINTER(ctypes.c_void_p)), ("grad_out", ctypes.POINTER(ctypes.c_void_p)),
                ("valid_len", ctypes.POINTER(ctypes.c_void_p)),
                ("stash_arena", ctypes.c_void_p), ("stash_arena_bytes", ctypes.c_size_t),
                ("workspace", ctypes.c_void_p), ("hip_stream", ctypes.c_void_p), ("lanes", ctypes.c_int),
                ("stash_mode", ctypes.c_int), ("recompute_scratch", ctypes.c_void_p),
                ("ends", ctypes.POINTER(EndsArgs))]


class Adam(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("step", ctypes.c_int), ("zero_grads", ctypes.c_int)]


class GemmProblem(ctypes.Structure):
    _fields_ = [("A", ctypes.c_void_p), ("B", ctypes.c_void_p), ("C", ctypes.c_void_p), ("bias", ctypes.c_void_p),
                ("aux", ctypes.c_void_p), ("aux_out", ctypes.c_void_p),
                ("M", ctypes.c_int), ("N", ctypes.c_int), ("K", ctypes.c_int),
                ("lda", ctypes.c_int), ("ldb", ctypes.c_int), ("ldc", ctypes.c_int),
                ("colsum", ctypes.c_void_p), ("colsum_scratch", ctypes.c_void_p)]


class PipelineArgs(ctypes.Structure):
    _fields_ = [("desc", ctypes.POINTER(ChunkDesc)),
                ("P", ctypes.c_int), ("W", ctypes.c_int), ("M", ctypes.c_int),
                ("weights", ctypes.POINTER(ctypes.c_void_p)), ("grads", ctypes.POINTER(ctypes.c_void_p)),
                ("x", ctypes.POINTER(ctypes.c_void_p)), ("dy", ctypes.POINTER(ctypes.c_void_p)),
                ("act", ctypes.POINTER(ctypes.c_void_p)), ("grad", ctypes.POINTER(ctypes.c_void_p)),
                ("valid_len", ctypes.POINTER(ctypes.c_void_p)),
                ("stash_arena", ctypes.POINTER(ctypes.c_void_p)), ("stash_arena_bytes", ctypes.POINTER(ctypes.c_size_t)),
                ("workspace", ctypes.c_void_p), ("hip_stream", ctypes.c_void_p), ("ends", ctypes.POINTER(EndsArgs))]


class LinkArgs(ctypes.Structure):
    _fields_ = [("act_recv", ctypes.POINTER(ctypes.c_void_p)), ("grad_recv", ctypes.POINTER(ctypes.c_void_p)),
                ("async_", ctypes.c_int), ("link_workgroups", ctypes.c_int)]


class HanayoError(RuntimeError):
    def __init__(self, code):
        self.code = code
        detail = _lib.hanayo_last_error().decode()
        super().__init__("%s (%d): %s" % (_lib.hanayo_strerror(code).decode(), code, detail))


EXPORTS = ("hanayo_strerror", "hanayo_last_error", "hanayo_stage_rank", "hanayo_rank_stage", "hanayo_schedule",
           "hanayo_schedule_scheme", "hanayo_bubble_model", "hanayo_actions_of",
           "hanayo_stash_plan", "hanayo_param_span", "hanayo_weight_bytes", "hanayo_grad_bytes",
           "hanayo_stash_bytes", "hanayo_workspace_bytes", "hanayo_act_bytes", "hanayo_chunk_forward",
           "hanayo_chunk_backward", "hanayo_stash_arena_bytes", "hanayo_stash_arena_bytes_input",
           "hanayo_recompute_scratch_bytes", "hanayo_executor_run", "hanayo_executor_plan", "hanayo_pipeline_run", "hanayo_replay", "hanayo_actions", "hanayo_replay_actions", "hanayo_pipeline_run_actions", "hanayo_device_info",
           "hanayo_op_gemm", "hanayo_op_gemm_group", "hanayo_op_gemm_config", "hanayo_op_copy", "hanayo_op_layernorm_forward", "hanayo_op_layernorm_backward", "hanayo_op_layernorm_backward_static", "hanayo_op_colsum_add",
           "hanayo_op_attention_forward", "hanayo_op_attention_backward",
           "hanayo_embed_forward", "hanayo_embed_backward", "hanayo_head_workspace_bytes", "hanayo_head_loss",
           "hanayo_adam_step", "hanayo_chunk_adam_step", "hanayo_ends_workspace_bytes")

_vp, _sz, _int = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
_descp = ctypes.POINTER(ChunkDesc)
_lib.hanayo_strerror.restype = ctypes.c_char_p
_lib.hanayo_strerror.argtypes = [_int]
_lib.hanayo_last_error.restype = ctypes.c_char_p
_lib.hanayo_last_error.argtypes = []
_lib.hanayo_stage_rank.argtypes = [_int, _int, _int, ctypes.POINTER(_int)]
_lib.hanayo_rank_stage.argtypes = [_int, _int, _int, _int, ctypes.POINTER(_int)]
_lib.hanayo_schedule.argtypes = [_int, _int, _int, _int, _vp, _sz, ctypes.POINTER(_sz)]
_lib.hanayo_schedule_scheme.argtypes = [_int, _int, _int, _int, _int, _vp, _sz, ctypes.POINTER(_sz)]
_dbl = ctypes.c_double
_lib.hanayo_bubble_model.argtypes = [_int, _int, _int, _int, _dbl, _dbl, _dbl] + [ctypes.POINTER(_dbl)] * 3
_lib.hanayo_stash_plan.argtypes = [_vp, _sz, _int, ctypes.POINTER(_int), _vp, _vp]
_lib.hanayo_param_span.argtypes = [_descp, _int, _int, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]
for _n in ("hanayo_weight_bytes", "hanayo_grad_bytes", "hanayo_stash_bytes", "hanayo_workspace_bytes",
           "hanayo_act_bytes"):
    getattr(_lib, _n).restype = _sz
    getattr(_lib, _n).argtypes = [_descp]
_lib.hanayo_chunk_forward.argtypes = [_descp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.hanayo_chunk_backward.argtypes = [_descp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.hanayo_stash_arena_bytes.restype = _sz
_lib.hanayo_stash_arena_bytes.argtypes = [_vp, _sz, _int, _descp]
_lib.hanayo_stash_arena_bytes_input.restype = _sz
_lib.hanayo_stash_arena_bytes_input.argtypes = [_vp, _sz, _int, _descp]
_lib.hanayo_recompute_scratch_bytes.restype = _sz
_lib.hanayo_recompute_scratch_bytes.argtypes = [_descp]
_lib.hanayo_executor_run.argtypes = [_vp, _sz, ctypes.POINTER(ExecArgs), ctypes.POINTER(_int)]
_lib.hanayo_executor_plan.argtypes = [_vp, _sz, _int, _int, _int, _int, _int, _vp, _vp, _vp, _vp]
_lib.hanayo_pipeline_run.argtypes = [_vp, _vp, ctypes.POINTER(PipelineArgs), _vp, _vp]
_lib.hanayo_replay.argtypes = [_vp, _vp, _int, _int, _int, _vp, ctypes.POINTER(ctypes.c_double), _vp]
_lib.hanayo_actions.argtypes = [_int, _int, _int, _int, _vp, _sz, ctypes.POINTER(_sz)]
_lib.hanayo_actions_of.argtypes = [_vp, _sz, _int, _int, _int, _vp, _sz, ctypes.POINTER(_sz)]
_lib.hanayo_replay_actions.argtypes = [_vp, _vp, _int, _int, _int, ctypes.c_double, ctypes.c_double, ctypes.c_double, _int,
                                       _vp, ctypes.POINTER(ctypes.c_double), _vp, _vp]
_lib.hanayo_pipeline_run_actions.argtypes = [_vp, _vp, ctypes.POINTER(PipelineArgs), ctypes.POINTER(LinkArgs), _vp, _vp]
_lib.hanayo_device_info.argtypes = [ctypes.c_char_p, _sz]
_lib.hanayo_op_gemm.argtypes = [_int, _vp, _vp, _vp] + [_int] * 9 + [_vp, _vp, _vp, _vp, _vp, _vp]
_lib.hanayo_op_gemm_group.argtypes = [_int, _int, _int, _int, _vp, _int, _vp]
_lib.hanayo_op_gemm_config.argtypes = [_int]
_lib.hanayo_op_copy.argtypes = [_vp, _vp, _sz, _vp]
_lib.hanayo_op_layernorm_forward.argtypes = [_int, _vp, _vp, _vp, _vp, _vp, _vp, _int, _int, ctypes.c_float, _vp]
_lib.hanayo_op_layernorm_backward.argtypes = [_int] + [_vp] * 9 + [_int, _int, _vp]
_lib.hanayo_op_layernorm_backward_static.argtypes = [_int] + [_vp] * 8 + [_int, _int, _vp]
_lib.hanayo_op_colsum_add.argtypes = [_int, _vp, _int, _int, _vp, _vp, _vp]
_lib.hanayo_op_attention_forward.argtypes = [_int, _vp, _vp, _vp, _vp, _int, _int, _int, _int, _int, _vp]
_lib.hanayo_op_attention_backward.argtypes = [_int] + [_vp] * 7 + [_int] * 5 + [_vp]
_endsp, _adamp = ctypes.POINTER(EndsDesc), ctypes.POINTER(Adam)
_lib.hanayo_embed_forward.argtypes = [_descp, _endsp, _vp, _vp, _vp, _vp, _vp]
_lib.hanayo_embed_backward.argtypes = [_descp, _endsp, _vp, _vp, _vp, _vp, _vp]
_lib.hanayo_head_workspace_bytes.restype = _sz
_lib.hanayo_head_workspace_bytes.argtypes = [_descp, _endsp]
_lib.hanayo_ends_workspace_bytes.restype = _sz
_lib.hanayo_ends_workspace_bytes.argtypes = [_descp, _endsp]
_lib.hanayo_head_loss.argtypes = [_descp, _endsp, _vp, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.hanayo_adam_step.argtypes = [_adamp, _int, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.hanayo_chunk_adam_step.argtypes = [_adamp, _descp, _vp, _vp, _vp, _vp, _vp, _vp]
EPI_NONE, EPI_BIAS, EPI_BIAS_GELU, EPI_BIAS_RES, EPI_MUL_DGELU, EPI_ADD, EPI_ACCUM_F32 = range(7)


def _check(rc):
    if rc != OK:
        raise HanayoError(rc)


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def make_desc(n_blocks, hidden, heads, ffn, seq, mb, norm, mask, dtype, ln_eps=1e-5):
    return ChunkDesc(n_blocks, hidden, heads, ffn, seq, mb, norm, mask, dtype, ln_eps)


def desc_for(wl):
    """Descriptor of a synth.Workload."""
    return make_desc(wl.n_blocks, wl.hidden, wl.heads, wl.ffn, wl.seq, wl.mb,
                     PRE_LN if wl.norm == "pre" else POST_LN,
                     MASK_CAUSAL if wl.causal else MASK_NONE,
                     BF16 if wl.dtype == "bf16" else FP32)


# ------------------------------------------------------------------ schedule

def hanayo_stage_rank(P, W, stage):
    out = _int()
    _check(_lib.hanayo_stage_rank(P, W, stage, ctypes.byref(out)))
    return out.value


def hanayo_rank_stage(P, W, rank, chunk):
    out = _int()
    _check(_lib.hanayo_rank_stage(P, W, rank, chunk, ctypes.byref(out)))
    return out.value


def hanayo_schedule(P, W, M, rank):
    """Ordered task list of one rank as a structured array (kind, chunk, rsvd, mb, stage)."""
    n = _sz()
    rc = _lib.hanayo_schedule(P, W, M, rank, None, 0, ctypes.byref(n))
    if rc != EBUFSIZE:
        _check(rc)
    out = np.zeros(n.value, dtype=TASK_DTYPE)
    _check(_lib.hanayo_schedule(P, W, M, rank, out.ctypes.data, out.size, ctypes.byref(n)))
    return out


SCHEME_HANAYO, SCHEME_CHIMERA_WAVE, SCHEME_GPIPE, SCHEME_1F1B = range(4)


def chunks_per_rank(W):
    """Buffer-table width of a placement: 2W chunks per device, one for the straight placement (W = 0)."""
    return 2 * W if W else 1


def hanayo_schedule_scheme(scheme, P, W, M, rank):
    """Ordered task list of one rank under a scheme (W = 0 for GPipe / 1F1B, 1 for Chimera-wave)."""
    n = _sz()
    rc = _lib.hanayo_schedule_scheme(scheme, P, W, M, rank, None, 0, ctypes.byref(n))
    if rc != EBUFSIZE:
        _check(rc)
    out = np.zeros(n.value, dtype=TASK_DTYPE)
    _check(_lib.hanayo_schedule_scheme(scheme, P, W, M, rank, out.ctypes.data, out.size, ctypes.byref(n)))
    return out


def hanayo_bubble_model(scheme, P, W, M, t_f, t_b, t_c):
    """Returns (ratio, idle, ratio_of_idle)."""
    r, i, q = _dbl(), _dbl(), _dbl()
    _check(_lib.hanayo_bubble_model(scheme, P, W, M, t_f, t_b, t_c, ctypes.byref(r), ctypes.byref(i), ctypes.byref(q)))
    return r.value, i.value, q.value


def hanayo_stash_plan(tasks, W):
    """Returns (peak_total, per_chunk[2W], slot[n])."""
    tasks = np.ascontiguousarray(tasks, dtype=TASK_DTYPE)
    peak = _int()
    per_chunk = np.zeros(chunks_per_rank(W), dtype=np.int32)
    slot = np.zeros(tasks.size, dtype=np.int32)
    _check(_lib.hanayo_stash_plan(tasks.ctypes.data, tasks.size, W, ctypes.byref(peak),
                                  per_chunk.ctypes.data, slot.ctypes.data))
    return peak.value, per_chunk, slot


# ------------------------------------------------------------------ sizes / layout

def hanayo_param_span(desc, block, param):
    off, cnt = _sz(), _sz()
    _check(_lib.hanayo_param_span(ctypes.byref(desc), block, param, ctypes.byref(off), ctypes.byref(cnt)))
    return off.value, cnt.value


def _size(fn, desc):
    v = fn(ctypes.byref(desc))
    if v == 0:
        raise HanayoError(EINVAL)
    return v


def hanayo_weight_bytes(desc):
    return _size(_lib.hanayo_weight_bytes, desc)


def hanayo_grad_bytes(desc):
    return _size(_lib.hanayo_grad_bytes, desc)


def hanayo_stash_bytes(desc):
    return _size(_lib.hanayo_stash_bytes, desc)


def hanayo_workspace_bytes(desc):
    return _size(_lib.hanayo_workspace_bytes, desc)


def hanayo_act_bytes(desc):
    return _size(_lib.hanayo_act_bytes, desc)


def hanayo_stash_arena_bytes(tasks, W, desc):
    tasks = np.ascontiguousarray(tasks, dtype=TASK_DTYPE)
    v = _lib.hanayo_stash_arena_bytes(tasks.ctypes.data, tasks.size, W, ctypes.byref(desc))
    if v == 0:
        raise HanayoError(ESTATE)
    return v


STASH_FULL, STASH_INPUT = 0, 1


def hanayo_stash_arena_bytes_input(tasks, W, desc):
    tasks = np.ascontiguousarray(tasks, dtype=TASK_DTYPE)
    v = _lib.hanayo_stash_arena_bytes_input(tasks.ctypes.data, tasks.size, W, ctypes.byref(desc))
    if v == 0:
        raise HanayoError(ESTATE)
    return v


def hanayo_recompute_scratch_bytes(desc):
    return _lib.hanayo_recompute_scratch_bytes(ctypes.byref(desc))


def hanayo_device_info():
    buf = ctypes.create_string_buffer(256)
    _check(_lib.hanayo_device_info(buf, 256))
    return buf.value.decode()


# ------------------------------------------------------------------ compute

def hanayo_chunk_forward(desc, weights, x, valid_len, y, stash_entry, workspace, stream=None):
    _check(_lib.hanayo_chunk_forward(ctypes.byref(desc), _ptr(weights), _ptr(x), _ptr(valid_len), _ptr(y),
                                     _ptr(stash_entry), _ptr(workspace), stream))


def hanayo_chunk_backward(desc, weights, grads, dy, valid_len, stash_entry, dx, workspace, stream=None):
    _check(_lib.hanayo_chunk_backward(ctypes.byref(desc), _ptr(weights), _ptr(grads), _ptr(dy), _ptr(valid_len),
                                      _ptr(stash_entry), _ptr(dx), _ptr(workspace), stream))


def hanayo_embed_forward(desc, ends, wte, wpe, tokens, x, stream=None):
    _check(_lib.hanayo_embed_forward(ctypes.byref(desc), ctypes.byref(ends), _ptr(wte), _ptr(wpe), _ptr(tokens), _ptr(x),
                                     stream))


def hanayo_embed_backward(desc, ends, tokens, dx, d_wte, d_wpe, stream=None):
    _check(_lib.hanayo_embed_backward(ctypes.byref(desc), ctypes.byref(ends), _ptr(tokens), _ptr(dx), _ptr(d_wte),
                                      _ptr(d_wpe), stream))


def hanayo_head_workspace_bytes(desc, ends):
    v = _lib.hanayo_head_workspace_bytes(ctypes.byref(desc), ctypes.byref(ends))
    if v == 0:
        raise HanayoError(EINVAL)
    return v


def hanayo_ends_workspace_bytes(desc, ends):
    v = _lib.hanayo_ends_workspace_bytes(ctypes.byref(desc), ctypes.byref(ends))
    if v == 0:
        raise HanayoError(EINVAL)
    return v


def make_ends_args(ends, wte, d_wte, wpe, d_wpe, head, d_head, lnf, d_lnf, tokens, labels, loss, loss_grad, loss_scale,
                   workspace):
    """hanayo_ends_args from tensors; tokens, labels, loss_grad are Python lists [M] of tensors."""
    tabs = [_table(t) for t in (tokens, labels, loss_grad)]
    a = EndsArgs(ends, _ptr(wte), _ptr(d_wte), _ptr(wpe), _ptr(d_wpe), _ptr(head), _ptr(d_head), _ptr(lnf), _ptr(d_lnf),
                 tabs[0], tabs[1], _ptr(loss), tabs[2], loss_scale, _ptr(workspace))
    a._keep = tabs
    return a


def hanayo_head_loss(desc, ends, lnf, head, y, labels, loss_scale, loss, dy, d_lnf, d_head, workspace, stream=None):
    _check(_lib.hanayo_head_loss(ctypes.byref(desc), ctypes.byref(ends), _ptr(lnf), _ptr(head), _ptr(y), _ptr(labels),
                                 loss_scale, _ptr(loss), _ptr(dy), _ptr(d_lnf), _ptr(d_head), _ptr(workspace), stream))


def hanayo_adam_step(adam, dtype, params, master, grads, m, v, count, stream=None):
    _check(_lib.hanayo_adam_step(ctypes.byref(adam), dtype, _ptr(params), _ptr(master), _ptr(grads), _ptr(m), _ptr(v),
                                 count, stream))


def hanayo_chunk_adam_step(adam, desc, weights, master, grads, m, v, stream=None):
    _check(_lib.hanayo_chunk_adam_step(ctypes.byref(adam), ctypes.byref(desc), _ptr(weights), _ptr(master), _ptr(grads),
                                       _ptr(m), _ptr(v), stream))


def hanayo_op_gemm(dtype, A, B, C, M, N, K, lda, ldb, ldc, a_t, b_t, epilogue, bias=None, aux=None, aux_out=None,
                   colsum=None, colsum_scratch=None, stream=None):
    _check(_lib.hanayo_op_gemm(dtype, _ptr(A), _ptr(B), _ptr(C), M, N, K, lda, ldb, ldc, int(a_t), int(b_t), epilogue,
                               _ptr(bias), _ptr(aux), _ptr(aux_out), _ptr(colsum), _ptr(colsum_scratch), stream))


def _problem_array(problems):
    arr = (GemmProblem * len(problems))()
    for q, p in zip(arr, problems):
        for name, _ in GemmProblem._fields_:
            v = p.get(name)
            setattr(q, name, v if isinstance(v, int) and name in ("M", "N", "K", "lda", "ldb", "ldc") else _ptr(v))
    return arr


def hanayo_op_gemm_group(dtype, a_t, b_t, epilogue, problems, stream=None):
    """problems: list of dicts with the keys of hanayo_gemm_problem (tensors or None, ints)."""
    arr = _problem_array(problems)
    _check(_lib.hanayo_op_gemm_group(dtype, int(a_t), int(b_t), epilogue, ctypes.addressof(arr), len(problems), stream))


def bound_op_gemm(*args, **kw):
    """hanayo_op_gemm with its arguments marshalled once: returns a callable for launch loops
    in which Python's per-call conversion cost would otherwise leave the GPU waiting."""
    names = ("dtype A B C M N K lda ldb ldc a_t b_t epilogue bias aux aux_out colsum colsum_scratch stream").split()
    vals = dict(zip(names, args))
    vals.update(kw)
    c = [vals["dtype"]] + [_ptr(vals[n]) for n in ("A", "B", "C")] + [int(vals[n]) for n in names[4:13]] + \
        [_ptr(vals.get(n)) for n in ("bias", "aux", "aux_out", "colsum", "colsum_scratch")] + [vals.get("stream")]
    fn = _lib.hanayo_op_gemm
    return lambda: _check(fn(*c))


def bound_op_gemm_group(dtype, a_t, b_t, epilogue, problems, stream=None):
    """hanayo_op_gemm_group with its arguments marshalled once (see bound_op_gemm)."""
    arr = _problem_array(problems)
    fn, addr, n = _lib.hanayo_op_gemm_group, ctypes.addressof(arr), len(problems)
    return lambda keep=arr: _check(fn(dtype, int(a_t), int(b_t), epilogue, addr, n, stream))


def hanayo_op_copy(dst, src, nbytes, stream=None):
    _check(_lib.hanayo_op_copy(_ptr(dst), _ptr(src), nbytes, stream))


def hanayo_op_gemm_config(config):
    _check(_lib.hanayo_op_gemm_config(int(config)))


def hanayo_op_layernorm_forward(dtype, x, gamma, beta, out, stats, copy_out, rows, hidden, eps, stream=None):
    _check(_lib.hanayo_op_layernorm_forward(dtype, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(out), _ptr(stats),
                                            _ptr(copy_out), rows, hidden, eps, stream))


def hanayo_op_layernorm_backward(dtype, dout, x, gamma, stats, addend, dz, dgamma, dbeta, scratch, rows, hidden,
                                 stream=None):
    _check(_lib.hanayo_op_layernorm_backward(dtype, _ptr(dout), _ptr(x), _ptr(gamma), _ptr(stats), _ptr(addend),
                                             _ptr(dz), _ptr(dgamma), _ptr(dbeta), _ptr(scratch), rows, hidden, stream))


def hanayo_op_layernorm_backward_static(dtype, dout, x, gamma, stats, addend, dz, dgamma, dbeta, rows, hidden,
                                        stream=None):
    _check(_lib.hanayo_op_layernorm_backward_static(dtype, _ptr(dout), _ptr(x), _ptr(gamma), _ptr(stats),
                                                    _ptr(addend), _ptr(dz), _ptr(dgamma), _ptr(dbeta), rows, hidden,
                                                    stream))


def hanayo_op_colsum_add(dtype, inp, rows, n, out, scratch, stream=None):
    _check(_lib.hanayo_op_colsum_add(dtype, _ptr(inp), rows, n, _ptr(out), _ptr(scratch), stream))


def hanayo_op_attention_forward(dtype, qkv, valid_len, ctx, lse, b, s, heads, head_dim, causal, stream=None):
    _check(_lib.hanayo_op_attention_forward(dtype, _ptr(qkv), _ptr(valid_len), _ptr(ctx), _ptr(lse), b, s, heads,
                                            head_dim, int(causal), stream))


def hanayo_op_attention_backward(dtype, qkv, valid_len, ctx, lse, dctx, dqkv, delta, b, s, heads, head_dim, causal,
                                 stream=None):
    _check(_lib.hanayo_op_attention_backward(dtype, _ptr(qkv), _ptr(valid_len), _ptr(ctx), _ptr(lse), _ptr(dctx),
                                             _ptr(dqkv), _ptr(delta), b, s, heads, head_dim, int(causal), stream))


def _table(items):
    arr = (ctypes.c_void_p * len(items))()
    for i, t in enumerate(items):
        arr[i] = _ptr(t)
    return arr


def hanayo_executor_plan(tasks, P, W, M, rank, lanes, desc=None, ends=None):
    """(lane [n], deps [n][5]) of the executor's lane plan; host only.  desc, ends: ChunkDesc and EndsDesc of a
    run with the model's ends, or None."""
    tasks = np.ascontiguousarray(tasks, dtype=TASK_DTYPE)
    lane = np.zeros(tasks.size, dtype=np.int32)
    deps = np.zeros((tasks.size, 5), dtype=np.int32)
    _check(_lib.hanayo_executor_plan(tasks.ctypes.data, tasks.size, P, W, M, rank, lanes,
                                     ctypes.addressof(desc) if desc is not None else None,
                                     ctypes.addressof(ends) if ends is not None else None, lane.ctypes.data,
                                     deps.ctypes.data))
    return lane, deps


def hanayo_executor_run(tasks, desc, P, W, M, rank, weights, grads, act_in, grad_in, act_out, grad_out,
                        valid_len, stash_arena, stash_arena_bytes, workspace, stream=None, lanes=1,
                        stash_mode=0, recompute_scratch=None, ends=None):
    """Tables are Python lists of tensors / None: weights, grads [2W]; act_*, grad_* [M*2W]
    indexed mb*2W+chunk; valid_len [M] or None.  Returns the stash peak seen."""
    tasks = np.ascontiguousarray(tasks, dtype=TASK_DTYPE)
    tabs = [_table(t) for t in (weights, grads, act_in, grad_in, act_out, grad_out)]
    vl = _table(valid_len) if valid_len is not None else None
    args = ExecArgs(ctypes.pointer(desc), P, W, M, rank, tabs[0], tabs[1], tabs[2], tabs[3], tabs[4], tabs[5],
                    vl, _ptr(stash_arena), stash_arena_bytes, _ptr(workspace), stream, lanes, stash_mode,
                    _ptr(recompute_scratch), ctypes.pointer(ends) if ends is not None else None)
    peak = _int()
    _check(_lib.hanayo_executor_run(tasks.ctypes.data, tasks.size, ctypes.byref(args), ctypes.byref(peak)))
    return peak.value


def _list_tables(lists):
    lists = [np.ascontiguousarray(t, dtype=TASK_DTYPE) for t in lists]
    ptrs = (ctypes.c_void_p * len(lists))(*[t.ctypes.data for t in lists])
    counts = (ctypes.c_size_t * len(lists))(*[t.size for t in lists])
    return lists, ptrs, counts


def hanayo_pipeline_run(lists, desc, P, W, M, weights, grads, x, dy, act, grad, valid_len, stash_arenas, workspace,
                        stream=None, timing=False, ends=None):
    """All P ranks' lists on this device with true dataflow.  Tables are Python lists of tensors:
    weights, grads [S]; x, dy [M]; act, grad [M*S] indexed mb*S+stage; valid_len [M] or None;
    stash_arenas [P].  Returns (stash peaks [P], per-rank arrays of task durations in ms or None)."""
    lists, ptrs, counts = _list_tables(lists)
    tabs = [_table(t) if t is not None else None for t in (weights, grads, x, dy, act, grad)]
    vl = _table(valid_len) if valid_len is not None else None
    arenas = _table(stash_arenas)
    arena_bytes = (ctypes.c_size_t * P)(*[t.numel() * t.element_size() for t in stash_arenas])
    args = PipelineArgs(ctypes.pointer(desc), P, W, M, tabs[0], tabs[1], tabs[2], tabs[3], tabs[4], tabs[5], vl,
                        arenas, arena_bytes, _ptr(workspace), stream, ctypes.pointer(ends) if ends is not None else None)
    peaks = (ctypes.c_int * P)()
    ms = [np.zeros(t.size, dtype=np.float32) for t in lists] if timing else None
    ms_tab = (ctypes.c_void_p * P)(*[a.ctypes.data for a in ms]) if timing else None
    _check(_lib.hanayo_pipeline_run(ptrs, counts, ctypes.byref(args), peaks, ms_tab))
    return list(peaks), ms


ACTION_DTYPE = np.dtype([("kind", np.uint8), ("chunk", np.uint8), ("peer", np.uint16), ("mb", np.uint32),
                         ("stage", np.uint32)])
F, B, SEND_ACT, RECV_ACT, SEND_GRAD, RECV_GRAD = range(6)


def hanayo_actions(P, W, M, rank):
    """Rank's action list (compute + send / receive actions) as a structured array."""
    n = _sz()
    rc = _lib.hanayo_actions(P, W, M, rank, None, 0, ctypes.byref(n))
    if rc != EBUFSIZE:
        _check(rc if rc != OK else ESTATE)
    out = np.zeros(n.value, dtype=ACTION_DTYPE)
    _check(_lib.hanayo_actions(P, W, M, rank, out.ctypes.data, out.size, ctypes.byref(n)))
    return out


def hanayo_actions_of(tasks, P, W, rank):
    """Action list of any task list of a rank (W = 0: straight placement)."""
    tasks = np.ascontiguousarray(tasks, dtype=TASK_DTYPE)
    n = _sz()
    rc = _lib.hanayo_actions_of(tasks.ctypes.data, tasks.size, P, W, rank, None, 0, ctypes.byref(n))
    if rc != EBUFSIZE:
        _check(rc)
    out = np.zeros(n.value, dtype=ACTION_DTYPE)
    _check(_lib.hanayo_actions_of(tasks.ctypes.data, tasks.size, P, W, rank, out.ctypes.data, out.size, ctypes.byref(n)))
    return out


def hanayo_replay_actions(lists, P, W, M, t_f=1.0, t_b=2.0, t_c=0.0, prefetch=False, cost=None):
    """The P interpreters simulated (see include/hanayo.h).  Returns (makespan, idle [P], waited [P])."""
    lists = [np.ascontiguousarray(t, dtype=ACTION_DTYPE) for t in lists]
    ptrs = (ctypes.c_void_p * len(lists))(*[t.ctypes.data for t in lists])
    counts = (ctypes.c_size_t * len(lists))(*[t.size for t in lists])
    cost_tab = None
    if cost is not None:
        cost = [np.ascontiguousarray(c, dtype=np.float32) for c in cost]
        if any(c.size != t.size for c, t in zip(cost, lists)):
            raise HanayoError(EINVAL)
        cost_tab = (ctypes.c_void_p * P)(*[c.ctypes.data for c in cost])
    makespan = ctypes.c_double()
    idle, waited = np.zeros(P), np.zeros(P)
    _check(_lib.hanayo_replay_actions(ptrs, counts, P, W, M, t_f, t_b, t_c, int(bool(prefetch)), cost_tab,
                                      ctypes.byref(makespan), idle.ctypes.data, waited.ctypes.data))
    return makespan.value, idle, waited


def hanayo_pipeline_run_actions(lists, desc, P, W, M, weights, grads, x, dy, act, grad, valid_len, stash_arenas,
                                workspace, act_recv, grad_recv, async_copies=True, link_workgroups=0, stream=None,
                                timing=False, ends=None):
    """All P ranks' ACTION lists on this device, transfers carried out as device copies (see include/hanayo.h).
    act_recv, grad_recv: lists [M*S] of tensors or None.  Returns (stash peaks [P], per-rank arrays of action
    durations in ms or None)."""
    lists = [np.ascontiguousarray(t, dtype=ACTION_DTYPE) for t in lists]
    ptrs = (ctypes.c_void_p * len(lists))(*[t.ctypes.data for t in lists])
    counts = (ctypes.c_size_t * len(lists))(*[t.size for t in lists])
    tabs = [_table(t) for t in (weights, grads, x, dy, act, grad)]
    vl = _table(valid_len) if valid_len is not None else None
    arenas = _table(stash_arenas)
    arena_bytes = (ctypes.c_size_t * P)(*[t.numel() * t.element_size() for t in stash_arenas])
    args = PipelineArgs(ctypes.pointer(desc), P, W, M, tabs[0], tabs[1], tabs[2], tabs[3], tabs[4], tabs[5], vl,
                        arenas, arena_bytes, _ptr(workspace), stream, ctypes.pointer(ends) if ends is not None else None)
    link = LinkArgs(_table(act_recv), _table(grad_recv), int(bool(async_copies)), int(link_workgroups))
    peaks = (ctypes.c_int * P)()
    ms = [np.zeros(t.size, dtype=np.float32) for t in lists] if timing else None
    ms_tab = (ctypes.c_void_p * P)(*[a.ctypes.data for a in ms]) if timing else None
    _check(_lib.hanayo_pipeline_run_actions(ptrs, counts, ctypes.byref(args), ctypes.byref(link), peaks, ms_tab))
    return list(peaks), ms


def hanayo_replay(lists, P, W, M, cost=None):
    """Replay of all ranks' lists with per-task durations cost[r][i] (None: forward 1, backward 2).
    Returns (makespan, idle per rank).  Host only."""
    lists, ptrs, counts = _list_tables(lists)
    cost_tab = None
    if cost is not None:
        cost = [np.ascontiguousarray(c, dtype=np.float32) for c in cost]
        for c, t in zip(cost, lists):
            if c.size != t.size:
                raise HanayoError(EINVAL)
        cost_tab = (ctypes.c_void_p * P)(*[c.ctypes.data for c in cost])
    makespan = ctypes.c_double()
    idle = np.zeros(P, dtype=np.float64)
    _check(_lib.hanayo_replay(ptrs, counts, P, W, M, cost_tab, ctypes.byref(makespan), idle.ctypes.data))
    return makespan.value, idle


# ------------------------------------------------------------------ packing (layout marshalling only)

def pack_params(desc, blocks):
    """list of per-block dicts of float32 arrays -> flat float32 array in the packed order."""
    total = hanayo_param_span(desc, desc.n_blocks - 1, N_PARAMS - 1)
    flat = np.zeros(total[0] + total[1], dtype=np.float32)
    for b, blk in enumerate(blocks):
        for i, name in enumerate(PARAM_NAMES):
            off, cnt = hanayo_param_span(desc, b, i)
            flat[off:off + cnt] = np.asarray(blk[name], dtype=np.float32).reshape(-1)
    return flat


def unpack_params(desc, flat, like):
    """flat array in the packed order -> list of per-block dicts shaped like `like`."""
    out = []
    for b, blk in enumerate(like):
        d = {}
        for i, name in enumerate(PARAM_NAMES):
            off, cnt = hanayo_param_span(desc, b, i)
            d[name] = np.asarray(flat[off:off + cnt]).reshape(np.shape(blk[name]))
        out.append(d)
    return out
