"""ctypes binding of liblynx.so: argument marshalling only.

Function names and argument order are those of include/lynx.h.  Device
buffers are passed as torch tensors (or raw integer addresses); torch is used
for device memory and streams, nothing else.  There is no fallback: if the
library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblynx.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2406_08756_amd.build` "
        "(there is no CPU or PyTorch fallback)")
_lib = C.CDLL(LIB_PATH)

LYNX_OK, LYNX_ERR_INVALID_ARG, LYNX_ERR_SHAPE, LYNX_ERR_STATE = 0, 1, 2, 3
LYNX_ERR_DEPENDENCY, LYNX_ERR_OOM, LYNX_ERR_HIP = 4, 5, 6
LYNX_F32, LYNX_BF16 = 0, 1
LYNX_RETAIN_STORE_ALL = 0x3FFF
LYNX_RETAIN_FULL_RECOMPUTE = 0x2001
LYNX_RETAIN_ATTENTION_ONLY = 0x3FFF & ~0x0038
LYNX_RETAIN_ELEMENTWISE_ONLY = 0x3FFF & ~0x0830
LYNX_SEG_ALL_MISSING = 0xFFFFFFFF
LYNX_NUM_ACTIVATIONS = 14
LYNX_PROFILE_SLOTS = 40
LYNX_STATIC_WORKSPACE_BYTES = 64 << 20
LYNX_FLAG_FUSED_ATTENTION = 1
PARAM_FIELDS = ("wqkv", "bqkv", "wo", "bo", "w1", "b1", "w2", "b2", "g1", "be1", "g2", "be2")


class lynx_layer_config(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("hidden", C.c_int32), ("local_heads", C.c_int32),
                ("head_dim", C.c_int32), ("local_ffn", C.c_int32), ("seq", C.c_int32),
                ("micro_batch", C.c_int32), ("tp_size", C.c_int32), ("tp_rank", C.c_int32),
                ("causal", C.c_int32), ("dropout_p", C.c_float), ("ln_eps", C.c_float),
                ("seed", C.c_uint64), ("layer_id", C.c_uint32), ("flags", C.c_uint32)]


class lynx_params(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_FIELDS]


class lynx_grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_FIELDS]


class lynx_policy_problem(C.Structure):
    _fields_ = [("n_ops", C.c_int32), ("cost", C.POINTER(C.c_double)), ("bytes", C.POINTER(C.c_double)),
                ("parents", C.POINTER(C.c_uint32)), ("comm_mask", C.c_uint32), ("needed_mask", C.c_uint32),
                ("ctime", C.c_double * 4), ("m_budget", C.c_double), ("m_static", C.c_double),
                ("n_layer", C.c_int32), ("n_batch", C.c_int32), ("last_stage", C.c_int32)]


class lynx_policy(C.Structure):
    _fields_ = [("retain_mask", C.c_uint32), ("phase_mask", C.c_uint32 * 5), ("critical_cost", C.c_double),
                ("recompute_cost", C.c_double), ("peak_bytes", C.c_double)]


class lynx_partition_problem(C.Structure):
    _fields_ = [("layer", C.POINTER(lynx_policy_problem)), ("n_total_layers", C.c_int32), ("n_stages", C.c_int32),
                ("t_fwd", C.c_double), ("t_bwd", C.c_double), ("static_per_layer", C.c_double),
                ("m_budget", C.c_double)]


class LynxError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lynx_status_string(status)} (status {status})")


_cfg_p = C.POINTER(lynx_layer_config)
_proto = {
    "lynx_activation_bytes": (C.c_size_t, [_cfg_p, C.c_int]),
    "lynx_workspace_bytes": (C.c_size_t, [_cfg_p, C.c_uint32]),
    "lynx_workspace_bytes_for_schedule": (C.c_size_t, [_cfg_p, C.c_uint32, C.POINTER(C.c_uint32)]),
    "lynx_layer_set_gradient_tap": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p]),
    "lynx_layer_create": (C.c_int, [_cfg_p, C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)]),
    "lynx_layer_create_static": (C.c_int, [_cfg_p, C.POINTER(C.c_void_p)]),
    "lynx_layer_destroy": (C.c_int, [C.c_void_p]),
    "lynx_layer_set_params": (C.c_int, [C.c_void_p, C.POINTER(lynx_params)]),
    "lynx_layer_forward": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64,
                                     C.c_void_p]),
    "lynx_recompute": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p]),
    "lynx_layer_backward": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(lynx_grads),
                                      C.c_void_p]),
    "lynx_layer_reset": (C.c_int, [C.c_void_p]),
    "lynx_layer_live_mask": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32)]),
    "lynx_layer_missing_mask": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32)]),
    "lynx_layer_live_bytes": (C.c_int, [C.c_void_p, C.POINTER(C.c_size_t)]),
    "lynx_layer_peak_bytes": (C.c_int, [C.c_void_p, C.POINTER(C.c_size_t)]),
    "lynx_layer_activation": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_void_p),
                                        C.POINTER(C.c_size_t)]),
    "lynx_dropout_mask": (C.c_int, [_cfg_p, C.c_uint64, C.c_int, C.c_void_p, C.c_void_p]),
    "lynx_layer_set_dry_run": (C.c_int, [C.c_void_p, C.c_int]),
    "lynx_layer_set_profiling": (C.c_int, [C.c_void_p, C.c_int]),
    "lynx_layer_profile_ms": (C.c_int, [C.c_void_p, C.POINTER(C.c_float)]),
    "lynx_profile_slot_name": (C.c_char_p, [C.c_int]),
    "lynx_status_string": (C.c_char_p, [C.c_int]),
    "lynx_comm_standin": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]),
    "lynx_policy_solve": (C.c_int, [C.POINTER(lynx_policy_problem), C.POINTER(lynx_policy)]),
    "lynx_partition_solve": (C.c_int, [C.POINTER(lynx_partition_problem), C.POINTER(C.c_int32),
                                       C.POINTER(C.c_double), C.POINTER(lynx_policy)]),
    "lynx_policy_layer_problem": (C.c_int, [_cfg_p, C.POINTER(lynx_policy_problem), C.POINTER(C.c_uint32),
                                            C.POINTER(C.c_double)]),
}
for _name, (_res, _args) in _proto.items():
    _f = getattr(_lib, _name)
    _f.restype, _f.argtypes = _res, _args
EXPORTED = tuple(_proto)


def _addr(buf) -> Optional[int]:
    """Device address of a torch tensor, or an integer address passed through."""
    if buf is None:
        return None
    if isinstance(buf, int):
        return buf
    return buf.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int, where: str) -> None:
    if status != LYNX_OK:
        raise LynxError(status, where)


def make_config(cfg) -> lynx_layer_config:
    """From any object with the config's field names (e.g. lynx_synth.LayerConfig)."""
    if isinstance(cfg, lynx_layer_config):
        return cfg
    return lynx_layer_config(int(cfg.dtype), cfg.hidden, cfg.local_heads, cfg.head_dim,
                             cfg.local_ffn, cfg.seq, cfg.micro_batch, cfg.tp_size, cfg.tp_rank,
                             int(cfg.causal), float(cfg.dropout_p), float(cfg.ln_eps),
                             int(cfg.seed), int(cfg.layer_id), int(getattr(cfg, "flags", 0)))


def lynx_status_string(status: int) -> str:
    return _lib.lynx_status_string(status).decode()


def lynx_activation_bytes(cfg, act_id: int) -> int:
    return _lib.lynx_activation_bytes(C.byref(make_config(cfg)), act_id)


def lynx_workspace_bytes(cfg, retain_mask: int) -> int:
    return _lib.lynx_workspace_bytes(C.byref(make_config(cfg)), retain_mask)


def lynx_workspace_bytes_for_schedule(cfg, retain_mask: int, phase_masks=None) -> int:
    pm = None if phase_masks is None else (C.c_uint32 * 4)(*[int(m) for m in phase_masks])
    return _lib.lynx_workspace_bytes_for_schedule(C.byref(make_config(cfg)), retain_mask, pm)


def lynx_layer_set_gradient_tap(layer: int, act_id: int, dst) -> None:
    _check(_lib.lynx_layer_set_gradient_tap(layer, act_id, _addr(dst)), "lynx_layer_set_gradient_tap")


def lynx_layer_create(cfg, workspace, workspace_bytes: int) -> int:
    handle = C.c_void_p()
    _check(_lib.lynx_layer_create(C.byref(make_config(cfg)), _addr(workspace), workspace_bytes,
                                  C.byref(handle)), "lynx_layer_create")
    return handle.value


def lynx_layer_create_static(cfg) -> int:
    handle = C.c_void_p()
    _check(_lib.lynx_layer_create_static(C.byref(make_config(cfg)), C.byref(handle)), "lynx_layer_create_static")
    return handle.value


def lynx_layer_destroy(layer: int) -> None:
    _check(_lib.lynx_layer_destroy(layer), "lynx_layer_destroy")


def _ptr_struct(cls, tensors: Dict[str, object]):
    return cls(*[_addr(tensors[n]) for n in PARAM_FIELDS])


def lynx_layer_set_params(layer: int, params: Dict[str, object]) -> None:
    st = _ptr_struct(lynx_params, params)
    _check(_lib.lynx_layer_set_params(layer, C.byref(st)), "lynx_layer_set_params")


def lynx_layer_forward(layer: int, x, out, retain_mask: int, step: int = 0, stream=None) -> None:
    _check(_lib.lynx_layer_forward(layer, _addr(x), _addr(out), retain_mask, step, _stream(stream)),
           "lynx_layer_forward")


def lynx_recompute(layer: int, segment_mask: int, stream=None) -> None:
    _check(_lib.lynx_recompute(layer, segment_mask, _stream(stream)), "lynx_recompute")


def lynx_layer_backward(layer: int, d_out, d_x, grads: Dict[str, object], stream=None) -> None:
    st = _ptr_struct(lynx_grads, grads)
    _check(_lib.lynx_layer_backward(layer, _addr(d_out), _addr(d_x), C.byref(st), _stream(stream)),
           "lynx_layer_backward")


def lynx_layer_reset(layer: int) -> None:
    _check(_lib.lynx_layer_reset(layer), "lynx_layer_reset")


def lynx_layer_live_mask(layer: int) -> int:
    v = C.c_uint32()
    _check(_lib.lynx_layer_live_mask(layer, C.byref(v)), "lynx_layer_live_mask")
    return v.value


def lynx_layer_missing_mask(layer: int) -> int:
    v = C.c_uint32()
    _check(_lib.lynx_layer_missing_mask(layer, C.byref(v)), "lynx_layer_missing_mask")
    return v.value


def lynx_layer_live_bytes(layer: int) -> int:
    v = C.c_size_t()
    _check(_lib.lynx_layer_live_bytes(layer, C.byref(v)), "lynx_layer_live_bytes")
    return v.value


def lynx_layer_peak_bytes(layer: int) -> int:
    v = C.c_size_t()
    _check(_lib.lynx_layer_peak_bytes(layer, C.byref(v)), "lynx_layer_peak_bytes")
    return v.value


def lynx_layer_activation(layer: int, act_id: int):
    """(device address or None, bytes)."""
    p, n = C.c_void_p(), C.c_size_t()
    _check(_lib.lynx_layer_activation(layer, act_id, C.byref(p), C.byref(n)), "lynx_layer_activation")
    return p.value, n.value


def lynx_dropout_mask(cfg, step: int, site: int, out, stream=None) -> None:
    _check(_lib.lynx_dropout_mask(C.byref(make_config(cfg)), step, site, _addr(out), _stream(stream)),
           "lynx_dropout_mask")


def lynx_layer_set_dry_run(layer: int, on: bool) -> None:
    _check(_lib.lynx_layer_set_dry_run(layer, int(on)), "lynx_layer_set_dry_run")


def lynx_layer_set_profiling(layer: int, on: bool) -> None:
    _check(_lib.lynx_layer_set_profiling(layer, int(on)), "lynx_layer_set_profiling")


def lynx_layer_profile_ms(layer: int):
    """{slot name: ms} for the slots that ran since the previous query."""
    buf = (C.c_float * LYNX_PROFILE_SLOTS)()
    _check(_lib.lynx_layer_profile_ms(layer, buf), "lynx_layer_profile_ms")
    return {lynx_profile_slot_name(i): buf[i] for i in range(LYNX_PROFILE_SLOTS) if buf[i] >= 0}


def lynx_profile_slot_name(slot: int) -> str:
    return _lib.lynx_profile_slot_name(slot).decode()


def lynx_comm_standin(dst, src, nbytes: int, workgroups: int, stream=None) -> None:
    _check(_lib.lynx_comm_standin(_addr(dst), _addr(src), nbytes, workgroups, _stream(stream)),
           "lynx_comm_standin")


def _mask_of(indices) -> int:
    m = 0
    for i in indices:
        m |= 1 << int(i)
    return m


def _policy_problem_struct(problem: dict):
    """(struct, keep-alive arrays) for a problem dict."""
    n = int(problem["n"])
    cost = (C.c_double * n)(*[float(v) for v in problem["cost"]])
    nbytes = (C.c_double * n)(*[float(v) for v in problem["bytes"]])
    parents = (C.c_uint32 * n)(*[_mask_of(q) for q in problem["parents"]])
    p = lynx_policy_problem()
    p.n_ops = n
    p.cost, p.bytes, p.parents = cost, nbytes, parents
    p.comm_mask, p.needed_mask = _mask_of(problem["comm"]), _mask_of(problem["needed"])
    for t in range(4):
        p.ctime[t] = float(problem["ctime"][t])
    p.m_budget, p.m_static = float(problem.get("m_budget", 0.0)), float(problem.get("m_static", 0.0))
    p.n_layer, p.n_batch = int(problem.get("n_layer", 1)), int(problem.get("n_batch", 1))
    p.last_stage = 1 if problem.get("last_stage") else 0
    return p, (cost, nbytes, parents)


def _policy_dict(out) -> dict:
    return {"retain_mask": int(out.retain_mask), "phase_mask": [int(m) for m in out.phase_mask],
            "critical_cost": float(out.critical_cost), "recompute_cost": float(out.recompute_cost),
            "peak_bytes": float(out.peak_bytes)}


def lynx_partition_solve(layer_problem: dict, n_total_layers: int, n_stages: int, t_fwd: float, t_bwd: float,
                         static_per_layer: float, m_budget: float):
    """Recomputation-aware greedy partition of identical layers over pipeline stages.
    Returns (layers per stage, time per stage, policy per stage) or None when the
    equal-share scheme does not fit the budget."""
    p, keep = _policy_problem_struct(layer_problem)
    pp = lynx_partition_problem()
    pp.layer = C.pointer(p)
    pp.n_total_layers, pp.n_stages = int(n_total_layers), int(n_stages)
    pp.t_fwd, pp.t_bwd = float(t_fwd), float(t_bwd)
    pp.static_per_layer, pp.m_budget = float(static_per_layer), float(m_budget)
    layers = (C.c_int32 * n_stages)()
    times = (C.c_double * n_stages)()
    policies = (lynx_policy * n_stages)()
    st = _lib.lynx_partition_solve(C.byref(pp), layers, times, policies)
    if st == LYNX_ERR_OOM:
        return None
    if st != LYNX_OK:
        raise LynxError(st, "lynx_partition_solve")
    return [int(v) for v in layers], [float(v) for v in times], [_policy_dict(q) for q in policies]


def lynx_policy_solve(problem: dict):
    """Solve a single-layer recomputation policy.  `problem` is a dict with n,
    cost[n], bytes[n], parents[n] (tuples of 1-based operator indices), comm and
    needed (sets of 1-based indices), ctime[4], m_budget, m_static, n_layer,
    n_batch, last_stage.  Returns a dict (retain_mask, phase_mask[5],
    critical_cost, recompute_cost, peak_bytes), or None when nothing fits."""
    p, keep = _policy_problem_struct(problem)
    out = lynx_policy()
    st = _lib.lynx_policy_solve(C.byref(p), C.byref(out))
    if st == LYNX_ERR_OOM:
        return None
    if st != LYNX_OK:
        raise LynxError(st, "lynx_policy_solve")
    return _policy_dict(out)


def lynx_policy_layer_problem(cfg, cost, ctime, m_budget, m_static=0.0, n_layer=1, n_batch=1,
                              last_stage=False) -> dict:
    """The problem dict of this library's 13-operator block for `cfg`: the
    dependency table, what backward reads and the M_i come from the library;
    cost[13] (C_i of OP_1..OP_13, e.g. from lynx_layer_profile_ms) and the rest
    from the caller."""
    c = cfg if isinstance(cfg, lynx_layer_config) else make_config(cfg)
    p = lynx_policy_problem()
    parents = (C.c_uint32 * 13)()
    nbytes = (C.c_double * 13)()
    st = _lib.lynx_policy_layer_problem(C.byref(c), C.byref(p), parents, nbytes)
    if st != LYNX_OK:
        raise LynxError(st, "lynx_policy_layer_problem")
    if len(cost) != 13:
        raise ValueError("cost must have 13 entries (OP_1..OP_13)")
    return {"n": 13, "cost": [float(v) for v in cost], "bytes": [float(v) for v in nbytes],
            "parents": [tuple(j for j in range(1, 14) if (int(parents[i]) >> j) & 1) for i in range(13)],
            "comm": set(), "needed": set(i for i in range(1, 14) if (int(p.needed_mask) >> i) & 1),
            "ctime": [float(v) for v in ctime], "m_budget": float(m_budget), "m_static": float(m_static),
            "n_layer": int(n_layer), "n_batch": int(n_batch), "last_stage": bool(last_stage)}
