"""ctypes binding of libhap.so: argument marshalling only.

Device buffers are torch tensors (any object with ``data_ptr()``) or raw integer addresses;
the stream is torch's current HIP stream unless given.  Every wrapper raises HapError on a
non-zero status and never falls back to another implementation: if the shared library has
not been built, importing this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(HERE, "libhap.so")

F32, BF16 = 0, 1
SHARD_BATCH, SHARD_FEATURE, SHARD_REDUCTION, REPLICATED = 0, 1, 2, 3
ACT_NONE, ACT_GELU_ERF = 0, 1

if not os.path.exists(lib_path):
    raise ImportError(
        f"{lib_path} is missing: build it with `python -m paper_2401_05965_amd.build` "
        "(or __graft_entry__.build()); there is no fallback path")
# PyTorch ships its own HIP runtime (same SONAME as the system one).  Two runtimes in one process do
# not work, so torch's copy must already be mapped when libhap.so is loaded: the dynamic linker then
# resolves libhap's libamdhip64.so.7 dependency to it, and both share devices, streams and memory.
import torch  # noqa: E402,F401  (load order matters; no torch API is used by the library)

lib = C.CDLL(lib_path)


class HapError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = lib.hap_last_error().decode()
        super().__init__(f"{where}: {lib.hap_strerror(status).decode()} ({status}): {detail}")


class Stage(C.Structure):
    _fields_ = [("flops_sharded", C.c_double), ("flops_fixed", C.c_double),
                ("comm_latency", C.c_double), ("comm_per_ratio", C.c_double)]


class _LinearDesc(C.Structure):
    _fields_ = [("tokens", C.c_int64), ("in_features", C.c_int64), ("out_features", C.c_int64),
                ("mode", C.c_int), ("m", C.c_int), ("offsets", C.POINTER(C.c_int64)),
                ("io_dtype", C.c_int), ("act", C.c_int), ("has_bias", C.c_int),
                ("ldx", C.c_int64), ("ldw", C.c_int64), ("ldy", C.c_int64),
                ("operands_are_full", C.c_int)]


class _AttnDesc(C.Structure):
    _fields_ = [("batch", C.c_int64), ("heads", C.c_int64), ("seq", C.c_int64), ("head_dim", C.c_int64),
                ("shard_over_heads", C.c_int), ("m", C.c_int), ("offsets", C.POINTER(C.c_int64)),
                ("io_dtype", C.c_int), ("stride_b", C.c_int64), ("stride_s", C.c_int64), ("stride_h", C.c_int64),
                ("o_stride_b", C.c_int64), ("o_stride_s", C.c_int64), ("o_stride_h", C.c_int64)]


class _MoeDesc(C.Structure):
    _fields_ = [("experts", C.c_int64), ("capacity", C.c_int64), ("in_features", C.c_int64), ("out_features", C.c_int64),
                ("m", C.c_int), ("offsets", C.POINTER(C.c_int64)),
                ("io_dtype", C.c_int), ("act", C.c_int), ("has_bias", C.c_int),
                ("ldx", C.c_int64), ("ldw", C.c_int64), ("ldy", C.c_int64),
                ("operands_are_full", C.c_int)]


class _GatherDesc(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("dim", C.c_int), ("m", C.c_int),
                ("offsets", C.POINTER(C.c_int64)), ("elem_bytes", C.c_int)]


class GatherDesc:
    """Python mirror of hap_gather_desc; keeps the offsets array alive."""

    def __init__(self, rows, cols, dim, offsets: Sequence[int], elem_bytes):
        offsets = list(offsets)
        self._offs = (C.c_int64 * len(offsets))(*offsets)
        self.m = len(offsets) - 1
        self.c = _GatherDesc(rows, cols, dim, self.m, C.cast(self._offs, C.POINTER(C.c_int64)), elem_bytes)


class LinearDesc:
    """Python mirror of hap_linear_desc; keeps the offsets array alive."""

    def __init__(self, tokens, in_features, out_features, mode, offsets: Optional[Sequence[int]], io_dtype,
                 act=ACT_NONE, has_bias=False, ldx=None, ldw=None, ldy=None, operands_are_full=True, m=None):
        offsets = list(offsets) if offsets is not None else None
        self._offs = (C.c_int64 * len(offsets))(*offsets) if offsets is not None else None
        self.m = (len(offsets) - 1) if (offsets is not None and m is None) else (m if m is not None else 1)
        self.c = _LinearDesc(tokens, in_features, out_features, mode, self.m,
                             C.cast(self._offs, C.POINTER(C.c_int64)) if self._offs is not None else None,
                             io_dtype, act, int(bool(has_bias)),
                             ldx if ldx is not None else in_features,
                             ldw if ldw is not None else out_features,
                             ldy if ldy is not None else out_features,
                             int(bool(operands_are_full)))


class MoeDesc:
    """Python mirror of hap_moe_desc; keeps the offsets array (expert ranges of the devices) alive."""

    def __init__(self, experts, capacity, in_features, out_features, offsets: Sequence[int], io_dtype,
                 act=ACT_NONE, has_bias=False, ldx=None, ldw=None, ldy=None, operands_are_full=True):
        offsets = list(offsets)
        self._offs = (C.c_int64 * len(offsets))(*offsets)
        self.m = len(offsets) - 1
        self.c = _MoeDesc(experts, capacity, in_features, out_features, self.m, C.cast(self._offs, C.POINTER(C.c_int64)),
                          io_dtype, act, int(bool(has_bias)),
                          ldx if ldx is not None else in_features,
                          ldw if ldw is not None else out_features,
                          ldy if ldy is not None else out_features,
                          int(bool(operands_are_full)))


class AttnDesc:
    def __init__(self, batch, heads, seq, head_dim, shard_over_heads, offsets, io_dtype=BF16,
                 stride_b=None, stride_s=None, stride_h=None, o_strides=None):
        offsets = list(offsets)
        self._offs = (C.c_int64 * len(offsets))(*offsets)
        self.m = len(offsets) - 1
        stride_h = head_dim if stride_h is None else stride_h
        stride_s = heads * head_dim if stride_s is None else stride_s
        stride_b = seq * stride_s if stride_b is None else stride_b
        self.c = _AttnDesc(batch, heads, seq, head_dim, int(bool(shard_over_heads)), self.m,
                           C.cast(self._offs, C.POINTER(C.c_int64)), io_dtype, stride_b, stride_s, stride_h,
                           *(o_strides if o_strides is not None else (0, 0, 0)))


lib.hap_strerror.restype = C.c_char_p
lib.hap_strerror.argtypes = [C.c_int]
lib.hap_last_error.restype = C.c_char_p
lib.hap_version.restype = C.c_char_p
lib.hap_debug_set_gemm_view_limit.restype = C.c_int64
lib.hap_allgather_capacity.restype = C.c_int64
for _n in ("hap_linear_fwd_workspace", "hap_linear_bwd_workspace", "hap_sfb_workspace", "hap_attn_bwd_workspace",
           "hap_layernorm_bwd_workspace", "hap_colsum_workspace", "hap_moe_linear_fwd_workspace", "hap_moe_linear_bwd_workspace"):
    if hasattr(lib, _n):
        getattr(lib, _n).restype = C.c_size_t


def _ptr(t) -> C.c_void_p:
    if t is None:
        return C.c_void_p(None)
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def _ws(ws):
    if ws is None:
        return C.c_void_p(None), C.c_size_t(0)
    return C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel() * ws.element_size())


def _check(status: int, where: str):
    if status != 0:
        raise HapError(status, where)


def _stages(stages):
    arr = (Stage * len(stages))()
    for i, s in enumerate(stages):
        arr[i] = s if isinstance(s, Stage) else Stage(*[float(v) for v in s])
    return arr


# ---------------------------------------------------------------- host

def hap_shard_ratios(speed: Sequence[float], stages):
    """stages: sequence of (flops_sharded, flops_fixed, comm_latency, comm_per_ratio). Returns (ratios, seconds)."""
    m = len(speed)
    sp = (C.c_double * m)(*[float(v) for v in speed])
    out = (C.c_double * m)()
    obj = C.c_double()
    _check(lib.hap_shard_ratios(C.c_int(m), sp, C.c_int(len(stages)), _stages(stages), out, C.byref(obj)), "hap_shard_ratios")
    return list(out), obj.value


def hap_iteration_time(speed, stages, ratios) -> float:
    m = len(speed)
    sec = C.c_double()
    _check(lib.hap_iteration_time(C.c_int(m), (C.c_double * m)(*map(float, speed)), C.c_int(len(stages)), _stages(stages),
                                  (C.c_double * m)(*map(float, ratios)), C.byref(sec)), "hap_iteration_time")
    return sec.value


def hap_shard_ratios_segments(speed: Sequence[float], stages, seg_offsets: Sequence[int]):
    """Per-segment ratios (Sec. 5.2).  Returns (g x m list of lists, seconds)."""
    m, g = len(speed), len(seg_offsets) - 1
    out = (C.c_double * (g * m))()
    obj = C.c_double()
    _check(lib.hap_shard_ratios_segments(C.c_int(m), (C.c_double * m)(*map(float, speed)), C.c_int(len(stages)), _stages(stages), C.c_int(g),
                                         (C.c_int * (g + 1))(*map(int, seg_offsets)), out, C.byref(obj)), "hap_shard_ratios_segments")
    return [list(out[k * m:(k + 1) * m]) for k in range(g)], obj.value


def hap_iteration_time_segments(speed, stages, seg_offsets, ratios) -> float:
    m, g = len(speed), len(seg_offsets) - 1
    flat = [float(v) for row in ratios for v in row]
    sec = C.c_double()
    _check(lib.hap_iteration_time_segments(C.c_int(m), (C.c_double * m)(*map(float, speed)), C.c_int(len(stages)), _stages(stages), C.c_int(g),
                                           (C.c_int * (g + 1))(*map(int, seg_offsets)), (C.c_double * (g * m))(*flat), C.byref(sec)),
           "hap_iteration_time_segments")
    return sec.value


class _GraphNode(C.Structure):
    _fields_ = [("op", C.c_int), ("a", C.c_int), ("b", C.c_int), ("rows", C.c_int64), ("cols", C.c_int64)]


class _Instr(C.Structure):
    _fields_ = [("kind", C.c_int), ("tensor", C.c_int), ("arg0", C.c_int), ("arg1", C.c_int)]


class _Net(C.Structure):
    _fields_ = [("latency", C.c_double), ("bandwidth", C.c_double), ("elem_bytes", C.c_int)]


class _SynthRules(C.Structure):
    _fields_ = [("placeholder_dims_mask", C.c_int), ("parameter_dims_mask", C.c_int), ("grouped_broadcast", C.c_int),
                ("replicated_matmul", C.c_int), ("placeholder_replicated", C.c_int)]


OPS = {"placeholder": 0, "parameter": 1, "matmul": 2, "unary": 3, "add": 4, "transpose": 5, "sum": 6}
INSTR_NAMES = ("placeholder", "placeholder-shard", "parameter", "parameter-shard", "matmul", "unary", "add", "transpose", "sum",
               "all-reduce", "reduce-scatter", "all-gather", "grouped-broadcast", "all-to-all")
FORM_NAMES = ("id", "ag0", "ag1", "ar")


def _graph(nodes):
    arr = (_GraphNode * len(nodes))()
    for i, n in enumerate(nodes):
        arr[i] = _GraphNode(OPS[n["op"]] if isinstance(n["op"], str) else n["op"], n.get("a", -1), n.get("b", -1), n["rows"], n["cols"])
    return arr


def _instr_tuple(i: _Instr):
    """(name, tensor, args...) in the notation of the paper's figures: dimensions for loads and collectives, input forms for computations."""
    name = INSTR_NAMES[i.kind]
    if name in ("placeholder", "parameter", "all-reduce"):
        return (name, i.tensor)
    if name in ("placeholder-shard", "parameter-shard", "reduce-scatter", "all-gather", "grouped-broadcast"):
        return (name, i.tensor, i.arg0)
    if name == "all-to-all":
        return (name, i.tensor, i.arg0, i.arg1)
    if name == "matmul":
        return (name, i.tensor, FORM_NAMES[i.arg0], FORM_NAMES[i.arg1])
    return (name, i.tensor, FORM_NAMES[i.arg0])


def _instr_struct(t):
    name = t[0]
    k = INSTR_NAMES.index(name)
    if name == "matmul":
        return _Instr(k, t[1], FORM_NAMES.index(t[2]), FORM_NAMES.index(t[3]))
    if name in ("unary", "add", "transpose", "sum"):
        return _Instr(k, t[1], FORM_NAMES.index(t[2]), 0)
    args = list(t[2:]) + [0, 0]
    return _Instr(k, t[1], args[0], args[1])


def hap_synthesize(nodes, ratios, speed, net, rules=None, capacity=64):
    """nodes: list of dicts (op, a, b, rows, cols); net: dict(latency, bandwidth, elem_bytes); rules: dict of the
    hap_synth_rules fields or None.  Returns (program as list of tuples, seconds, partial programs expanded)."""
    m = len(ratios)
    prog = (_Instr * capacity)()
    n = C.c_int(); sec = C.c_double(); exp = C.c_int64()
    r = _rules(rules)
    _check(lib.hap_synthesize(C.c_int(len(nodes)), _graph(nodes), C.c_int(m), (C.c_double * m)(*map(float, ratios)),
                              (C.c_double * m)(*map(float, speed)), C.byref(_Net(net["latency"], net["bandwidth"], net["elem_bytes"])), r,
                              prog, C.c_int(capacity), C.byref(n), C.byref(sec), C.byref(exp)), "hap_synthesize")
    return [_instr_tuple(prog[i]) for i in range(n.value)], sec.value, exp.value


def _rules(rules):
    if rules is None:
        return None
    dm = lambda dims: sum(1 << d for d in dims)
    return C.byref(_SynthRules(dm(rules.get("placeholder_dims", (0, 1))), dm(rules.get("parameter_dims", (0, 1))),
                               int(rules.get("grouped_broadcast", True)), int(rules.get("replicated_matmul", True)),
                               int(rules.get("placeholder_replicated", True))))


def hap_program_stages(nodes, program, m, net, capacity=64):
    """Stage tuples (flops_sharded, flops_fixed, comm_latency, comm_per_ratio) of a program, as hap_shard_ratios takes them."""
    arr = (_Instr * max(len(program), 1))(*[_instr_struct(t) for t in program])
    st = (Stage * capacity)()
    n = C.c_int()
    _check(lib.hap_program_stages(C.c_int(len(nodes)), _graph(nodes), C.c_int(len(program)), arr, C.c_int(m),
                                  C.byref(_Net(net["latency"], net["bandwidth"], net["elem_bytes"])), st, C.c_int(capacity), C.byref(n)),
           "hap_program_stages")
    return [(st[i].flops_sharded, st[i].flops_fixed, st[i].comm_latency, st[i].comm_per_ratio) for i in range(n.value)]


def hap_optimize(nodes, speed, net, rules=None, max_steps=10, capacity=64):
    """Alternating optimisation of Sec. 3.1.  Returns (program, ratios, seconds, steps)."""
    m = len(speed)
    prog = (_Instr * capacity)()
    n = C.c_int(); sec = C.c_double(); steps = C.c_int()
    B = (C.c_double * m)()
    _check(lib.hap_optimize(C.c_int(len(nodes)), _graph(nodes), C.c_int(m), (C.c_double * m)(*map(float, speed)),
                            C.byref(_Net(net["latency"], net["bandwidth"], net["elem_bytes"])), _rules(rules), C.c_int(max_steps),
                            prog, C.c_int(capacity), C.byref(n), B, C.byref(sec), C.byref(steps)), "hap_optimize")
    return [_instr_tuple(prog[i]) for i in range(n.value)], list(B), sec.value, steps.value


def hap_program_time(nodes, program, ratios, speed, net) -> float:
    m = len(ratios)
    arr = (_Instr * max(len(program), 1))(*[_instr_struct(t) for t in program])
    sec = C.c_double()
    _check(lib.hap_program_time(C.c_int(len(nodes)), _graph(nodes), C.c_int(len(program)), arr, C.c_int(m), (C.c_double * m)(*map(float, ratios)),
                                (C.c_double * m)(*map(float, speed)), C.byref(_Net(net["latency"], net["bandwidth"], net["elem_bytes"])),
                                C.byref(sec)), "hap_program_time")
    return sec.value


def hap_round_shards(ratios: Sequence[float], dim_len: int, granule: int = 1):
    m = len(ratios)
    sizes = (C.c_int64 * m)()
    offs = (C.c_int64 * (m + 1))()
    _check(lib.hap_round_shards(C.c_int(m), (C.c_double * m)(*map(float, ratios)), C.c_int64(dim_len), C.c_int64(granule),
                                sizes, offs), "hap_round_shards")
    return list(sizes), list(offs)


# ---------------------------------------------------------------- device

def hap_version() -> str:
    return lib.hap_version().decode()


def hap_strerror(status: int) -> str:
    return lib.hap_strerror(C.c_int(int(status))).decode()


def hap_last_error() -> str:
    return (lib.hap_last_error() or b"").decode()


def hap_linear_fwd_workspace(desc: LinearDesc, shard_index: int) -> int:
    return int(lib.hap_linear_fwd_workspace(C.byref(desc.c), C.c_int(shard_index)))


def hap_linear_bwd_workspace(desc: LinearDesc, shard_index: int) -> int:
    return int(lib.hap_linear_bwd_workspace(C.byref(desc.c), C.c_int(shard_index)))


def hap_sharded_linear_fwd(desc: LinearDesc, shard_index, X, W, bias, Y, preact=None, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib.hap_sharded_linear_fwd(C.byref(desc.c), C.c_int(shard_index), _ptr(X), _ptr(W), _ptr(bias), _ptr(Y),
                                      _ptr(preact), wp, wb, _stream(stream)), "hap_sharded_linear_fwd")


def hap_sharded_linear_bwd(desc: LinearDesc, shard_index, X, W, preact, dY, dX, dW, dW_dtype, dbias, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib.hap_sharded_linear_bwd(C.byref(desc.c), C.c_int(shard_index), _ptr(X), _ptr(W), _ptr(preact), _ptr(dY),
                                      _ptr(dX), _ptr(dW), C.c_int(dW_dtype), _ptr(dbias), wp, wb, _stream(stream)),
           "hap_sharded_linear_bwd")


def hap_sharded_linear_bwd_dact(desc: LinearDesc, shard_index, X, W, preact, dY, dX, dW, dW_dtype, dbias, x_preact, x_act,
                                ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib.hap_sharded_linear_bwd_dact(C.byref(desc.c), C.c_int(shard_index), _ptr(X), _ptr(W), _ptr(preact), _ptr(dY),
                                           _ptr(dX), _ptr(dW), C.c_int(dW_dtype), _ptr(dbias), _ptr(x_preact), C.c_int(x_act),
                                           wp, wb, _stream(stream)), "hap_sharded_linear_bwd_dact")


def hap_sfb_grad(Xs, dYs, rows, in_features, out_features, ldx, ldy, in_dtype, dW, lddw, accumulate=False, ws=None, stream=None):
    m = len(rows)
    xp = (C.c_void_p * m)(*[_ptr(t) for t in Xs])
    yp = (C.c_void_p * m)(*[_ptr(t) for t in dYs])
    wp, wb = _ws(ws)
    _check(lib.hap_sfb_grad(C.c_int(m), xp, yp, (C.c_int64 * m)(*map(int, rows)), C.c_int64(in_features), C.c_int64(out_features),
                            C.c_int64(ldx), C.c_int64(ldy), C.c_int(in_dtype), _ptr(dW), C.c_int64(lddw), C.c_int(int(accumulate)),
                            wp, wb, _stream(stream)), "hap_sfb_grad")


def hap_sfb_grad_static(Xs, dYs, rows, in_features, out_features, ldx, ldy, in_dtype, dW, lddw, accumulate=False, stream=None):
    m = len(rows)
    xp = (C.c_void_p * m)(*[_ptr(t) for t in Xs])
    yp = (C.c_void_p * m)(*[_ptr(t) for t in dYs])
    _check(lib.hap_sfb_grad_static(C.c_int(m), xp, yp, (C.c_int64 * m)(*map(int, rows)), C.c_int64(in_features), C.c_int64(out_features),
                                   C.c_int64(ldx), C.c_int64(ldy), C.c_int(in_dtype), _ptr(dW), C.c_int64(lddw), C.c_int(int(accumulate)),
                                   _stream(stream)), "hap_sfb_grad_static")


def hap_sfb_workspace(m, rows, in_features, out_features) -> int:
    return int(lib.hap_sfb_workspace(C.c_int(m), (C.c_int64 * m)(*map(int, rows)), C.c_int64(in_features), C.c_int64(out_features)))


def hap_moe_linear_fwd_workspace(desc: MoeDesc, shard_index: int) -> int:
    return int(lib.hap_moe_linear_fwd_workspace(C.byref(desc.c), C.c_int(shard_index)))


def hap_moe_linear_bwd_workspace(desc: MoeDesc, shard_index: int) -> int:
    return int(lib.hap_moe_linear_bwd_workspace(C.byref(desc.c), C.c_int(shard_index)))


def hap_moe_linear_fwd(desc: MoeDesc, shard_index, X, W, bias, rows, Y, preact=None, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib.hap_moe_linear_fwd(C.byref(desc.c), C.c_int(shard_index), _ptr(X), _ptr(W), _ptr(bias), _ptr(rows), _ptr(Y),
                                  _ptr(preact), wp, wb, _stream(stream)), "hap_moe_linear_fwd")


def hap_moe_linear_bwd(desc: MoeDesc, shard_index, X, W, preact, dY, rows, dX, dW, dW_dtype, dbias, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib.hap_moe_linear_bwd(C.byref(desc.c), C.c_int(shard_index), _ptr(X), _ptr(W), _ptr(preact), _ptr(dY), _ptr(rows),
                                  _ptr(dX), _ptr(dW), C.c_int(dW_dtype), _ptr(dbias), wp, wb, _stream(stream)), "hap_moe_linear_bwd")


def hap_moe_linear_bwd_dact(desc: MoeDesc, shard_index, X, W, preact, dY, rows, dX, dW, dW_dtype, dbias, x_preact, x_act, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib.hap_moe_linear_bwd_dact(C.byref(desc.c), C.c_int(shard_index), _ptr(X), _ptr(W), _ptr(preact), _ptr(dY), _ptr(rows),
                                       _ptr(dX), _ptr(dW), C.c_int(dW_dtype), _ptr(dbias), _ptr(x_preact), C.c_int(x_act), wp, wb,
                                       _stream(stream)), "hap_moe_linear_bwd_dact")


def hap_allgather_capacity(desc: GatherDesc) -> int:
    return int(lib.hap_allgather_capacity(C.byref(desc.c)))


def hap_allgather_pad(desc: GatherDesc, shard_index, shard, ld_shard, slot, ld_slot, stream=None):
    _check(lib.hap_allgather_pad(C.byref(desc.c), C.c_int(shard_index), _ptr(shard), C.c_int64(ld_shard), _ptr(slot), C.c_int64(ld_slot),
                                 _stream(stream)), "hap_allgather_pad")


def hap_allgather_assemble(desc: GatherDesc, pieces, ld_pieces, out, ld_out, stream=None):
    m = desc.m
    pp = (C.c_void_p * m)(*[_ptr(t) for t in pieces])
    _check(lib.hap_allgather_assemble(C.byref(desc.c), pp, (C.c_int64 * m)(*map(int, ld_pieces)), _ptr(out), C.c_int64(ld_out),
                                      _stream(stream)), "hap_allgather_assemble")


def hap_reducescatter_split(desc: GatherDesc, full, ld_full, slots, ld_slots, stream=None):
    m = desc.m
    pp = (C.c_void_p * m)(*[_ptr(t) for t in slots])
    _check(lib.hap_reducescatter_split(C.byref(desc.c), _ptr(full), C.c_int64(ld_full), pp, (C.c_int64 * m)(*map(int, ld_slots)),
                                       _stream(stream)), "hap_reducescatter_split")


def hap_attn_bwd_workspace(desc: AttnDesc, shard_index: int) -> int:
    return int(lib.hap_attn_bwd_workspace(C.byref(desc.c), C.c_int(shard_index)))


def hap_sharded_attn_fwd(desc: AttnDesc, shard_index, Q, K, V, O, lse, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib.hap_sharded_attn_fwd(C.byref(desc.c), C.c_int(shard_index), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(lse),
                                    wp, wb, _stream(stream)), "hap_sharded_attn_fwd")


def hap_sharded_attn_bwd(desc: AttnDesc, shard_index, Q, K, V, O, lse, dO, dQ, dK, dV, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib.hap_sharded_attn_bwd(C.byref(desc.c), C.c_int(shard_index), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(lse),
                                    _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV), wp, wb, _stream(stream)), "hap_sharded_attn_bwd")


def hap_layernorm_fwd(rows, n, io_dtype, x, gamma, beta, y, mean, rstd, stream=None):
    _check(lib.hap_layernorm_fwd(C.c_int64(rows), C.c_int64(n), C.c_int(io_dtype), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(y),
                                 _ptr(mean), _ptr(rstd), _stream(stream)), "hap_layernorm_fwd")


def hap_layernorm_bwd_workspace(rows, n) -> int:
    return int(lib.hap_layernorm_bwd_workspace(C.c_int64(rows), C.c_int64(n)))


def hap_layernorm_bwd(rows, n, io_dtype, x, gamma, mean, rstd, dy, dx, dgamma, dbeta, ws, stream=None, dresidual=None):
    wp, wb = _ws(ws)
    _check(lib.hap_layernorm_bwd(C.c_int64(rows), C.c_int64(n), C.c_int(io_dtype), _ptr(x), _ptr(gamma), _ptr(mean), _ptr(rstd),
                                 _ptr(dy), _ptr(dresidual), _ptr(dx), _ptr(dgamma), _ptr(dbeta), wp, wb, _stream(stream)), "hap_layernorm_bwd")


def hap_gelu_bwd(rows, cols, io_dtype, preact, ldp, dy, lddy, out, ldo, stream=None):
    _check(lib.hap_gelu_bwd(C.c_int64(rows), C.c_int64(cols), C.c_int(io_dtype), _ptr(preact), C.c_int64(ldp), _ptr(dy),
                            C.c_int64(lddy), _ptr(out), C.c_int64(ldo), _stream(stream)), "hap_gelu_bwd")


def hap_add(rows, cols, io_dtype, a, lda, b, ldb, bias, out, ldo, stream=None):
    _check(lib.hap_add(C.c_int64(rows), C.c_int64(cols), C.c_int(io_dtype), _ptr(a), C.c_int64(lda), _ptr(b), C.c_int64(ldb),
                       _ptr(bias), _ptr(out), C.c_int64(ldo), _stream(stream)), "hap_add")


def hap_colsum_workspace(rows, cols) -> int:
    return int(lib.hap_colsum_workspace(C.c_int64(rows), C.c_int64(cols)))


def hap_colsum(rows, cols, io_dtype, a, lda, out, ws, stream=None):
    wp, wb = _ws(ws)
    _check(lib.hap_colsum(C.c_int64(rows), C.c_int64(cols), C.c_int(io_dtype), _ptr(a), C.c_int64(lda), _ptr(out), wp, wb,
                          _stream(stream)), "hap_colsum")


def hap_debug_set_gemm_view_limit(nbytes: int) -> int:
    """Testing aid: operand-view size from which the GEMM engine cuts a product into pieces (0 restores the default).
    Returns the number of products run in pieces so far."""
    return int(lib.hap_debug_set_gemm_view_limit(C.c_int64(int(nbytes))))


def hap_device_info():
    """(compute units, peak engine clock in kHz) of the current device."""
    cu, khz = C.c_int(0), C.c_int(0)
    _check(lib.hap_device_info(C.byref(cu), C.byref(khz)), "hap_device_info")
    return cu.value, khz.value


def hap_probe_mfma_bf16(random_operands: bool, iters: int, scratch, stream=None) -> float:
    """Launches the MFMA issue-rate probe; returns the flops of the launch (the caller times it)."""
    fl = C.c_double()
    _check(lib.hap_probe_mfma_bf16(C.c_int(int(bool(random_operands))), C.c_int(iters), _ptr(scratch), C.byref(fl), _stream(stream)),
           "hap_probe_mfma_bf16")
    return fl.value
