"""ctypes binding of librelayhip.so: the same entry points as include/relayhip.h,
argument marshalling only.  PyTorch appears here solely as the owner of device
memory and streams (tensor.data_ptr(), current stream handle)."""
from __future__ import annotations

import ctypes
import json
import os
from ctypes import POINTER, byref, c_char_p, c_double, c_int32, c_int64, c_size_t, c_void_p
from typing import Dict, List, Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librelayhip.so")

RL_F32, RL_BF16 = 0, 1
STATIC_WORKSPACE_BYTES = 16 << 20
RL_MAX_RANK = 6
DTYPES = {"f32": RL_F32, "bf16": RL_BF16}
DTYPE_BYTES = {"f32": 4, "bf16": 2}

OPS = {"dense": 0, "conv2d": 1, "bias_add": 2, "add": 3, "sub": 4, "mul": 5, "div": 6, "neg": 7, "sq": 8, "relu": 9,
       "sigmoid": 10, "tanh": 11, "maxpool2d": 12, "global_avgpool": 13, "flatten": 14, "lstm_gates": 15, "cast": 16,
       "concat": 17, "layout_transform": 18, "dense_grad_x": 19, "dense_grad_w": 20, "conv2d_grad_x": 21, "conv2d_grad_w": 22}

STATUS = {0: "ok", -1: "null", -2: "kind", -3: "shape", -4: "type", -5: "group", -6: "binding", -7: "workspace",
          -8: "align", -9: "unsupported", -10: "hip"}


class rl_type(ctypes.Structure):
    _fields_ = [("dtype", c_int32), ("rank", c_int32), ("dims", c_int64 * RL_MAX_RANK)]


class rl_attr_contract(ctypes.Structure):
    _fields_ = [("out_dtype", c_int32)]


class rl_attr_conv2d(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("stride_h", "stride_w", "pad_h", "pad_w", "dilation_h", "dilation_w", "groups", "out_dtype")]


class rl_attr_axis(ctypes.Structure):
    _fields_ = [("axis", c_int32)]


class rl_attr_pool2d(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("kernel_h", "kernel_w", "stride_h", "stride_w", "pad_h", "pad_w")]


class rl_attr_cast(ctypes.Structure):
    _fields_ = [("to", c_int32)]


class rl_attr_layout(ctypes.Structure):
    _fields_ = [("perm", c_int32 * RL_MAX_RANK)]


class rl_binding(ctypes.Structure):
    _fields_ = [("value_id", c_int32), ("dev_ptr", c_void_p)]


class rl_recurrent(ctypes.Structure):
    _fields_ = [("x_id", c_int32), ("h_in_id", c_int32), ("c_in_id", c_int32), ("h_out_id", c_int32), ("c_out_id", c_int32),
                ("x_seq_dev", c_void_p), ("x_step_bytes", c_size_t), ("h0_dev", c_void_p), ("c_dev", c_void_p),
                ("h_seq_dev", c_void_p), ("h_step_bytes", c_size_t)]


PLAN_OPT_FIELDS = ("no_lp", "no_lp_256", "no_ws", "ws_all", "no_stem", "no_stem_pool", "no_dma", "no_c64", "no_run", "no_run_ks",
                   "no_pair", "s2_pair", "no_splitk", "no_hoist", "no_stem_direct", "no_wgrad", "no_grad_fwd", "no_out_transpose", "no_dense_chain")


class rl_plan_opts(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32)] + [(n, c_int32) for n in PLAN_OPT_FIELDS]


def make_opts(opts: Optional[Dict[str, int]]):
    """{field: value} -> rl_plan_opts (None stays None: the planner's own choices)."""
    if opts is None:
        return None
    o = rl_plan_opts()
    o.struct_size = ctypes.sizeof(rl_plan_opts)
    for k, v in opts.items():
        if k not in PLAN_OPT_FIELDS:
            raise KeyError(f"unknown plan option {k!r}")
        setattr(o, k, int(v))
    return o


class RelayError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"relayhip error {status} ({STATUS.get(status, '?')}): {text}")
        self.status = status
        self.category = STATUS.get(status, "?")


_lib = None

# every symbol include/relayhip.h declares
SYMBOLS = ["rl_ctx_create", "rl_ctx_destroy", "rl_last_error", "rl_graph_create", "rl_graph_destroy", "rl_graph_input",
           "rl_graph_param", "rl_graph_op", "rl_graph_group", "rl_graph_output", "rl_graph_autogroup", "rl_graph_group_of", "rl_plan_create", "rl_plan_destroy",
           "rl_plan_describe", "rl_plan_workspace_bytes", "rl_plan_packed_bytes", "rl_plan_prepack", "rl_plan_run",
           "rl_plan_run_static", "rl_plan_run_recurrent", "rl_plan_recurrent_workspace_bytes", "rl_prep_fold_batchnorm", "rl_plan_profile", "rl_calibrate_mfma_bf16"]


def lib():
    """Load the HIP library; there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(or paper_1810_00952_amd/build.py)")
        # One HIP runtime per process.  PyTorch (which the callers use for device memory) ships its own copy of
        # libamdhip64 under the same SONAME and opens it by path; if this library pulled in the system copy first,
        # the process would hold two runtimes and the second one to initialise finds no device.  With torch loaded
        # first the dynamic linker resolves this library's dependency to the copy that is already there.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        L.rl_ctx_create.argtypes = [POINTER(c_void_p)]
        L.rl_ctx_destroy.argtypes = [c_void_p]; L.rl_ctx_destroy.restype = None
        L.rl_last_error.argtypes = [c_void_p]; L.rl_last_error.restype = c_char_p
        L.rl_graph_create.argtypes = [c_void_p, POINTER(c_void_p)]
        L.rl_graph_destroy.argtypes = [c_void_p]; L.rl_graph_destroy.restype = None
        L.rl_graph_input.argtypes = [c_void_p, POINTER(rl_type), POINTER(c_int32)]
        L.rl_graph_param.argtypes = [c_void_p, POINTER(rl_type), POINTER(c_int32)]
        L.rl_graph_op.argtypes = [c_void_p, c_int32, POINTER(c_int32), c_int32, c_void_p, c_size_t, POINTER(rl_type), c_int32,
                                  POINTER(c_int32), POINTER(c_int32)]
        L.rl_graph_group.argtypes = [c_void_p, POINTER(c_int32), c_int32, POINTER(c_int32)]
        L.rl_graph_output.argtypes = [c_void_p, c_int32]
        L.rl_graph_autogroup.argtypes = [c_void_p, POINTER(c_int32)]
        L.rl_graph_group_of.argtypes = [c_void_p, c_int32, POINTER(c_int32)]
        L.rl_plan_create.argtypes = [c_void_p, POINTER(rl_plan_opts), POINTER(c_void_p)]
        L.rl_plan_destroy.argtypes = [c_void_p]; L.rl_plan_destroy.restype = None
        L.rl_plan_describe.argtypes = [c_void_p, c_char_p, c_size_t, POINTER(c_size_t)]
        L.rl_plan_workspace_bytes.argtypes = [c_void_p, POINTER(c_size_t)]
        L.rl_plan_recurrent_workspace_bytes.argtypes = [c_void_p, c_int32, POINTER(c_size_t)]
        L.rl_plan_packed_bytes.argtypes = [c_void_p, c_int32, POINTER(c_size_t)]
        L.rl_plan_prepack.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_void_p]
        L.rl_plan_run.argtypes = [c_void_p, POINTER(rl_binding), c_int32, c_void_p, c_size_t, c_void_p]
        L.rl_plan_run_static.argtypes = [c_void_p, POINTER(rl_binding), c_int32, c_void_p]
        L.rl_plan_profile.argtypes = [c_void_p, POINTER(rl_binding), c_int32, c_void_p, c_size_t, c_void_p, c_int32,
                                      POINTER(ctypes.c_float), c_int32, POINTER(c_int32)]
        L.rl_plan_run_recurrent.argtypes = [c_void_p, c_int32, POINTER(rl_recurrent), POINTER(rl_binding), c_int32, c_void_p,
                                            c_size_t, c_void_p]
        L.rl_prep_fold_batchnorm.argtypes = [c_void_p] + [c_void_p] * 5 + [c_double, c_void_p, c_int32, c_void_p, c_int64, c_int64, c_void_p]
        L.rl_calibrate_mfma_bf16.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_void_p]
        for s in SYMBOLS:
            if getattr(L, s).restype is not None and s != "rl_last_error":
                getattr(L, s).restype = c_int32
        _lib = L
    return _lib


def make_type(dtype, shape: Sequence[int]) -> rl_type:
    t = rl_type()
    t.dtype = DTYPES.get(dtype, -1) if isinstance(dtype, str) else int(dtype)
    t.rank = len(shape)
    for i, d in enumerate(shape[:RL_MAX_RANK]):
        t.dims[i] = int(d)
    return t


class Context:
    def __init__(self):
        self._h = c_void_p()
        st = lib().rl_ctx_create(byref(self._h))
        if st != 0:
            raise RelayError(st, "rl_ctx_create failed")

    def last_error(self) -> str:
        return lib().rl_last_error(self._h).decode()

    def check(self, st: int):
        if st != 0:
            raise RelayError(st, self.last_error())

    def fold_batchnorm(self, w, gamma, beta, mean, var, eps, w_out, out_dtype: str, b_out, O: int, per_o: int, stream=None):
        """rl_prep_fold_batchnorm on device pointers (ints)."""
        self.check(lib().rl_prep_fold_batchnorm(self._h, w, gamma, beta, mean, var, c_double(eps), w_out, DTYPES[out_dtype], b_out,
                                                c_int64(O), c_int64(per_o), c_void_p(stream or 0)))

    def calibrate_mfma_bf16(self, scratch_ptr: int, workgroups: int, iters: int, stream=None) -> float:
        """rl_calibrate_mfma_bf16; returns the flops the enqueued kernel performs."""
        self.check(lib().rl_calibrate_mfma_bf16(self._h, c_void_p(scratch_ptr), workgroups, iters, c_void_p(stream or 0)))
        return float(workgroups) * 8 * 16 * iters * 32768.0

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.rl_ctx_destroy(self._h)
            self._h = None


def _attrs_for(kind: str, attrs: Dict):
    od = attrs.get("out_dtype")
    if kind in ("dense", "dense_grad_x", "dense_grad_w"):
        return rl_attr_contract(DTYPES[od]) if od is not None else None
    if kind in ("conv2d", "conv2d_grad_x", "conv2d_grad_w"):
        s, p = attrs.get("stride", (1, 1)), attrs.get("pad", (0, 0))
        d = attrs.get("dilation", (1, 1))
        return rl_attr_conv2d(s[0], s[1], p[0], p[1], d[0], d[1], attrs.get("groups", 1), DTYPES[od] if od is not None else -1)
    if kind in ("bias_add", "concat"):
        return rl_attr_axis(attrs.get("axis", 1))
    if kind == "maxpool2d":
        k, s, p = attrs["kernel"], attrs.get("stride", (1, 1)), attrs.get("pad", (0, 0))
        return rl_attr_pool2d(k[0], k[1], s[0], s[1], p[0], p[1])
    if kind == "cast":
        return rl_attr_cast(DTYPES.get(attrs.get("to"), -1))
    if kind == "layout_transform":
        perm = [int(v) for v in attrs.get("perm", ())]
        if len(perm) > RL_MAX_RANK:
            perm = perm[:RL_MAX_RANK - 1] + [-1]        # cannot be marshalled: let the library reject it
        return rl_attr_layout((c_int32 * RL_MAX_RANK)(*(perm + [-1] * (RL_MAX_RANK - len(perm)))))
    return None


class Graph:
    def __init__(self, ctx: Context):
        self.ctx = ctx
        self._h = c_void_p()
        ctx.check(lib().rl_graph_create(ctx._h, byref(self._h)))

    def input(self, dtype, shape) -> int:
        vid = c_int32()
        self.ctx.check(lib().rl_graph_input(self._h, byref(make_type(dtype, shape)), byref(vid)))
        return vid.value

    def param(self, dtype, shape) -> int:
        vid = c_int32()
        self.ctx.check(lib().rl_graph_param(self._h, byref(make_type(dtype, shape)), byref(vid)))
        return vid.value

    def op(self, kind, inputs: Sequence[int], out_types: Sequence[Tuple[str, Sequence[int]]], **attrs) -> Tuple[int, List[int]]:
        code = OPS.get(kind, -1) if isinstance(kind, str) else int(kind)
        ins = (c_int32 * max(1, len(inputs)))(*inputs)
        outs_t = (rl_type * len(out_types))(*[make_type(dt, sh) for dt, sh in out_types])
        a = _attrs_for(kind, attrs) if isinstance(kind, str) else None
        op_id = c_int32()
        out_ids = (c_int32 * len(out_types))()
        self.ctx.check(lib().rl_graph_op(self._h, code, ins, len(inputs), byref(a) if a is not None else None,
                                         ctypes.sizeof(a) if a is not None else 0, outs_t, len(out_types), byref(op_id), out_ids))
        return op_id.value, list(out_ids)

    def group(self, op_ids: Sequence[int]) -> int:
        gid = c_int32()
        arr = (c_int32 * max(1, len(op_ids)))(*op_ids)
        self.ctx.check(lib().rl_graph_group(self._h, arr, len(op_ids), byref(gid)))
        return gid.value

    def output(self, vid: int) -> None:
        self.ctx.check(lib().rl_graph_output(self._h, vid))

    def autogroup(self) -> int:
        n = c_int32()
        self.ctx.check(lib().rl_graph_autogroup(self._h, byref(n)))
        return n.value

    def group_of(self, op_id: int) -> int:
        gid = c_int32()
        self.ctx.check(lib().rl_graph_group_of(self._h, op_id, byref(gid)))
        return gid.value

    def groups(self, n_ops: int) -> List[List[int]]:
        """Members of every group, in group order (ops without a group are left out)."""
        by = {}
        for o in range(n_ops):
            gi = self.group_of(o)
            if gi >= 0:
                by.setdefault(gi, []).append(o)
        return [by[k] for k in sorted(by)]

    def plan(self, opts: Optional[Dict[str, int]] = None) -> "Plan":
        return Plan(self, opts)

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.rl_graph_destroy(self._h)
            self._h = None


def graph_from_spec(ctx: Context, spec, auto_groups: bool = False) -> Graph:
    """Replay a plain-data graph description (values, calls with declared result
    types, groups, outputs) through the C ABI, call by call.  Value and op ids
    of the description and of the library coincide because both are append-only.
    auto_groups: ignore the description's groups and let rl_graph_autogroup form them."""
    g = Graph(ctx)
    first_out = {op.outputs[0]: oi for oi, op in enumerate(spec.ops)}
    for vid, v in enumerate(spec.values):
        if v.role == "input":
            got = g.input(v.type.dtype, v.type.shape)
        elif v.role == "param":
            got = g.param(v.type.dtype, v.type.shape)
        elif vid in first_out:
            oi = first_out[vid]
            op = spec.ops[oi]
            o_id, outs = g.op(op.kind, op.inputs, [(spec.values[o].type.dtype, spec.values[o].type.shape) for o in op.outputs],
                              **op.attrs)
            if o_id != oi or outs != list(op.outputs):
                raise AssertionError("id drift between description and library")
            continue
        else:
            continue            # second result of a two-result call, already declared
        if got != vid:
            raise AssertionError("id drift between description and library")
    if auto_groups:
        for o in spec.outputs:
            g.output(o)
        g.autogroup()
        return g
    for grp in spec.groups:
        g.group(grp)
    for o in spec.outputs:
        g.output(o)
    return g


class Plan:
    def __init__(self, graph: Graph, opts: Optional[Dict[str, int]] = None):
        self.ctx = graph.ctx
        self._h = c_void_p()
        o = make_opts(opts)
        self.ctx.check(lib().rl_plan_create(graph._h, byref(o) if o is not None else None, byref(self._h)))

    def describe(self) -> dict:
        need = c_size_t()
        self.ctx.check(lib().rl_plan_describe(self._h, None, 0, byref(need)))
        buf = ctypes.create_string_buffer(need.value)
        self.ctx.check(lib().rl_plan_describe(self._h, buf, need.value, byref(need)))
        return json.loads(buf.value.decode())

    def recurrent_workspace_bytes(self, steps: int) -> int:
        n = c_size_t(0)
        self.ctx.check(lib().rl_plan_recurrent_workspace_bytes(self._h, steps, byref(n)))
        return n.value

    def workspace_bytes(self) -> int:
        n = c_size_t()
        self.ctx.check(lib().rl_plan_workspace_bytes(self._h, byref(n)))
        return n.value

    def packed_bytes(self, vid: int) -> int:
        n = c_size_t()
        self.ctx.check(lib().rl_plan_packed_bytes(self._h, vid, byref(n)))
        return n.value

    def prepack(self, vid: int, src_ptr: int, dst_ptr: int, stream: int = 0) -> None:
        self.ctx.check(lib().rl_plan_prepack(self._h, vid, c_void_p(src_ptr), c_void_p(dst_ptr), c_void_p(stream)))

    @staticmethod
    def _bindings(b: Dict[int, int]):
        arr = (rl_binding * max(1, len(b)))()
        for i, (vid, ptr) in enumerate(b.items()):
            arr[i].value_id = vid
            arr[i].dev_ptr = ptr
        return arr

    def run(self, bindings: Dict[int, int], workspace_ptr: int = 0, workspace_bytes: int = 0, stream: int = 0) -> None:
        self.ctx.check(lib().rl_plan_run(self._h, self._bindings(bindings), len(bindings), c_void_p(workspace_ptr),
                                         c_size_t(workspace_bytes), c_void_p(stream)))

    def run_static(self, bindings: Dict[int, int], stream: int = 0) -> None:
        """rl_plan_run_static: the library's built-in workspace (STATIC_WORKSPACE_BYTES at most), no device allocation."""
        self.ctx.check(lib().rl_plan_run_static(self._h, self._bindings(bindings), len(bindings), c_void_p(stream)))

    def profile(self, bindings: Dict[int, int], workspace_ptr: int, workspace_bytes: int, stream: int, reps: int) -> List[float]:
        """Mean milliseconds per plan step over `reps` runs (synchronises)."""
        n = c_int32()
        cap = 4096
        buf = (ctypes.c_float * cap)()
        self.ctx.check(lib().rl_plan_profile(self._h, self._bindings(bindings), len(bindings), c_void_p(workspace_ptr),
                                             c_size_t(workspace_bytes), c_void_p(stream), reps, buf, cap, byref(n)))
        return list(buf[:n.value])

    def run_recurrent(self, steps: int, roles: Dict[str, int], x_seq: int, x_step_bytes: int, h0: int, c: int, h_seq: int,
                      h_step_bytes: int, param_bindings: Dict[int, int], workspace_ptr: int = 0, workspace_bytes: int = 0,
                      stream: int = 0) -> None:
        io = rl_recurrent(roles["x"], roles["h_in"], roles["c_in"], roles["h_out"], roles["c_out"], x_seq, x_step_bytes, h0, c,
                          h_seq, h_step_bytes)
        self.ctx.check(lib().rl_plan_run_recurrent(self._h, steps, byref(io), self._bindings(param_bindings), len(param_bindings),
                                                   c_void_p(workspace_ptr), c_size_t(workspace_bytes), c_void_p(stream)))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.rl_plan_destroy(self._h)
            self._h = None
