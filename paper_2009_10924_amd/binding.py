"""ctypes binding of libfusion_stitching.so: argument marshalling only.

Names follow include/fusion_stitching.h.  Every step of the hot path runs inside
the library's HIP kernels; PyTorch appears only as the owner of device memory and
of the stream handle.  There is no CPU fallback: if the library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

FS_MAX_RANK = 4
DTYPE = {"f32": 0, "f16": 1, "bf16": 2, "i32": 3}
DTYPE_NAME = {v: k for k, v in DTYPE.items()}
OPCODE = {
    "add": 0, "sub": 1, "mul": 2, "div": 3, "max": 4, "scale": 5, "add_scalar": 6, "square": 7,
    "exp": 8, "rsqrt": 9, "tanh": 10, "gelu_tanh": 11, "gelu_tanh_grad": 12, "broadcast": 13,
    "log": 19, "sigmoid": 20, "relu": 21, "abs": 22, "sqrt": 23,
    "reduce_sum": 14, "reduce_max": 15, "reduce_mean": 16, "transpose": 17, "convert": 18,
}
SCHEME = {"auto": 0, "unfused": 1, "local": 2, "wave": 3, "lds": 4, "global": 5}
SCHEME_NAME = {v: k for k, v in SCHEME.items()}
ERROR_NAME = {0: "FS_OK", -1: "FS_ERR_INVALID_ARG", -2: "FS_ERR_SHAPE", -3: "FS_ERR_DTYPE", -4: "FS_ERR_CYCLE",
              -5: "FS_ERR_UNSUPPORTED_PATTERN", -6: "FS_ERR_LOCALITY", -7: "FS_ERR_WORKSPACE",
              -8: "FS_ERR_ALIGN", -9: "FS_ERR_HIP", -10: "FS_ERR_HOST"}

EXPORTS = [
    "fs_graph_create", "fs_graph_destroy", "fs_graph_input", "fs_graph_op", "fs_graph_output",
    "fs_graph_finalize", "fs_plan_create", "fs_plan_destroy", "fs_plan_query", "fs_plan_candidate", "fs_plan_describe",
    "fs_plan_source", "fs_codegen_enable", "fs_codegen_available", "fs_execute", "fs_execute_static", "fs_stream_copy", "fs_stream_probe", "fs_last_error", "fs_version",
    "fs_pack_create", "fs_pack_destroy", "fs_pack_query", "fs_pack_execute",
    "fs_explore", "fs_explore_score", "fs_program_destroy", "fs_program_query", "fs_program_pattern", "fs_program_execute",
    "fs_program_describe", "fs_program_execute_stage", "fs_graph_external",
]
FS_PACK_MAX_MEMBERS = 256
FS_STATIC_SCRATCH_BYTES = 4 << 20


class FsError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{ERROR_NAME.get(code, code)}: {text}")
        self.code = code
        self.text = text


class fs_attr_scalar(C.Structure):
    _fields_ = [("value", C.c_double)]


class fs_attr_axis(C.Structure):
    _fields_ = [("axis", C.c_int32)]


class fs_attr_perm(C.Structure):
    _fields_ = [("perm", C.c_int32 * FS_MAX_RANK)]


class fs_attr_dims(C.Structure):
    _fields_ = [("rank", C.c_int32), ("dims", C.c_int64 * FS_MAX_RANK)]


class fs_attr_dtype(C.Structure):
    _fields_ = [("dtype", C.c_int32)]


class fs_plan_opts(C.Structure):
    _fields_ = [("candidate", C.c_int32), ("block_threads", C.c_int32),
                ("lanes_per_row", C.c_int32), ("vecs_per_lane", C.c_int32)]


class fs_plan_info(C.Structure):
    _fields_ = [
        ("scheme", C.c_int32), ("n_kernels", C.c_int32), ("block", C.c_int32 * 3), ("grid", C.c_int32 * 3),
        ("lanes_per_row", C.c_int32), ("vecs_per_lane", C.c_int32), ("rows_per_block", C.c_int32),
        ("lds_bytes", C.c_int32), ("vgprs", C.c_int32), ("waves_per_simd", C.c_int32),
        ("n_candidates", C.c_int32), ("candidate", C.c_int32),
        ("workspace_bytes", C.c_int64), ("bytes_min", C.c_int64), ("bytes_moved_model", C.c_int64),
        ("predicted_us", C.c_double), ("pattern", C.c_char * 32), ("kernel", C.c_char * 64),
    ]

    def as_dict(self) -> Dict:
        return {
            "scheme": SCHEME_NAME.get(self.scheme, self.scheme), "n_kernels": self.n_kernels,
            "block": list(self.block), "grid": list(self.grid), "lanes_per_row": self.lanes_per_row,
            "vecs_per_lane": self.vecs_per_lane, "rows_per_block": self.rows_per_block,
            "lds_bytes": self.lds_bytes, "vgprs": self.vgprs, "waves_per_simd": self.waves_per_simd,
            "n_candidates": self.n_candidates, "candidate": self.candidate,
            "workspace_bytes": self.workspace_bytes, "bytes_min": self.bytes_min,
            "bytes_moved_model": self.bytes_moved_model, "predicted_us": self.predicted_us,
            "pattern": self.pattern.decode(), "kernel": self.kernel.decode(),
        }


class fs_pack_info(C.Structure):
    _fields_ = [
        ("n_members", C.c_int32), ("n_kernels", C.c_int32), ("grid", C.c_int32), ("block", C.c_int32),
        ("vgprs", C.c_int32), ("n_inputs", C.c_int32), ("n_outputs", C.c_int32), ("generated", C.c_int32),
        ("bytes_min", C.c_int64), ("predicted_us", C.c_double), ("predicted_separate_us", C.c_double),
    ]

    def as_dict(self) -> Dict:
        return {k: getattr(self, k) for k, _ in self._fields_ if k != "reserved"}


class fs_explore_opts(C.Structure):
    _fields_ = [("top_k", C.c_int32), ("beam_width", C.c_int32), ("no_packing", C.c_int32), ("no_remote_fusion", C.c_int32),
                ("no_joint_folds", C.c_int32)]


class fs_program_info(C.Structure):
    _fields_ = [
        ("n_ops", C.c_int32), ("n_patterns", C.c_int32), ("n_single_ops", C.c_int32), ("n_steps", C.c_int32),
        ("n_kernels", C.c_int32), ("n_packs", C.c_int32), ("beam_plans", C.c_int32), ("n_joint_folds", C.c_int32),
        ("workspace_bytes", C.c_int64), ("bytes_min", C.c_int64), ("bytes_moved_model", C.c_int64),
        ("f_total_us", C.c_double), ("predicted_us", C.c_double), ("predicted_unfused_us", C.c_double),
        ("n_stages", C.c_int32), ("reserved", C.c_int32),
    ]

    def as_dict(self) -> Dict:
        return {k: getattr(self, k) for k, _ in self._fields_ if k != "reserved"}


_LIB: Optional[C.CDLL] = None


def lib_path() -> str:
    """In-tree library; FUSION_STITCHING_LIB overrides it (e.g. a sanitizer build of the host code)."""
    return os.environ.get("FUSION_STITCHING_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libfusion_stitching.so")


def load() -> C.CDLL:
    """Loads the in-tree library; raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python -m paper_2009_10924_amd.build` (there is no fallback path)")
    # PyTorch ships its own HIP runtime (same soname).  A process must hold exactly one
    # runtime, so torch's is loaded first and the library binds to it.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(path)
    vp, i32, i64p = C.c_void_p, C.c_int32, C.POINTER(C.c_int64)
    lib.fs_graph_create.argtypes = [C.POINTER(vp)]
    lib.fs_graph_create.restype = i32
    lib.fs_graph_destroy.argtypes = [vp]
    lib.fs_graph_destroy.restype = None
    lib.fs_graph_input.argtypes = [vp, i32, i32, i64p]
    lib.fs_graph_input.restype = i32
    lib.fs_graph_op.argtypes = [vp, i32, i32, C.POINTER(i32), vp, C.c_size_t]
    lib.fs_graph_op.restype = i32
    lib.fs_graph_output.argtypes = [vp, i32, i32]
    lib.fs_graph_output.restype = i32
    lib.fs_graph_finalize.argtypes = [vp]
    lib.fs_graph_finalize.restype = i32
    lib.fs_plan_create.argtypes = [vp, i32, C.POINTER(fs_plan_opts), C.POINTER(vp)]
    lib.fs_plan_create.restype = i32
    lib.fs_plan_destroy.argtypes = [vp]
    lib.fs_plan_destroy.restype = None
    lib.fs_plan_query.argtypes = [vp, C.POINTER(fs_plan_info)]
    lib.fs_plan_query.restype = i32
    lib.fs_plan_candidate.argtypes = [vp, i32, C.POINTER(fs_plan_info)]
    lib.fs_plan_candidate.restype = i32
    lib.fs_plan_describe.argtypes = [vp, C.c_char_p, C.c_size_t]
    lib.fs_plan_describe.restype = C.c_int64
    lib.fs_program_describe.argtypes = [vp, C.c_char_p, C.c_size_t]
    lib.fs_program_describe.restype = C.c_int64
    lib.fs_plan_source.argtypes = [vp, C.c_char_p, C.c_size_t]
    lib.fs_plan_source.restype = C.c_int64
    lib.fs_codegen_enable.argtypes = [C.c_int32]
    lib.fs_codegen_enable.restype = C.c_int32
    lib.fs_codegen_available.argtypes = []
    lib.fs_codegen_available.restype = C.c_int32
    lib.fs_execute.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp, C.c_size_t, vp]
    lib.fs_execute.restype = i32
    lib.fs_execute_static.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp]
    lib.fs_execute_static.restype = i32
    lib.fs_stream_copy.argtypes = [vp, vp, C.c_size_t, vp]
    lib.fs_stream_copy.restype = i32
    lib.fs_stream_probe.argtypes = [vp, vp, C.c_size_t, C.c_size_t, i32, i32, i32, vp]
    lib.fs_stream_probe.restype = i32
    lib.fs_explore.argtypes = [vp, C.POINTER(fs_explore_opts), C.POINTER(vp)]
    lib.fs_explore.restype = i32
    lib.fs_explore_score.argtypes = [vp, C.POINTER(i32), i32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.fs_explore_score.restype = i32
    lib.fs_program_destroy.argtypes = [vp]
    lib.fs_program_destroy.restype = None
    lib.fs_program_query.argtypes = [vp, C.POINTER(fs_program_info)]
    lib.fs_program_query.restype = i32
    lib.fs_program_pattern.argtypes = [vp, i32, C.POINTER(i32), i32, C.POINTER(i32), C.POINTER(C.c_double), C.POINTER(i32),
                                       C.POINTER(fs_plan_info)]
    lib.fs_program_pattern.restype = i32
    lib.fs_program_execute.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp, C.c_size_t, vp]
    lib.fs_program_execute.restype = i32
    lib.fs_program_execute_stage.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), vp, C.c_size_t, vp]
    lib.fs_program_execute_stage.restype = i32
    lib.fs_graph_external.argtypes = [vp, i32, i32]
    lib.fs_graph_external.restype = i32
    lib.fs_pack_create.argtypes = [C.POINTER(vp), i32, C.POINTER(vp)]
    lib.fs_pack_create.restype = i32
    lib.fs_pack_destroy.argtypes = [vp]
    lib.fs_pack_destroy.restype = None
    lib.fs_pack_query.argtypes = [vp, C.POINTER(fs_pack_info)]
    lib.fs_pack_query.restype = i32
    lib.fs_pack_execute.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp]
    lib.fs_pack_execute.restype = i32
    lib.fs_last_error.argtypes = []
    lib.fs_last_error.restype = C.c_char_p
    lib.fs_version.argtypes = []
    lib.fs_version.restype = C.c_char_p
    _LIB = lib
    return lib


def _check(code: int) -> int:
    if code < 0:
        raise FsError(code, load().fs_last_error().decode())
    return code


class Graph:
    """fs_graph handle.  Tensors are addressed by the ids the library returns."""

    def __init__(self):
        self._lib = load()
        h = C.c_void_p()
        _check(self._lib.fs_graph_create(C.byref(h)))
        self.handle = h
        self.names: Dict[str, int] = {}

    def __del__(self):
        if getattr(self, "handle", None):
            self._lib.fs_graph_destroy(self.handle)
            self.handle = None

    def input(self, dtype: str, dims: Sequence[int]) -> int:
        arr = (C.c_int64 * max(1, len(dims)))(*dims)
        return _check(self._lib.fs_graph_input(self.handle, DTYPE[dtype], len(dims), arr))

    def op(self, opcode: str, inputs: Sequence[int], **attr) -> int:
        ins = (C.c_int32 * max(1, len(inputs)))(*inputs)
        a = None
        if opcode in ("scale", "add_scalar"):
            a = fs_attr_scalar(float(attr["value"]))
        elif opcode in ("reduce_sum", "reduce_max", "reduce_mean"):
            a = fs_attr_axis(int(attr["axis"]))
        elif opcode == "transpose":
            perm = list(attr["perm"]) + [0] * (FS_MAX_RANK - len(attr["perm"]))
            a = fs_attr_perm((C.c_int32 * FS_MAX_RANK)(*perm))
        elif opcode == "broadcast":
            dims = list(attr["dims"])
            a = fs_attr_dims(len(dims), (C.c_int64 * FS_MAX_RANK)(*(dims + [1] * (FS_MAX_RANK - len(dims)))))
        elif opcode == "convert":
            a = fs_attr_dtype(DTYPE[attr["dtype"]])
        if a is None:
            return _check(self._lib.fs_graph_op(self.handle, OPCODE[opcode], len(inputs), ins, None, 0))
        return _check(self._lib.fs_graph_op(self.handle, OPCODE[opcode], len(inputs), ins,
                                            C.cast(C.byref(a), C.c_void_p), C.sizeof(a)))

    def output(self, tensor: int, store_as: str) -> None:
        _check(self._lib.fs_graph_output(self.handle, tensor, DTYPE[store_as]))

    def finalize(self) -> None:
        _check(self._lib.fs_graph_finalize(self.handle))

    @classmethod
    def from_spec(cls, spec) -> "Graph":
        """Replays a workload descriptor (inputs / ops / outputs by name) through the C ABI."""
        g = cls()
        for t in spec.inputs:
            g.names[t.name] = g.input(t.dtype, t.dims)
        external = list(getattr(spec, "external", ()))
        for op in spec.ops:
            g.names[op.out] = g.op(op.opcode, [g.names[n] for n in op.inputs], **op.attr)
            # a dependence through an external computation is declared as soon as its source exists (and before
            # anything reads the input it leads to)
            for src, dst in external:
                if src == op.out:
                    _check(g._lib.fs_graph_external(g.handle, g.names[src], g.names[dst]))
        for name, dtype in spec.outputs:
            g.output(g.names[name], dtype)
        g.finalize()
        return g


class Plan:
    def __init__(self, graph: Graph, scheme: str = "auto", candidate: int = -1, block_threads: int = 0,
                 lanes_per_row: int = 0, vecs_per_lane: int = 0):
        self._lib = load()
        self._graph = graph
        # `candidate` here is the 0-based index fs_plan_info reports (-1: choose); the C struct counts from 1 (0: choose)
        opts = fs_plan_opts(candidate + 1 if candidate >= 0 else 0, block_threads, lanes_per_row, vecs_per_lane)
        h = C.c_void_p()
        _check(self._lib.fs_plan_create(graph.handle, SCHEME[scheme], C.byref(opts), C.byref(h)))
        self.handle = h
        self.info = self.query()

    def __del__(self):
        if getattr(self, "handle", None):
            self._lib.fs_plan_destroy(self.handle)
            self.handle = None

    def query(self) -> Dict:
        info = fs_plan_info()
        _check(self._lib.fs_plan_query(self.handle, C.byref(info)))
        return info.as_dict()

    def describe(self) -> str:
        need = self._lib.fs_plan_describe(self.handle, None, 0)
        if need < 0:
            _check(int(need))
        buf = C.create_string_buffer(int(need))
        self._lib.fs_plan_describe(self.handle, buf, int(need))
        return buf.value.decode()

    def source(self) -> str:
        """HIP source of the plan's generated kernel ('' if it runs a compiled-in kernel)."""
        need = self._lib.fs_plan_source(self.handle, None, 0)
        if need < 0:
            _check(int(need))
        buf = C.create_string_buffer(int(need))
        self._lib.fs_plan_source(self.handle, buf, int(need))
        return buf.value.decode()

    def candidates(self) -> List[Dict]:
        out = []
        for i in range(self.info["n_candidates"]):
            info = fs_plan_info()
            _check(self._lib.fs_plan_candidate(self.handle, i, C.byref(info)))
            out.append(info.as_dict())
        return out

    def execute_ptrs(self, inputs: Sequence[int], outputs: Sequence[int], workspace: int, workspace_bytes: int,
                     stream: int) -> None:
        ins = (C.c_void_p * max(1, len(inputs)))(*inputs)
        outs = (C.c_void_p * max(1, len(outputs)))(*outputs)
        _check(self._lib.fs_execute(self.handle, ins, outs, C.c_void_p(workspace), workspace_bytes, C.c_void_p(stream)))

    def bind(self, inputs: Sequence[int], outputs: Sequence[int], workspace: int, workspace_bytes: int, stream: int):
        """Marshals the arguments once; the returned callable only crosses the C ABI (for tight launch loops)."""
        ins = (C.c_void_p * max(1, len(inputs)))(*inputs)
        outs = (C.c_void_p * max(1, len(outputs)))(*outputs)
        ws, nb, st = C.c_void_p(workspace), C.c_size_t(workspace_bytes), C.c_void_p(stream)
        fn, handle = self._lib.fs_execute, self.handle

        def call(_keep=(ins, outs)):
            code = fn(handle, ins, outs, ws, nb, st)
            if code < 0:
                _check(code)
        return call

    def execute(self, inputs, outputs, workspace=None, stream: Optional[int] = None) -> None:
        """inputs / outputs: torch device tensors in declaration order; workspace: a uint8 tensor (its contents on entry do not matter)."""
        import torch
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        ws_ptr = workspace.data_ptr() if workspace is not None else 0
        ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
        self.execute_ptrs([t.data_ptr() for t in inputs], [t.data_ptr() for t in outputs], ws_ptr, ws_bytes, stream)

    def make_workspace(self, device="cuda"):
        import torch
        n = int(self.info["workspace_bytes"])
        return torch.zeros(max(n, 16), dtype=torch.uint8, device=device) if n > 0 else None

    def execute_static_ptrs(self, inputs: Sequence[int], outputs: Sequence[int], stream: int) -> None:
        """fs_execute_static: the plan's scratch is the library's static device array, nothing is allocated."""
        ins = (C.c_void_p * max(1, len(inputs)))(*inputs)
        outs = (C.c_void_p * max(1, len(outputs)))(*outputs)
        _check(self._lib.fs_execute_static(self.handle, ins, outs, C.c_void_p(stream)))


class Pack:
    """Several independent plans executed as one packed launch per 32 members."""

    def __init__(self, plans: Sequence[Plan]):
        self._lib = load()
        arr = (C.c_void_p * max(1, len(plans)))(*[p.handle for p in plans])
        h = C.c_void_p()
        _check(self._lib.fs_pack_create(arr, len(plans), C.byref(h)))
        self.handle = h
        info = fs_pack_info()
        _check(self._lib.fs_pack_query(self.handle, C.byref(info)))
        self.info = info.as_dict()

    def __del__(self):
        if getattr(self, "handle", None):
            self._lib.fs_pack_destroy(self.handle)
            self.handle = None

    def bind(self, inputs: Sequence[int], outputs: Sequence[int], stream: int):
        """inputs / outputs: device addresses, member after member; returns a pre-marshalled call."""
        ins = (C.c_void_p * max(1, len(inputs)))(*inputs)
        outs = (C.c_void_p * max(1, len(outputs)))(*outputs)
        st = C.c_void_p(stream)
        fn, handle = self._lib.fs_pack_execute, self.handle

        def call(_keep=(ins, outs)):
            code = fn(handle, ins, outs, st)
            if code < 0:
                _check(code)
        return call

    def execute_ptrs(self, inputs: Sequence[int], outputs: Sequence[int], stream: int) -> None:
        self.bind(inputs, outputs, stream)()


def codegen_enable(on: bool) -> bool:
    """Process-wide switch for offering generated kernels; returns the previous setting."""
    return bool(load().fs_codegen_enable(1 if on else 0))


def codegen_available() -> bool:
    return bool(load().fs_codegen_available())


class codegen:
    """`with codegen(False): ...` plans, scores and explores without generated kernels inside the block."""

    def __init__(self, on: bool):
        self.on = on

    def __enter__(self):
        self.before = codegen_enable(self.on)
        return self

    def __exit__(self, *exc):
        codegen_enable(self.before)
        return False


def explore_score(graph: Graph, ops: Sequence[int]) -> float:
    """Delta-evaluator score (microseconds) of `ops` taken as one fusion pattern; raises FsError if they cannot be one."""
    return explore_score_ex(graph, ops)[0]


def explore_score_ex(graph: Graph, ops: Sequence[int]):
    """(f_us, f_optimistic_us, status): status 0 = runnable as one pattern; a negative fs_error otherwise, with f_us None.
    f_optimistic_us is set for every pattern without a cyclic dependence."""
    arr = (C.c_int32 * max(1, len(ops)))(*ops)
    f, fo = C.c_double(), C.c_double()
    code = load().fs_explore_score(graph.handle, arr, len(ops), C.byref(f), C.byref(fo))
    if code == -1:
        _check(code)
    return (f.value if code == 0 else None), fo.value, code


class Program:
    """Fusion plan found for a multi-pattern graph, and its execution."""

    def __init__(self, graph: Graph, top_k: int = 0, beam_width: int = 0, no_packing: bool = False, no_remote_fusion: bool = False,
                 no_joint_folds: bool = False):
        self._lib = load()
        self._graph = graph
        opts = fs_explore_opts(top_k, beam_width, 1 if no_packing else 0, 1 if no_remote_fusion else 0, 1 if no_joint_folds else 0)
        h = C.c_void_p()
        _check(self._lib.fs_explore(graph.handle, C.byref(opts), C.byref(h)))
        self.handle = h
        info = fs_program_info()
        _check(self._lib.fs_program_query(self.handle, C.byref(info)))
        self.info = info.as_dict()

    def __del__(self):
        if getattr(self, "handle", None):
            self._lib.fs_program_destroy(self.handle)
            self.handle = None

    def patterns(self) -> List[Dict]:
        out = []
        for i in range(self.info["n_patterns"] + self.info["n_single_ops"]):
            n, f, pack, info = C.c_int32(), C.c_double(), C.c_int32(), fs_plan_info()
            _check(self._lib.fs_program_pattern(self.handle, i, None, 0, C.byref(n), C.byref(f), C.byref(pack), C.byref(info)))
            ops = (C.c_int32 * max(1, n.value))()
            _check(self._lib.fs_program_pattern(self.handle, i, ops, n.value, None, None, None, None))
            out.append({"ops": list(ops)[:n.value], "f_us": f.value, "pack": pack.value, "info": info.as_dict()})
        return out

    def describe(self) -> str:
        need = self._lib.fs_program_describe(self.handle, None, 0)
        if need < 0:
            _check(int(need))
        buf = C.create_string_buffer(int(need))
        self._lib.fs_program_describe(self.handle, buf, int(need))
        return buf.value.decode()

    def make_workspace(self, device="cuda"):
        import torch
        n = int(self.info["workspace_bytes"])
        return torch.zeros(max(n, 256), dtype=torch.uint8, device=device)

    def bind(self, inputs: Sequence[int], outputs: Sequence[int], workspace: int, workspace_bytes: int, stream: int):
        ins = (C.c_void_p * max(1, len(inputs)))(*inputs)
        outs = (C.c_void_p * max(1, len(outputs)))(*outputs)
        ws, nb, st = C.c_void_p(workspace), C.c_size_t(workspace_bytes), C.c_void_p(stream)
        fn, handle = self._lib.fs_program_execute, self.handle

        def call(_keep=(ins, outs)):
            code = fn(handle, ins, outs, ws, nb, st)
            if code < 0:
                _check(code)
        return call

    def bind_stage(self, stage: int, inputs: Sequence[int], outputs: Sequence[int], workspace: int, workspace_bytes: int, stream: int):
        """The steps of one stage (programs whose graph declares external computations run stage by stage)."""
        ins = (C.c_void_p * max(1, len(inputs)))(*inputs)
        outs = (C.c_void_p * max(1, len(outputs)))(*outputs)
        ws, nb, st = C.c_void_p(workspace), C.c_size_t(workspace_bytes), C.c_void_p(stream)
        fn, handle = self._lib.fs_program_execute_stage, self.handle

        def call(_keep=(ins, outs)):
            code = fn(handle, stage, ins, outs, ws, nb, st)
            if code < 0:
                _check(code)
        return call


def stream_copy(dst, src, stream: Optional[int] = None) -> None:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    nbytes = src.numel() * src.element_size()
    _check(load().fs_stream_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes, C.c_void_p(stream)))


def bind_copy(dst_ptr: int, src_ptr: int, nbytes: int, stream: int):
    """Pre-marshalled fs_stream_copy call (for tight timing loops)."""
    fn = load().fs_stream_copy
    d, s_, n, st = C.c_void_p(dst_ptr), C.c_void_p(src_ptr), C.c_size_t(nbytes), C.c_void_p(stream)

    def call():
        code = fn(d, s_, n, st)
        if code < 0:
            _check(code)
    return call


def bind_probe(dst_ptr: int, src_ptr: int, stream_bytes: int, reads: int, writes: int, vecs_per_lane: int, stream: int,
               pitch_bytes: int = 0):
    """Pre-marshalled fs_stream_probe call."""
    fn = load().fs_stream_probe
    d, s_, n, st = C.c_void_p(dst_ptr), C.c_void_p(src_ptr), C.c_size_t(stream_bytes), C.c_void_p(stream)
    pitch = C.c_size_t(pitch_bytes)

    def call():
        code = fn(d, s_, n, pitch, reads, writes, vecs_per_lane, st)
        if code < 0:
            _check(code)
    return call


# ---- torch <-> storage helpers (memory plumbing, no arithmetic) --------------------
def torch_dtype(name: str):
    import torch
    return {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i32": torch.int32}[name]


def to_device(array, dtype: str, device="cuda"):
    """numpy storage array (bf16 as uint16 bit patterns) -> torch device tensor of the storage dtype."""
    import numpy as np
    import torch
    if dtype == "bf16":
        t = torch.from_numpy(np.ascontiguousarray(array).view(np.int16)).view(torch.bfloat16)
    else:
        t = torch.from_numpy(np.ascontiguousarray(array))
    return t.to(device)


def to_host(tensor, dtype: str):
    """torch device tensor -> numpy storage array (bf16 as uint16 bit patterns)."""
    import numpy as np
    import torch
    t = tensor.detach().cpu().contiguous()
    if dtype == "bf16":
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def alloc_outputs(spec, device="cuda"):
    """Uninitialised device tensors for the outputs of a workload descriptor, shapes from the plan's graph."""
    import torch
    shapes = output_shapes(spec)
    return [torch.empty(shapes[name], dtype=torch_dtype(dt), device=device) for name, dt in spec.outputs]


def output_shapes(spec) -> Dict[str, tuple]:
    """Shape bookkeeping for a descriptor (no values involved)."""
    dims = {t.name: tuple(t.dims) for t in spec.inputs}
    for op in spec.ops:
        a = dims[op.inputs[0]]
        if len(op.inputs) == 2:
            b = dims[op.inputs[1]]
            r = max(len(a), len(b))
            pa, pb = (1,) * (r - len(a)) + a, (1,) * (r - len(b)) + b
            dims[op.out] = tuple(max(x, y) for x, y in zip(pa, pb))
        elif op.opcode.startswith("reduce_"):
            ax = op.attr["axis"]
            dims[op.out] = a[:ax] + (1,) + a[ax + 1:]
        elif op.opcode == "transpose":
            dims[op.out] = tuple(a[p] for p in op.attr["perm"])
        elif op.opcode == "broadcast":
            dims[op.out] = tuple(op.attr["dims"])
        else:
            dims[op.out] = a
    return dims
