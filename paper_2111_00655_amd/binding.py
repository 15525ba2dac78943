"""ctypes binding of libcollage_mi.so: one Python function per C entry point,
with the same name.  Argument marshalling only; every step of the path runs in
the library.  A failing call raises ClgError carrying the status code and the
library's message.  The library must have been built (python -m
paper_2111_00655_amd.build); there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
# CLG_LIBRARY selects another build of the library (the host-sanitized one for CPU-only runs)
LIB_PATH = os.environ.get("CLG_LIBRARY") or os.path.join(HERE, "libcollage_mi.so")

MAX_DIMS = 6
MAX_PATTERN_ARGS = 8
MAX_CONSTRAINTS = 4
MAX_MATCH_NODES = 16
COST_INF = 1 << 60
WILDCARD = -1

OP_KINDS = ("conv2d", "conv2d_transpose", "dense", "batch_matmul", "bias_add", "add",
            "mul_scalar", "relu", "gelu", "tanh", "softmax", "layer_norm", "max_pool2d",
            "global_avg_pool2d", "take", "reshape", "transpose", "avg_pool2d", "concat",
            "conv3d", "max_pool3d", "global_avg_pool3d")
OP_ID = {k: i for i, k in enumerate(OP_KINDS)}
ATTR_ID = {k: i for i, k in enumerate(("groups", "kernel_h", "kernel_w", "stride_h", "stride_w",
                                       "pad_h", "pad_w", "transpose_b", "axis"))}
STATUS = {0: "OK", -1: "INVALID_ARG", -2: "SHAPE_MISMATCH", -3: "NO_KERNEL", -4: "NOT_A_COVER",
          -5: "OVERLAP", -6: "UNKNOWN_ID", -7: "WORKSPACE_TOO_SMALL", -8: "HIP_ERROR",
          -9: "OUT_OF_MEMORY", -10: "IO_ERROR", -11: "BUFFER_TOO_SMALL"}
F32, I32 = 0, 1


class ClgError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code
        self.status = STATUS.get(code, str(code))


class Attrs(C.Structure):
    _fields_ = [("stride", C.c_int32 * 2), ("pad", C.c_int32 * 2), ("kernel", C.c_int32 * 2),
                ("groups", C.c_int32), ("axis", C.c_int32), ("transpose_b", C.c_int32),
                ("ndims", C.c_int32), ("dims", C.c_int64 * MAX_DIMS), ("scalar", C.c_double),
                ("eps", C.c_double), ("stride_d", C.c_int32), ("pad_d", C.c_int32), ("kernel_d", C.c_int32),
                ("reserved_", C.c_int32)]


class AttrConstraint(C.Structure):
    _fields_ = [("attr", C.c_int32), ("lo", C.c_int64), ("hi", C.c_int64)]


class PatternRule(C.Structure):
    _fields_ = [("op_class", C.c_int32 * len(OP_KINDS)), ("max_ops", C.c_int32), ("grow_from_elemwise", C.c_int32)]


RULE_NONE, RULE_FUSABLE, RULE_ELEMWISE = 0, 1, 2


class PatternNode(C.Structure):
    _fields_ = [("op", C.c_int32), ("n_args", C.c_int32), ("args", C.c_int32 * MAX_PATTERN_ARGS),
                ("n_constraints", C.c_int32), ("constraints", AttrConstraint * MAX_CONSTRAINTS)]


class Match(C.Structure):
    _fields_ = [("pattern", C.c_int32), ("backend", C.c_int32), ("first", C.c_int32),
                ("sink", C.c_int32), ("n_nodes", C.c_int32), ("nodes", C.c_int32 * MAX_MATCH_NODES),
                ("binding", C.c_int32 * MAX_MATCH_NODES)]


class EsOpts(C.Structure):
    _fields_ = [("population", C.c_int32), ("generations", C.c_int32), ("tournament", C.c_int32),
                ("patience", C.c_int32), ("p_init", C.c_double), ("p_mutate", C.c_double),
                ("p_flip", C.c_double), ("p_cross", C.c_double), ("seed_ones", C.c_int32), ("reserved_", C.c_int32)]


FITNESS_FN = C.CFUNCTYPE(C.c_double, C.POINTER(C.c_uint8), C.c_size_t, C.c_void_p)


def make_es_opts(population=8, generations=10, tournament=3, patience=0,
                 p_init=0.25, p_mutate=0.5, p_flip=0.1, p_cross=0.5, seed_ones=False):
    return EsOpts(population, generations, tournament, patience, p_init, p_mutate, p_flip, p_cross, int(bool(seed_ones)), 0)


class MeasureOpts(C.Structure):
    _fields_ = [("warmup", C.c_int32), ("batches", C.c_int32), ("reps", C.c_int32)]


class ProfileOpts(C.Structure):
    _fields_ = [("warmup", C.c_int32), ("batches", C.c_int32), ("min_batch_us", C.c_int32),
                ("max_launches", C.c_int32), ("seed", C.c_uint64), ("no_cache", C.c_int32)]


class KernelInfo(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("match", C.c_int32), ("bound", C.c_int32),
                ("flops", C.c_double), ("bytes", C.c_double)]


# every symbol include/collage_mi.h declares: name -> (restype, argtypes)
_P = C.c_void_p
_i32p, _i64p, _szp = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_size_t)
SYMBOLS = {
    "clg_create": (C.c_int32, [C.POINTER(_P), C.c_int32]),
    "clg_destroy": (C.c_int32, [_P]),
    "clg_last_error": (C.c_char_p, []),
    "clg_version": (C.c_int32, []),
    "clg_graph_create": (C.c_int32, [_P, C.POINTER(_P)]),
    "clg_graph_destroy": (C.c_int32, [_P]),
    "clg_graph_input": (C.c_int32, [_P, C.c_int32, C.c_int32, _i64p, _i32p]),
    "clg_graph_const": (C.c_int32, [_P, C.c_int32, C.c_int32, _i64p, _P, _i32p]),
    "clg_graph_op": (C.c_int32, [_P, C.c_int32, C.c_int32, _i32p, C.POINTER(Attrs), _i32p]),
    "clg_graph_mark_output": (C.c_int32, [_P, C.c_int32]),
    "clg_graph_num_nodes": (C.c_int32, [_P, _i32p]),
    "clg_graph_node_shape": (C.c_int32, [_P, C.c_int32, _i32p, _i32p, _i64p]),
    "clg_register_backend": (C.c_int32, [_P, C.c_char_p, _i32p]),
    "clg_register_pattern": (C.c_int32, [_P, C.c_int32, C.POINTER(PatternNode), C.c_int32, _i32p]),
    "clg_num_patterns": (C.c_int32, [_P, _i32p]),
    "clg_get_pattern": (C.c_int32, [_P, C.c_int32, _i32p, C.POINTER(PatternNode), C.c_int32, _i32p]),
    "clg_generate_patterns": (C.c_int32, [_P, _P, C.c_int32, C.POINTER(PatternRule), _i32p]),
    "clg_match_all": (C.c_int32, [_P, _P, C.POINTER(Match), C.c_size_t, _szp]),
    "clg_profile_match": (C.c_int32, [_P, _P, C.c_int32, C.POINTER(ProfileOpts), _i64p]),
    "clg_profile_all": (C.c_int32, [_P, _P, C.POINTER(ProfileOpts), _i64p, C.c_size_t]),
    "clg_profile_empty": (C.c_int32, [_P, C.POINTER(ProfileOpts), _i64p]),
    "clg_cost_log_load": (C.c_int32, [_P, C.c_char_p]),
    "clg_cost_log_save": (C.c_int32, [_P, C.c_char_p]),
    "clg_cost_log_size": (C.c_int32, [_P, _szp]),
    "clg_match_key": (C.c_int32, [_P, _P, C.c_int32, C.c_char_p, C.c_size_t]),
    "clg_search_dp": (C.c_int32, [_P, _P, _i64p, C.c_size_t, C.c_int64, _i32p, C.c_size_t, _szp, _i64p]),
    "clg_search_stats": (C.c_int32, [_P, _i64p]),
    "clg_compile": (C.c_int32, [_P, _P, _i32p, C.c_size_t, C.POINTER(_P)]),
    "clg_plan_destroy": (C.c_int32, [_P]),
    "clg_plan_workspace_bytes": (C.c_int32, [_P, _szp]),
    "clg_plan_num_kernels": (C.c_int32, [_P, _szp]),
    "clg_plan_kernel_info": (C.c_int32, [_P, C.c_size_t, C.POINTER(KernelInfo)]),
    "clg_plan_set_lanes": (C.c_int32, [_P, C.c_int32]),
    "clg_plan_num_lanes": (C.c_int32, [_P, _i32p]),
    "clg_plan_set_handover": (C.c_int32, [_P, C.POINTER(C.c_uint8), C.c_size_t, C.c_int32]),
    "clg_plan_measure": (C.c_int32, [_P, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p, C.c_size_t,
                                     C.c_void_p, C.POINTER(MeasureOpts), _i64p]),
    "clg_search_graph_level": (C.c_int32, [_P, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p, C.c_size_t,
                                           C.c_void_p, C.c_int32, C.POINTER(EsOpts), C.POINTER(C.c_uint32), C.c_size_t,
                                           C.POINTER(MeasureOpts), C.POINTER(C.c_uint8), _i64p, _i64p, _i64p,
                                           C.POINTER(C.c_double), _i32p]),
    "clg_evolve": (C.c_int32, [C.c_size_t, C.POINTER(EsOpts), C.POINTER(C.c_uint32), C.c_size_t, FITNESS_FN,
                               C.c_void_p, C.POINTER(C.c_uint8), C.POINTER(C.c_double), C.POINTER(C.c_int64),
                               C.POINTER(C.c_double), _i32p]),
    "clg_plan_reads_constant": (C.c_int32, [_P, C.c_int32, _i32p, C.POINTER(C.c_size_t)]),
    "clg_plan_num_launches": (C.c_int32, [_P, C.POINTER(C.c_size_t)]),
    "clg_plan_region_of": (C.c_int32, [_P, C.c_size_t, _i32p]),
    "clg_execute": (C.c_int32, [_P, C.POINTER(_P), C.POINTER(_P), _P, C.c_size_t, _P]),
    "clg_execute_static": (C.c_int32, [_P, C.POINTER(_P), C.POINTER(_P), _P]),
    "clg_execute_timed": (C.c_int32, [_P, C.POINTER(_P), C.POINTER(_P), _P, C.c_size_t, _P, _i64p, C.c_size_t]),
}

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run python -m paper_2111_00655_amd.build")
        # PyTorch ships its own copy of the HIP runtime under the same soname.  The
        # process must end up with ONE runtime that both PyTorch (device memory,
        # streams) and this library use, and PyTorch only works with its own: load
        # PyTorch first so that the library binds to the copy already in memory.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        _lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(_lib, name)
            fn.restype = res
            fn.argtypes = args
    return _lib


def _check(rc):
    if rc != 0:
        raise ClgError(rc, (lib().clg_last_error() or b"").decode(errors="replace"))


def _dims(shape):
    return (C.c_int64 * len(shape))(*[int(d) for d in shape])


# ---- context ----------------------------------------------------------------------
def clg_version():
    return lib().clg_version()


def clg_last_error():
    return (lib().clg_last_error() or b"").decode(errors="replace")


def clg_create(device=0):
    h = _P()
    _check(lib().clg_create(C.byref(h), int(device)))
    return h


def clg_destroy(ctx):
    _check(lib().clg_destroy(ctx))


# ---- graph --------------------------------------------------------------------------
def clg_graph_create(ctx):
    h = _P()
    _check(lib().clg_graph_create(ctx, C.byref(h)))
    return h


def clg_graph_destroy(g):
    _check(lib().clg_graph_destroy(g))


def clg_graph_input(g, dtype, shape):
    node = C.c_int32()
    _check(lib().clg_graph_input(g, int(dtype), len(shape), _dims(shape), C.byref(node)))
    return node.value


def clg_graph_const(g, dtype, shape, dev_ptr):
    node = C.c_int32()
    _check(lib().clg_graph_const(g, int(dtype), len(shape), _dims(shape), _P(dev_ptr or 0), C.byref(node)))
    return node.value


def make_attrs(**kw):
    a = Attrs()
    a.stride_d, a.pad_d, a.kernel_d = 1, 0, 1
    for k in ("stride", "pad", "kernel"):
        if k in kw:
            v = kw[k]
            if len(v) == 3:                  # (depth, height, width) of the 3-D operators
                setattr(a, k + "_d", int(v[0]))
                v = v[1:]
            getattr(a, k)[0], getattr(a, k)[1] = int(v[0]), int(v[1])
    a.groups = int(kw.get("groups", 1))
    a.axis = int(kw.get("axis", 1))
    a.transpose_b = 1 if kw.get("transpose_b", True) else 0
    if "dims" in kw:
        a.ndims = len(kw["dims"])
        for i, d in enumerate(kw["dims"]):
            a.dims[i] = int(d)
    a.scalar = float(kw.get("scalar", 0.0))
    a.eps = float(kw.get("eps", 0.0))
    return a


def clg_graph_op(g, op_kind, in_nodes, attrs=None):
    node = C.c_int32()
    kind = OP_ID[op_kind] if isinstance(op_kind, str) else int(op_kind)
    arr = (C.c_int32 * len(in_nodes))(*[int(i) for i in in_nodes])
    _check(lib().clg_graph_op(g, kind, len(in_nodes), arr, C.byref(attrs) if attrs is not None else None,
                              C.byref(node)))
    return node.value


def clg_graph_mark_output(g, node):
    _check(lib().clg_graph_mark_output(g, int(node)))


def clg_graph_num_nodes(g):
    n = C.c_int32()
    _check(lib().clg_graph_num_nodes(g, C.byref(n)))
    return n.value


def clg_graph_node_shape(g, node):
    dt, nd = C.c_int32(), C.c_int32()
    dims = (C.c_int64 * MAX_DIMS)()
    _check(lib().clg_graph_node_shape(g, int(node), C.byref(dt), C.byref(nd), dims))
    return dt.value, tuple(dims[i] for i in range(nd.value))


# ---- registry ------------------------------------------------------------------------
def clg_register_backend(ctx, name):
    b = C.c_int32()
    _check(lib().clg_register_backend(ctx, name.encode(), C.byref(b)))
    return b.value


def flatten_pattern(pat):
    """Nested pattern (op, args, constraints) / "*" -> PatternNode array in
    post-order (arguments left to right, then the node; root last)."""
    nodes = []

    def rec(p):
        n = PatternNode()
        if p == "*":
            n.op = WILDCARD
            nodes.append(n)
            return len(nodes) - 1
        op, args, cons = p
        idx = [rec(a) for a in args]
        n.op = OP_ID[op]
        n.n_args = len(idx)
        for k, i in enumerate(idx):
            n.args[k] = i
        n.n_constraints = len(cons)
        for k, (name, (lo, hi)) in enumerate(cons):
            n.constraints[k].attr = ATTR_ID[name]
            n.constraints[k].lo = lo
            n.constraints[k].hi = hi
        nodes.append(n)
        return len(nodes) - 1

    rec(pat)
    return (PatternNode * len(nodes))(*nodes)


def clg_register_pattern(ctx, backend, pattern):
    arr = pattern if isinstance(pattern, C.Array) else flatten_pattern(pattern)
    pid = C.c_int32()
    _check(lib().clg_register_pattern(ctx, int(backend), arr, len(arr), C.byref(pid)))
    return pid.value


def clg_num_patterns(ctx):
    n = C.c_int32()
    _check(lib().clg_num_patterns(ctx, C.byref(n)))
    return n.value


def clg_get_pattern(ctx, pattern):
    """(backend id, nested pattern (op, args, constraints)) of a registered pattern."""
    n, be = C.c_int32(), C.c_int32()
    _check(lib().clg_get_pattern(ctx, int(pattern), C.byref(be), None, 0, C.byref(n)))
    arr = (PatternNode * n.value)()
    _check(lib().clg_get_pattern(ctx, int(pattern), C.byref(be), arr, n.value, C.byref(n)))
    attr_names = {v: k for k, v in ATTR_ID.items()}

    def rec(i):
        nd = arr[i]
        if nd.op == WILDCARD:
            return "*"
        cons = tuple(sorted((attr_names[nd.constraints[k].attr], (int(nd.constraints[k].lo), int(nd.constraints[k].hi)))
                            for k in range(nd.n_constraints)))
        return (OP_KINDS[nd.op], tuple(rec(nd.args[k]) for k in range(nd.n_args)), cons)

    return be.value, rec(n.value - 1)


def make_rule(op_class, max_ops, grow_from_elemwise):
    """op_class: operator kind name -> RULE_NONE / RULE_FUSABLE / RULE_ELEMWISE (missing kinds: none)."""
    r = PatternRule()
    for k, name in enumerate(OP_KINDS):
        r.op_class[k] = int(op_class.get(name, RULE_NONE))
    r.max_ops = int(max_ops)
    r.grow_from_elemwise = 1 if grow_from_elemwise else 0
    return r


def clg_generate_patterns(ctx, g, backend, rule):
    n = C.c_int32()
    _check(lib().clg_generate_patterns(ctx, g, int(backend), C.byref(rule), C.byref(n)))
    return n.value


# ---- graph-level search ---------------------------------------------------------------
def clg_evolve(n, opts, rand, fitness):
    """fitness: Python callable on a list of digits.  Returns (best digits, best cost,
    evaluations, history up to the generations run)."""
    raised = []

    def call(digits, count, _user):
        try:
            return float(fitness([digits[i] for i in range(count)]))
        except BaseException as e:            # must not unwind through the C frames
            raised.append(e)
            return float("nan")
    r = (C.c_uint32 * max(len(rand), 1))(*[int(x) for x in rand])
    best = (C.c_uint8 * max(n, 1))()
    cost, evals, gens = C.c_double(), C.c_int64(), C.c_int32()
    hist = (C.c_double * (opts.generations + 1))()
    rc = lib().clg_evolve(n, C.byref(opts), r, len(rand), FITNESS_FN(call), None, best, C.byref(cost),
                          C.byref(evals), hist, C.byref(gens))
    if raised:
        raise raised[0]
    _check(rc)
    return [best[i] for i in range(n)], cost.value, evals.value, [hist[i] for i in range(gens.value + 1)]


# ---- matches ------------------------------------------------------------------------
def clg_match_all(ctx, g):
    n = C.c_size_t()
    _check(lib().clg_match_all(ctx, g, None, 0, C.byref(n)))
    arr = (Match * max(n.value, 1))()
    _check(lib().clg_match_all(ctx, g, arr, n.value, C.byref(n)))
    return [arr[i] for i in range(n.value)]


# ---- measurer ------------------------------------------------------------------------
def clg_profile_match(ctx, g, match, opts=None):
    c = C.c_int64()
    _check(lib().clg_profile_match(ctx, g, int(match), C.byref(opts) if opts is not None else None, C.byref(c)))
    return c.value


def clg_profile_all(ctx, g, n_matches, opts=None):
    out = np.zeros(max(n_matches, 1), np.int64)
    _check(lib().clg_profile_all(ctx, g, C.byref(opts) if opts is not None else None,
                                 out.ctypes.data_as(_i64p), n_matches))
    return out[:n_matches]


def clg_profile_empty(ctx, opts=None):
    c = C.c_int64()
    _check(lib().clg_profile_empty(ctx, C.byref(opts) if opts is not None else None, C.byref(c)))
    return c.value


def clg_cost_log_load(ctx, path):
    _check(lib().clg_cost_log_load(ctx, os.fsencode(path)))


def clg_cost_log_save(ctx, path):
    _check(lib().clg_cost_log_save(ctx, os.fsencode(path)))


def clg_cost_log_size(ctx):
    n = C.c_size_t()
    _check(lib().clg_cost_log_size(ctx, C.byref(n)))
    return n.value


def clg_match_key(ctx, g, match):
    buf = C.create_string_buffer(1024)
    _check(lib().clg_match_key(ctx, g, int(match), buf, len(buf)))
    return buf.value.decode()


# ---- search ------------------------------------------------------------------------
def clg_search_dp(ctx, g, cost_ns, eps_ns=0):
    cost = np.ascontiguousarray(cost_ns, dtype=np.int64)
    n_nodes = clg_graph_num_nodes(g)
    chosen = np.zeros(max(n_nodes, 1), np.int32)
    n, total = C.c_size_t(), C.c_int64()
    _check(lib().clg_search_dp(ctx, g, cost.ctypes.data_as(_i64p), cost.size, int(eps_ns),
                               chosen.ctypes.data_as(_i32p), chosen.size, C.byref(n), C.byref(total)))
    return total.value, tuple(int(v) for v in chosen[:n.value])


def clg_search_stats(g):
    s = (C.c_int64 * 5)()
    _check(lib().clg_search_stats(g, s))
    return dict(N=s[0], P=s[1], F=s[2], S=s[3], states=s[4])


# ---- compile / execute ------------------------------------------------------------------
def clg_compile(ctx, g, matches):
    ids = np.ascontiguousarray(matches, dtype=np.int32)
    h = _P()
    _check(lib().clg_compile(ctx, g, ids.ctypes.data_as(_i32p), ids.size, C.byref(h)))
    return h


def clg_plan_destroy(plan):
    _check(lib().clg_plan_destroy(plan))


def clg_plan_workspace_bytes(plan):
    n = C.c_size_t()
    _check(lib().clg_plan_workspace_bytes(plan, C.byref(n)))
    return n.value


def clg_plan_num_kernels(plan):
    n = C.c_size_t()
    _check(lib().clg_plan_num_kernels(plan, C.byref(n)))
    return n.value


def clg_plan_set_lanes(plan, lanes):
    _check(lib().clg_plan_set_lanes(plan, int(lanes)))


def clg_plan_num_lanes(plan):
    n = C.c_int32()
    _check(lib().clg_plan_num_lanes(plan, C.byref(n)))
    return n.value


def clg_plan_kernel_info(plan, index):
    info = KernelInfo()
    _check(lib().clg_plan_kernel_info(plan, int(index), C.byref(info)))
    return dict(name=info.name.decode(), match=info.match, bound=("mfma", "hbm")[info.bound],
                flops=info.flops, bytes=info.bytes)


def _ptr_array(ptrs):
    return (_P * max(len(ptrs), 1))(*[_P(int(p)) for p in ptrs])


def clg_execute(plan, inputs, outputs, workspace, ws_bytes, stream=0):
    """inputs / outputs: sequences of device addresses (ints); workspace: device address."""
    _check(lib().clg_execute(plan, _ptr_array(inputs), _ptr_array(outputs), _P(int(workspace) or None),
                             int(ws_bytes), _P(int(stream) or None)))


def clg_plan_reads_constant(plan, node):
    """(whether executions read the caller's buffer of this constant, bytes of the plan's packed copies of it)"""
    reads, packed = C.c_int32(0), C.c_size_t(0)
    _check(lib().clg_plan_reads_constant(plan, int(node), C.byref(reads), C.byref(packed)))
    return bool(reads.value), packed.value


def clg_plan_num_launches(plan):
    n = C.c_size_t(0)
    _check(lib().clg_plan_num_launches(plan, C.byref(n)))
    return n.value


def clg_plan_region_of(plan, index):
    r = C.c_int32(0)
    _check(lib().clg_plan_region_of(plan, int(index), C.byref(r)))
    return r.value


STATIC_WORKSPACE_BYTES = 32 << 20


def clg_execute_static(plan, inputs, outputs, stream=0):
    """clg_execute on the library's own fixed workspace: nothing is allocated anywhere."""
    _check(lib().clg_execute_static(plan, _ptr_array(inputs), _ptr_array(outputs), _P(int(stream) or None)))


def clg_execute_timed(plan, inputs, outputs, workspace, ws_bytes, stream=0):
    n = clg_plan_num_kernels(plan)
    ns = np.zeros(max(n, 1), np.int64)
    _check(lib().clg_execute_timed(plan, _ptr_array(inputs), _ptr_array(outputs), _P(int(workspace) or None),
                                   int(ws_bytes), _P(int(stream) or None), ns.ctypes.data_as(_i64p), ns.size))
    return ns[:n]


def clg_plan_set_handover(plan, digits, lanes=2):
    d = (C.c_uint8 * max(len(digits), 1))(*[int(x) for x in digits])
    _check(lib().clg_plan_set_handover(plan, d, len(digits), int(lanes)))


def clg_plan_measure(plan, inputs, outputs, workspace, ws_bytes, stream=0, warmup=5, batches=5, reps=20):
    ns = C.c_int64()
    m = MeasureOpts(warmup, batches, reps)
    _check(lib().clg_plan_measure(plan, _ptr_array(inputs), _ptr_array(outputs), _P(int(workspace) or None),
                                  int(ws_bytes), _P(int(stream) or None), C.byref(m), C.byref(ns)))
    return ns.value


def clg_search_graph_level(plan, inputs, outputs, workspace, ws_bytes, stream, lanes, opts, rand,
                           warmup=3, batches=3, reps=20):
    """Returns (best digits, best ns, seed ns, evaluations, history)."""
    n = clg_plan_num_kernels(plan)
    r = (C.c_uint32 * max(len(rand), 1))(*[int(x) for x in rand])
    best = (C.c_uint8 * max(n, 1))()
    best_ns, seed_ns, evals, gens = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int32()
    hist = (C.c_double * (opts.generations + 1))()
    m = MeasureOpts(warmup, batches, reps)
    _check(lib().clg_search_graph_level(plan, _ptr_array(inputs), _ptr_array(outputs), _P(int(workspace) or None),
                                        int(ws_bytes), _P(int(stream) or None), int(lanes), C.byref(opts), r, len(rand),
                                        C.byref(m), best, C.byref(best_ns), C.byref(seed_ns), C.byref(evals), hist,
                                        C.byref(gens)))
    return [best[i] for i in range(n)], best_ns.value, seed_ns.value, evals.value, [hist[i] for i in range(gens.value + 1)]
