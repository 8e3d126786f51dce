"""ctypes binding of libdynbatch.so: same names as the C ABI, argument marshalling only.

PyTorch tensors provide device memory and the current HIP stream; every step of the two hot
paths runs inside the library's kernels.  There is no fallback: if the library has not been
built, importing this module raises.
"""
from __future__ import annotations

import ctypes as ct
import os
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdynbatch.so")

DYNB_F32, DYNB_BF16 = 0, 1
DYNB_SCHED_IMPROVED, DYNB_SCHED_STANDARD, DYNB_SCHED_NAIVE, DYNB_SCHED_DEPTH = 0, 1, 2, 3
DYNB_PLAN_THROUGHPUT = 8
DYNB_PLAN_BALANCE = 4
DYNB_PLAN_PERSISTENT = 16
DYNB_PLAN_KEEP = 32
ERRORS = {-1: "DYNB_E_INVAL", -2: "DYNB_E_MALFORMED", -3: "DYNB_E_NOMEM", -4: "DYNB_E_WORKSPACE",
          -5: "DYNB_E_UNSUPPORTED", -6: "DYNB_E_HIP"}

EXPORTS = ["dynb_last_error", "dynbatch_plan", "dynbatch_plan_dag", "dynbatch_plan_view", "dynbatch_plan_free",
           "dynbatch_plan_device_bytes", "dynbatch_plan_upload", "dynbatch_workspace_bytes",
           "dynbatch_packed_weights_bytes", "dynbatch_pack_weights",
           "dynbatch_classify_workspace_bytes", "dynbatch_classify", "dynbatch_backward_workspace_bytes", "dynbatch_backward",
           "dynbatch_execute", "dynbatch_execute_check", "dynb_set_spin_limit", "moe_workspace_bytes", "moe_forward", "moe_forward_static", "moe_forward_naive",
           "dynb_timing_enable", "dynb_probe_mfma_bf16", "dynb_probe_copy", "dynb_probe_read",
           "dynb_timing_read"]


class DynbError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{ERRORS.get(code, code)}: {msg}")
        self.code = code
        self.name = ERRORS.get(code, str(code))


I32P = ct.POINTER(ct.c_int32)


class _PlanView(ct.Structure):
    _fields_ = [(n, ct.c_int32) for n in ("n_examples", "n_nodes", "n_levels", "n_buckets", "n_compute_nodes",
                                          "n_launches", "max_launch_nodes", "n_slots")] + \
               [(n, I32P) for n in ("node_level", "node_type", "child0", "child1", "root", "bucket_level",
                                    "bucket_type", "bucket_start", "bucket_count", "members", "in0", "in1", "out",
                                    "node_launch", "item_node")] + \
               [("n_tickets", ct.c_int32), ("tickets", I32P)] + \
               [(n, I32P) for n in ("grad_dst0", "grad_dst1", "fn_first", "fn_items")] + \
               [("n_types", ct.c_int32), ("n_wg_units", ct.c_int32), ("wg_units", I32P), ("wg_order", I32P)]


class _Shape(ct.Structure):
    _fields_ = [("C", ct.c_int32), ("H", ct.c_int32), ("W", ct.c_int32), ("dtype", ct.c_int32)]


class _Weights(ct.Structure):
    _fields_ = [(n, ct.c_void_p) for n in ("w1", "b1", "w3a", "b3a", "w3b", "b3b", "packed")]


class _Grads(ct.Structure):
    _fields_ = [(n, ct.c_void_p) for n in ("dfeats", "dw1", "db1", "dw3a", "db3a", "dw3b", "db3b")]


class _HeadShape(ct.Structure):
    _fields_ = [(n, ct.c_int32) for n in ("C", "H", "W", "dtype", "Cc", "F", "n_answers")]


class _HeadWeights(ct.Structure):
    _fields_ = [(n, ct.c_void_p) for n in ("wc", "bc", "wf1", "bf1", "wf2", "bf2")]


class _MoeShape(ct.Structure):
    _fields_ = [(n, ct.c_int32) for n in ("T", "d", "h", "E", "k", "dtype")] + [("flags", ct.c_uint32)]


class _StageTime(ct.Structure):
    _fields_ = [("tag", ct.c_int32), ("units", ct.c_int32), ("ms", ct.c_float)]


class _MoeAux(ct.Structure):
    _fields_ = [(n, ct.c_void_p) for n in ("logits", "topk_idx", "topk_w", "counts", "offsets", "perm", "inv")]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    L = ct.CDLL(LIB_PATH)
    L.dynb_last_error.restype = ct.c_char_p
    L.dynbatch_plan.argtypes = [I32P, I32P, ct.c_int32, ct.POINTER(ct.c_uint8), ct.c_int32, ct.c_uint32,
                                ct.POINTER(ct.c_void_p)]
    L.dynbatch_plan_dag.argtypes = [I32P, I32P, I32P, I32P, I32P, ct.c_int32, ct.POINTER(ct.c_uint8), ct.c_int32, ct.c_uint32,
                                    ct.POINTER(ct.c_void_p)]
    L.dynbatch_plan_view.argtypes = [ct.c_void_p, ct.POINTER(_PlanView)]
    L.dynbatch_plan_free.argtypes = [ct.c_void_p]
    L.dynbatch_plan_free.restype = None
    L.dynbatch_plan_device_bytes.argtypes = [ct.c_void_p]
    L.dynbatch_plan_device_bytes.restype = ct.c_size_t
    L.dynbatch_plan_upload.argtypes = [ct.c_void_p, ct.c_void_p, ct.c_size_t, ct.c_void_p]
    L.dynbatch_workspace_bytes.argtypes = [ct.c_void_p, ct.POINTER(_Shape)]
    L.dynbatch_workspace_bytes.restype = ct.c_size_t
    L.dynbatch_execute.argtypes = [ct.c_void_p, ct.POINTER(_Shape), ct.POINTER(_Weights), ct.c_void_p, ct.c_void_p,
                                   ct.c_void_p, ct.c_size_t, ct.c_void_p]
    L.dynbatch_backward_workspace_bytes.argtypes = [ct.c_void_p, ct.POINTER(_Shape)]
    L.dynbatch_backward_workspace_bytes.restype = ct.c_size_t
    L.dynbatch_backward.argtypes = [ct.c_void_p, ct.POINTER(_Shape), ct.POINTER(_Weights), ct.c_void_p, ct.c_void_p, ct.c_void_p,
                                    ct.c_void_p, ct.POINTER(_Grads), ct.c_void_p, ct.c_size_t, ct.c_void_p]
    L.dynbatch_classify_workspace_bytes.argtypes = [ct.POINTER(_HeadShape), ct.c_int32]
    L.dynbatch_classify_workspace_bytes.restype = ct.c_size_t
    L.dynbatch_classify.argtypes = [ct.POINTER(_HeadShape), ct.POINTER(_HeadWeights), ct.c_void_p, ct.c_int32, ct.c_void_p,
                                    ct.c_void_p, ct.c_void_p, ct.c_size_t, ct.c_void_p]
    L.dynbatch_execute_check.argtypes = [ct.c_void_p, ct.POINTER(_Shape), ct.c_void_p, ct.c_void_p]
    L.dynb_set_spin_limit.argtypes = [ct.c_int32]
    L.dynb_set_spin_limit.restype = ct.c_int32
    L.dynbatch_packed_weights_bytes.argtypes = [ct.POINTER(_Shape), ct.c_int32]
    L.dynbatch_packed_weights_bytes.restype = ct.c_size_t
    L.dynbatch_pack_weights.argtypes = [ct.POINTER(_Shape), ct.c_int32, ct.POINTER(_Weights), ct.c_void_p, ct.c_size_t,
                                        ct.c_void_p]
    L.moe_workspace_bytes.argtypes = [ct.POINTER(_MoeShape)]
    L.moe_workspace_bytes.restype = ct.c_size_t
    L.moe_forward.argtypes = [ct.POINTER(_MoeShape), ct.c_void_p, ct.c_void_p, ct.c_void_p, ct.c_void_p, ct.c_void_p,
                              ct.c_void_p, ct.c_void_p, ct.POINTER(_MoeAux), ct.c_void_p, ct.c_size_t, ct.c_void_p]
    L.moe_forward_naive.argtypes = L.moe_forward.argtypes + [ct.c_int32]
    L.moe_forward_static.argtypes = L.moe_forward.argtypes[:9] + [ct.c_void_p]
    L.dynb_probe_mfma_bf16.argtypes = [ct.c_int32, ct.c_int32, ct.c_void_p, ct.c_void_p, ct.POINTER(ct.c_double)]
    L.dynb_probe_copy.argtypes = [ct.c_void_p, ct.c_void_p, ct.c_size_t, ct.c_void_p]
    L.dynb_probe_read.argtypes = [ct.c_void_p, ct.c_size_t, ct.c_void_p, ct.c_void_p]
    L.dynb_timing_enable.argtypes = [ct.c_int]
    L.dynb_timing_read.argtypes = [ct.POINTER(_StageTime), ct.c_int32, ct.POINTER(ct.c_int32)]
    return L


lib = _load()


def _check(rc: int):
    if rc != 0:
        raise DynbError(rc, lib.dynb_last_error().decode())


def _stream(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ct.c_void_p(s.cuda_stream)


def _ptr(t):
    return None if t is None else ct.c_void_p(t.data_ptr())


def _scratch(nbytes: int, device, stream):
    """Device buffer the binding allocates on the caller's behalf.  If the work runs on another stream than
    the current one, the allocator is told so: it must not hand the block out again before that work is done."""
    import torch
    t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device=device)
    if stream is not None and stream != torch.cuda.current_stream():
        t.record_stream(stream)
    return t


# ------------------------------------------------------------------------------------------ planner
class Plan:
    """Owner of a dynb_plan*; keeps the uploaded index-list buffer alive."""

    def __init__(self, handle, B):
        self.handle = handle
        self.B = B
        self.dev_buf = None
        self._free = lib.dynbatch_plan_free      # kept here: module globals may be gone at interpreter shutdown

    def free(self):
        h, self.handle = getattr(self, "handle", None), None
        if h:
            self._free(h)

    def __del__(self):
        try:
            self.free()
        except Exception:                        # nothing useful can be done in a finalizer
            pass


def dynbatch_plan(prog, prog_off, arity, flags: int = DYNB_SCHED_IMPROVED) -> Plan:
    prog = np.ascontiguousarray(prog, dtype=np.int32)
    prog_off = np.ascontiguousarray(prog_off, dtype=np.int32)
    arity = np.ascontiguousarray(arity, dtype=np.uint8)
    h = ct.c_void_p()
    if len(prog) == 0:
        prog = np.zeros(1, np.int32)      # keep the pointer non-NULL; lengths come from prog_off
    _check(lib.dynbatch_plan(prog.ctypes.data_as(I32P), prog_off.ctypes.data_as(I32P), len(prog_off) - 1,
                             arity.ctypes.data_as(ct.POINTER(ct.c_uint8)), len(arity), flags, ct.byref(h)))
    return Plan(h, len(prog_off) - 1)


def dynbatch_plan_dag(node_type, arg0, arg1, node_off, root, arity, flags: int = DYNB_SCHED_IMPROVED) -> Plan:
    """Plan of a batch of dependency graphs (argument indices local to each example, -1 = none)."""
    a = [np.ascontiguousarray(v, dtype=np.int32) for v in (node_type, arg0, arg1, node_off, root)]
    arity = np.ascontiguousarray(arity, dtype=np.uint8)
    for i in range(3):
        if len(a[i]) == 0:
            a[i] = np.zeros(1, np.int32)  # keep the pointers non-NULL; lengths come from node_off
    h = ct.c_void_p()
    B = len(a[3]) - 1
    if len(a[4]) != B:
        raise ValueError("root must have one entry per example")
    _check(lib.dynbatch_plan_dag(*[v.ctypes.data_as(I32P) for v in a], B,
                                 arity.ctypes.data_as(ct.POINTER(ct.c_uint8)), len(arity), flags, ct.byref(h)))
    return Plan(h, B)


def dynbatch_plan_view(plan: Plan) -> SimpleNamespace:
    v = _PlanView()
    _check(lib.dynbatch_plan_view(plan.handle, ct.byref(v)))

    def arr(p, n):
        return np.ctypeslib.as_array(p, shape=(n,)).copy() if n > 0 else np.zeros(0, np.int32)

    N, nb, B = v.n_nodes, v.n_buckets, v.n_examples
    return SimpleNamespace(
        n_examples=B, n_nodes=N, n_levels=v.n_levels, n_buckets=nb, n_compute_nodes=v.n_compute_nodes,
        n_launches=v.n_launches, max_launch_nodes=v.max_launch_nodes, n_slots=v.n_slots,
        node_level=arr(v.node_level, N), node_type=arr(v.node_type, N), child0=arr(v.child0, N),
        child1=arr(v.child1, N), root=arr(v.root, B), bucket_level=arr(v.bucket_level, nb),
        bucket_type=arr(v.bucket_type, nb), bucket_start=arr(v.bucket_start, nb),
        bucket_count=arr(v.bucket_count, nb), members=arr(v.members, N), in0=arr(v.in0, N), in1=arr(v.in1, N),
        out=arr(v.out, N), node_launch=arr(v.node_launch, N), item_node=arr(v.item_node, v.n_compute_nodes),
        n_tickets=v.n_tickets, tickets=arr(v.tickets, v.n_tickets),
        grad_dst0=arr(v.grad_dst0, v.n_compute_nodes if v.grad_dst0 else 0),
        grad_dst1=arr(v.grad_dst1, v.n_compute_nodes if v.grad_dst1 else 0),
        fn_first=arr(v.fn_first, v.n_types + 1 if v.fn_first else 0),
        fn_items=arr(v.fn_items, v.n_compute_nodes if v.fn_items else 0),
        n_types=v.n_types, n_wg_units=v.n_wg_units,
        wg_units=arr(v.wg_units, 8 * v.n_wg_units if v.wg_units else 0).reshape(-1, 8),
        wg_order=arr(v.wg_order, v.n_wg_units if v.wg_order else 0))


def dynbatch_plan_device_bytes(plan: Plan) -> int:
    return int(lib.dynbatch_plan_device_bytes(plan.handle))


def dynbatch_plan_upload(plan: Plan, dev_buf=None, stream=None):
    import torch
    n = dynbatch_plan_device_bytes(plan)
    if dev_buf is None:
        dev_buf = _scratch(n, "cuda", stream)
    _check(lib.dynbatch_plan_upload(plan.handle, _ptr(dev_buf), dev_buf.numel() * dev_buf.element_size(), _stream(stream)))
    plan.dev_buf = dev_buf
    return dev_buf


# ------------------------------------------------------------------------------------------ executor
def _shape_of(feats) -> _Shape:
    import torch
    B, H, W, C = feats.shape
    if feats.dtype == torch.float32:
        dt = DYNB_F32
    elif feats.dtype == torch.bfloat16:
        dt = DYNB_BF16
    else:
        raise TypeError("feats must be float32 or bfloat16")
    return _Shape(C, H, W, dt)


def dynbatch_workspace_bytes(plan: Plan, C: int, H: int, W: int, dtype: int) -> int:
    return int(lib.dynbatch_workspace_bytes(plan.handle, ct.byref(_Shape(C, H, W, dtype))))


def _weights_struct(weights: dict) -> _Weights:
    return _Weights(*[(t.data_ptr() if t is not None else None) for t in
                      (weights.get(k) for k in ("w1", "b1", "w3a", "b3a", "w3b", "b3b", "packed"))])


def dynbatch_packed_weights_bytes(C: int, H: int, W: int, dtype: int, n_types: int) -> int:
    return int(lib.dynbatch_packed_weights_bytes(ct.byref(_Shape(C, H, W, dtype)), n_types))


def dynbatch_pack_weights(weights: dict, C: int, H: int, W: int, dtype: int, packed=None, stream=None):
    """One-time preparation: returns a device buffer to pass as weights["packed"]."""
    import torch
    n_types = int(weights["w3a"].shape[0])
    shape = _Shape(C, H, W, dtype)
    if packed is None:
        packed = torch.empty(max(int(lib.dynbatch_packed_weights_bytes(ct.byref(shape), n_types)), 256),
                             dtype=torch.uint8, device=weights["w3a"].device)
    w = _weights_struct({**weights, "packed": None})
    _check(lib.dynbatch_pack_weights(ct.byref(shape), n_types, ct.byref(w), _ptr(packed),
                                     packed.numel() * packed.element_size(), _stream(stream)))
    return packed


def dynbatch_execute(plan: Plan, weights: dict, feats, out=None, workspace=None, stream=None):
    """weights: dict with device tensors w1,b1,w3a,b3a,w3b,b3b (biases float32 or None; w1 may be None)
    and optionally packed (from dynbatch_pack_weights).
    feats: device [B,H,W,C] float32 or bfloat16, contiguous.  Returns out [B,H,W,C]."""
    import torch
    assert feats.is_cuda and feats.is_contiguous() and feats.shape[0] == plan.B
    shape = _shape_of(feats)
    for key in ("w1", "w3a", "w3b"):
        t = weights.get(key)
        assert t is None or (t.is_cuda and t.is_contiguous() and t.dtype == feats.dtype), key
    for key in ("b1", "b3a", "b3b"):
        t = weights.get(key)
        assert t is None or (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32), key
    if out is None:
        out = torch.empty_like(feats)
        if stream is not None and stream != torch.cuda.current_stream():
            out.record_stream(stream)
    assert out.is_cuda and out.is_contiguous() and out.shape == feats.shape and out.dtype == feats.dtype
    if workspace is None:
        workspace = _scratch(lib.dynbatch_workspace_bytes(plan.handle, ct.byref(shape)), feats.device, stream)
    w = _weights_struct(weights)
    _check(lib.dynbatch_execute(plan.handle, ct.byref(shape), ct.byref(w), _ptr(feats), _ptr(out), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)))
    return out


def dynbatch_execute_check(plan: Plan, feats, workspace, stream=None) -> None:
    """After executing a DYNB_PLAN_PERSISTENT plan: waits for the stream and raises DynbError(DYNB_E_HIP) if a
    bounded wait of the dependency-driven kernel expired."""
    _check(lib.dynbatch_execute_check(plan.handle, ct.byref(_shape_of(feats)), _ptr(workspace), _stream(stream)))


def dynb_set_spin_limit(polls: int) -> int:
    return int(lib.dynb_set_spin_limit(int(polls)))


# ------------------------------------------------------------------------------------------ backward pass
def dynbatch_backward_workspace_bytes(plan: Plan, C: int, H: int, W: int, dtype: int) -> int:
    return int(lib.dynbatch_backward_workspace_bytes(plan.handle, ct.byref(_Shape(C, H, W, dtype))))


def dynbatch_backward(plan: Plan, weights: dict, feats, out, forward_workspace, dout, workspace=None, stream=None, grads=None) -> dict:
    """Backward pass of an executed DYNB_PLAN_KEEP plan.  dout: device float32 [B,H,W,C].  Returns a dict of device
    float32 tensors dfeats, dw1, db1, dw3a, db3a, dw3b, db3b in the shapes of feats and of the weights (`grads`: such
    a dict from an earlier call, to be overwritten)."""
    import torch
    shape = _shape_of(feats)
    assert dout.is_cuda and dout.is_contiguous() and dout.dtype == torch.float32 and dout.shape == feats.shape
    f32 = lambda t: torch.empty(t.shape, dtype=torch.float32, device=feats.device)
    C = shape.C
    n_types = weights["w3a"].shape[0]
    g = grads if grads is not None else dict(
        dfeats=f32(feats), dw3a=f32(weights["w3a"]), dw3b=f32(weights["w3b"]),
        db3a=torch.empty((n_types, C), dtype=torch.float32, device=feats.device),
        db3b=torch.empty((n_types, C), dtype=torch.float32, device=feats.device),
        dw1=torch.empty((n_types, C, 2 * C), dtype=torch.float32, device=feats.device),
        db1=torch.empty((n_types, C), dtype=torch.float32, device=feats.device))
    for k in ("dfeats", "dw1", "db1", "dw3a", "db3a", "dw3b", "db3b"):
        assert g[k].is_cuda and g[k].is_contiguous() and g[k].dtype == torch.float32
    if workspace is None:
        n = int(lib.dynbatch_backward_workspace_bytes(plan.handle, ct.byref(shape)))
        if n == 0:
            _check(lib.dynbatch_backward(plan.handle, ct.byref(shape), None, None, None, None, None, None, None, 0, None))
        workspace = _scratch(n, feats.device, stream)
    gs = _Grads(*[g[k].data_ptr() for k in ("dfeats", "dw1", "db1", "dw3a", "db3a", "dw3b", "db3b")])
    w = _weights_struct(weights)
    _check(lib.dynbatch_backward(plan.handle, ct.byref(shape), ct.byref(w), _ptr(feats), _ptr(out), _ptr(forward_workspace),
                                 _ptr(dout), ct.byref(gs), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream(stream)))
    return g


# ------------------------------------------------------------------------------------------ classifier head
def _head_shape(roots, head: dict) -> _HeadShape:
    import torch
    B, H, W, C = roots.shape
    dt = DYNB_F32 if roots.dtype == torch.float32 else DYNB_BF16
    Cc, F, A = head["wc"].shape[0], head["wf1"].shape[0], head["wf2"].shape[0]
    assert head["wc"].shape == (Cc, C) and head["wf1"].shape == (F, H * W * Cc) and head["wf2"].shape == (A, F)
    return _HeadShape(C, H, W, dt, Cc, F, A)


def dynbatch_classify_workspace_bytes(C, H, W, dtype, Cc, F, n_answers, B) -> int:
    return int(lib.dynbatch_classify_workspace_bytes(ct.byref(_HeadShape(C, H, W, dtype, Cc, F, n_answers)), B))


def dynbatch_classify(roots, head: dict, probs=None, want_logits: bool = False, workspace=None, stream=None):
    """roots: device [B,H,W,C] float32 or bfloat16 (the output of dynbatch_execute); head: dict of device tensors
    wc [Cc,C], wf1 [F,H*W*Cc], wf2 [A,F] in the dtype of roots and bc, bf1, bf2 float32 or None.
    Returns probs [B,A] float32 (and the logits if wanted)."""
    import torch
    assert roots.is_cuda and roots.is_contiguous() and roots.dtype in (torch.float32, torch.bfloat16)
    for key in ("wc", "wf1", "wf2"):
        assert head[key].is_cuda and head[key].is_contiguous() and head[key].dtype == roots.dtype, key
    for key in ("bc", "bf1", "bf2"):
        t = head.get(key)
        assert t is None or (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32), key
    shape = _head_shape(roots, head)
    B, A = roots.shape[0], shape.n_answers
    if probs is None:
        probs = torch.empty((B, A), dtype=torch.float32, device=roots.device)
    logits = torch.empty((B, A), dtype=torch.float32, device=roots.device) if want_logits else None
    if workspace is None:
        workspace = _scratch(lib.dynbatch_classify_workspace_bytes(ct.byref(shape), B), roots.device, stream)
    w = _HeadWeights(*[(head.get(k).data_ptr() if head.get(k) is not None else None) for k in ("wc", "bc", "wf1", "bf1", "wf2", "bf2")])
    _check(lib.dynbatch_classify(ct.byref(shape), ct.byref(w), _ptr(roots), B, _ptr(probs), _ptr(logits), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream)))
    return (probs, logits) if want_logits else probs


# ------------------------------------------------------------------------------------------ MoE
def moe_workspace_bytes(T: int, d: int, h: int, E: int, k: int, dtype: int = DYNB_BF16) -> int:
    return int(lib.moe_workspace_bytes(ct.byref(_MoeShape(T, d, h, E, k, dtype))))


MOE_STATIC_SCRATCH_BYTES = 48 << 20
MOE_SEPARATE_PERMUTE = 1


def moe_forward_static(x, Wg, Wn, noise, W1, W2, k: int, out, aux=None, stream=None):
    """moe_forward without a workspace: the library's built-in device array holds the scratch data and the
    call allocates nothing, so `out` (and the aux tensors, if wanted: a namespace like moe_forward returns)
    must be given."""
    T, d = x.shape
    E, h = W1.shape[0], W1.shape[1]
    shape = _MoeShape(T, d, h, E, k, DYNB_BF16)
    aux_c = None
    if aux is not None:
        aux_c = _MoeAux(*[getattr(aux, n).data_ptr() for n in
                          ("logits", "topk_idx", "topk_w", "counts", "offsets", "perm", "inv")])
    _check(lib.moe_forward_static(ct.byref(shape), _ptr(x), _ptr(Wg), _ptr(Wn), _ptr(noise), _ptr(W1), _ptr(W2),
                                  _ptr(out), ct.byref(aux_c) if aux_c is not None else None, _stream(stream)))
    return out


def moe_forward(x, Wg, Wn, noise, W1, W2, k: int, out=None, want_aux: bool = False, workspace=None, stream=None,
                naive_stride: int = 0, flags: int = 0):
    """x [T,d] bf16; Wg, Wn [E,d] bf16; noise [T,E] f32 or None; W1 [E,h,d]; W2 [E,d,h] bf16 (all device,
    contiguous).  Returns out [T,d] bf16, or (out, aux namespace of device tensors) if want_aux.
    naive_stride >= 1 calls moe_forward_naive (one expert call per use) instead."""
    import torch
    T, d = x.shape
    E, h = W1.shape[0], W1.shape[1]
    for t in (x, Wg, W1, W2):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.bfloat16
    assert Wg.shape == (E, d) and W1.shape == (E, h, d) and W2.shape == (E, d, h)
    assert Wn is None or (Wn.is_cuda and Wn.is_contiguous() and Wn.dtype == torch.bfloat16 and Wn.shape == (E, d))
    assert noise is None or (noise.is_cuda and noise.is_contiguous() and noise.dtype == torch.float32
                             and noise.shape == (T, E))
    shape = _MoeShape(T, d, h, E, k, DYNB_BF16, flags)
    side = stream is not None and stream != torch.cuda.current_stream()
    if out is None:
        out = torch.empty_like(x)
        if side:
            out.record_stream(stream)
    if workspace is None:
        n = int(lib.moe_workspace_bytes(ct.byref(shape)))
        if n == 0:
            _check(lib.moe_forward(ct.byref(shape), None, None, None, None, None, None, None, None, None, 0, None))
        workspace = _scratch(n, x.device, stream)
    aux_t, aux_c = None, None
    if want_aux:
        dev = x.device
        aux_t = SimpleNamespace(
            logits=torch.empty((T, E), dtype=torch.float32, device=dev),
            topk_idx=torch.empty((T, k), dtype=torch.int32, device=dev),
            topk_w=torch.empty((T, k), dtype=torch.float32, device=dev),
            counts=torch.empty(E, dtype=torch.int32, device=dev),
            offsets=torch.empty(E + 1, dtype=torch.int32, device=dev),
            perm=torch.empty(T * k, dtype=torch.int32, device=dev),
            inv=torch.empty(T * k, dtype=torch.int32, device=dev))
        if side:
            for t_ in vars(aux_t).values():
                t_.record_stream(stream)
        aux_c = _MoeAux(*[getattr(aux_t, n).data_ptr() for n in
                          ("logits", "topk_idx", "topk_w", "counts", "offsets", "perm", "inv")])
    args = (ct.byref(shape), _ptr(x), _ptr(Wg), _ptr(Wn), _ptr(noise), _ptr(W1), _ptr(W2), _ptr(out),
            ct.byref(aux_c) if aux_c is not None else None, _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream))
    if naive_stride:
        _check(lib.moe_forward_naive(*args, naive_stride))
    else:
        _check(lib.moe_forward(*args))
    return (out, aux_t) if want_aux else out


# ------------------------------------------------------------------------------------------ timing
MOE_STAGES = ("gate", "topk", "sort", "permute", "ffn1", "ffn2", "combine")


def dynb_timing_enable(mode) -> None:
    """0/False off, 1/True one event per launch group or stage, 2 one event pair around all launch groups."""
    _check(lib.dynb_timing_enable(int(mode)))


def dynb_timing_read():
    """Stages of the last timed call: list of (tag, units, ms)."""
    n = ct.c_int32(0)
    _check(lib.dynb_timing_read(None, 0, ct.byref(n)))
    if n.value == 0:
        return []
    buf = (_StageTime * n.value)()
    _check(lib.dynb_timing_read(buf, n.value, ct.byref(n)))
    return [(b.tag, b.units, b.ms) for b in buf]


# ------------------------------------------------------------------------------------------ measurement helpers
def dynb_probe_mfma_bf16(iters: int, workgroups: int, sink, stream=None) -> float:
    """Enqueues the register-only MFMA loop; returns its flop count (time it with events on the stream)."""
    fl = ct.c_double(0.0)
    _check(lib.dynb_probe_mfma_bf16(iters, workgroups, _ptr(sink), _stream(stream), ct.byref(fl)))
    return fl.value


def dynb_probe_read(src, sink, stream=None) -> int:
    """Reads all of `src` (device tensor) and stores nothing; returns the number of bytes read."""
    n = src.numel() * src.element_size()
    _check(lib.dynb_probe_read(_ptr(src), n, _ptr(sink), _stream(stream)))
    return n


def dynb_probe_copy(dst, src, stream=None) -> int:
    """Enqueues the plain copy kernel over two equally sized device tensors; returns the bytes copied."""
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    _check(lib.dynb_probe_copy(_ptr(dst), _ptr(src), n, _stream(stream)))
    return n
