"""ctypes binding of libdsbd.so: argument marshalling only.

The structures mirror include/dsbd.h field by field.  Tensors are torch CUDA(HIP) tensors; their
data pointers and the current stream's handle are passed through unchanged.
"""
import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))

DSBD_NOT_REACHED, DSBD_ACCEPTED, DSBD_REJECTED, DSBD_PRUNED, DSBD_ROOT = 0, 1, 2, 3, 4
DSBD_FAULT_TOPOLOGY, DSBD_FAULT_TOKEN, DSBD_FAULT_NONFINITE = 1, 2, 4
DSBD_FAULT_ZERO_RESIDUAL, DSBD_FAULT_BOUNDS, DSBD_FAULT_SYNC_TIMEOUT = 8, 16, 32

_ERRORS = {-1: "invalid argument", -2: "unsupported shape", -3: "workspace too small", -4: "HIP runtime error"}


class DsbdError(RuntimeError):
    def __init__(self, code, where):
        super().__init__("%s failed: %s (%d)" % (where, _ERRORS.get(code, "unknown"), code))
        self.code = code


class _Forest(C.Structure):
    _fields_ = [("n_prompts", C.c_int32), ("n_trees", C.c_int32), ("n_nodes", C.c_int32),
                ("tree_prompt", C.c_void_p), ("tree_off", C.c_void_p), ("parent", C.c_void_p),
                ("token", C.c_void_p), ("draft_rank", C.c_void_p),
                ("max_tree_nodes", C.c_int32), ("max_depth", C.c_int32), ("max_prompt_trees", C.c_int32)]


class _KV(C.Structure):
    _fields_ = [("k_ptr", C.c_void_p), ("v_ptr", C.c_void_p), ("len", C.c_void_p),
                ("k_shared_ptr", C.c_void_p), ("v_shared_ptr", C.c_void_p), ("shared_len", C.c_void_p),
                ("token_stride", C.c_int64), ("head_stride", C.c_int64), ("max_len", C.c_int32)]


class _DraftIn(C.Structure):
    _fields_ = [("n_prompts", C.c_int32), ("n_beams", C.c_int32), ("max_prompt_beams", C.c_int32), ("V", C.c_int32),
                ("beam_off", C.c_void_p), ("logits_draft", C.c_void_p), ("beam_logp_draft", C.c_void_p),
                ("u", C.c_void_p)]


class _DraftOut(C.Structure):
    _fields_ = [("parent", C.c_void_p), ("token", C.c_void_p), ("logp_draft", C.c_void_p)]


class _ForestOut(C.Structure):
    _fields_ = [("tree_prompt", C.c_void_p), ("tree_off", C.c_void_p), ("parent", C.c_void_p), ("token", C.c_void_p),
                ("draft_rank", C.c_void_p), ("node_of_root", C.c_void_p), ("node_of", C.c_void_p),
                ("max_tree_nodes", C.c_void_p)]


class _Params(C.Structure):
    _fields_ = [("W_L", C.c_int32), ("W_min", C.c_int32), ("W_cap", C.c_int32), ("t", C.c_float),
                ("top_k", C.c_int32), ("top_p", C.c_float)]


class _VerifyIn(C.Structure):
    _fields_ = [("V", C.c_int32), ("logits_target", C.c_void_p), ("logits_draft", C.c_void_p),
                ("beam_logp_target", C.c_void_p), ("beam_logp_draft", C.c_void_p),
                ("u_accept", C.c_void_p), ("u_resid", C.c_void_p), ("u_fill", C.c_void_p)]


class _VerifyOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "node_status", "lse_target", "lse_draft", "node_logp_target", "node_logp_draft", "l_last", "layer_width",
        "n_out", "out_parent", "out_token", "out_node", "out_logp_target", "out_logp_draft", "near_tie_count")]


class _NextBeams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "n_next", "src_tree", "src_out", "path_len", "path", "token", "logp_target", "logp_draft")]


class _KVDst(C.Structure):
    _fields_ = [("k_ptr", C.c_void_p), ("v_ptr", C.c_void_p), ("len", C.c_void_p), ("capacity", C.c_int32)]


def lib_path():
    return os.path.join(_HERE, "libdsbd.so")


_lib = None


def load_library():
    """Loads libdsbd.so; raises ImportError if it has not been built. There is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError("libdsbd.so not found at %s: build it with `python -m paper_2409_16560_amd.build`" % path)
    lib = C.CDLL(path)
    lib.dsbd_forest_attention_workspace_bytes.restype = C.c_size_t
    lib.dsbd_forest_attention_workspace_bytes.argtypes = [C.POINTER(_Forest), C.POINTER(_KV), C.c_int32, C.c_int32, C.c_int32]
    lib.dsbd_forest_attention.restype = C.c_int32
    lib.dsbd_forest_attention.argtypes = [C.POINTER(_Forest), C.POINTER(_KV), C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.dsbd_verify_forest_workspace_bytes.restype = C.c_size_t
    lib.dsbd_verify_forest_workspace_bytes.argtypes = [C.POINTER(_Forest), C.c_int32, C.POINTER(_Params)]
    lib.dsbd_verify_forest.restype = C.c_int32
    lib.dsbd_verify_forest.argtypes = [C.POINTER(_Forest), C.POINTER(_VerifyIn), C.POINTER(_Params),
                                       C.POINTER(_VerifyOut), C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.dsbd_select_beams.restype = C.c_int32
    lib.dsbd_select_beams.argtypes = [C.POINTER(_Forest), C.POINTER(_VerifyOut), C.c_int32, C.c_int32,
                                      C.POINTER(_NextBeams), C.c_void_p, C.c_void_p]
    lib.dsbd_verify_forest_select.restype = C.c_int32
    lib.dsbd_verify_forest_select.argtypes = [C.POINTER(_Forest), C.POINTER(_VerifyIn), C.POINTER(_Params),
                                              C.POINTER(_VerifyOut), C.c_int32, C.POINTER(_NextBeams), C.c_void_p,
                                              C.c_size_t, C.c_void_p, C.c_void_p]
    lib.dsbd_commit_kv.restype = C.c_int32
    lib.dsbd_commit_kv.argtypes = [C.POINTER(_Forest), C.POINTER(_KV), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                   C.POINTER(_NextBeams), C.c_int32, C.POINTER(_KVDst), C.c_void_p, C.c_void_p]
    lib.dsbd_draft_layer_workspace_bytes.restype = C.c_size_t
    lib.dsbd_draft_layer_workspace_bytes.argtypes = [C.POINTER(_DraftIn), C.c_int32, C.c_int32, C.c_float]
    lib.dsbd_draft_layer.restype = C.c_int32
    lib.dsbd_draft_layer.argtypes = [C.POINTER(_DraftIn), C.c_int32, C.c_int32, C.c_float, C.POINTER(_DraftOut),
                                     C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.dsbd_build_forest.restype = C.c_int32
    lib.dsbd_build_forest.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.POINTER(_ForestOut), C.c_void_p, C.c_void_p]
    lib.dsbd_init.restype = C.c_int32
    lib.dsbd_init.argtypes = []
    lib.dsbd_verify_forest_static_capacity.restype = C.c_size_t
    lib.dsbd_verify_forest_static_capacity.argtypes = []
    lib.dsbd_verify_forest_static.restype = C.c_int32
    lib.dsbd_verify_forest_static.argtypes = [C.POINTER(_Forest), C.POINTER(_VerifyIn), C.POINTER(_Params),
                                              C.POINTER(_VerifyOut), C.c_void_p, C.c_void_p]
    lib.dsbd_stream_read_probe.restype = C.c_int32
    lib.dsbd_stream_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.POINTER(C.c_float), C.c_void_p]
    lib.dsbd_reload_knobs.restype = None
    lib.dsbd_reload_knobs.argtypes = []
    lib.dsbd_timing_enable.restype = C.c_int32
    lib.dsbd_timing_enable.argtypes = [C.c_int32, C.c_int32]
    lib.dsbd_timing_collect.restype = C.c_int32
    lib.dsbd_timing_collect.argtypes = [C.POINTER(C.c_float), C.c_int32]
    lib.dsbd_version.restype = C.c_char_p
    _lib = lib
    return lib


def dsbd_version():
    return load_library().dsbd_version().decode()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _i32(t, dev):
    return torch.as_tensor(t, dtype=torch.int32).to(dev).contiguous()


class Forest:
    """Draft forest on the device plus the host-side bounds the library wants."""

    def __init__(self, tree_prompt, tree_off, parent, token=None, draft_rank=None, *, n_prompts, max_tree_nodes,
                 max_depth, max_prompt_trees, device="cuda"):
        self.tree_prompt = _i32(tree_prompt, device)
        self.tree_off = _i32(tree_off, device)
        self.parent = _i32(parent, device)
        self.token = None if token is None else _i32(token, device)
        self.draft_rank = None if draft_rank is None else _i32(draft_rank, device)
        self.n_prompts = int(n_prompts)
        self.n_trees = int(self.tree_prompt.numel())
        self.n_nodes = int(self.parent.numel())
        self.max_tree_nodes, self.max_depth, self.max_prompt_trees = int(max_tree_nodes), int(max_depth), int(max_prompt_trees)
        self.device = self.parent.device

    def c_struct(self):
        return _Forest(self.n_prompts, self.n_trees, self.n_nodes, _ptr(self.tree_prompt), _ptr(self.tree_off),
                       _ptr(self.parent), _ptr(self.token), _ptr(self.draft_rank),
                       self.max_tree_nodes, self.max_depth, self.max_prompt_trees)


class PrefixKV:
    """Per-beam prefix caches: lists of bf16 tensors [L_b, Hkv, D] (token-major) or [Hkv, L_b, D] (head-major).
    k_shared / v_shared: optional per-tree tensors for the shared leading segment (the same tensor object for
    the beams of one prompt)."""

    def __init__(self, k: List[torch.Tensor], v: List[torch.Tensor], k_shared=None, v_shared=None,
                 head_major=False):
        dev = k[0].device
        self.keep = (k, v, k_shared, v_shared)
        # the strides come from any cache that holds tokens (an empty tensor's strides say nothing); the shared
        # segments have the layout of the beams' own
        held = [t for t in list(k) + [t for t in (k_shared or []) if t is not None] if t.numel() > 0]
        ref = held[0] if held else k[0]
        if head_major:
            self.token_stride, self.head_stride = ref.stride(1), ref.stride(0)
            lens = [t.shape[1] for t in k]
        else:
            self.token_stride, self.head_stride = ref.stride(0), ref.stride(1)
            lens = [t.shape[0] for t in k]
        for t in list(k) + list(v):
            assert t.dtype == torch.bfloat16 and (t.numel() == 0 or t.stride(-1) == 1)
        # the library takes ONE token stride and ONE head stride for all caches and cannot check them against the
        # allocations: caches whose strides differ (head-major tensors of different lengths, say) would be read out
        # of bounds, so they are refused here
        ts_ax, hs_ax = (1, 0) if head_major else (0, 1)
        for t in held + [t for t in list(v) + [t for t in (v_shared or []) if t is not None] if t.numel() > 0]:
            if t.dim() != 3 or (t.stride(ts_ax), t.stride(hs_ax)) != (self.token_stride, self.head_stride):
                raise ValueError("PrefixKV: every cache must have the same token and head strides (got %s against %s); "
                                 "allocate head-major caches with one common capacity and pass views of them"
                                 % ((t.stride(ts_ax), t.stride(hs_ax)), (self.token_stride, self.head_stride)))
        self.k_ptr = torch.tensor([t.data_ptr() for t in k], dtype=torch.int64, device=dev)
        self.v_ptr = torch.tensor([t.data_ptr() for t in v], dtype=torch.int64, device=dev)
        self.len = torch.tensor(lens, dtype=torch.int32, device=dev)
        self.max_len = max(lens) if lens else 0
        self.k_shared_ptr = self.v_shared_ptr = self.shared_len = None
        if k_shared is not None:
            ax = 1 if head_major else 0
            sl = [0 if t is None else t.shape[ax] for t in k_shared]
            self.k_shared_ptr = torch.tensor([0 if t is None else t.data_ptr() for t in k_shared], dtype=torch.int64, device=dev)
            self.v_shared_ptr = torch.tensor([0 if t is None else t.data_ptr() for t in v_shared], dtype=torch.int64, device=dev)
            self.shared_len = torch.tensor(sl, dtype=torch.int32, device=dev)
            self.max_len = max(a + b for a, b in zip(lens, sl))

    def c_struct(self):
        return _KV(_ptr(self.k_ptr), _ptr(self.v_ptr), _ptr(self.len), _ptr(self.k_shared_ptr),
                   _ptr(self.v_shared_ptr), _ptr(self.shared_len), self.token_stride, self.head_stride, self.max_len)


def _check(rc, where):
    if rc != 0:
        raise DsbdError(rc, where)


def dsbd_forest_attention_workspace_bytes(forest: Forest, kv: PrefixKV, Hq, Hkv, D):
    f, k = forest.c_struct(), kv.c_struct()
    return int(load_library().dsbd_forest_attention_workspace_bytes(C.byref(f), C.byref(k), Hq, Hkv, D))


def dsbd_forest_attention(forest: Forest, kv: PrefixKV, q, k_tree, v_tree, scale=0.0, out=None, lse=None,
                          anc_mask_out=None, workspace=None, fault=None, stream=None, want_lse=True):
    """q [N,Hq,D], k_tree/v_tree [N,Hkv,D] bf16.  Returns (out bf16 [N,Hq,D], lse f32 [N,Hq], fault i32[1])."""
    lib = load_library()
    N, Hq, D = q.shape
    Hkv = k_tree.shape[1]
    dev = q.device
    f, k = forest.c_struct(), kv.c_struct()
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((N, Hq), dtype=torch.float32, device=dev)
    if fault is None:
        fault = torch.zeros(1, dtype=torch.int32, device=dev)
    if workspace is None:
        nbytes = int(lib.dsbd_forest_attention_workspace_bytes(C.byref(f), C.byref(k), Hq, Hkv, D))
        if nbytes == 0 and N > 0:
            raise DsbdError(-2, "dsbd_forest_attention_workspace_bytes")
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    rc = lib.dsbd_forest_attention(C.byref(f), C.byref(k), _ptr(q), _ptr(k_tree), _ptr(v_tree), Hq, Hkv, D,
                                   float(scale), _ptr(out), _ptr(lse), _ptr(anc_mask_out), _ptr(workspace),
                                   workspace.numel(), _ptr(fault), _stream(stream))
    _check(rc, "dsbd_forest_attention")
    return out, lse, fault


@dataclass
class VerifyResult:
    node_status: torch.Tensor
    lse_target: torch.Tensor
    lse_draft: torch.Tensor
    node_logp_target: torch.Tensor
    node_logp_draft: torch.Tensor
    l_last: torch.Tensor
    layer_width: torch.Tensor
    n_out: torch.Tensor
    out_parent: torch.Tensor
    out_token: torch.Tensor
    out_node: torch.Tensor
    out_logp_target: torch.Tensor
    out_logp_draft: torch.Tensor
    near_tie_count: torch.Tensor
    fault: torch.Tensor
    W_cap: int = 0

    def c_struct(self):
        return _VerifyOut(*[_ptr(getattr(self, n)) for n, _ in _VerifyOut._fields_])

    @staticmethod
    def allocate(forest: Forest, W_cap: int):
        dev, N, P, Lw = forest.device, forest.n_nodes, forest.n_prompts, forest.max_depth + 2
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        return VerifyResult(
            e((N,), torch.uint8), e((N,), torch.float32), e((N,), torch.float32), e((N,), torch.float32),
            e((N,), torch.float32), e((P,), torch.int32), e((P, Lw), torch.int32), e((P,), torch.int32),
            e((P, W_cap), torch.int32), e((P, W_cap), torch.int32), e((P, W_cap), torch.int32),
            e((P, W_cap), torch.float64), e((P, W_cap), torch.float64), e((P,), torch.int32),
            torch.zeros(1, dtype=torch.int32, device=dev), W_cap)


def _params(W_L, W_min, W_cap, t, top_k=0, top_p=1.0):
    return _Params(int(W_L), int(W_min), int(W_cap), float(t), int(top_k), float(top_p))


def dsbd_verify_forest_workspace_bytes(forest: Forest, V, W_L=0, W_min=1, W_cap=16, t=-1.0, top_k=0, top_p=1.0):
    f, p = forest.c_struct(), _params(W_L, W_min, W_cap, t, top_k, top_p)
    return int(load_library().dsbd_verify_forest_workspace_bytes(C.byref(f), int(V), C.byref(p)))


def dsbd_verify_forest(forest: Forest, logits_target, logits_draft, beam_logp_target, beam_logp_draft,
                       u_accept, u_resid, u_fill, W_L=0, W_min=1, W_cap=16, t=-1.0, result: VerifyResult = None,
                       workspace=None, stream=None, top_k=0, top_p=1.0):
    """Layer-wise verification; logits [N,V] f32, beam_logp [T] f64, uniforms f32.  top_k / top_p: the warping
    operation on the joints (0 / 1.0: none).  Returns VerifyResult."""
    lib = load_library()
    N, V = logits_target.shape
    f, p = forest.c_struct(), _params(W_L, W_min, W_cap, t, top_k, top_p)
    for t_, dt in ((logits_target, torch.float32), (logits_draft, torch.float32), (beam_logp_target, torch.float64),
                   (beam_logp_draft, torch.float64), (u_accept, torch.float32), (u_resid, torch.float32),
                   (u_fill, torch.float32)):
        assert t_.dtype == dt and t_.is_contiguous()
    assert u_resid.numel() == forest.n_prompts * (forest.max_depth + 2)
    assert u_fill.numel() == forest.n_prompts * (forest.max_depth + 2) * W_cap
    vin = _VerifyIn(int(V), _ptr(logits_target), _ptr(logits_draft), _ptr(beam_logp_target), _ptr(beam_logp_draft),
                    _ptr(u_accept), _ptr(u_resid), _ptr(u_fill))
    if result is None:
        result = VerifyResult.allocate(forest, W_cap)
    if workspace is None:
        nbytes = int(lib.dsbd_verify_forest_workspace_bytes(C.byref(f), int(V), C.byref(p)))
        if nbytes == 0 and N > 0:
            raise DsbdError(-2, "dsbd_verify_forest_workspace_bytes")
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=logits_target.device)
    vout = result.c_struct()
    rc = lib.dsbd_verify_forest(C.byref(f), C.byref(vin), C.byref(p), C.byref(vout), _ptr(workspace),
                                workspace.numel(), _ptr(result.fault), _stream(stream))
    _check(rc, "dsbd_verify_forest")
    return result


def dsbd_verify_forest_select(forest: Forest, logits_target, logits_draft, beam_logp_target, beam_logp_draft,
                              u_accept, u_resid, u_fill, W_L=0, W_min=1, W_cap=16, t=-1.0, keep_one=False,
                              result: VerifyResult = None, next_beams: "NextBeams" = None, workspace=None, stream=None,
                              top_k=0, top_p=1.0):
    """dsbd_verify_forest and dsbd_select_beams in one call.  Returns (VerifyResult, NextBeams); faults of both are
    reported in VerifyResult.fault."""
    lib = load_library()
    N, V = logits_target.shape
    f, p = forest.c_struct(), _params(W_L, W_min, W_cap, t, top_k, top_p)
    for t_, dt in ((logits_target, torch.float32), (logits_draft, torch.float32), (beam_logp_target, torch.float64),
                   (beam_logp_draft, torch.float64), (u_accept, torch.float32), (u_resid, torch.float32),
                   (u_fill, torch.float32)):
        assert t_.dtype == dt and t_.is_contiguous()
    assert u_resid.numel() == forest.n_prompts * (forest.max_depth + 2)
    assert u_fill.numel() == forest.n_prompts * (forest.max_depth + 2) * W_cap
    vin = _VerifyIn(int(V), _ptr(logits_target), _ptr(logits_draft), _ptr(beam_logp_target), _ptr(beam_logp_draft),
                    _ptr(u_accept), _ptr(u_resid), _ptr(u_fill))
    if result is None:
        result = VerifyResult.allocate(forest, W_cap)
    if next_beams is None:
        next_beams = NextBeams.allocate(forest, W_cap)
    if workspace is None:
        nbytes = int(lib.dsbd_verify_forest_workspace_bytes(C.byref(f), int(V), C.byref(p)))
        if nbytes == 0 and N > 0:
            raise DsbdError(-2, "dsbd_verify_forest_workspace_bytes")
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=logits_target.device)
    vout, nx = result.c_struct(), next_beams.c_struct()
    rc = lib.dsbd_verify_forest_select(C.byref(f), C.byref(vin), C.byref(p), C.byref(vout), int(bool(keep_one)),
                                       C.byref(nx), _ptr(workspace), workspace.numel(), _ptr(result.fault),
                                       _stream(stream))
    _check(rc, "dsbd_verify_forest_select")
    return result, next_beams


def dsbd_init():
    """Optional set-up for the current device (second stream, address of the static scratch array)."""
    _check(load_library().dsbd_init(), "dsbd_init")


def dsbd_verify_forest_static_capacity() -> int:
    return int(load_library().dsbd_verify_forest_static_capacity())


def dsbd_verify_forest_static(forest: Forest, logits_target, logits_draft, beam_logp_target, beam_logp_draft,
                              u_accept, u_resid, u_fill, result: VerifyResult, W_L=0, W_min=1, W_cap=16, t=-1.0,
                              stream=None, top_k=0, top_p=1.0):
    """dsbd_verify_forest without a workspace argument (the library's static device array serves as one).  The
    caller passes the result arrays: this wrapper allocates nothing either."""
    lib = load_library()
    N, V = logits_target.shape
    f, p = forest.c_struct(), _params(W_L, W_min, W_cap, t, top_k, top_p)
    vin = _VerifyIn(int(V), _ptr(logits_target), _ptr(logits_draft), _ptr(beam_logp_target), _ptr(beam_logp_draft),
                    _ptr(u_accept), _ptr(u_resid), _ptr(u_fill))
    vout = result.c_struct()
    rc = lib.dsbd_verify_forest_static(C.byref(f), C.byref(vin), C.byref(p), C.byref(vout), _ptr(result.fault),
                                       _stream(stream))
    _check(rc, "dsbd_verify_forest_static")
    return result


@dataclass
class NextBeams:
    n_next: torch.Tensor
    src_tree: torch.Tensor
    src_out: torch.Tensor
    path_len: torch.Tensor
    path: torch.Tensor
    token: torch.Tensor
    logp_target: torch.Tensor
    logp_draft: torch.Tensor
    fault: torch.Tensor

    def c_struct(self):
        return _NextBeams(*[_ptr(getattr(self, n)) for n, _ in _NextBeams._fields_])

    @staticmethod
    def allocate(forest: Forest, W_cap: int):
        dev, P, plen = forest.device, forest.n_prompts, forest.max_depth + 1
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        return NextBeams(e((P,), torch.int32), e((P, W_cap), torch.int32), e((P, W_cap), torch.int32),
                         e((P, W_cap), torch.int32), e((P, W_cap, plen), torch.int32), e((P, W_cap), torch.int32),
                         e((P, W_cap), torch.float64), e((P, W_cap), torch.float64),
                         torch.zeros(1, dtype=torch.int32, device=dev))


def dsbd_select_beams(forest: Forest, verified: VerifyResult, keep_one=False, result: NextBeams = None, stream=None):
    lib = load_library()
    f, v = forest.c_struct(), verified.c_struct()
    if result is None:
        result = NextBeams.allocate(forest, verified.W_cap)
    nx = result.c_struct()
    rc = lib.dsbd_select_beams(C.byref(f), C.byref(v), int(verified.W_cap), int(bool(keep_one)), C.byref(nx),
                               _ptr(result.fault), _stream(stream))
    _check(rc, "dsbd_select_beams")
    return result


class KVDst:
    """Destination caches of the next beams: one bf16 tensor per slot (p, j) of the plan (None for slots that are
    never used), laid out like the source caches ([cap, Hkv, D], or [Hkv, cap, D] with head_major)."""

    def __init__(self, k: List[Optional[torch.Tensor]], v: List[Optional[torch.Tensor]], src: PrefixKV, head_major=False):
        ref = next(t for t in k if t is not None)
        dev = ref.device
        ax = 1 if head_major else 0
        for t in list(k) + list(v):
            if t is None:
                continue
            assert t.dtype == torch.bfloat16 and t.stride(-1) == 1
            ts, hs = (t.stride(1), t.stride(0)) if head_major else (t.stride(0), t.stride(1))
            assert (ts, hs) == (src.token_stride, src.head_stride), "destinations use the layout of the sources"
        self.keep = (k, v)
        self.capacity = min(t.shape[ax] for t in list(k) + list(v) if t is not None)
        self.k_ptr = torch.tensor([0 if t is None else t.data_ptr() for t in k], dtype=torch.int64, device=dev)
        self.v_ptr = torch.tensor([0 if t is None else t.data_ptr() for t in v], dtype=torch.int64, device=dev)
        self.len = torch.zeros(len(k), dtype=torch.int32, device=dev)

    def c_struct(self):
        return _KVDst(_ptr(self.k_ptr), _ptr(self.v_ptr), _ptr(self.len), int(self.capacity))


def dsbd_commit_kv(forest: Forest, src: PrefixKV, k_tree, v_tree, plan: NextBeams, W_cap: int, dst: KVDst,
                   fault=None, stream=None):
    """Copies the surviving caches into the next beams' buffers (appending the tree rows of each beam's path).
    Returns (dst.len as [P, W_cap] int32 tensor, fault i32[1])."""
    lib = load_library()
    f, k, nx, d = forest.c_struct(), src.c_struct(), plan.c_struct(), dst.c_struct()
    assert dst.k_ptr.numel() == forest.n_prompts * W_cap
    Hkv, D = k_tree.shape[1], k_tree.shape[2]
    if fault is None:
        fault = torch.zeros(1, dtype=torch.int32, device=k_tree.device)
    rc = lib.dsbd_commit_kv(C.byref(f), C.byref(k), _ptr(k_tree), _ptr(v_tree), int(Hkv), int(D), C.byref(nx),
                            int(W_cap), C.byref(d), _ptr(fault), _stream(stream))
    _check(rc, "dsbd_commit_kv")
    return dst.len.view(forest.n_prompts, W_cap), fault


DSBD_KERNEL_ATTENTION, DSBD_KERNEL_VOCAB_STATS, DSBD_KERNEL_VERIFY_LAYERS, DSBD_KERNEL_KV_COMMIT = 1, 2, 3, 4


def dsbd_draft_layer(beam_off, logits_draft, beam_logp_draft, u, W_S, *, max_prompt_beams, top_k=0, top_p=1.0,
                     workspace=None, fault=None, stream=None):
    """One beam-sampling step of the small model.  beam_off i32[P+1] (device), logits_draft f32[n_beams,V],
    beam_logp_draft f64[n_beams], u f32[P,W_S].  Returns (parent i32[P,W_S] rows of the input, token i32[P,W_S],
    logp f64[P,W_S], fault i32[1])."""
    lib = load_library()
    n_beams, V = logits_draft.shape
    P = beam_off.numel() - 1
    dev = logits_draft.device
    assert beam_off.dtype == torch.int32 and logits_draft.dtype == torch.float32 and logits_draft.is_contiguous()
    assert beam_logp_draft.dtype == torch.float64 and u.dtype == torch.float32 and u.is_contiguous()
    assert u.numel() == P * W_S and beam_logp_draft.numel() == n_beams
    din = _DraftIn(int(P), int(n_beams), int(max_prompt_beams), int(V), _ptr(beam_off), _ptr(logits_draft),
                   _ptr(beam_logp_draft), _ptr(u))
    parent = torch.empty((P, W_S), dtype=torch.int32, device=dev)
    token = torch.empty((P, W_S), dtype=torch.int32, device=dev)
    logp = torch.empty((P, W_S), dtype=torch.float64, device=dev)
    dout = _DraftOut(_ptr(parent), _ptr(token), _ptr(logp))
    if fault is None:
        fault = torch.zeros(1, dtype=torch.int32, device=dev)
    if workspace is None:
        nbytes = int(lib.dsbd_draft_layer_workspace_bytes(C.byref(din), int(W_S), int(top_k), float(top_p)))
        if nbytes == 0:
            raise DsbdError(-2, "dsbd_draft_layer_workspace_bytes")
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    rc = lib.dsbd_draft_layer(C.byref(din), int(W_S), int(top_k), float(top_p), C.byref(dout), _ptr(workspace),
                              workspace.numel(), _ptr(fault), _stream(stream))
    _check(rc, "dsbd_draft_layer")
    return parent, token, logp, fault


def dsbd_build_forest(root_off, layer_parent, layer_token, root_token=None, *, n_roots, max_prompt_trees,
                      fault=None, stream=None):
    """Forest layout of gamma sampled layers.  root_off i32[P+1] (device), layer_parent / layer_token
    i32[gamma, P*W_S] (device), root_token i32[n_roots] or None.  Returns (Forest, node_of_root i32[n_roots],
    node_of i32[gamma, P*W_S], max_tree_nodes i32[1] (device), fault i32[1]); the Forest carries the bound of 64
    nodes per tree, the device value says what the largest tree really holds."""
    lib = load_library()
    dev = root_off.device
    P = root_off.numel() - 1
    gamma = int(layer_parent.shape[0]) if layer_parent is not None and layer_parent.numel() > 0 else 0
    W_S = int(layer_parent.shape[1]) // P if gamma else 0
    N = int(n_roots) + gamma * P * W_S
    i32 = lambda n: torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    tree_prompt, tree_off, parent, token, rank = i32(n_roots), i32(n_roots + 1), i32(N), i32(N), i32(N)
    node_of_root, node_of, mx = i32(n_roots), i32(gamma * P * W_S), i32(1)
    fo = _ForestOut(_ptr(tree_prompt), _ptr(tree_off), _ptr(parent), _ptr(token), _ptr(rank), _ptr(node_of_root),
                    _ptr(node_of), _ptr(mx))
    if fault is None:
        fault = torch.zeros(1, dtype=torch.int32, device=dev)
    for t_ in (root_off, layer_parent, layer_token, root_token):
        assert t_ is None or (t_.dtype == torch.int32 and t_.is_contiguous())
    rc = lib.dsbd_build_forest(int(P), int(n_roots), gamma, W_S, _ptr(root_off), _ptr(root_token),
                               _ptr(layer_parent) if gamma else None, _ptr(layer_token) if gamma else None,
                               C.byref(fo), _ptr(fault), _stream(stream))
    _check(rc, "dsbd_build_forest")
    f = Forest(tree_prompt[:n_roots], tree_off[:n_roots + 1], parent[:N], token[:N], rank[:N], n_prompts=P,
               max_tree_nodes=64, max_depth=gamma, max_prompt_trees=int(max_prompt_trees), device=dev)
    return f, node_of_root[:n_roots], node_of[:gamma * P * W_S].view(gamma, P * W_S) if gamma else node_of[:0], mx, fault


def dsbd_stream_read_probe(buf: torch.Tensor, reps: int = 10, stream=None) -> float:
    """GB/s of a plain streaming read over `buf` (a device tensor of at least 1 MiB), best of `reps`."""
    ms = C.c_float(0.0)
    nbytes = buf.numel() * buf.element_size()
    _check(load_library().dsbd_stream_read_probe(_ptr(buf), nbytes, int(reps), C.byref(ms), _stream(stream)),
           "dsbd_stream_read_probe")
    return nbytes / (ms.value * 1e-3) / 1e9


def dsbd_reload_knobs():
    """Read the tuning overrides (DSBD_* environment variables) again; the library reads them once per process."""
    load_library().dsbd_reload_knobs()


def dsbd_timing_enable(kernel: int, capacity: int = 0):
    """Record HIP events around every launch of one library kernel (0 switches the hook off)."""
    _check(load_library().dsbd_timing_enable(int(kernel), int(capacity)), "dsbd_timing_enable")


def dsbd_timing_collect(max_n: int = 4096):
    """Milliseconds of every recorded launch since the last collect (waits for the events)."""
    buf = (C.c_float * max_n)()
    n = load_library().dsbd_timing_collect(buf, max_n)
    if n < 0:
        raise DsbdError(n, "dsbd_timing_collect")
    return [float(buf[i]) for i in range(n)]
