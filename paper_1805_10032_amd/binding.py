"""ctypes binding of the Zeno HIP library (include/zeno.h).

Argument marshalling only: every function takes torch tensors that already
live on the GPU, passes their device pointers and the current HIP stream to
the C entry point of the same name, and returns the output tensors.  There is
no CPU fallback: a missing library or a tensor on the wrong device raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ZENO_HIP_LIB") or os.path.join(_HERE, "lib", "libzeno_hip.so")

ZENO_MAX_LAYERS = 8
ZENO_MAX_CANDIDATES = 1024
LOSS = {"squared": 0, "softmax_ce": 1}
FWD = {"fp32": 0, "bf16": 1}
STATUS = {0: "ok", 1: "invalid argument", 2: "unsupported size", 3: "workspace", 4: "device", 5: "host memory"}

EXPORTS = ["zeno_model_create", "zeno_cnn_model_create", "zeno_model_destroy", "zeno_model_num_params",
           "zeno_score_workspace_bytes", "zeno_score", "zeno_score_static", "zeno_aggregate", "zeno_aggregate_update", "zeno_mean",
           "zeno_median", "zeno_krum_workspace_bytes", "zeno_krum", "zeno_status_string", "zeno_profile_enable", "zeno_profile_collect",
           "zeno_score_plan_check"]

KERNEL_NAMES = ["pack", "layer_base", "layer_cand", "loss", "combine", "average", "mean", "median", "average_update",
                "krum", "conv_base", "conv_cand", "aux"]
ZENO_MAX_CONV = 8


class ZenoError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: status {status} ({STATUS.get(int(status), '?')})")


class _ModelDesc(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32),
                ("dims", ctypes.c_int32 * (ZENO_MAX_LAYERS + 1)),
                ("has_bias", ctypes.c_int32),
                ("loss", ctypes.c_int32),
                ("fwd", ctypes.c_int32)]


class _CnnDesc(ctypes.Structure):
    _fields_ = [("in_h", ctypes.c_int32), ("in_w", ctypes.c_int32), ("in_c", ctypes.c_int32),
                ("n_conv", ctypes.c_int32),
                ("conv_c", ctypes.c_int32 * ZENO_MAX_CONV),
                ("conv_stride", ctypes.c_int32 * ZENO_MAX_CONV),
                ("fc_out", ctypes.c_int32), ("has_bias", ctypes.c_int32), ("loss", ctypes.c_int32)]


class _ProfileRecord(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("layer", ctypes.c_int32), ("ms", ctypes.c_float),
                ("algorithmic_bytes", ctypes.c_double), ("waves", ctypes.c_int32), ("k_split", ctypes.c_int32),
                ("streaming", ctypes.c_int32), ("row_blocks", ctypes.c_int32), ("merged", ctypes.c_int32),
                ("second", ctypes.c_int32), ("k_slices", ctypes.c_int32),
                ("candidates", ctypes.c_int32),
                ("tail_candidates", ctypes.c_int32)]


class _Batch(ctypes.Structure):
    _fields_ = [("n_r", ctypes.c_int32),
                ("features", ctypes.c_void_p),
                ("labels", ctypes.c_void_p),
                ("targets", ctypes.c_void_p)]


_lib = None


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_1805_10032_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    lib.zeno_model_create.argtypes = [ctypes.POINTER(_ModelDesc), ctypes.POINTER(vp)]
    lib.zeno_model_create.restype = ctypes.c_int
    lib.zeno_cnn_model_create.argtypes = [ctypes.POINTER(_CnnDesc), ctypes.POINTER(vp)]
    lib.zeno_cnn_model_create.restype = ctypes.c_int
    lib.zeno_model_destroy.argtypes = [vp]
    lib.zeno_model_destroy.restype = None
    lib.zeno_model_num_params.argtypes = [vp]
    lib.zeno_model_num_params.restype = i64
    lib.zeno_score_workspace_bytes.argtypes = [vp, i32, i32]
    lib.zeno_score_workspace_bytes.restype = ctypes.c_size_t
    lib.zeno_score.argtypes = [vp, vp, vp, i64, i32, ctypes.POINTER(_Batch), f32, f32, vp, vp,
                               ctypes.c_size_t, vp]
    lib.zeno_score.restype = ctypes.c_int
    lib.zeno_score_static.argtypes = [vp, vp, vp, i64, i32, ctypes.POINTER(_Batch), f32, f32, vp, vp]
    lib.zeno_score_static.restype = ctypes.c_int
    lib.zeno_aggregate.argtypes = [vp, i64, vp, i32, i64, i32, vp, vp, vp]
    lib.zeno_aggregate.restype = ctypes.c_int
    lib.zeno_aggregate_update.argtypes = [vp, i64, vp, i32, i64, i32, f32, vp, vp, vp, vp, vp]
    lib.zeno_aggregate_update.restype = ctypes.c_int
    lib.zeno_mean.argtypes = [vp, i64, i32, i64, vp, vp]
    lib.zeno_mean.restype = ctypes.c_int
    lib.zeno_median.argtypes = [vp, i64, i32, i64, vp, vp]
    lib.zeno_median.restype = ctypes.c_int
    lib.zeno_krum_workspace_bytes.argtypes = [i32]
    lib.zeno_krum_workspace_bytes.restype = ctypes.c_size_t
    lib.zeno_krum.argtypes = [vp, i64, i32, i64, i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.zeno_krum.restype = ctypes.c_int
    lib.zeno_score_plan_check.argtypes = [vp, i32, i32]
    lib.zeno_score_plan_check.restype = ctypes.c_int
    lib.zeno_profile_enable.argtypes = [i32]
    lib.zeno_profile_enable.restype = ctypes.c_int
    lib.zeno_profile_collect.argtypes = [ctypes.POINTER(_ProfileRecord), i32]
    lib.zeno_profile_collect.restype = i32
    lib.zeno_status_string.argtypes = [ctypes.c_int]
    lib.zeno_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError(f"{name} must be a CUDA/HIP tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _rows(G: torch.Tensor):
    """(pointer, ldg) of a candidate matrix: rows contiguous, ldg >= d floats apart
    (a column slice of a wider allocation is accepted as it is, nothing is copied)."""
    if not isinstance(G, torch.Tensor) or not G.is_cuda or G.dtype != torch.float32 or G.dim() != 2:
        raise ValueError("G must be a 2-D float32 CUDA/HIP tensor")
    m, d = G.shape
    if d > 1 and G.stride(1) != 1:
        raise ValueError("the rows of G must be contiguous")
    ldg = int(G.stride(0)) if m > 1 else int(d)
    if ldg < d:
        raise ValueError("the rows of G overlap")
    return G.data_ptr(), ldg


def candidate_pitch(d: int, align: int = 32) -> int:
    """Row pitch in floats for an [m x d] candidate matrix: d rounded up to `align` floats, and, for
    line-aligned layouts (align a multiple of 32 floats = 128 bytes), to an ODD number of 128-byte
    lines.  With an even number of lines the rows of all candidates start at the same offset modulo
    256 bytes, and the workgroups that stream the same columns of 16 candidates at the same time then
    lean on the same memory channels (measured on the 14 GB workload: 2 % slower)."""
    align = max(1, int(align))
    ldg = (int(d) + align - 1) // align * align
    if align % 32 == 0 and (ldg // 32) % 2 == 0:
        ldg += 32
    return ldg


def alloc_candidates(m: int, d: int, device=None, align: int = 32) -> torch.Tensor:
    """An [m x d] float32 view whose rows start `align`-float (128-byte) aligned, an odd number of
    128-byte lines apart: the layout the streaming kernels are fastest on."""
    buf = torch.empty((int(m), candidate_pitch(d, align)), dtype=torch.float32,
                      device=device or torch.device("cuda", torch.cuda.current_device()))
    return buf[:, :int(d)]


class ZenoModel:
    """Host-side model handle (zeno_model_create / zeno_model_destroy)."""

    def __init__(self, dims, has_bias=True, loss="softmax_ce", fwd="fp32"):
        lib = load_library()
        desc = _ModelDesc()
        if not 2 <= len(dims) <= ZENO_MAX_LAYERS + 1:
            raise ZenoError(1, "ZenoModel")
        desc.n_layers = len(dims) - 1
        for i, v in enumerate(dims):
            desc.dims[i] = int(v)
        desc.has_bias = int(bool(has_bias))
        desc.loss = LOSS[loss]
        desc.fwd = FWD[fwd]
        handle = ctypes.c_void_p()
        st = lib.zeno_model_create(ctypes.byref(desc), ctypes.byref(handle))
        if st != 0:
            raise ZenoError(st, "zeno_model_create")
        self._lib = lib
        self._h = handle
        self.dims, self.has_bias, self.loss, self.fwd = list(dims), bool(has_bias), loss, fwd

    @property
    def num_params(self) -> int:
        return int(self._lib.zeno_model_num_params(self._h))

    def workspace_bytes(self, m: int, n_r: int) -> int:
        return int(self._lib.zeno_score_workspace_bytes(self._h, int(m), int(n_r)))

    def plan_check(self, m: int, n_r: int) -> int:
        """Status of the host-side check that every launch of zeno_score stays inside its workspace slots."""
        return int(self._lib.zeno_score_plan_check(self._h, int(m), int(n_r)))

    def close(self):
        if self._h is not None and self._h.value:
            self._lib.zeno_model_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class ZenoCnnModel(ZenoModel):
    """Handle of a convolutional model (zeno_cnn_model_create): desc = dict(in_h, in_w, in_c, conv_c=[...],
    conv_stride=[...], fc_out, has_bias); fp32 forward."""

    def __init__(self, desc, loss="softmax_ce"):
        lib = load_library()
        cd = _CnnDesc()
        cd.in_h, cd.in_w, cd.in_c = int(desc["in_h"]), int(desc["in_w"]), int(desc["in_c"])
        conv_c, conv_stride = list(desc["conv_c"]), list(desc["conv_stride"])
        if not (1 <= len(conv_c) <= ZENO_MAX_CONV) or len(conv_c) != len(conv_stride):
            raise ZenoError(1, "ZenoCnnModel")
        cd.n_conv = len(conv_c)
        for i, (c, s) in enumerate(zip(conv_c, conv_stride)):
            cd.conv_c[i], cd.conv_stride[i] = int(c), int(s)
        cd.fc_out = int(desc["fc_out"])
        cd.has_bias = int(bool(desc["has_bias"]))
        cd.loss = LOSS[loss]
        handle = ctypes.c_void_p()
        st = lib.zeno_cnn_model_create(ctypes.byref(cd), ctypes.byref(handle))
        if st != 0:
            raise ZenoError(st, "zeno_cnn_model_create")
        self._lib = lib
        self._h = handle
        self.desc = dict(desc)
        self.dims = [cd.in_h * cd.in_w * cd.in_c, cd.fc_out]      # input width of a sample, output width
        self.has_bias, self.loss, self.fwd = bool(desc["has_bias"]), loss, "fp32"


def alloc_workspace(model: ZenoModel, m: int, n_r: int, device=None) -> torch.Tensor:
    """A byte tensor of the size zeno_score asks for (torch's allocator returns
    at least 256-byte aligned blocks)."""
    n = model.workspace_bytes(m, n_r)
    if n == 0:
        raise ZenoError(1, "zeno_score_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device or torch.device("cuda", torch.cuda.current_device()))


def zeno_score(model: ZenoModel, x, G, features, gamma, rho, *, labels=None, targets=None,
               scores=None, workspace=None):
    """scores[i] = f_r(x) - f_r(x - gamma G[i]) - rho ||G[i]||^2  (Definition 2)."""
    lib = load_library()
    m, d = int(G.shape[0]), int(G.shape[1])
    if d != model.num_params or x.numel() != d:
        raise ValueError("x / G do not match the model's parameter count")
    n_r = int(features.shape[0])
    if features.shape[1] != model.dims[0]:
        raise ValueError("features do not match the model's input width")
    batch = _Batch()
    batch.n_r = n_r
    batch.features = _dev(features, torch.float32, "features")
    batch.labels = _dev(labels, torch.int32, "labels") if labels is not None else None
    batch.targets = _dev(targets, torch.float32, "targets") if targets is not None else None
    if scores is None:
        scores = torch.empty(m, dtype=torch.float32, device=G.device)
    if workspace is None:
        workspace = alloc_workspace(model, m, n_r, G.device)
    g_ptr, ldg = _rows(G)
    st = lib.zeno_score(model._h, _dev(x, torch.float32, "x"), g_ptr, ldg, m,
                        ctypes.byref(batch), float(gamma), float(rho),
                        _dev(scores, torch.float32, "scores"),
                        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream())
    if st != 0:
        raise ZenoError(st, "zeno_score")
    return scores


STATIC_SCRATCH_BYTES = 32 << 20


def zeno_score_static(model: ZenoModel, x, G, features, gamma, rho, *, labels=None, targets=None, scores=None):
    """zeno_score on the library's static scratch array: no workspace, nothing allocated by the call
    (pass `scores` to keep the binding from allocating the output either)."""
    lib = load_library()
    m, d = int(G.shape[0]), int(G.shape[1])
    if d != model.num_params or x.numel() != d:
        raise ValueError("x / G do not match the model's parameter count")
    if features.shape[1] != model.dims[0]:
        raise ValueError("features do not match the model's input width")
    batch = _Batch()
    batch.n_r = int(features.shape[0])
    batch.features = _dev(features, torch.float32, "features")
    batch.labels = _dev(labels, torch.int32, "labels") if labels is not None else None
    batch.targets = _dev(targets, torch.float32, "targets") if targets is not None else None
    if scores is None:
        scores = torch.empty(m, dtype=torch.float32, device=G.device)
    g_ptr, ldg = _rows(G)
    st = lib.zeno_score_static(model._h, _dev(x, torch.float32, "x"), g_ptr, ldg, m, ctypes.byref(batch),
                               float(gamma), float(rho), _dev(scores, torch.float32, "scores"), _stream())
    if st != 0:
        raise ZenoError(st, "zeno_score_static")
    return scores


def zeno_aggregate(G, scores, b, *, out=None, selected=None, want_selected=True):
    """Zeno_b: mean of the m-b highest-scoring rows (Definition 3).  Returns (out, selected)."""
    lib = load_library()
    m, d = int(G.shape[0]), int(G.shape[1])
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=G.device)
    if selected is None and want_selected and 0 <= b < m:
        selected = torch.empty(m - b, dtype=torch.int32, device=G.device)
    g_ptr, ldg = _rows(G)
    st = lib.zeno_aggregate(g_ptr, ldg, _dev(scores, torch.float32, "scores"), m, d, int(b),
                            _dev(out, torch.float32, "out"),
                            _dev(selected, torch.int32, "selected") if selected is not None else None,
                            _stream())
    if st != 0:
        raise ZenoError(st, "zeno_aggregate")
    return out, selected


def zeno_aggregate_update(G, scores, b, gamma, x, *, x_next=None, out=None, want_out=True, selected=None,
                          want_selected=True):
    """Zeno_b and the server's SGD step in one pass: x_next = x - gamma * Zeno_b(G)
    (Algorithm 1, server side).  x_next=x updates in place.  Returns (x_next, out, selected)."""
    lib = load_library()
    m, d = int(G.shape[0]), int(G.shape[1])
    if x.numel() != d:
        raise ValueError("x does not match the width of G")
    if x_next is None:
        x_next = torch.empty(d, dtype=torch.float32, device=G.device)
    if out is None and want_out:
        out = torch.empty(d, dtype=torch.float32, device=G.device)
    if selected is None and want_selected and 0 <= b < m:
        selected = torch.empty(m - b, dtype=torch.int32, device=G.device)
    g_ptr, ldg = _rows(G)
    st = lib.zeno_aggregate_update(g_ptr, ldg, _dev(scores, torch.float32, "scores"), m, d, int(b), float(gamma),
                                   _dev(x, torch.float32, "x"), _dev(x_next, torch.float32, "x_next"),
                                   _dev(out, torch.float32, "out") if out is not None else None,
                                   _dev(selected, torch.int32, "selected") if selected is not None else None,
                                   _stream())
    if st != 0:
        raise ZenoError(st, "zeno_aggregate_update")
    return x_next, out, selected


def zeno_mean(G, *, out=None):
    lib = load_library()
    m, d = int(G.shape[0]), int(G.shape[1])
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=G.device)
    g_ptr, ldg = _rows(G)
    st = lib.zeno_mean(g_ptr, ldg, m, d, _dev(out, torch.float32, "out"), _stream())
    if st != 0:
        raise ZenoError(st, "zeno_mean")
    return out


def zeno_median(G, *, out=None):
    lib = load_library()
    m, d = int(G.shape[0]), int(G.shape[1])
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=G.device)
    g_ptr, ldg = _rows(G)
    st = lib.zeno_median(g_ptr, ldg, m, d, _dev(out, torch.float32, "out"), _stream())
    if st != 0:
        raise ZenoError(st, "zeno_median")
    return out


def zeno_krum(G, b, *, out=None, want_scores=True, workspace=None):
    """Krum_b (Definition 5).  Returns (out, chosen index tensor [1], krum scores or None)."""
    lib = load_library()
    m, d = int(G.shape[0]), int(G.shape[1])
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=G.device)
    chosen = torch.empty(1, dtype=torch.int32, device=G.device)
    ks = torch.empty(m, dtype=torch.float32, device=G.device) if want_scores else None
    if workspace is None:
        n = int(lib.zeno_krum_workspace_bytes(m))
        workspace = torch.empty(max(n, 256), dtype=torch.uint8, device=G.device)
    g_ptr, ldg = _rows(G)
    st = lib.zeno_krum(g_ptr, ldg, m, d, int(b), _dev(out, torch.float32, "out"), _dev(chosen, torch.int32, "chosen"),
                       _dev(ks, torch.float32, "krum_scores") if ks is not None else None,
                       _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream())
    if st != 0:
        raise ZenoError(st, "zeno_krum")
    return out, chosen, ks


def profile_enable(on: bool = True):
    load_library().zeno_profile_enable(1 if on else 0)


def profile_collect(max_records: int = 4096, detail: bool = False):
    """[(kernel name, layer, ms, algorithmic bytes)] of the launches since the last collect; with
    detail=True a dict per launch that also names the launch shape of the layer kernels."""
    buf = (_ProfileRecord * max_records)()
    n = load_library().zeno_profile_collect(buf, max_records)
    if detail:
        return [dict(kernel=KERNEL_NAMES[r.kernel], layer=int(r.layer), ms=float(r.ms), bytes=float(r.algorithmic_bytes),
                     waves=int(r.waves), k_split=int(r.k_split), streaming=int(r.streaming),
                     row_blocks=int(r.row_blocks), merged=int(r.merged), second=int(r.second), k_slices=int(r.k_slices),
                     candidates=int(r.candidates),
                     tail_candidates=int(r.tail_candidates))
                for r in (buf[i] for i in range(n))]
    return [(KERNEL_NAMES[buf[i].kernel], int(buf[i].layer), float(buf[i].ms), float(buf[i].algorithmic_bytes))
            for i in range(n)]
