"""ctypes binding of include/mst.h: argument marshalling only -- every step of the hot
path runs inside libmst_hip.so.  There is no CPU fallback: if the library is missing the
import of a compute entry point raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))

MST_F32, MST_BF16 = 0, 1
MST_PATH_AUTO, MST_PATH_SPARSE, MST_PATH_DENSE = 0, 1, 2

_STATUS = {0: "MST_OK", -1: "MST_ERR_ARG", -2: "MST_ERR_SHAPE", -3: "MST_ERR_WORKSPACE",
           -4: "MST_ERR_STATE", -5: "MST_ERR_HIP"}


class MstError(RuntimeError):
    def __init__(self, fn: str, code: int, hip: int = 0):
        self.code = code
        super().__init__("%s -> %s (%d)%s" % (fn, _STATUS.get(code, "?"), code,
                                              " hipError=%d" % hip if code == -5 else ""))


class _ScheduleCfgC(C.Structure):
    _fields_ = [("S_M", C.c_double), ("N", C.c_int32), ("Delta_W", C.c_int64), ("T_U", C.c_int64),
                ("Delta_R", C.c_int64), ("zeta", C.POINTER(C.c_double)), ("n_zeta", C.c_int32)]


class UpdateStats(C.Structure):
    _fields_ = [("nnz_before", C.c_int64), ("nnz_after", C.c_int64), ("n_prune", C.c_int64),
                ("n_grow", C.c_int64), ("n_rand", C.c_int64), ("n_grad", C.c_int64)]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


class FormatStats(C.Structure):
    _fields_ = [("nnz", C.c_int64), ("row_view_slots", C.c_int64), ("col_view_slots", C.c_int64),
                ("row_view_efficiency", C.c_double), ("col_view_efficiency", C.c_double),
                ("heavy_rows", C.c_int64), ("heavy_entries", C.c_int64)]

    def as_dict(self):
        return {k: (int(getattr(self, k)) if t is C.c_int64 else float(getattr(self, k))) for k, t in self._fields_}


class TransformerShape(C.Structure):
    _fields_ = [("L", C.c_int64), ("N_embd", C.c_int64), ("D_ffw", C.c_int64), ("D_vocab", C.c_int64),
                ("n_layers", C.c_int64)]


class TransformerFlops(C.Structure):
    _fields_ = [(k, C.c_double) for k in ("kqv", "scores", "reduce", "proj", "ffw1", "ffw2", "lm", "forward",
                                          "backward", "total")]

    def as_dict(self):
        return {k: float(getattr(self, k)) for k, _ in self._fields_}


def lib_path() -> str:
    return os.path.join(HERE, "libmst_hip.so")


_lib = None


def lib() -> C.CDLL:
    """Loads libmst_hip.so (building it first if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    L = C.CDLL(path)
    vp, i32, i64, u64, dbl, sz = C.c_void_p, C.c_int, C.c_int64, C.c_uint64, C.c_double, C.c_size_t
    sig = {
        "mst_version": (C.c_char_p, []),
        "mst_last_hip_error": (i32, []),
        "mst_layer_device_bytes": (sz, [i32, i32, i64]),
        "mst_workspace_bytes": (sz, [i32, i32, i64, i32]),
        "mst_layer_create": (i32, [C.POINTER(vp), i32, i32, i64, vp, sz]),
        "mst_layer_destroy": (i32, [vp]),
        "mst_layer_load_dense": (i32, [vp, vp, vp, vp, sz, vp]),
        "mst_layer_export_dense": (i32, [vp, vp, vp, vp]),
        "mst_layer_values": (i32, [vp, C.POINTER(vp), C.POINTER(i64)]),
        "mst_layer_sync_values": (i32, [vp, vp]),
        "mst_layer_indices": (i32, [vp, vp, vp]),
        "mst_layer_set_path": (i32, [vp, i32]),
        "mst_layer_uses_dense": (i32, [vp, i32, i32, i32]),
        "mst_layer_set_prune_lambda": (i32, [vp, C.c_float]),
        "mst_spmm_force_shape": (i32, [i32, i32]),
        "mst_layer_nnz": (i64, [vp]),
        "mst_sparse_fc_fwd": (i32, [vp, vp, vp, i32, i32, vp]),
        "mst_sparse_fc_bwd_input": (i32, [vp, vp, vp, i32, i32, vp]),
        "mst_sparse_fc_bwd_weight": (i32, [vp, vp, vp, vp, i32, i32, vp, sz, vp]),
        "mst_sparse_fc_bwd_weight_static": (i32, [vp, vp, vp, vp, i32, i32, vp]),
        "mst_static_scratch_bytes": (sz, []),
        "mst_sparse_fc_bwd": (i32, [vp, vp, vp, vp, vp, i32, i32, vp, sz, vp]),
        "mst_bwd_force_shape": (i32, [i32, i32]),
        "mst_gemm_force_fp32_mfma": (i32, [i32]),
        "mst_gemm_last_tile": (i32, []),
        "mst_heavy_rows": (i32, [i32]),
        "mst_gather_active": (i32, [vp, vp, vp, vp]),
        "mst_layer_format_stats": (i32, [vp, C.POINTER(FormatStats), vp]),
        "mst_probe_lds_read": (i32, [vp, i32, i32, i32, vp]),
        "mst_update_due": (i32, [i64, i64]),
        "mst_update_seed": (u64, [u64, i64, C.c_int32, C.c_int32]),
        "mst_dense_grad": (i32, [vp, vp, vp, i32, i32, i32, i32, vp, sz, vp]),
        "mst_update_counts": (i32, [i64, i64, dbl, dbl, dbl, C.POINTER(UpdateStats)]),
        "mst_mask_update_from_scores": (i32, [vp, vp, dbl, dbl, dbl, u64, vp, sz, C.POINTER(UpdateStats), vp]),
        "mst_mask_update_from_scores_multi": (i32, [i32, vp, vp, vp, dbl, dbl, vp, vp, vp, vp, vp]),
        "mst_mask_update": (i32, [vp, vp, vp, i32, i32, dbl, dbl, dbl, u64, vp, sz, C.POINTER(UpdateStats), vp]),
        "mst_sparse_fc_bwd_weight_update": (i32, [vp, vp, vp, vp, i32, i32, dbl, dbl, dbl, u64, vp, sz,
                                                  C.POINTER(UpdateStats), vp]),
        "mst_schedule_density": (i32, [C.POINTER(_ScheduleCfgC), i64, C.POINTER(dbl), C.POINTER(dbl)]),
        "mst_erdos_renyi_density": (i32, [i32, C.POINTER(i32), C.POINTER(i32), dbl, C.POINTER(dbl)]),
        "mst_flops_fc_forward": (i32, [i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(dbl), C.POINTER(dbl)]),
        "mst_flops_transformer": (i32, [C.POINTER(TransformerShape), dbl, dbl, C.POINTER(TransformerFlops)]),
        "mst_strided_attention_mask": (i32, [vp, i32, i32, vp]),
        "mst_strided_attention_count": (i32, [i32, i32, C.POINTER(i64)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


EXPORTS = ["mst_version", "mst_last_hip_error", "mst_layer_device_bytes", "mst_workspace_bytes",
           "mst_layer_create", "mst_layer_destroy", "mst_layer_load_dense", "mst_layer_export_dense",
           "mst_layer_values", "mst_layer_sync_values", "mst_layer_indices", "mst_layer_set_path", "mst_layer_uses_dense", "mst_layer_set_prune_lambda",
           "mst_spmm_force_shape",
           "mst_layer_nnz", "mst_sparse_fc_fwd", "mst_sparse_fc_bwd_input", "mst_sparse_fc_bwd_weight", "mst_sparse_fc_bwd_weight_static",
           "mst_static_scratch_bytes", "mst_sparse_fc_bwd", "mst_bwd_force_shape", "mst_gemm_force_fp32_mfma", "mst_gemm_last_tile", "mst_heavy_rows",
           "mst_gather_active", "mst_layer_format_stats", "mst_probe_lds_read", "mst_update_due", "mst_update_seed",
           "mst_dense_grad", "mst_update_counts", "mst_mask_update_from_scores", "mst_mask_update_from_scores_multi", "mst_mask_update",
           "mst_sparse_fc_bwd_weight_update",
           "mst_schedule_density", "mst_erdos_renyi_density", "mst_flops_fc_forward", "mst_flops_transformer",
           "mst_strided_attention_mask", "mst_strided_attention_count"]


def _check(fn: str, code: int):
    if code != 0:
        raise MstError(fn, code, lib().mst_last_hip_error() if code == -5 else 0)


def _ptr(t) -> int:
    """Device (or host) address of a torch tensor / raw int address / None."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


# ------------------------------------------------------------------ host-only calls

class ScheduleCfg:
    """Hyper-parameters of the sparsity-variation and update-fraction schedules."""

    def __init__(self, S_M=0.96, N=5, Delta_W=2000, T_U=100000, Delta_R=2000,
                 zeta: Optional[Sequence[float]] = None):
        self.S_M, self.N, self.Delta_W, self.T_U, self.Delta_R = S_M, N, Delta_W, T_U, Delta_R
        self.zeta = list(zeta) if zeta is not None else [0.3] * (N + 1)

    def _c(self):
        arr = (C.c_double * len(self.zeta))(*self.zeta)
        return _ScheduleCfgC(self.S_M, self.N, self.Delta_W, self.T_U, self.Delta_R, arr, len(self.zeta)), arr


def mst_schedule_density(cfg: ScheduleCfg, step: int):
    """(density, zeta) at a training step."""
    c, keep = cfg._c()
    d, z = C.c_double(), C.c_double()
    _check("mst_schedule_density", lib().mst_schedule_density(C.byref(c), step, C.byref(d), C.byref(z)))
    return d.value, z.value


def mst_update_counts(n_total: int, nnz: int, target_density: float, zeta: float, rand_ratio: float) -> dict:
    st = UpdateStats()
    _check("mst_update_counts", lib().mst_update_counts(n_total, nnz, target_density, zeta, rand_ratio, C.byref(st)))
    return st.as_dict()


def mst_layer_device_bytes(O: int, I: int, nnz_capacity: int) -> int:
    return int(lib().mst_layer_device_bytes(O, I, nnz_capacity))


def mst_workspace_bytes(O: int, I: int, nnz_capacity: int, T: int) -> int:
    return int(lib().mst_workspace_bytes(O, I, nnz_capacity, T))


# ------------------------------------------------------------------ layer handle

class Layer:
    """Owns the torch byte buffer that backs one mst_layer_t and the handle itself."""

    def __init__(self, O: int, I: int, nnz_capacity: int, device="cuda:0"):
        import torch
        self.O, self.I, self.cap = O, I, nnz_capacity
        nbytes = mst_layer_device_bytes(O, I, nnz_capacity)
        if nbytes == 0:
            raise MstError("mst_layer_device_bytes", -2)
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        h = C.c_void_p()
        _check("mst_layer_create", lib().mst_layer_create(C.byref(h), O, I, nnz_capacity, self.buf.data_ptr(), nbytes))
        self.h = h
        self._destroy = lib().mst_layer_destroy      # kept for __del__ at interpreter shutdown

    def close(self):
        if getattr(self, "h", None):
            self._destroy(self.h)
            self.h = None

    __del__ = close

    @property
    def nnz(self) -> int:
        return int(lib().mst_layer_nnz(self.h))

    def load_dense(self, W, M, ws, stream=None):
        _check("mst_layer_load_dense",
               lib().mst_layer_load_dense(self.h, _ptr(W), _ptr(M), _ptr(ws), ws.numel(), _stream(stream)))

    def export_dense(self, W=None, M=None, stream=None):
        _check("mst_layer_export_dense", lib().mst_layer_export_dense(self.h, _ptr(W), _ptr(M), _stream(stream)))

    def values(self):
        """fp32 torch view (no copy) of the active weights in ascending flat-index order."""
        import torch
        p, n = C.c_void_p(), C.c_int64()
        _check("mst_layer_values", lib().mst_layer_values(self.h, C.byref(p), C.byref(n)))
        off = p.value - self.buf.data_ptr()
        return self.buf[off: off + 4 * n.value].view(torch.float32)

    def sync_values(self, stream=None):
        _check("mst_layer_sync_values", lib().mst_layer_sync_values(self.h, _stream(stream)))

    def indices(self, out, stream=None):
        _check("mst_layer_indices", lib().mst_layer_indices(self.h, _ptr(out), _stream(stream)))

    def format_stats(self, stream=None) -> dict:
        st = FormatStats()
        _check("mst_layer_format_stats", lib().mst_layer_format_stats(self.h, C.byref(st), _stream(stream)))
        return st.as_dict()

    def set_path(self, path: int):
        _check("mst_layer_set_path", lib().mst_layer_set_path(self.h, path))

    def uses_dense(self, act: int, T: int, weight_gradient=False) -> bool:
        """weight_gradient: False / 0 = Y and dX, True / 1 = the weight gradient, 2 = mst_sparse_fc_bwd."""
        rc = lib().mst_layer_uses_dense(self.h, act, T, int(weight_gradient))
        _check("mst_layer_uses_dense", min(rc, 0))
        return rc == 1

    def set_prune_lambda(self, lam: float):
        _check("mst_layer_set_prune_lambda", lib().mst_layer_set_prune_lambda(self.h, float(lam)))


# ------------------------------------------------------------------ device calls

def mst_spmm_force_shape(tokens_per_workgroup: int = 0, quads_per_wavefront: int = 0):
    _check("mst_spmm_force_shape", lib().mst_spmm_force_shape(tokens_per_workgroup, quads_per_wavefront))


def mst_sparse_fc_fwd(layer: Layer, X, Y, T: int, act: int = MST_F32, stream=None):
    _check("mst_sparse_fc_fwd", lib().mst_sparse_fc_fwd(layer.h, _ptr(X), _ptr(Y), T, act, _stream(stream)))


def mst_sparse_fc_bwd_input(layer: Layer, dY, dX, T: int, act: int = MST_F32, stream=None):
    _check("mst_sparse_fc_bwd_input",
           lib().mst_sparse_fc_bwd_input(layer.h, _ptr(dY), _ptr(dX), T, act, _stream(stream)))


def mst_sparse_fc_bwd_weight(layer: Layer, dY, X, dW, T: int, ws, act: int = MST_F32, stream=None):
    _check("mst_sparse_fc_bwd_weight",
           lib().mst_sparse_fc_bwd_weight(layer.h, _ptr(dY), _ptr(X), _ptr(dW), T, act, _ptr(ws), ws.numel(),
                                          _stream(stream)))


def mst_sparse_fc_bwd_weight_static(layer: Layer, dY, X, dW, T: int, act: int = MST_F32, stream=None):
    _check("mst_sparse_fc_bwd_weight_static",
           lib().mst_sparse_fc_bwd_weight_static(layer.h, _ptr(dY), _ptr(X), _ptr(dW), T, act, _stream(stream)))


def mst_static_scratch_bytes() -> int:
    return int(lib().mst_static_scratch_bytes())


def mst_bwd_force_shape(wavefronts_per_workgroup: int = 0, quads_per_wavefront: int = 0):
    _check("mst_bwd_force_shape", lib().mst_bwd_force_shape(wavefronts_per_workgroup, quads_per_wavefront))


def mst_gemm_last_tile() -> int:
    return lib().mst_gemm_last_tile()


def mst_heavy_rows(on: int = 1):
    _check("mst_heavy_rows", lib().mst_heavy_rows(on))


def mst_gemm_force_fp32_mfma(on):
    """False / 0: automatic; True / 1: plain fp32 MFMA kernel; 128 or 256: split kernel with that tile."""
    _check("mst_gemm_force_fp32_mfma", lib().mst_gemm_force_fp32_mfma(int(on)))


def mst_sparse_fc_bwd(layer: Layer, dY, X, dX, dW, T: int, ws, act: int = MST_F32, stream=None):
    _check("mst_sparse_fc_bwd",
           lib().mst_sparse_fc_bwd(layer.h, _ptr(dY), _ptr(X), _ptr(dX), _ptr(dW), T, act, _ptr(ws), ws.numel(),
                                   _stream(stream)))


def mst_gather_active(layer: Layer, G, dW, stream=None):
    _check("mst_gather_active", lib().mst_gather_active(layer.h, _ptr(G), _ptr(dW), _stream(stream)))


def mst_probe_lds_read(out, width: int, iters: int, blocks: int, stream=None):
    _check("mst_probe_lds_read", lib().mst_probe_lds_read(_ptr(out), width, iters, blocks, _stream(stream)))


def mst_update_due(step: int, delta_t: int) -> bool:
    r = lib().mst_update_due(int(step), int(delta_t))
    if r < 0:
        raise MstError("mst_update_due", r)
    return bool(r)


def mst_update_seed(run_seed: int, step: int, n_layers: int, layer: int) -> int:
    return int(lib().mst_update_seed(int(run_seed) & 0xFFFFFFFFFFFFFFFF, int(step), int(n_layers), int(layer)))


def mst_dense_grad(dY, X, G, T: int, O: int, I: int, act: int = MST_F32, ws=None, stream=None):
    _check("mst_dense_grad",
           lib().mst_dense_grad(_ptr(dY), _ptr(X), _ptr(G), T, O, I, act, _ptr(ws),
                                ws.numel() if ws is not None else 0, _stream(stream)))


def mst_mask_update_from_scores(layer: Layer, G, target_density: float, zeta: float, rand_ratio: float,
                                rng_seed: int, ws, stream=None) -> dict:
    st = UpdateStats()
    _check("mst_mask_update_from_scores",
           lib().mst_mask_update_from_scores(layer.h, _ptr(G), target_density, zeta, rand_ratio, rng_seed,
                                             _ptr(ws), ws.numel(), C.byref(st), _stream(stream)))
    return st.as_dict()


def mst_mask_update_from_scores_multi(layers, G, target_density, zeta: float, rand_ratio: float, rng_seed, ws,
                                      streams) -> list:
    """One native call for several layers, layer j on streams[j] (arrays marshalled here, nothing else)."""
    n = len(layers)
    hs = (C.c_void_p * n)(*[L.h.value for L in layers])
    gs = (C.c_void_p * n)(*[_ptr(g) for g in G])
    ds = (C.c_double * n)(*[float(d) for d in target_density])
    seeds = (C.c_uint64 * n)(*[int(x) for x in rng_seed])
    wss = (C.c_void_p * n)(*[_ptr(w) for w in ws])
    wbs = (C.c_size_t * n)(*[w.numel() for w in ws])
    sts = (UpdateStats * n)()
    ss = (C.c_void_p * n)(*[_stream(x) for x in streams])
    _check("mst_mask_update_from_scores_multi",
           lib().mst_mask_update_from_scores_multi(n, hs, gs, ds, zeta, rand_ratio, seeds, wss, wbs, sts, ss))
    return [st.as_dict() for st in sts]


def mst_mask_update(layer: Layer, dY, X, T: int, target_density: float, zeta: float, rand_ratio: float,
                    rng_seed: int, ws, act: int = MST_F32, stream=None) -> dict:
    st = UpdateStats()
    _check("mst_mask_update",
           lib().mst_mask_update(layer.h, _ptr(dY), _ptr(X), T, act, target_density, zeta, rand_ratio, rng_seed,
                                 _ptr(ws), ws.numel(), C.byref(st), _stream(stream)))
    return st.as_dict()


def mst_sparse_fc_bwd_weight_update(layer: Layer, dY, X, dW, T: int, target_density: float, zeta: float,
                                    rand_ratio: float, rng_seed: int, ws, act: int = MST_F32, stream=None) -> dict:
    st = UpdateStats()
    _check("mst_sparse_fc_bwd_weight_update",
           lib().mst_sparse_fc_bwd_weight_update(layer.h, _ptr(dY), _ptr(X), _ptr(dW), T, act, target_density, zeta,
                                                 rand_ratio, rng_seed, _ptr(ws), ws.numel(), C.byref(st),
                                                 _stream(stream)))
    return st.as_dict()


def _shape_arrays(shapes):
    n = len(shapes)
    O = (C.c_int * max(n, 1))(*[int(o) for o, _ in shapes])
    I = (C.c_int * max(n, 1))(*[int(i) for _, i in shapes])
    return n, O, I


def mst_erdos_renyi_density(shapes, global_density: float):
    """shapes = [(O_l, I_l)] -> per-layer densities."""
    n, O, I = _shape_arrays(shapes)
    out = (C.c_double * max(n, 1))()
    _check("mst_erdos_renyi_density", lib().mst_erdos_renyi_density(n, O, I, float(global_density), out))
    return [float(out[l]) for l in range(n)]


def mst_flops_fc_forward(shapes, density) -> float:
    n, O, I = _shape_arrays(shapes)
    if len(density) != n:
        raise ValueError("one density per layer")
    d = (C.c_double * max(n, 1))(*[float(x) for x in density])
    out = C.c_double(0.0)
    _check("mst_flops_fc_forward", lib().mst_flops_fc_forward(n, O, I, d, C.byref(out)))
    return float(out.value)


def mst_flops_transformer(L: int, N_embd: int, D_ffw: int, D_vocab: int, n_layers: int, density: float,
                          q_atten: float) -> dict:
    shape = TransformerShape(int(L), int(N_embd), int(D_ffw), int(D_vocab), int(n_layers))
    out = TransformerFlops()
    _check("mst_flops_transformer", lib().mst_flops_transformer(C.byref(shape), float(density), float(q_atten),
                                                                 C.byref(out)))
    return out.as_dict()


def mst_strided_attention_mask(M, L: int, stride: int, stream=None):
    """M: uint8 device tensor of L * L elements."""
    _check("mst_strided_attention_mask", lib().mst_strided_attention_mask(_ptr(M), int(L), int(stride), _stream(stream)))


def mst_strided_attention_count(L: int, stride: int) -> int:
    out = C.c_int64(0)
    _check("mst_strided_attention_count", lib().mst_strided_attention_count(int(L), int(stride), C.byref(out)))
    return int(out.value)
