"""ctypes binding of libcham (argument marshalling only; every step runs in the HIP kernels).

PyTorch is used for device memory and the current stream, nothing else.  The functions carry
the names of the C entry points declared in ``include/cham.h``.  There is no CPU fallback:
if the library is not built, or no GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcham.so")

F_FORCE_EXACT, F_STREAMING, F_RESIDENT, F_NO_MFMA = 1, 2, 4, 8
F_VALUES_BELOW_2048 = 16
OUT_EMPTY, OUT_KEPT, OUT_SYNTH, OUT_DROPPED = 0, 1, 2, 3

EXPORTS = [
    "cham_version", "cham_strerror", "cham_last_hip_error", "cham_sweep_workspace_bytes",
    "cham_kmeans_sweep", "cham_select_k", "cham_select_k_host", "cham_snap_workspace_bytes",
    "cham_snap_centroids", "cham_synth_workspace_bytes", "cham_synthesize", "cham_hash_config",
    "cham_hash_rows", "cham_sweep_knee_workspace_bytes", "cham_kmeans_sweep_knee", "cham_synthesize_table",
    "cham_visited_table_clear", "cham_visited_table_insert_hashes", "cham_visited_table_insert_configs",
    "cham_update_configs", "cham_sweep_path", "cham_sweep_path_kernel", "cham_sweep_passes",
    "cham_static_init", "cham_kmeans_sweep_static",
    "cham_sweep_workspace_bytes_u16", "cham_sweep_path_u16", "cham_kmeans_sweep_u16", "cham_sweep_knee_workspace_bytes_u16",
    "cham_kmeans_sweep_knee_u16", "cham_snap_workspace_bytes_u16", "cham_snap_centroids_u16",
    "cham_synth_workspace_bytes_u16", "cham_synthesize_u16", "cham_synthesize_table_u16",
    "cham_visited_table_insert_configs_u16", "cham_hash_config_u16", "cham_hash_rows_u16",
]


class ChamError(RuntimeError):
    pass


_lib = None


def load() -> C.CDLL:
    """Load libcham.so (built in-tree by ``build.build_lib``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ChamError(f"{LIB_PATH} is not built; run `python -m paper_2001_08743_amd.build`")
        # PyTorch ships its own copy of the HIP runtime: it has to be in the process first, so that the
        # library binds to that same runtime (its kernels then see the device and streams torch uses).
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = C.CDLL(LIB_PATH)
        vp, i32, i64, u64, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_double
        lib.cham_version.restype = i32
        lib.cham_strerror.restype = C.c_char_p
        lib.cham_strerror.argtypes = [i32]
        lib.cham_last_hip_error.restype = i32
        lib.cham_sweep_workspace_bytes.restype = i64
        lib.cham_sweep_workspace_bytes.argtypes = [i64, i32, vp, i32, vp, i32, i32, i32]
        lib.cham_kmeans_sweep.restype = i32
        lib.cham_kmeans_sweep.argtypes = [vp, i64, i32, vp, i32, vp, i32, i32, i32, vp,
                                          vp, vp, vp, vp, vp, vp, vp, i64, i32, vp]
        lib.cham_sweep_path.restype = i32
        lib.cham_sweep_path.argtypes = [i64, i32, vp, i32, vp, i32, i32]
        lib.cham_sweep_path_u16.restype = i32
        lib.cham_sweep_path_u16.argtypes = [i64, i32, vp, i32, vp, i32, i32]
        lib.cham_sweep_path_kernel.restype = C.c_char_p
        lib.cham_sweep_path_kernel.argtypes = [i32]
        lib.cham_sweep_passes.restype = i32
        lib.cham_sweep_passes.argtypes = [vp, i64, i64, i32, vp, i32, vp, i32, i32, vp, vp]
        lib.cham_static_init.restype = i32
        lib.cham_static_init.argtypes = []
        lib.cham_kmeans_sweep_static.restype = i32
        lib.cham_kmeans_sweep_static.argtypes = [vp, i64, i32, vp, i32, vp, i32, i32, i32, vp,
                                                 vp, vp, vp, vp, vp, vp, i32, vp]
        lib.cham_sweep_knee_workspace_bytes.restype = i64
        lib.cham_sweep_knee_workspace_bytes.argtypes = [i64, i32, vp, i32, vp, i32, i32, i32]
        lib.cham_kmeans_sweep_knee.restype = i32
        lib.cham_kmeans_sweep_knee.argtypes = [vp, i64, i32, vp, i32, vp, i32, i32, i32, vp, f64, i32,
                                               vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, vp]
        lib.cham_synthesize_table.restype = i32
        lib.cham_synthesize_table.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp, i64, vp,
                                              vp, vp, vp, vp, i64, vp]
        lib.cham_visited_table_clear.restype = i32
        lib.cham_visited_table_clear.argtypes = [vp, i64, vp]
        lib.cham_visited_table_insert_hashes.restype = i32
        lib.cham_visited_table_insert_hashes.argtypes = [vp, i64, vp, i64, vp, vp]
        lib.cham_visited_table_insert_configs.restype = i32
        lib.cham_visited_table_insert_configs.argtypes = [vp, i64, vp, i64, i32, vp, vp, i64, vp, vp]
        lib.cham_update_configs.restype = i32
        lib.cham_update_configs.argtypes = [vp, vp, i64, i32, i32, vp, u64, vp, i64, vp, i64, vp, vp, vp]
        lib.cham_select_k.restype = i32
        lib.cham_select_k.argtypes = [vp, vp, i32, i32, f64, vp, vp]
        lib.cham_select_k_host.restype = i32
        lib.cham_select_k_host.argtypes = [vp, vp, i32, f64]
        lib.cham_snap_workspace_bytes.restype = i64
        lib.cham_snap_workspace_bytes.argtypes = [i64, i32, vp, i32, vp, i32]
        lib.cham_snap_centroids.restype = i32
        lib.cham_snap_centroids.argtypes = [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, i64, i32, vp]
        lib.cham_synth_workspace_bytes.restype = i64
        lib.cham_synth_workspace_bytes.argtypes = [i64, i32, vp, i32, vp, i32]
        lib.cham_synthesize.restype = i32
        lib.cham_synthesize.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp, i64, vp,
                                        vp, vp, vp, vp, i64, vp]
        lib.cham_hash_config.restype = u64
        lib.cham_hash_config.argtypes = [vp, i32, u64]
        lib.cham_hash_rows.restype = i32
        lib.cham_hash_rows.argtypes = [vp, i64, i32, vp, u64, vp, vp]
        # the entry points for two-byte knobs take the same argument lists
        for name in EXPORTS:
            if name.endswith("_u16"):
                base = getattr(lib, name[:-4])
                getattr(lib, name).restype = base.restype
                getattr(lib, name).argtypes = base.argtypes
        _lib = lib
    return _lib


def _knob_dtypes(sfx: str):
    """(numpy dtype of host rows, torch dtype of device knob buffers) for an entry-point suffix.
    Two-byte knobs live in int16 tensors (same bits as uint16)."""
    torch = _torch()
    return (np.uint8, torch.uint8) if sfx == "" else (np.uint16, torch.int16)


def knobs_to_host(t) -> np.ndarray:
    """Device knob tensor (uint8, or int16 holding uint16 bits) as a numpy array of unsigned values."""
    a = t.cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def _check(rc: int):
    if rc < 0:
        lib = load()
        msg = lib.cham_strerror(int(rc)).decode()
        raise ChamError(f"libcham error {rc}: {msg} (hip error {lib.cham_last_hip_error()})")
    return rc


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise ChamError("no GPU visible: libcham has no CPU path")
    return torch


def _hp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dp(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    torch = _torch()
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _host_lists(task_off, ks):
    to = np.ascontiguousarray(task_off, dtype=np.int64)
    k = np.ascontiguousarray(ks, dtype=np.int32)
    return to, k


def to_soa(rows: np.ndarray, device="cuda:0", pad_to: int = 64):
    """Upload row-major rows [N, d] (uint8, or uint16 for two-byte knobs) as the structure-of-arrays
    matrix X [d, ld] the library reads."""
    torch = _torch()
    dt = np.uint16 if np.asarray(rows).dtype == np.uint16 else np.uint8
    rows = np.ascontiguousarray(rows, dtype=dt)
    n, d = rows.shape
    ld = max(pad_to, (n + pad_to - 1) // pad_to * pad_to)
    host = np.zeros((d, ld), dtype=dt)
    host[:, :n] = rows.T
    if dt == np.uint16:
        host = host.view(np.int16)
    return torch.from_numpy(host).to(device), ld


def cham_version() -> int:
    return int(load().cham_version())


def cham_hash_config(cfg, salt: int = 0) -> int:
    cfg = np.ascontiguousarray(cfg, dtype=np.uint8)
    return int(load().cham_hash_config(_hp(cfg), C.c_int32(cfg.shape[0]), C.c_uint64(int(salt))))


def cham_hash_config_u16(cfg, salt: int = 0) -> int:
    cfg = np.ascontiguousarray(cfg, dtype=np.uint16)
    return int(load().cham_hash_config_u16(_hp(cfg), C.c_int32(cfg.shape[0]), C.c_uint64(int(salt))))


def cham_select_k_host(curve, status=None, threshold: float = 2.5) -> int:
    curve = np.ascontiguousarray(curve, dtype=np.float64)
    st = None if status is None else np.ascontiguousarray(status, dtype=np.int32)
    return int(load().cham_select_k_host(_hp(curve), _hp(st), C.c_int32(len(curve)), C.c_double(threshold)))


def cham_hash_rows(rows_dev, salts_dev=None, salt_all: int = 0, _sfx: str = ""):
    """rows_dev: device uint8 [n, d] row-major; salts_dev: device int64/uint64 [n] or None."""
    torch = _torch()
    assert rows_dev.dtype == _knob_dtypes(_sfx)[1]
    n, d = rows_dev.shape
    out = torch.empty(n, dtype=torch.int64, device=rows_dev.device)
    _check(getattr(load(), "cham_hash_rows" + _sfx)(_dp(rows_dev), C.c_int64(n), C.c_int32(d), _dp(salts_dev),
                                                    C.c_uint64(int(salt_all)), _dp(out), _stream()))
    return out


def cham_hash_rows_u16(rows_dev, salts_dev=None, salt_all: int = 0):
    """rows_dev: device int16 tensor [n, d] holding uint16 knob values, row-major."""
    return cham_hash_rows(rows_dev, salts_dev, salt_all, _sfx="_u16")


def cham_sweep_workspace_bytes(ld, d, task_off, ks, n_iter, flags=0, _sfx: str = "") -> int:
    to, k = _host_lists(task_off, ks)
    fn = getattr(load(), "cham_sweep_workspace_bytes" + _sfx)
    return _check(fn(C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(len(to) - 1),
                     _hp(k), C.c_int32(len(k)), C.c_int32(n_iter), C.c_int32(flags)))


def cham_sweep_knee_workspace_bytes(ld, d, task_off, ks, n_iter, flags=0, _sfx: str = "") -> int:
    to, k = _host_lists(task_off, ks)
    fn = getattr(load(), "cham_sweep_knee_workspace_bytes" + _sfx)
    return _check(fn(C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(len(to) - 1), _hp(k), C.c_int32(len(k)),
                     C.c_int32(n_iter), C.c_int32(flags)))


def cham_sweep_workspace_bytes_u16(ld, d, task_off, ks, n_iter, flags=0) -> int:
    return cham_sweep_workspace_bytes(ld, d, task_off, ks, n_iter, flags, _sfx="_u16")


def cham_sweep_knee_workspace_bytes_u16(ld, d, task_off, ks, n_iter, flags=0) -> int:
    return cham_sweep_knee_workspace_bytes(ld, d, task_off, ks, n_iter, flags, _sfx="_u16")


def cham_kmeans_sweep(X, ld: int, d: int, task_off, ks: Sequence[int], n_iter: int, init_centroids=None,
                      want_labels: bool = False, want_trace: bool = False, flags: int = 0,
                      out: Optional[dict] = None, workspace=None, _sfx: str = ""):
    """Run the sweep; returns a dict of device tensors (centroids, counts, inertia, status, labels, trace)."""
    torch = _torch()
    lib = load()
    assert X.dtype == _knob_dtypes(_sfx)[1]
    to, k = _host_lists(task_off, ks)
    T, n_k, Ksum = len(to) - 1, len(k), int(k.sum())
    dev = X.device
    if out is None:
        out = {}
        out["centroids"] = torch.empty((T, Ksum, d), dtype=torch.float64, device=dev)
        out["counts"] = torch.empty((T, Ksum), dtype=torch.int32, device=dev)
        out["inertia"] = torch.empty((T, n_k), dtype=torch.float64, device=dev)
        out["status"] = torch.empty((T, n_k), dtype=torch.int32, device=dev)
        out["labels"] = torch.zeros((n_k, ld), dtype=torch.uint8, device=dev) if want_labels else None
        out["trace"] = torch.empty((T, n_k, n_iter + 1), dtype=torch.float64, device=dev) if want_trace else None
    if workspace is None:
        nbytes = cham_sweep_workspace_bytes(ld, d, to, k, n_iter, flags, _sfx=_sfx)
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    rc = getattr(lib, "cham_kmeans_sweep" + _sfx)(_dp(X), C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(T), _hp(k), C.c_int32(n_k),
                               C.c_int32(n_iter), C.c_int32(0 if init_centroids is None else 1),
                               _dp(init_centroids), _dp(out["centroids"]), _dp(out["counts"]),
                               _dp(out["inertia"]), _dp(out["status"]), _dp(out.get("labels")),
                               _dp(out.get("trace")), _dp(workspace), C.c_int64(workspace.numel()),
                               C.c_int32(flags), _stream())
    _check(rc)
    out["workspace"] = workspace
    out["koff"] = np.concatenate([[0], np.cumsum(k)]).astype(np.int64)
    return out


def cham_sweep_path(ld: int, d: int, task_off, ks, flags: int = 0, _sfx: str = "") -> int:
    to, k = _host_lists(task_off, ks)
    return _check(getattr(load(), "cham_sweep_path" + _sfx)(C.c_int64(ld), C.c_int32(d), _hp(to),
                                                            C.c_int32(len(to) - 1), _hp(k), C.c_int32(len(k)),
                                                            C.c_int32(flags)))


def cham_sweep_path_u16(ld: int, d: int, task_off, ks, flags: int = 0) -> int:
    return cham_sweep_path(ld, d, task_off, ks, flags, _sfx="_u16")


def cham_sweep_path_kernel(path: int) -> str:
    return load().cham_sweep_path_kernel(C.c_int32(path)).decode()


def cham_sweep_passes(workspace, ld: int, d: int, task_off, ks, flags: int = 0, passes=None):
    """Labelling passes per (task, k) that the last sweep using ``workspace`` ran; device int32 [T, n_k]."""
    torch = _torch()
    to, k = _host_lists(task_off, ks)
    T, n_k = len(to) - 1, len(k)
    if passes is None:
        passes = torch.empty((T, n_k), dtype=torch.int32, device=workspace.device)
    _check(load().cham_sweep_passes(_dp(workspace), C.c_int64(workspace.numel()), C.c_int64(ld), C.c_int32(d),
                                    _hp(to), C.c_int32(T), _hp(k), C.c_int32(n_k), C.c_int32(flags), _dp(passes),
                                    _stream()))
    return passes


def cham_static_init() -> None:
    _torch()
    _check(load().cham_static_init())


def cham_kmeans_sweep_static(X, ld: int, d: int, task_off, ks: Sequence[int], n_iter: int, out: dict,
                             init_centroids=None, flags: int = 0):
    """cham_kmeans_sweep on the library's static scratch buffer; ``out`` holds the caller's output tensors
    (centroids, counts, inertia, status and optionally labels, trace).  Nothing is allocated here."""
    to, k = _host_lists(task_off, ks)
    rc = load().cham_kmeans_sweep_static(_dp(X), C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(len(to) - 1), _hp(k),
                                         C.c_int32(len(k)), C.c_int32(n_iter),
                                         C.c_int32(0 if init_centroids is None else 1), _dp(init_centroids),
                                         _dp(out["centroids"]), _dp(out["counts"]), _dp(out["inertia"]),
                                         _dp(out["status"]), _dp(out.get("labels")), _dp(out.get("trace")),
                                         C.c_int32(flags), _stream())
    _check(rc)
    return out


def cham_kmeans_sweep_u16(X, ld: int, d: int, task_off, ks: Sequence[int], n_iter: int, **kw):
    """cham_kmeans_sweep for two-byte knobs: X is a device int16 tensor [d, ld] holding uint16 values."""
    return cham_kmeans_sweep(X, ld, d, task_off, ks, n_iter, _sfx="_u16", **kw)


def cham_kmeans_sweep_knee(X, ld: int, d: int, task_off, ks: Sequence[int], n_iter: int, threshold: float = 2.5,
                           chunk: int = 8, init_centroids=None, want_labels: bool = False,
                           want_trace: bool = False, flags: int = 0, out: Optional[dict] = None, workspace=None,
                           _sfx: str = ""):
    """Run the sweep in chunks and stop every task at its knee; returns the same dict plus ``chosen``."""
    torch = _torch()
    lib = load()
    assert X.dtype == _knob_dtypes(_sfx)[1]
    to, k = _host_lists(task_off, ks)
    T, n_k, Ksum = len(to) - 1, len(k), int(k.sum())
    dev = X.device
    if out is None:
        out = {}
        out["centroids"] = torch.empty((T, Ksum, d), dtype=torch.float64, device=dev)
        out["counts"] = torch.empty((T, Ksum), dtype=torch.int32, device=dev)
        out["inertia"] = torch.empty((T, n_k), dtype=torch.float64, device=dev)
        out["status"] = torch.empty((T, n_k), dtype=torch.int32, device=dev)
        out["chosen"] = torch.empty(T, dtype=torch.int32, device=dev)
        out["labels"] = torch.zeros((n_k, ld), dtype=torch.uint8, device=dev) if want_labels else None
        out["trace"] = torch.empty((T, n_k, n_iter + 1), dtype=torch.float64, device=dev) if want_trace else None
    if workspace is None:
        nbytes = cham_sweep_knee_workspace_bytes(ld, d, to, k, n_iter, flags, _sfx=_sfx)
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    rc = getattr(lib, "cham_kmeans_sweep_knee" + _sfx)(_dp(X), C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(T), _hp(k),
                                    C.c_int32(n_k), C.c_int32(n_iter), C.c_int32(0 if init_centroids is None else 1),
                                    _dp(init_centroids), C.c_double(threshold), C.c_int32(chunk),
                                    _dp(out["centroids"]), _dp(out["counts"]), _dp(out["inertia"]),
                                    _dp(out["status"]), _dp(out["chosen"]), _dp(out.get("labels")),
                                    _dp(out.get("trace")), _dp(workspace), C.c_int64(workspace.numel()),
                                    C.c_int32(flags), _stream())
    _check(rc)
    out["workspace"] = workspace
    out["koff"] = np.concatenate([[0], np.cumsum(k)]).astype(np.int64)
    return out


def cham_kmeans_sweep_knee_u16(X, ld: int, d: int, task_off, ks: Sequence[int], n_iter: int, **kw):
    return cham_kmeans_sweep_knee(X, ld, d, task_off, ks, n_iter, _sfx="_u16", **kw)


def cham_select_k(inertia, status, threshold: float = 2.5, chosen=None):
    torch = _torch()
    T, n_k = inertia.shape
    if chosen is None:
        chosen = torch.empty(T, dtype=torch.int32, device=inertia.device)
    _check(load().cham_select_k(_dp(inertia), _dp(status), C.c_int32(T), C.c_int32(n_k), C.c_double(threshold),
                                _dp(chosen), _stream()))
    return chosen


def cham_snap_centroids(X, ld: int, d: int, task_off, ks, chosen_idx, centroids, flags: int = 0,
                        out: Optional[dict] = None, workspace=None, _sfx: str = ""):
    torch = _torch()
    assert X.dtype == _knob_dtypes(_sfx)[1]
    to, k = _host_lists(task_off, ks)
    T, n_k, kmax = len(to) - 1, len(k), int(k[-1])
    dev = X.device
    if out is None:
        out = dict(labels_sel=torch.zeros(ld, dtype=torch.uint8, device=dev),
                   pick_row=torch.empty((T, kmax), dtype=torch.int32, device=dev),
                   pick_cfg=torch.empty((T, kmax, d), dtype=_knob_dtypes(_sfx)[1], device=dev))
    if workspace is None:
        nbytes = _check(getattr(load(), "cham_snap_workspace_bytes" + _sfx)(
            C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(T), _hp(k), C.c_int32(n_k)))
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    _check(getattr(load(), "cham_snap_centroids" + _sfx)(_dp(X), C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(T), _hp(k),
                                      C.c_int32(n_k), _dp(chosen_idx), _dp(centroids), _dp(out["labels_sel"]),
                                      _dp(out["pick_row"]), _dp(out["pick_cfg"]), _dp(workspace),
                                      C.c_int64(workspace.numel()), C.c_int32(flags), _stream()))
    out["workspace"] = workspace
    return out


def cham_snap_centroids_u16(X, ld: int, d: int, task_off, ks, chosen_idx, centroids, **kw):
    return cham_snap_centroids(X, ld, d, task_off, ks, chosen_idx, centroids, _sfx="_u16", **kw)


def cham_synthesize(X, ld: int, d: int, task_off, cards, valid, ks, chosen_idx, labels_sel, pick_row, pick_cfg,
                    visited, task_salt=None, out: Optional[dict] = None, workspace=None, _sfx: str = ""):
    """visited: device int64/uint64 tensor, sorted ascending as unsigned 64-bit words."""
    torch = _torch()
    assert X.dtype == _knob_dtypes(_sfx)[1] and pick_cfg.dtype == X.dtype
    to, k = _host_lists(task_off, ks)
    T, n_k, kmax = len(to) - 1, len(k), int(k[-1])
    cards = np.ascontiguousarray(cards, dtype=np.uint16).reshape(T, d)
    salts = None if task_salt is None else np.ascontiguousarray(task_salt, dtype=np.uint64)
    dev = X.device
    if out is None:
        out = dict(out_cfg=torch.empty((T, kmax, d), dtype=_knob_dtypes(_sfx)[1], device=dev),
                   out_flag=torch.empty((T, kmax), dtype=torch.uint8, device=dev),
                   out_count=torch.empty(T, dtype=torch.int32, device=dev))
    if workspace is None:
        nbytes = _check(getattr(load(), "cham_synth_workspace_bytes" + _sfx)(
            C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(T), _hp(k), C.c_int32(n_k)))
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    n_vis = 0 if visited is None else int(visited.numel())
    _check(getattr(load(), "cham_synthesize" + _sfx)(_dp(X), C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(T), _hp(cards),
                                  _dp(valid), _hp(k), C.c_int32(n_k), _dp(chosen_idx), _dp(labels_sel),
                                  _dp(pick_row), _dp(pick_cfg), _dp(visited) if n_vis else None,
                                  C.c_int64(n_vis), _hp(salts), _dp(out["out_cfg"]), _dp(out["out_flag"]),
                                  _dp(out["out_count"]), _dp(workspace), C.c_int64(workspace.numel()), _stream()))
    out["workspace"] = workspace
    return out


def cham_synthesize_u16(X, ld: int, d: int, task_off, cards, valid, ks, chosen_idx, labels_sel, pick_row,
                        pick_cfg, visited, **kw):
    return cham_synthesize(X, ld, d, task_off, cards, valid, ks, chosen_idx, labels_sel, pick_row, pick_cfg,
                           visited, _sfx="_u16", **kw)


def cham_synthesize_table(X, ld: int, d: int, task_off, cards, valid, ks, chosen_idx, labels_sel, pick_row,
                          pick_cfg, table, task_salt=None, out: Optional[dict] = None, workspace=None,
                          _sfx: str = ""):
    """cham_synthesize with the visited set held in a device table (int64/uint64 tensor of 2^m slots)."""
    torch = _torch()
    assert X.dtype == _knob_dtypes(_sfx)[1] and pick_cfg.dtype == X.dtype
    to, k = _host_lists(task_off, ks)
    T, n_k, kmax = len(to) - 1, len(k), int(k[-1])
    cards = np.ascontiguousarray(cards, dtype=np.uint16).reshape(T, d)
    salts = None if task_salt is None else np.ascontiguousarray(task_salt, dtype=np.uint64)
    dev = X.device
    if out is None:
        out = dict(out_cfg=torch.empty((T, kmax, d), dtype=_knob_dtypes(_sfx)[1], device=dev),
                   out_flag=torch.empty((T, kmax), dtype=torch.uint8, device=dev),
                   out_count=torch.empty(T, dtype=torch.int32, device=dev))
    if workspace is None:
        nbytes = _check(getattr(load(), "cham_synth_workspace_bytes" + _sfx)(
            C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(T), _hp(k), C.c_int32(n_k)))
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    _check(getattr(load(), "cham_synthesize_table" + _sfx)(_dp(X), C.c_int64(ld), C.c_int32(d), _hp(to), C.c_int32(T), _hp(cards),
                                        _dp(valid), _hp(k), C.c_int32(n_k), _dp(chosen_idx), _dp(labels_sel),
                                        _dp(pick_row), _dp(pick_cfg), _dp(table), C.c_int64(table.numel()),
                                        _hp(salts), _dp(out["out_cfg"]), _dp(out["out_flag"]),
                                        _dp(out["out_count"]), _dp(workspace), C.c_int64(workspace.numel()),
                                        _stream()))
    out["workspace"] = workspace
    return out


def cham_synthesize_table_u16(X, ld: int, d: int, task_off, cards, valid, ks, chosen_idx, labels_sel, pick_row,
                              pick_cfg, table, **kw):
    return cham_synthesize_table(X, ld, d, task_off, cards, valid, ks, chosen_idx, labels_sel, pick_row, pick_cfg,
                                 table, _sfx="_u16", **kw)


def cham_visited_table_clear(table):
    _check(load().cham_visited_table_clear(_dp(table), C.c_int64(table.numel()), _stream()))
    return table


def cham_visited_table_insert_hashes(table, hashes, overflow=None):
    _check(load().cham_visited_table_insert_hashes(_dp(table), C.c_int64(table.numel()), _dp(hashes),
                                                   C.c_int64(hashes.numel()), _dp(overflow), _stream()))


def cham_visited_table_insert_configs_u16(table, cfgs, d: int, **kw):
    return cham_visited_table_insert_configs(table, cfgs, d, _sfx="_u16", **kw)


def cham_visited_table_insert_configs(table, cfgs, d: int, flags=None, salts=None, rows_per_salt: int = 1,
                                      overflow=None, _sfx: str = ""):
    assert cfgs.dtype == _knob_dtypes(_sfx)[1]
    n = cfgs.numel() // d
    _check(getattr(load(), "cham_visited_table_insert_configs" + _sfx)(_dp(table), C.c_int64(table.numel()), _dp(cfgs), C.c_int64(n),
                                                    C.c_int32(d), _dp(flags), _dp(salts), C.c_int64(rows_per_salt),
                                                    _dp(overflow), _stream()))


def cham_update_configs(theta, actions, cards, salt: int = 0, seen_table=None, unique_rows=None, n_unique=None,
                        overflow=None):
    """theta [B][d] uint8 (in place), actions [S][B][d] int8, cards [d] (device int16/uint16 tensor)."""
    B, d = theta.shape
    n_steps = actions.shape[0] if actions.dim() == 3 else 1
    _check(load().cham_update_configs(_dp(theta), _dp(actions), C.c_int64(B), C.c_int32(d), C.c_int32(n_steps),
                                      _dp(cards), C.c_uint64(salt), _dp(seen_table),
                                      C.c_int64(0 if seen_table is None else seen_table.numel()), _dp(unique_rows),
                                      C.c_int64(0 if unique_rows is None else unique_rows.shape[0]), _dp(n_unique),
                                      _dp(overflow), _stream()))
    return theta


class DeviceWorkload:
    """A workload's inputs resident on the GPU, plus a driver for the whole path."""

    def __init__(self, wl, device="cuda:0"):
        torch = _torch()
        self.wl = wl
        self.device = device
        self.X, self.ld = to_soa(wl.rows, device)
        self.sfx = "_u16" if wl.rows.dtype == np.uint16 else ""      # which family of entry points
        self.d = wl.d
        v = np.zeros(self.ld, dtype=np.uint8)
        v[:wl.n_total] = wl.valid
        self.valid = torch.from_numpy(v).to(device)
        self.visited = None

    def build_visited(self):
        """Hash the visited configurations on the device and sort them (input preparation)."""
        torch = _torch()
        from . import workloads
        wl = self.wl
        if len(wl.visited_cfg):
            host = np.ascontiguousarray(wl.visited_cfg)
            rows = torch.from_numpy(host.view(np.int16) if self.sfx else host).to(self.device)
            salts = torch.from_numpy(wl.salts[wl.visited_task].astype(np.int64)).to(self.device)
            h = cham_hash_rows(rows, salts, _sfx=self.sfx).cpu().numpy().view(np.uint64)
        else:
            h = np.zeros(0, dtype=np.uint64)
        arr = workloads.finalize_visited(h, wl.visited_raw, wl.n_visited)
        self.visited_host = arr
        self.visited = torch.from_numpy(arr.view(np.int64).copy()).to(self.device)
        return self.visited

    def run(self, threshold: Optional[float] = None, flags: int = 0, want_labels: bool = False,
            want_trace: bool = False, bufs: Optional[dict] = None):
        """sweep -> select -> snap -> synthesize on the current stream; no host synchronisation."""
        wl = self.wl
        thr = wl.threshold if threshold is None else threshold
        if self.visited is None:
            self.build_visited()
        b = bufs or {}
        # two-byte knobs: cardinalities of at most 2048 are the caller's promise of values below 2048
        sweep_flags = flags | (F_VALUES_BELOW_2048 if self.sfx and int(np.max(wl.cards)) <= 2048 else 0)
        sw = cham_kmeans_sweep(self.X, self.ld, self.d, wl.task_off, wl.ks, wl.n_iter, flags=sweep_flags,
                               want_labels=want_labels, want_trace=want_trace,
                               out=b.get("sweep"), workspace=b.get("sweep_ws"), _sfx=self.sfx)
        chosen = cham_select_k(sw["inertia"], sw["status"], thr, chosen=b.get("chosen"))
        sn = cham_snap_centroids(self.X, self.ld, self.d, wl.task_off, wl.ks, chosen, sw["centroids"],
                                 flags=flags, out=b.get("snap"), workspace=b.get("snap_ws"), _sfx=self.sfx)
        sy = cham_synthesize(self.X, self.ld, self.d, wl.task_off, wl.cards, self.valid, wl.ks, chosen,
                             sn["labels_sel"], sn["pick_row"], sn["pick_cfg"], self.visited,
                             task_salt=wl.salts, out=b.get("synth"), workspace=b.get("synth_ws"), _sfx=self.sfx)
        return dict(sweep=sw, chosen=chosen, snap=sn, synth=sy)
