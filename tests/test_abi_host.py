"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
public header declares, rejects bad arguments before touching the device, and its host-side
helpers follow the paper's rules."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2001_08743_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2001_08743_amd import build
        build.build_lib()
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cham.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cham_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert "cham_kmeans_sweep" in names and "cham_synthesize" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_version_and_strerror(lib):
    assert lib.cham_version() >= 100
    assert lib.cham_strerror(0) == b"ok"
    for code in range(-10, 0):
        assert len(lib.cham_strerror(code)) > 3


def test_knee_rule_on_host(lib):
    # Algorithm 1: previous_loss starts at infinity; stop at the first k with thr*loss >= previous
    assert binding.cham_select_k_host([100, 30, 20, 19], None, 2.5) == 2
    assert binding.cham_select_k_host([100, 50], None, 2.0) == 1
    assert binding.cham_select_k_host([81, 27, 9, 3], None, 2.5) == 3
    assert binding.cham_select_k_host([5.0], None, 2.5) == 0
    assert binding.cham_select_k_host([100, 0, 30, 20], [0, 1, 0, 0], 2.5) == 3
    assert binding.cham_select_k_host([0, 0], [1, 1], 2.5) == -1


def test_host_hash_matches_published_fnv1a_vectors(lib, golden_dir):
    for line in open(os.path.join(golden_dir, "fnv1a64_vectors.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        s, digest = line.split()
        data = b"" if s == "EMPTY" else s.encode()
        cfg = np.frombuffer(data, dtype=np.uint8) if data else np.zeros(0, np.uint8)
        assert binding.cham_hash_config(cfg, 0) == int(digest, 16)


def _sweep_rc(lib, X=1024, ld=64, d=4, task_off=(0, 10), ks=(1, 2), n_iter=1, init_mode=0, ws=4096, ws_bytes=1 << 20,
              flags=0, outs=4096, fn="cham_kmeans_sweep"):
    to = np.asarray(task_off, dtype=np.int64)
    k = np.asarray(ks, dtype=np.int32)
    vp = C.c_void_p
    return getattr(lib, fn)(vp(X), C.c_int64(ld), C.c_int32(d), to.ctypes.data_as(vp), C.c_int32(len(to) - 1),
                                 k.ctypes.data_as(vp), C.c_int32(len(k)), C.c_int32(n_iter), C.c_int32(init_mode),
                                 None, vp(outs), vp(outs), vp(outs), vp(outs), None, None, vp(ws),
                                 C.c_int64(ws_bytes), C.c_int32(flags), None)


def test_argument_errors_are_reported_before_any_device_work(lib):
    # pointers below are fake non-null addresses: every case must be rejected before they are used
    assert _sweep_rc(lib, X=0) == -1                       # null X
    assert _sweep_rc(lib, d=0) == -2
    assert _sweep_rc(lib, d=33) == -2
    assert _sweep_rc(lib, ld=62) == -2                     # ld not a multiple of 4
    assert _sweep_rc(lib, X=1026) == -2                    # misaligned X
    assert _sweep_rc(lib, ld=8, task_off=(0, 10)) == -2    # rows beyond ld
    assert _sweep_rc(lib, ks=(2, 2)) == -3                 # not strictly increasing
    assert _sweep_rc(lib, ks=(0, 2)) == -3
    assert _sweep_rc(lib, ks=(1, 257)) == -3
    assert _sweep_rc(lib, task_off=(0, 10, 5)) == -4       # decreasing offsets
    assert _sweep_rc(lib, task_off=(-4, 10)) == -4
    assert _sweep_rc(lib, n_iter=-1) == -2
    assert _sweep_rc(lib, init_mode=1) == -1               # init centroids missing
    assert _sweep_rc(lib, init_mode=7) == -8
    assert _sweep_rc(lib, flags=1 << 20) == -8
    assert _sweep_rc(lib, outs=0) == -1                    # null outputs
    assert _sweep_rc(lib, ws=0) == -6
    assert _sweep_rc(lib, ws_bytes=16) == -6
    assert _sweep_rc(lib, ws=4100) == -6                   # workspace not 256-byte aligned


def test_workspace_queries(lib):
    n = binding.cham_sweep_workspace_bytes(4096, 12, [0, 4096], list(range(2, 65)), 50)
    assert n >= 63 * 4096 and n % 256 == 0
    with pytest.raises(binding.ChamError):
        binding.cham_sweep_workspace_bytes(4095, 12, [0, 4095], [2, 3], 5)


def test_knee_sweep_workspace_and_argument_errors(lib):
    base = binding.cham_sweep_workspace_bytes(4096, 12, [0, 2048, 4096], list(range(2, 65)), 50)
    knee = binding.cham_sweep_knee_workspace_bytes(4096, 12, [0, 2048, 4096], list(range(2, 65)), 50)
    assert knee >= base + 2 * 4 and knee % 256 == 0
    to = (C.c_int64 * 2)(0, 16)
    ks = (C.c_int32 * 2)(2, 3)
    one = C.c_void_p(256)                                   # non-null, never dereferenced: errors come first
    args = lambda chunk, chosen: lib.cham_kmeans_sweep_knee(one, C.c_int64(16), C.c_int32(4), to, C.c_int32(1), ks,
                                                            C.c_int32(2), C.c_int32(3), C.c_int32(0), None,
                                                            C.c_double(2.5), C.c_int32(chunk), one, one, one, one,
                                                            chosen, None, None, one, C.c_int64(1 << 20),
                                                            C.c_int32(0), None)
    assert args(1, None) == -1                              # missing chosen_idx
    assert args(0, one) == -3                               # chunk < 1


def test_visited_table_argument_errors(lib):
    one = C.c_void_p(256)
    assert lib.cham_visited_table_clear(None, C.c_int64(16), None) == -1
    assert lib.cham_visited_table_clear(one, C.c_int64(12), None) == -2          # not a power of two
    assert lib.cham_visited_table_clear(C.c_void_p(260), C.c_int64(16), None) == -2   # misaligned
    assert lib.cham_visited_table_insert_hashes(one, C.c_int64(16), None, C.c_int64(3), None, None) == -1
    assert lib.cham_visited_table_insert_configs(one, C.c_int64(16), one, C.c_int64(3), C.c_int32(40), None, None,
                                                 C.c_int64(1), None, None) == -2
    assert lib.cham_visited_table_insert_configs(one, C.c_int64(16), one, C.c_int64(3), C.c_int32(4), None, None,
                                                 C.c_int64(0), None, None) == -2


def test_two_byte_knob_argument_errors_and_limits(lib):
    u16 = dict(fn="cham_kmeans_sweep_u16")
    assert _sweep_rc(lib, X=0, **u16) == -1
    assert _sweep_rc(lib, d=65, **u16) == -2
    assert _sweep_rc(lib, X=1028, **u16) == -2                # 4- but not 8-byte aligned
    assert _sweep_rc(lib, ld=62, **u16) == -2
    assert _sweep_rc(lib, ks=(1, 257), **u16) == -3
    assert _sweep_rc(lib, flags=binding.F_STREAMING, **u16) == -8
    assert _sweep_rc(lib, d=64, ks=(2, 126), **u16) == -3     # centroids and sums of 126 x 64 knobs exceed LDS
    assert _sweep_rc(lib, d=64, ks=(2, 125), ws=0, **u16) == -6   # 125 fits: the next check is the workspace
    assert _sweep_rc(lib, d=48, ks=(167,), **u16) == -3
    assert _sweep_rc(lib, d=40, ks=(200,), **u16) == -3
    assert _sweep_rc(lib, d=40, ks=(199,), ws=0, **u16) == -6
    assert _sweep_rc(lib, d=56, ks=(144,), **u16) == -3
    assert _sweep_rc(lib, d=32, ks=(248,), **u16) == -3
    assert _sweep_rc(lib, d=24, ks=(256,), ws=0, **u16) == -6
    # workspace queries follow the same limits
    assert binding.cham_sweep_workspace_bytes_u16(4096, 64, [0, 4096], [2, 125], 5) > 0
    with pytest.raises(binding.ChamError):
        binding.cham_sweep_workspace_bytes_u16(4096, 64, [0, 4096], [2, 126], 5)
    with pytest.raises(binding.ChamError):
        binding.cham_sweep_workspace_bytes(4096, 64, [0, 4096], [2, 3], 5)        # byte knobs stop at 32
    # no f16 copy of the rows in the two-byte workspace
    assert binding.cham_sweep_workspace_bytes_u16(4096, 12, [0, 4096], [2, 3], 5) < \
        binding.cham_sweep_workspace_bytes(4096, 12, [0, 4096], [2, 3], 5)
    one = C.c_void_p(256)
    assert lib.cham_visited_table_insert_configs_u16(one, C.c_int64(16), one, C.c_int64(3), C.c_int32(65), None, None,
                                                     C.c_int64(1), None, None) == -2


def test_two_byte_host_hash_equals_the_byte_hash_below_256_and_takes_whole_values_above(lib):
    rng = np.random.default_rng(4)
    for _ in range(20):
        cfg = rng.integers(0, 256, size=int(rng.integers(1, 40)))
        salt = int(rng.integers(0, 2 ** 40))
        assert binding.cham_hash_config_u16(cfg, salt) == binding.cham_hash_config(cfg, salt)
    M = 1 << 64
    h = 0xCBF29CE484222325
    for v in (300, 65535, 0, 256):
        h = ((h ^ v) * 0x100000001B3) % M
    assert binding.cham_hash_config_u16([300, 65535, 0, 256], 0) == h


def test_sweep_path_query(lib):
    ks64 = list(range(1, 65))
    assert binding.cham_sweep_path(4096, 24, [0, 4096], ks64) == 0            # resident, matrix cores
    assert binding.cham_sweep_path_kernel(0) == "resident_mfma_kernel"
    assert binding.cham_sweep_path(8192, 24, [0, 8192], ks64) == 1            # task too large for one workgroup
    assert binding.cham_sweep_path(4096, 16, [0, 4096], [16, 128]) == 1       # k above 64
    assert binding.cham_sweep_path_kernel(1) == "stream_assign_kernel"
    assert binding.cham_sweep_path(4096, 32, [0, 4096], ks64) == 2            # no spare knob slot
    assert binding.cham_sweep_path(4096, 24, [0, 4096], ks64, flags=binding.F_NO_MFMA) == 2
    assert binding.cham_sweep_path_kernel(2) == "resident_sweep_kernel"
    with pytest.raises(binding.ChamError):
        binding.cham_sweep_path(4096, 24, [0, 4096], [3, 2])


def test_sweep_path_query_for_two_byte_knobs(lib):
    """Sweeps over two-byte knobs run on the vector ALU unless the caller promises values below 2048 and the
    matrix-core kernel's limits hold: d <= 63, and (d <= 31, 4096 rows, k <= 64) or (2048 rows, k <= 32)."""
    P = binding.F_VALUES_BELOW_2048
    ks64, ks32 = list(range(1, 65)), list(range(1, 33))
    path = binding.cham_sweep_path_u16
    assert path(2048, 40, [0, 2048], ks32) == 2                                # no promise
    assert path(2048, 40, [0, 2048], ks32, flags=P) == 0
    assert path(2048, 63, [0, 2048], ks32, flags=P) == 0
    assert path(2048, 64, [0, 2048], ks32, flags=P) == 2                       # no room for the spare slot
    assert path(2048, 40, [0, 2048], ks32 + [33], flags=P) == 2                # k above 32 with more than 31 knobs
    assert path(2112, 40, [0, 2049], ks32, flags=P) == 2                       # task above 2048 rows
    assert path(4096, 31, [0, 4096], ks64, flags=P) == 0
    assert path(4096, 32, [0, 4096], ks64, flags=P) == 2
    assert path(4160, 31, [0, 4097], ks64, flags=P) == 2
    assert path(4096, 16, [0, 4096], [16, 128], flags=P) == 2
    assert path(2048, 40, [0, 2048], ks32, flags=P | binding.F_NO_MFMA) == 2
    assert path(2048, 40, [0, 2048], ks32, flags=P | binding.F_FORCE_EXACT) == 2
    with pytest.raises(binding.ChamError):
        path(2048, 40, [0, 2048], ks32, flags=binding.F_STREAMING)
    with pytest.raises(binding.ChamError):
        path(2048, 64, [0, 2048], [126], flags=P)                               # beyond the vector kernel's LDS
    # the workspace of the promised path holds the f16 copy of the rows: 64 halves a row above 31 knobs, 32 below
    w0 = binding.cham_sweep_workspace_bytes_u16(2048, 40, [0, 2048], ks32, 10)
    w1 = binding.cham_sweep_workspace_bytes_u16(2048, 40, [0, 2048], ks32, 10, flags=P)
    w2 = binding.cham_sweep_workspace_bytes_u16(2048, 24, [0, 2048], ks32, 10, flags=P)
    w3 = binding.cham_sweep_workspace_bytes_u16(2048, 24, [0, 2048], ks32, 10)
    assert w1 - w0 == 2048 * 64 * 2 and w2 - w3 == 2048 * 32 * 2
    # the byte entry points accept and ignore the promise
    assert binding.cham_sweep_path(4096, 24, [0, 4096], ks64, flags=P) == 0


def test_static_sweep_rejects_bad_arguments_and_sizes_before_any_device_work(lib):
    vp = C.c_void_p

    def rc(X=1024, ld=64, d=4, task_off=(0, 10), ks=(1, 2), n_iter=1, init_mode=0, flags=0, outs=4096):
        to = np.asarray(task_off, dtype=np.int64)
        k = np.asarray(ks, dtype=np.int32)
        return lib.cham_kmeans_sweep_static(vp(X), C.c_int64(ld), C.c_int32(d), to.ctypes.data_as(vp),
                                            C.c_int32(len(to) - 1), k.ctypes.data_as(vp), C.c_int32(len(k)),
                                            C.c_int32(n_iter), C.c_int32(init_mode), None, vp(outs), vp(outs),
                                            vp(outs), vp(outs), None, None, C.c_int32(flags), None)

    assert rc(d=0) == -2
    assert rc(ks=(2, 2)) == -3
    assert rc(task_off=(0, 10, 5)) == -4
    assert rc(flags=1 << 20) == -8
    # 1 Mi rows need 64 MiB of packed rows alone: beyond the static buffer
    assert rc(ld=1 << 20, task_off=(0, 1 << 20)) == -10
    # 2000 tasks: the host-side tables no longer fit on the stack
    assert rc(ld=4000, task_off=tuple(range(0, 4002, 2))) == -10
    assert len(lib.cham_strerror(-10)) > 20
    # the documented limit and the workspace query agree
    text = open(os.path.join(ROOT, "include", "cham.h")).read()
    m = re.search(r"#define\s+CHAM_STATIC_SCRATCH_BYTES\s+\((\d+) \* (\d+) \* (\d+)\)", text)
    limit = int(m.group(1)) * int(m.group(2)) * int(m.group(3))
    ks = list(range(2, 33))
    assert binding.cham_sweep_workspace_bytes(65536, 12, np.arange(0, 65537, 1024), ks, 30) <= limit
