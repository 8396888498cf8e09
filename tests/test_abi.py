"""The C-ABI library loads on a machine without a GPU and exports every declared symbol."""
import ctypes
import os
import re

from paper_2311_10359_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fikit.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(fikit_[a-z_]+)\s*\(", text))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(build.LIB):
        build.build_library()
    lib = ctypes.CDLL(build.LIB)
    names = declared_functions()
    assert names == set(binding.EXPORTS)
    for name in names:
        assert hasattr(lib, name), name


def test_host_only_entry_points():
    lib = binding.load()
    assert lib.fikit_version() >= 1
    assert binding.status_string(0) == "ok"
    for st in range(-8, 0):
        assert binding.status_string(st) not in ("ok", "unknown status")
    assert binding.status_string(-99) == "unknown status"
    # workspace queries are pure host arithmetic: monotone in the sizes, 0 beyond the size limit
    a = binding.fikit_profile_workspace_bytes(1000, 2)
    b = binding.fikit_profile_workspace_bytes(100000, 2)
    c = binding.fikit_profile_workspace_bytes(100000, 2000)
    assert 0 < a < b <= c
    assert binding.fikit_profile_workspace_bytes(1 << 32, 1) == 0
    assert binding.fikit_gapfill_workspace_bytes(1000, 2, 1) >= 3 * 8 * 1000
    assert binding.fikit_gapfill_workspace_bytes(1 << 33, 2, 1) == 0


def test_host_side_argument_checks_need_no_gpu():
    """NULL pointers, misalignment and size limits are rejected before any HIP call."""
    lib = binding.load()
    n_rows = ctypes.c_uint64(7)
    null = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(0x1000)         # never dereferenced on these paths
    odd = ctypes.c_void_p(0x1004)
    assert lib.fikit_profile(fake, 10, null, 1, null, fake, 10, fake, ctypes.byref(n_rows), fake, 1 << 30, null) == -1
    assert n_rows.value == 0
    assert lib.fikit_profile(odd, 10, fake, 1, null, fake, 10, fake, ctypes.byref(n_rows), fake, 1 << 30, null) == -1
    assert lib.fikit_profile(fake, 1 << 32, fake, 1, null, fake, 10, fake, ctypes.byref(n_rows), fake, 1 << 30, null) == -1
    assert lib.fikit_profile(fake, 10, fake, 0, null, fake, 10, fake, ctypes.byref(n_rows), fake, 1 << 30, null) == -1
    assert lib.fikit_profile(fake, 10, fake, 1, null, fake, 10, fake, None, fake, 1 << 30, null) == -1
    assert lib.fikit_profile(fake, 10, fake, 1, null, fake, 10, fake, ctypes.byref(n_rows), fake, 64, null) == -2
    p = binding._GapfillParams(-5, 0)
    assert lib.fikit_gapfill(fake, fake, 1, fake, fake, fake, fake, 1, ctypes.byref(p), fake, fake, fake, fake, fake,
                             fake, 1 << 20, null) == -1
    p = binding._GapfillParams(0, 0)
    assert lib.fikit_gapfill(fake, fake, 1, fake, fake, null, fake, 1, ctypes.byref(p), fake, fake, fake, fake, fake,
                             fake, 1 << 20, null) == -1
    assert lib.fikit_gapfill(fake, fake, 1, fake, fake, fake, fake, 1, None, fake, fake, fake, fake, fake,
                             fake, 1 << 20, null) == -1
    p = binding._GapfillParams(0, 0, 2, 0)   # no such predictor
    assert lib.fikit_gapfill(fake, fake, 1, fake, fake, fake, fake, 1, ctypes.byref(p), fake, fake, fake, fake, fake,
                             fake, 1 << 20, null) == -1
    r = binding._ReplayParams(0, 0, 1, 7)
    assert lib.fikit_gapfill_replay(fake, fake, 1, fake, fake, fake, fake, fake, 1, ctypes.byref(r), fake, fake, fake, fake,
                                    fake, fake, 1 << 20, null) == -1
    r = binding._ReplayParams(0, -1, 0, 0)
    assert lib.fikit_gapfill_replay(fake, fake, 1, fake, fake, fake, fake, fake, 1, ctypes.byref(r), fake, fake, fake, fake,
                                    fake, fake, 1 << 20, null) == -1
    p = binding._GapfillParams(0, 0, 0, 0)
    assert lib.fikit_prio_fill(fake, fake, 1, fake, fake, fake, null, fake, fake, 1, ctypes.byref(p), fake, fake, fake, fake,
                               fake, fake, 1 << 20, null) == -1
    assert lib.fikit_prio_fill(fake, fake, 1, fake, fake, fake, fake, fake, fake, 1, None, fake, fake, fake, fake,
                               fake, fake, 1 << 20, null) == -1
    p = binding._GapfillParams(0, 0, 0, 1)   # reserved must be 0
    assert lib.fikit_prio_fill(fake, fake, 1, fake, fake, fake, fake, fake, fake, 1, ctypes.byref(p), fake, fake, fake, fake,
                               fake, fake, 1 << 20, null) == -1
    assert lib.fikit_prio_fill_workspace_bytes(1 << 33, 1, 1) == 0
    assert lib.fikit_pairing_best(fake, fake, 1, 1, fake, fake, null, fake, fake, fake, fake, fake, 1 << 20, null) == -1
    assert lib.fikit_pairing_best(fake, fake, 1, 1, fake, fake, fake, fake, odd, fake, fake, fake, 1 << 20, null) == -1
    assert lib.fikit_pairing_best(fake, fake, 1, 1, fake, fake, fake, fake, fake, fake, fake, fake, 16, null) == -2
    assert lib.fikit_pairing_best(fake, fake, 1 << 31, 1, fake, fake, fake, fake, fake, fake, fake, fake, 1 << 20, null) == -1
    assert lib.fikit_pairing_workspace_bytes(1000) >= 8000
    assert lib.fikit_profile_merge(fake, fake, fake, fake, 1, fake, 10, fake, None, fake, 1 << 20, null) == -1
    assert lib.fikit_profile_merge(fake, null, fake, fake, 1, fake, 10, fake, ctypes.byref(n_rows), fake, 1 << 20, null) == -1
    assert lib.fikit_profile_merge(fake, fake, fake, fake, 1, fake, 10, fake, ctypes.byref(n_rows), fake, 16, null) == -2
    assert lib.fikit_profile_merge(fake, fake, fake, fake, 0, fake, 10, fake, ctypes.byref(n_rows), fake, 1 << 20, null) == -1
    assert lib.fikit_profile_merge_workspace_bytes(1000) >= 4004
    # the variant on the built-in scratch buffer refuses what does not fit it, before any HIP call
    p = binding._GapfillParams(500, 0, 0, 0)
    assert lib.fikit_gapfill_static(fake, binding.FIKIT_STATIC_MAX_IDS + 1, fake, 2, fake, fake, fake, fake, 1, ctypes.byref(p),
                                    fake, 1, fake, fake, fake, fake, fake, null) == binding.FIKIT_TOO_LARGE
    assert lib.fikit_gapfill_static(fake, 100, fake, binding.FIKIT_STATIC_MAX_TASKS + 1, fake, fake, fake, fake, 1,
                                    ctypes.byref(p), fake, 1, fake, fake, fake, fake, fake, null) == binding.FIKIT_TOO_LARGE
    assert lib.fikit_gapfill_static(fake, 100, fake, 2, fake, fake, fake, fake, 1, ctypes.byref(p), fake, 1, fake, fake, fake,
                                    fake, null, null) == -1     # no status word
    assert lib.fikit_gapfill_static(fake, 100, fake, 2, fake, fake, fake, fake, 1, None, fake, 1, fake, fake, fake,
                                    fake, fake, null) == -1
    assert lib.fikit_measure(fake, 10, null, 1, fake, fake, fake, 256, null) == -1
    assert lib.fikit_measure(fake, 10, fake, 1, fake, fake, fake, 16, null) == -2
    assert lib.fikit_measure_workspace_bytes() == 256
