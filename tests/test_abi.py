"""CPU-only checks of the C-ABI library: it loads, exports every function include/*.h declares,
and its argument validation (which runs before any HIP call) returns the documented codes."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2502_05202_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.load_library()


def declared_functions():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include")))
                   if h.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tli_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def _build(lib, d2t, Vt):
    arr = np.ascontiguousarray(d2t, dtype=np.int32)
    out = ctypes.c_void_p()
    S = ctypes.c_int32(-5)
    rc = lib.tli_build_map(arr.ctypes.data_as(ctypes.c_void_p), arr.shape[0], Vt, ctypes.byref(out), ctypes.byref(S))
    return rc, out, S.value


def test_build_map_validation(lib):
    assert _build(lib, [0, 1, 7], 7)[0] == -2          # 7 is not in [0, 7)
    assert _build(lib, [0, -2, 1], 7)[0] == -2         # only -1 marks "not shared"
    assert _build(lib, [3, 1, 3], 7)[0] == -3          # two drafter ids on one target id
    rc, out, S = _build(lib, [-1, -1, -1], 7)          # disjoint vocabularies
    assert rc == -4 and out.value is None and S == 0
    assert lib.tli_build_map(None, 3, 7, ctypes.byref(ctypes.c_void_p()), None) == -1
    arr = np.zeros(3, np.int32)
    assert lib.tli_build_map(arr.ctypes.data_as(ctypes.c_void_p), 0, 7, ctypes.byref(ctypes.c_void_p()), None) == -1
    assert lib.tli_build_map(arr.ctypes.data_as(ctypes.c_void_p), 3, 0, ctypes.byref(ctypes.c_void_p()), None) == -1
    assert lib.tli_build_map(arr.ctypes.data_as(ctypes.c_void_p), 3, 7, None, None) == -1
    assert lib.tli_build_map(arr.ctypes.data_as(ctypes.c_void_p), 3, (1 << 30) + 1, ctypes.byref(ctypes.c_void_p()), None) == -1
    assert binding.tli_workspace_bytes(1, 1, (1 << 30) + 1, 10, binding.TLI_F32) == 0


def test_status_strings_and_workspace(lib):
    assert binding.status_string(0) == "TLI_OK"
    assert binding.status_string(-3) == "TLI_ERR_NOT_INJECTIVE"
    assert binding.status_string(99) == "TLI_ERR_UNKNOWN"
    big = binding.tli_workspace_bytes(256, 8, 256000, 128256, binding.TLI_BF16)
    small = binding.tli_workspace_bytes(1, 3, 64, 48, binding.TLI_F32)
    assert 0 < small < big < (1 << 30)
    assert big % 256 == 0
    for bad in ((0, 8, 10, 10), (1, 0, 10, 10), (1, 65, 10, 10), (1, 1, 0, 10), (1, 1, 10, 0)):
        assert binding.tli_workspace_bytes(*bad, binding.TLI_F32) == 0
    assert binding.tli_workspace_bytes(1, 1, 10, 10, 7) == 0


def test_hot_calls_reject_null_arguments(lib):
    z = ctypes.c_void_p(0)
    assert lib.tli_draft_sample(z, z, 0, 8, 1, 1.0, z, z, z, z, z, z, 1, z, 0, z) == -1
    assert lib.tli_verify(z, z, z, 0, 1, 1, 1.0, 1.0, z, z, z, z, z, z, z, z, z, z, z, z, 0, z) == -1
    assert lib.tli_map_info(z, None, None, None) == -1
    lib.tli_free_map(z)  # freeing NULL is a no-op
    assert lib.tli_calib_read(z, 4096, 4096, 0, z, z) == -1
    assert lib.tli_calib_copy(z, z, 16, z) == -1
    assert lib.tli_device_info(None) == -1


def test_new_entry_points_reject_null_arguments(lib):
    z = ctypes.c_void_p(0)
    assert lib.tli_union_draft_sample(z, z, 0, 8, 1, 1.0, z, z, z, z, z, z, 1, z, 0, z) == -1
    assert lib.tli_draft_sample_compact(z, z, 0, 8, 1, 1.0, z, z, z, z, z, z, 1, z, 0, z) == -1
    assert lib.tli_union_verify(z, z, z, 0, 1, 1, 1.0, 1.0, z, z, z, z, z, z, z, z, z, z, z, z, 0, z) == -1
    assert lib.tli_verify_compact(z, z, z, 8, 0, 1, 1, 1.0, 1.0, z, z, z, z, z, z, z, z, z, z, z, z, 0, z) == -1
    assert lib.tli_acceptance_rates(z, z, z, 0, 1, 1, 1.0, 1.0, z, z, z, z, 0, z) == -1
    assert lib.tli_sample_rows(z, 0, 8, 1, 8, 1.0, z, z, z, z, z, 1, z, 0, z) == -1
    assert lib.tli_sample_rows(z, 0, 8, 1, 8, 0.0, z, z, z, z, z, 1, z, 0, z) == -1
    assert lib.tli_greedy_draft(z, z, 0, 8, 1, z, z, z, 1, z, 0, z) == -1
    assert lib.tli_exact_match_verify(z, 0, 1, 1, 8, 1.0, z, z, z, z, z, z, z, 0, z) == -1
    assert lib.tli_warp_rows(z, z, 0, 8, 1, 8, 1.0, 5, 0.9, z, 8, z, z, z, z, 0, z) == -1
    assert lib.tli_acceptance_rates_workspace_bytes(z, 1, 1, 0) == 0
    assert lib.tli_sample_rows_workspace_bytes(0, 8, 0) == 0 and lib.tli_sample_rows_workspace_bytes(4, 1000, 1) > 0
    assert lib.tli_exact_match_workspace_bytes(2, 64, 100, 0) == 0 and lib.tli_exact_match_workspace_bytes(2, 3, 100, 0) > 0
    assert lib.tli_warp_workspace_bytes(3, 100, 1) > 0 and lib.tli_warp_workspace_bytes(3, 100, 9) == 0


def test_map_tables_replayed_on_the_host(lib):
    """tli_map_dry_run builds the map's tables without a device and replays what the residual-scan kernel does
    with them (sweep of the drafter row into LDS slots, walk of every chunk's pair list): in bounds, every slot
    written once, every shared pair visited once with both sides matching d2t.  Shapes: one and several parts for
    both storage types, sparse and identical vocabularies, a single shared token, rows of more than 1024 chunks,
    shared ids bunched at one end of either vocabulary."""
    from paper_2502_05202_amd import synth
    cases = [(64, 48, 32), (128256, 32000, 24000), (151936, 49152, 40000), (256000, 128256, 90000),
             (202048, 128256, 60000), (2048 * 3, 2048 * 3, 2048 * 3), (70000, 60000, 50000), (8, 8, 1),
             (1024 * 1100 + 12, 3000, 2000), (50000, 20000, 1)]
    for Vt, Vd, S in cases:
        d2t = synth.make_d2t(Vd, Vt, S, seed=Vt + S)
        r = binding.tli_map_dry_run(d2t, Vt)
        assert r["status"] == 0 and r["failed_check"] == 0 and r["num_shared"] == S, (Vt, Vd, S, r)
        assert r["nparts"][0] >= r["nparts"][1] >= 1  # fp32 logits take twice the LDS of bf16 ones
    assert binding.tli_map_dry_run(synth.make_d2t(128256, 256000, 90000, seed=1), 256000)["nparts"] == (4, 2)
    # bunched: the first S drafter ids map to the last S target ids, in reverse
    Vd, Vt, S = 40000, 90000, 30000
    d2t = np.full(Vd, -1, np.int32)
    d2t[:S] = Vt - 1 - np.arange(S)
    assert binding.tli_map_dry_run(d2t, Vt)["status"] == 0
    # the same argument checks as tli_build_map
    assert binding.tli_map_dry_run([0, 1, 7], 7)["status"] == -2
    assert binding.tli_map_dry_run([3, 1, 3], 7)["status"] == -3
    assert binding.tli_map_dry_run([-1, -1], 7)["status"] == -4
    assert binding.status_string(-7) == "TLI_ERR_INTERNAL"


def test_d2t_from_token_strings(lib):
    """Vocabularies are sets of strings; the shared tokens are the equal strings (the paper's notation paragraph and
    its three tiny examples)."""
    ex = binding.tli_d2t_from_strings
    assert ex(["a", "b", "c"], ["a", "b"]).tolist() == [0, 1, -1]      # T={a,b}, D={a,b,c}
    assert ex(["b"], ["a"]).tolist() == [-1]                            # disjoint
    assert ex(["b"], ["a", "b"]).tolist() == [1]
    assert ex(["a", "b"], ["a"]).tolist() == [0, -1]
    # any bytes, the empty string and prefixes of one another are tokens of their own
    assert ex([b"\x00", b"", b"ab", b"a\x00b"], [b"a\x00b", b"abc", b"", b"\x00\x00"]).tolist() == [-1, 2, -1, 0]
    rng = np.random.default_rng(3)
    words = [f"tok{i}" for i in rng.permutation(5000)]
    D, T = words[:3000], list(reversed(words[1000:4500]))
    want = {w: i for i, w in enumerate(T)}
    assert ex(D, T).tolist() == [want.get(w, -1) for w in D]
    with pytest.raises(binding.TliError):
        ex(["a", "a"], ["a"])                                           # a set has no duplicates
    with pytest.raises(binding.TliError):
        ex(["a"], ["b", "b"])
    # what comes out is what tli_build_map takes
    assert binding.tli_map_dry_run(ex(D, T), len(T))["num_shared"] == 2000


def test_map_builder_under_address_and_ub_sanitizers(tmp_path):
    """The host-side table builder (argument checks, parts, staging tables, pair lists, the host replay of the residual
    scan's indexing, the string join) is plain C++ in a file of its own: built here with g++ -fsanitize=address,undefined
    -- no HIP, no device -- and driven over the workloads' vocabulary shapes, bunched and identical vocabularies,
    invalid maps, the string join, and a seeded fuzz of (Vd, Vt, S, layout of the shared ids).  A sanitizer report, a
    failed consistency check or an unexpected status fails the test."""
    import subprocess

    csrc = os.path.join(ROOT, "paper_2502_05202_amd", "csrc")
    exe = str(tmp_path / "hostmap_san")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-static-libubsan",  # the runtimes inside the executable: no library order to mind
                    "-I", os.path.join(ROOT, "include"), "-I", csrc, os.path.join(csrc, "tli_host_map.cpp"),
                    os.path.join(ROOT, "tests", "hostmap_san_driver.cpp"), "-o", exe], check=True)
    cases = [
        (48, 64, 32, 1, 0), (32000, 128256, 24000, 2, 0), (49152, 151936, 40000, 3, 0), (128256, 256000, 90000, 4, 0),
        (128256, 202048, 60000, 5, 0),                       # the five workloads
        (60000, 70000, 50000, 6, 1), (130000, 130000, 130000, 7, 2), (4096, 8200, 1, 8, 0),
        (5000, 2048 * 1100 + 8, 3000, 9, 0),                 # a row of more than 1024 chunks
        (9000, 7000, 500, 10, 3), (9000, 7000, 500, 11, 3), (9000, 7000, 500, 12, 3),   # the three refusals
        (3000, 5000, 1200, 13, 4), (20000, 9000, 8000, 14, 4),                          # through token strings
    ]
    rng = np.random.default_rng(2025)
    for i in range(24):  # seeded fuzz
        Vd, Vt = int(rng.integers(8, 200000)), int(rng.integers(8, 300000))
        S = int(rng.integers(1, min(Vd, Vt) + 1))
        cases.append((Vd, Vt, S, 100 + i, int(rng.integers(0, 2))))
    args = [str(v) for c in cases for v in c]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe] + args, capture_output=True, text=True, env=env)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-3000:]
    assert res.stdout.count("failed_check 0") == len(cases)
