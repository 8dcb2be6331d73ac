"""CPU-side checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2506_00812_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2506_00812_amd.build import build
        build(verbose=False)
    return binding.load_library()


def test_header_symbols_are_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "vecflow.h")).read()
    declared = sorted(set(re.findall(r"\b(vf_[a-z_]+)\s*\(", hdr)))
    assert declared == sorted(binding.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_stats_struct_matches_header():
    hdr = open(os.path.join(ROOT, "include", "vecflow.h")).read()
    body = re.search(r"typedef struct vf_stats \{(.*?)\} vf_stats;", hdr, re.S).group(1)
    names = [n.strip() for line in body.split(";") for n in line.replace("int64_t", "").replace("int32_t", "").split(",")
             if n.strip()]
    assert names == [n for n, _ in binding.VfStats._fields_]


def test_profile_struct_matches_header():
    hdr = open(os.path.join(ROOT, "include", "vecflow.h")).read()
    body = re.search(r"typedef struct vf_profile \{(.*?)\} vf_profile;", hdr, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = [n.strip() for line in body.split(";")
             for n in re.sub(r"\b(float|double|int64_t|int32_t)\b", "", line).split(",") if n.strip()]
    assert names == [n for n, _ in binding.VfProfile._fields_]


def test_search_multi_rejects_bad_mode_without_gpu(lib):
    assert lib.vf_search_multi(None, None, 0, None, None, 9, 10, 32, 1, 8, 0, None, None, None) == -1
    assert b"mode" in lib.vf_last_error()


def test_build_rejects_bad_arguments_without_gpu(lib):
    h = C.c_void_p()
    off = np.array([0, 1, 2], dtype=np.int64)
    ids = np.array([0, 5], dtype=np.int32)
    fake = C.c_void_p(4096)    # never dereferenced: validation fails first
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    cases = [
        dict(dtype=7, dim=16, n_labels=8, T=40, R=8),        # dtype
        dict(dtype=0, dim=17, n_labels=8, T=40, R=8),        # dim not a multiple of 16
        dict(dtype=1, dim=6, n_labels=8, T=40, R=8),         # float dim not a multiple of 4
        dict(dtype=0, dim=16, n_labels=8, T=8, R=8),         # T < R + 1
        dict(dtype=0, dim=16, n_labels=8, T=400, R=65),      # R too large
        dict(dtype=0, dim=16, n_labels=4, T=40, R=8),        # label id 5 outside the vocabulary
    ]
    for c in cases:
        rc = lib.vf_build_index(fake, c["dtype"], 2, c["dim"], p(off), p(ids), c["n_labels"], c["T"], c["R"], None, None,
                                C.byref(h))
        assert rc == -1, c
        assert lib.vf_last_error()
        assert not h.value
    assert lib.vf_build_index(None, 0, 2, 16, p(off), p(ids), 8, 40, 8, None, None, C.byref(h)) == -1
    # vectors longer than the contraction kernel's LDS tile allows; an allocator with a missing function
    assert lib.vf_build_index(fake, 1, 2, 256, p(off), p(ids), 8, 40, 8, None, None, C.byref(h)) == -1
    assert b"992" in lib.vf_last_error()
    half = binding.VfAllocator(binding.ALLOC_FN(lambda n, c: None), binding.FREE_FN(0), None)
    assert lib.vf_build_index(fake, 0, 2, 16, p(off), p(ids), 8, 40, 8, C.byref(half), None, C.byref(h)) == -1
    assert b"allocator" in lib.vf_last_error()
    lib.vf_index_free(None)    # allowed


def test_tuning_names_and_ranges_without_gpu(lib):
    """vf_tune with a NULL index changes the process-wide defaults: every documented name is accepted, unknown
    names and values out of range are rejected with VF_EINVAL, and nothing throws across the ABI."""
    hdr = open(os.path.join(ROOT, "include", "vecflow.h")).read()
    doc = re.search(r"Names: (.*?)\.  Returns VF_EINVAL", hdr, re.S).group(1)
    names = re.findall(r'"([a-z_0-9]+)"', doc)
    assert len(names) == 26
    defaults = dict(seg_groups=16, seg_groups_heavy=16, heavy_rows=9, tile_rows=16, zero_copy_bytes=8192, scan_valu=1,
                    scan16=1, scan_bf16=1, scan_bf16_margin=22, scan_bf16_slots=1, scan_bf16_seg_groups=24, beam_lat_waves=1024, overlap=1, seed_exact=0, seed_slack=1.0, seed_margin=8, seed_margin_bf16=24, seed_cache=1,
                    seed_bf16=1, seed_bf16_min_batch=512, seed_fb_window=131072, seed_select=0, seed_seg_seeds=0, build16=1, build_panel_kb=4096,
                    build_progress=0)
    assert sorted(names) == sorted(defaults)
    for n in names:
        assert lib.vf_tune(None, n.encode(), float(defaults[n])) == 0, n
    assert lib.vf_tune(None, b"no_such_knob", 1.0) == -1
    assert b"no_such_knob" in lib.vf_last_error()
    assert lib.vf_tune(None, b"tile_rows", 33.0) == -1
    assert lib.vf_tune(None, b"tile_rows", 7.5) == -1
    assert lib.vf_tune(None, b"seed_slack", -1.0) == -1
    assert lib.vf_tune(None, b"seed_slack", float("nan")) == -1
    assert lib.vf_tune(None, None, 1.0) == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(binding.VecflowError):
        binding.load_library()


def test_bench_reads_the_committed_counter_summary():
    """bench.py takes `roofline.traffic` from the rocprofv3 counter summary under profiles/ and prefers the
    parameters that summary was taken at: the summary must parse, and it must cover the three search kernels."""
    import importlib.util
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("vf_bench", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    params = bench.committed_params("c2")
    assert params is not None and len(params) == 4 and params in bench.CANDIDATES
    for kernel in ("beam_kernel", "seed_mfma_kernel", "scan_bf16_kernel"):
        t = bench.committed_traffic(kernel, "c2", params)
        assert t is not None and 10_000_000 < t < 5_000_000_000, (kernel, t)
    assert bench.committed_traffic("beam_kernel", "c2", (1, 1, 1, 1)) is None      # other parameters: no figure
    assert bench.committed_params("no such workload") is None
