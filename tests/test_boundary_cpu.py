"""The C interface without a GPU: the library loads, exports every declared symbol, and its
host-side argument checks answer with error codes (no compute is launched here)."""
import ctypes as C
import os
import re

import pytest

import paper_2305_03152_amd as spp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "spp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spp_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(spp.LIB_PATH):
        from paper_2305_03152_amd import build
        build.build()
    return spp.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(spp.EXPORTS) == names


def test_mfg_bound_host_logic(lib):
    nb, eb = spp.mfg_bound(1024, (15, 10, 5), 2_400_000)
    assert nb == [1024, 16384, 180224, 1081344] and eb == [0, 15360, 163840, 901120]
    nb, eb = spp.mfg_bound(256, (15, 10, 5), 10_000)
    assert nb == [256, 4096, 10000, 10000] and eb == [0, 3840, 40960, 50000]
    with pytest.raises(spp.SppError):
        spp.mfg_bound(4, (65,), 100)          # fanout above SPP_MAX_FANOUT
    with pytest.raises(spp.SppError):
        spp.mfg_bound(4, (1,) * 9, 100)       # more hops than SPP_MAX_L


def test_null_arguments_are_errors_not_crashes(lib):
    assert lib.spp_ctx_sync(None) == -1
    assert b"null" in lib.spp_last_error()
    assert lib.spp_gather_last_stats(None, None) == -1
    assert lib.spp_cache_set_limit(None, 0) == -1
    lib.spp_ctx_destroy(None)
    lib.spp_graph_destroy(None)
    lib.spp_cache_destroy(None)


def test_product_path_fails_loudly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    with pytest.raises(spp.SppError):
        spp.Context(0)


def test_binding_constants_match_the_header():
    """Flags, limits and timer indices are typed twice (C header, ctypes binding): they must agree."""
    from paper_2305_03152_amd import api
    text = open(os.path.join(ROOT, "include", "spp.h")).read()
    defines = {k: int(v.rstrip("u"), 0) for k, v in re.findall(r"#define\s+(SPP_[A-Z0-9_]+)\s+(0x[0-9a-fA-F]+u?|\d+)\b", text)}
    for name in ("SPP_MAX_L", "SPP_MAX_FANOUT", "SPP_SYNC", "SPP_VIP_INCLUDE_HOP0", "SPP_GRAPH_IN_LISTS", "SPP_NO_JOIN",
                 "SPP_STORE_ORDER"):
        assert defines[name] == getattr(api, name), name
    assert defines["SPP_MAX_GATHER_LISTS"] == 64 and defines["SPP_MAX_SAMPLE_BATCHES"] == 64
    enums = {k: int(v) for k, v in re.findall(r"\b(SPP_T_[A-Z_]+)\s*=\s*(\d+)", text)}
    for name in ("SPP_T_VIP_TOTAL", "SPP_T_VIP_HOP_FIRST", "SPP_T_SAMPLE", "SPP_T_GATHER_HIT", "SPP_T_GATHER_MISS",
                 "SPP_T_GATHER_CLASSIFY", "SPP_T_COUNT"):
        assert enums[name] == getattr(api, name), name
    # struct layouts the binding mirrors: sizes as the C compiler sees them
    import subprocess, tempfile
    src = '#include "spp.h"\n#include <stdio.h>\nint main(void){printf("%zu %zu %zu %zu %zu\\n", sizeof(spp_mfg), ' \
          'sizeof(spp_gather_stats), sizeof(spp_gather_list), sizeof(spp_sample_item), sizeof(spp_id_list));return 0;}\n'
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "s.c")
        open(c, "w").write(src)
        exe = os.path.join(d, "s")
        subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), c, "-o", exe], check=True)
        sizes = [int(x) for x in subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split()]
    assert sizes == [C.sizeof(api._MfgStruct), C.sizeof(api._GatherStats), C.sizeof(api._GatherList), C.sizeof(api._SampleItem),
                     C.sizeof(api._IdList)]


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
