"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every declared symbol, rejects invalid calls before touching HIP, and its index
helpers (multiply-shift division, XCD tile ordering) are exact."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1610_03618_amd as cm
from paper_1610_03618_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INVALID = 1


def _declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(cnnmem_\w+)\s*\(", text))


def test_library_is_built_and_exports_every_declared_symbol():
    assert sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h")) == \
        ["cnnmem.h", "cnnmem_debug.h"]
    assert os.path.exists(hip_build.LIB_PATH)
    lib = ctypes.CDLL(hip_build.LIB_PATH)
    declared = _declared_symbols("cnnmem.h")
    assert {"cnnmem_transform", "cnnmem_pool", "cnnmem_softmax", "cnnmem_pool_out_dims",
            "cnnmem_status_string", "cnnmem_version"} <= declared
    for name in declared:
        assert hasattr(lib, name), name


def test_test_hooks_live_in_a_library_of_their_own():
    hooks = ctypes.CDLL(hip_build.HOOKS_LIB_PATH)
    product = ctypes.CDLL(hip_build.LIB_PATH)
    declared = _declared_symbols("cnnmem_debug.h")
    assert declared == {"cnnmem_debug_fastdiv", "cnnmem_debug_smalldiv_mismatches", "cnnmem_debug_xcd_tile",
                        "cnnmem_debug_canonical_permutation"}
    for name in declared:
        assert hasattr(hooks, name), name
        assert not hasattr(product, name), f"{name} is exported by the product library"
    assert cm.test_hooks().cnnmem_debug_fastdiv(17, 0) == 0xFFFFFFFF      # no quotient, no SIGFPE


def test_version_and_status_strings():
    assert cm.cnnmem_version() >= 100
    assert cm.cnnmem_status_string(0) == "ok"
    assert "invalid" in cm.cnnmem_status_string(1)
    assert cm.cnnmem_status_string(77) == "unknown status"


def test_pool_out_dims_follows_floor_rule():
    assert cm.cnnmem_pool_out_dims(12, 12, 4, 4, 2, 2, 0, 0) == (0, 5, 5)        # Fig. 8
    assert cm.cnnmem_pool_out_dims(32, 32, 3, 3, 2, 2, 0, 0) == (0, 15, 15)
    assert cm.cnnmem_pool_out_dims(224, 112, 2, 2, 2, 2, 0, 0) == (0, 112, 56)
    assert cm.cnnmem_pool_out_dims(5, 7, 3, 3, 2, 1, 1, 1) == (0, 3, 7)
    assert cm.cnnmem_pool_out_dims(2, 2, 3, 3, 1, 1, 0, 0)[0] == INVALID       # window > image
    assert cm.cnnmem_pool_out_dims(8, 8, 3, 3, 0, 1, 0, 0)[0] == INVALID       # zero stride
    assert cm.cnnmem_pool_out_dims(8, 8, 3, 3, 1, 1, 2, 0)[0] == INVALID       # pad > k/2
    lib = cm.library()
    assert lib.cnnmem_pool_out_dims(8, 8, 2, 2, 2, 2, 0, 0, None, None) == INVALID


FAKE = 0x1000  # a non-null, 16-byte aligned address that is never dereferenced: every call below is rejected on the host


@pytest.mark.parametrize("kwargs", [
    dict(src=None), dict(dst=None), dict(N=0), dict(C=-1), dict(H=0), dict(W=0),
    dict(src_layout=2), dict(dst_layout=-1), dict(src=FAKE + 2),
])
def test_transform_rejects_invalid_arguments_on_host(kwargs):
    a = dict(src=FAKE, dst=FAKE + 4096, N=2, C=2, H=2, W=2, src_layout=cm.NCHW, dst_layout=cm.CHWN)
    a.update(kwargs)
    assert cm.cnnmem_transform(a["src"], a["dst"], a["N"], a["C"], a["H"], a["W"], a["src_layout"],
                               a["dst_layout"], stream=0) == INVALID


@pytest.mark.parametrize("kwargs", [
    dict(src=None), dict(dst=None), dict(N=0), dict(C=0), dict(H=0), dict(W=-3), dict(layout=5),
    dict(mode=2), dict(kh=0), dict(kw=0), dict(sh=0), dict(sw=-1), dict(ph=-1), dict(pw=-1),
    dict(ph=2), dict(pw=2), dict(kh=9), dict(kw=9), dict(dst=FAKE + 1),
])
def test_pool_rejects_invalid_arguments_on_host(kwargs):
    a = dict(src=FAKE, dst=FAKE + 4096, N=2, C=2, H=8, W=8, layout=cm.NCHW, mode=cm.POOL_MAX,
             kh=3, kw=3, sh=2, sw=2, ph=0, pw=0)
    a.update(kwargs)
    assert cm.cnnmem_pool(a["src"], a["dst"], a["N"], a["C"], a["H"], a["W"], a["layout"], a["mode"],
                          a["kh"], a["kw"], a["sh"], a["sw"], a["ph"], a["pw"], stream=0) == INVALID


@pytest.mark.parametrize("tuning", [dict(rows_per_lane=5), dict(rows_per_lane=-1), dict(cols_per_lane=3),
                                    dict(workgroups_per_cu=9), dict(workgroups_per_cu=1), dict(workgroups_per_cu=-2),
                                    dict(nchw_kernel=3), dict(slab_lanes=300)])
def test_pool_tuned_rejects_out_of_range_tuning_on_host(tuning):
    assert cm.cnnmem_pool_tuned(FAKE, FAKE + 4096, 2, 2, 8, 8, cm.NCHW, cm.POOL_MAX, 3, 3, 2, 2, 0, 0,
                                tuning=tuning, stream=0) == INVALID
    # and a valid tuning does not rescue an invalid call
    assert cm.cnnmem_pool_tuned(None, FAKE, 2, 2, 8, 8, cm.NCHW, cm.POOL_MAX, 3, 3, 2, 2, 0, 0,
                                tuning=dict(rows_per_lane=2), stream=0) == INVALID


@pytest.mark.parametrize("kwargs", [dict(logits=None), dict(probs=None), dict(N=0), dict(classes=0),
                                    dict(logits=FAKE + 3)])
def test_softmax_rejects_invalid_arguments_on_host(kwargs):
    a = dict(logits=FAKE, probs=FAKE + 4096, N=4, classes=10)
    a.update(kwargs)
    assert cm.cnnmem_softmax(a["logits"], a["probs"], a["N"], a["classes"], stream=0) == INVALID


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(2, 3)
    with pytest.raises(ValueError):
        cm.cnnmem_softmax(x, x, 2, 3, stream=0)


def test_fastdiv_is_exact():
    lib = cm.test_hooks()
    rng = np.random.default_rng(5)
    divisors = [1, 2, 3, 4, 5, 7, 13, 27, 28, 32, 55, 112, 729, 3025, 21841, 65536, 65537,
                (1 << 31) - 1] + rng.integers(1, 1 << 31, size=40).tolist()
    for d in divisors:
        ns = [0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, (1 << 31) - 1, (1 << 31) - d] + \
            rng.integers(0, 1 << 31, size=200).tolist()
        for n in ns:
            if 0 <= n < (1 << 31):
                assert lib.cnnmem_debug_fastdiv(n, d) == n // d, (n, d)


def test_small_number_divider_is_exact_where_a_quotient_can_first_go_wrong():
    lib = cm.test_hooks()
    # every divisor up to 4096 against every multiple of it below 2^20 and its two neighbours
    assert lib.cnnmem_debug_smalldiv_mismatches(1 << 20, 4096) == 0
    assert lib.cnnmem_debug_smalldiv_mismatches(1 << 16, 65535) == 0
    assert lib.cnnmem_debug_smalldiv_mismatches((1 << 20) + 1, 4) == -1       # beyond what the divider promises
    assert lib.cnnmem_debug_smalldiv_mismatches(16, 0) == -1


@pytest.mark.parametrize("nblocks", [1, 2, 7, 8, 9, 15, 16, 17, 63, 64, 100, 1001, 4096, 12289])
def test_xcd_tile_order_is_a_bijection_and_groups_by_xcd(nblocks):
    lib = cm.test_hooks()
    tiles = [lib.cnnmem_debug_xcd_tile(b, nblocks) for b in range(nblocks)]
    assert sorted(tiles) == list(range(nblocks))
    # blocks dealt to one XCD (same id mod 8) get consecutive tiles
    for x in range(min(8, nblocks)):
        mine = [tiles[b] for b in range(x, nblocks, 8)]
        assert mine == list(range(mine[0], mine[0] + len(mine)))


@pytest.mark.parametrize("dtype", [3, -1, 99])
def test_dtype_entry_points_reject_unknown_formats_on_host(dtype):
    assert cm.cnnmem_transform_dtype(FAKE, FAKE + 4096, 2, 2, 2, 2, cm.NCHW, cm.CHWN, dtype, stream=0) == INVALID
    assert cm.cnnmem_pool_dtype(FAKE, FAKE + 4096, 2, 2, 4, 4, cm.NCHW, cm.POOL_MAX, 2, 2, 2, 2, 0, 0, dtype,
                                stream=0) == INVALID
    assert cm.cnnmem_softmax_dtype(FAKE, FAKE + 4096, 2, 10, dtype, stream=0) == INVALID


@pytest.mark.parametrize("dtype", [1, 2])
def test_dtype_entry_points_validate_like_the_fp32_ones(dtype):
    assert cm.cnnmem_transform_dtype(FAKE, FAKE + 4096, 0, 2, 2, 2, cm.NCHW, cm.CHWN, dtype, stream=0) == INVALID
    assert cm.cnnmem_transform_dtype(FAKE + 1, FAKE + 4096, 2, 2, 2, 2, cm.NCHW, cm.CHWN, dtype, stream=0) == INVALID
    assert cm.cnnmem_transform_dtype(FAKE, FAKE + 4096, 2, 2, 2, 2, cm.NCHW, 7, dtype, stream=0) == INVALID
    assert cm.cnnmem_pool_dtype(FAKE, FAKE + 4096, 2, 2, 4, 4, cm.NCHW, cm.POOL_MAX, 9, 9, 2, 2, 0, 0, dtype,
                                stream=0) == INVALID
    assert cm.cnnmem_pool_dtype(FAKE, FAKE + 4097, 2, 2, 4, 4, cm.NCHW, cm.POOL_MAX, 2, 2, 2, 2, 0, 0, dtype,
                                stream=0) == INVALID
    assert cm.cnnmem_pool_dtype(None, FAKE, 2, 2, 4, 4, cm.NCHW, cm.POOL_MAX, 2, 2, 2, 2, 0, 0, dtype, stream=0) == INVALID
    assert cm.cnnmem_softmax_dtype(FAKE, FAKE + 4096, 2, 0, dtype, stream=0) == INVALID
    assert cm.cnnmem_softmax_dtype(FAKE + 1, FAKE + 4096, 2, 10, dtype, stream=0) == INVALID


def test_headers_compile_as_plain_c(tmp_path):
    """The ABI headers are plain C: no torch, no HIP, no C++."""
    import subprocess
    src = tmp_path / "use_headers.c"
    src.write_text('#include "cnnmem.h"\n#include "cnnmem_debug.h"\n'
                   'int main(void) { cnnmem_pool_tuning t = {0, 0, 0, 0, 0}; cnnmem_layer l = {CNNMEM_LAYER_POOL, 1, 1};\n'
                   '  (void)t; (void)l; return CNNMEM_F16 + CNNMEM_POOL_AVG + CNNMEM_CHWN > 0 ? 0 : 1; }\n')
    include = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", include, "-c", str(src),
                    "-o", str(tmp_path / "use_headers.o")], check=True)


def test_binding_refuses_tensors_smaller_than_the_call_needs():
    """A bare pointer carries no size, so the binding is where an undersized tensor is caught, before any launch
    (the size is looked at first, so the check can be exercised here without a GPU)."""
    import torch
    from paper_1610_03618_amd import binding

    assert binding._prod(2, 3, 4, 5) == 120 and binding._prod(2, 0, 4, 5) is None
    assert binding._pooled(16, 64, 32, 32, 3, 3, 2, 2, 0, 0) == 16 * 64 * 15 * 15
    assert binding._pooled(1, 1, 2, 2, 3, 3, 1, 1, 0, 0) is None        # window larger than the image
    small, enough = torch.zeros(10), torch.zeros(16)
    with pytest.raises(ValueError, match="needs 16"):
        cm.cnnmem_transform(FAKE, small, 2, 2, 2, 2, cm.NCHW, cm.CHWN, stream=0)
    with pytest.raises(ValueError, match="needs 16"):
        cm.cnnmem_pool(small, enough, 1, 1, 4, 4, cm.NCHW, cm.POOL_MAX, 2, 2, 2, 2, 0, 0, stream=0)
    with pytest.raises(ValueError, match="needs 4"):
        cm.cnnmem_pool(FAKE, torch.zeros(3), 1, 1, 4, 4, cm.NCHW, cm.POOL_MAX, 2, 2, 2, 2, 0, 0, stream=0)
    with pytest.raises(ValueError, match="needs 12"):
        cm.cnnmem_softmax(small, small, 3, 4, stream=0)
    with pytest.raises(ValueError, match="needs 24"):
        cm.cnnmem_permute(enough, enough, (1, 2, 3, 4), (3, 2, 1, 0), stream=0)
    with pytest.raises(ValueError, match="needs 16"):
        cm.cnnmem_pool_backward(FAKE, FAKE, small, 1, 1, 4, 4, cm.NCHW, cm.POOL_MAX, 2, 2, 2, 2, 0, 0, stream=0)
    # large enough: the next check (CPU memory is refused) is reached
    with pytest.raises(ValueError, match="GPU memory"):
        cm.cnnmem_transform(enough, enough, 2, 2, 2, 2, cm.NCHW, cm.CHWN, stream=0)


def test_probe_library_is_separate_and_validates_on_the_host():
    """The memory-system probes of `bench.py --workload access_patterns` live in a library of their own and
    refuse arguments that would address past the buffers before they launch anything."""
    probes = ctypes.CDLL(hip_build.PROBES_LIB_PATH)
    product = ctypes.CDLL(hip_build.LIB_PATH)
    p, i, ll = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong
    probes.cnnmem_probe_tile_pattern.argtypes = [p, p, ll, ll, i, i, i, i, p]
    probes.cnnmem_probe_chunk_copy.argtypes = [p, p, ll, i, i, p]
    for name in ("cnnmem_probe_tile_pattern", "cnnmem_probe_chunk_copy"):
        assert not hasattr(product, name)
    tile = probes.cnnmem_probe_tile_pattern
    assert tile(None, FAKE, 1024, 128, 32, 128, 1, 0, None) == INVALID            # null pointer
    assert tile(FAKE, FAKE + 4096, 1024, 128, 32, 64, 1, 0, None) == INVALID      # tile of 2048 floats: no kernel
    assert tile(FAKE, FAKE + 4096, 1024, 100, 32, 128, 1, 0, None) == INVALID     # images not a multiple of the tile
    assert tile(FAKE, FAKE + 4096, 16, 128, 32, 128, 1, 0, None) == INVALID       # fewer rows than one tile
    assert tile(FAKE + 4, FAKE + 4096, 1024, 128, 32, 128, 1, 0, None) == INVALID  # misaligned
    chunk = probes.cnnmem_probe_chunk_copy
    assert chunk(FAKE, FAKE + 4096, 1000, 4096, 3, None) == INVALID               # not whole chunks
    assert chunk(FAKE, FAKE + 4096, 1024, 24, 3, None) == INVALID                 # chunk not a multiple of 16 bytes
    assert chunk(FAKE, None, 1024, 4096, 3, None) == INVALID
