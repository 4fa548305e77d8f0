"""Host-only checks of the C ABI: the built library exports what include/pcgrl.h declares, and
its defaults agree with the workload tables.  No GPU call is made."""
import ctypes as C
import os
import re

import pytest

from paper_2408_12525_amd import binding, build, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "pcgrl.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pcgrl_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_entry_point():
    binding.load()                      # compiles the library first if it was never built
    lib = C.CDLL(build.LIB)
    names = header_functions()
    assert {"pcgrl_create", "pcgrl_reset", "pcgrl_step", "pcgrl_metrics"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


@pytest.mark.parametrize("problem", [wl.BINARY, wl.MAZE, wl.DUNGEON])
def test_default_config_matches_workload_table(problem):
    c = binding.pcgrl_config_default(problem)
    w, lo, hi = wl.default_reward_table(problem)
    M = wl.num_metrics(problem)
    assert list(c.weights)[:M] == w and list(c.target_lo)[:M] == lo and list(c.target_hi)[:M] == hi
    K = wl.NUM_TILES[problem]
    cdf = list(c.init_cdf)
    assert cdf[K - 1] == 2**32 - 1 and all(cdf[i] <= cdf[i + 1] for i in range(K - 1))


def test_host_side_argument_errors_need_no_gpu():
    L = binding.load()
    assert L.pcgrl_create(None, None, 0) == -1
    assert L.pcgrl_config_default(7, C.byref(binding.PcgrlConfig())) == -2
    assert L.pcgrl_destroy(None) == 0
    assert L.pcgrl_strerror(-2).decode().startswith("configuration")
    h = C.c_void_p()
    bad = binding.make_config(wl.workload("maze16", batch=4, obs_w=99))
    assert L.pcgrl_create(C.byref(h), C.byref(bad), 0) == -2 and not h


SHIFT_ASM = """
_Z3fooPi:
	v_and_b32_e32 v{amt}, 31, v41
	v_lshlrev_b64 v[60:61], v{amt}, v[42:43]
	v_lshrrev_b64 v[4:5], s7, v[42:43]
	s_endpgm
	.amdhsa_kernel _Z3fooPi
		.amdhsa_next_free_vgpr {n}
	.end_amdhsa_kernel
"""


def test_build_scan_finds_a_shift_amount_in_the_highest_allocated_register():
    """The check the build runs on the compiler's device assembly (64-bit vector shifts whose
    amount sits in the last register of the kernel's allocation, which comes in blocks of eight):
    found where it is, not found one register lower, with a larger allocation, or with the amount
    in a scalar register."""
    n, found = build.scan_shift_amounts(SHIFT_ASM.format(amt=63, n=64))
    assert n == 1 and len(found) == 1 and found[0][0] == "_Z3fooPi" and found[0][1] == 64
    assert build.scan_shift_amounts(SHIFT_ASM.format(amt=63, n=58))[1] != []      # 58 registers are handed out as 64
    assert build.scan_shift_amounts(SHIFT_ASM.format(amt=62, n=64))[1] == []
    assert build.scan_shift_amounts(SHIFT_ASM.format(amt=63, n=65))[1] == []
    assert build.scan_shift_amounts(SHIFT_ASM.format(amt=71, n=65))[1] != []


def test_built_library_passed_the_scan():
    """build() refuses to hand out a library with such a shift; the report it leaves says how many
    kernels it looked at."""
    import json
    binding.load()
    if not os.path.exists(build.SCAN_REPORT):      # a library from before the check: build again
        build.build(force=True)
    rep = json.load(open(build.SCAN_REPORT))
    assert rep["findings"] == [] and rep["kernels"] >= 80
