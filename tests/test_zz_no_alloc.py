"""The entry point that allocates nothing (pcgrl_exact_diameter_static) against the entry point it
is a variant of, through the C ABI: same results, on two calls in a row that share the library's
static scratch array, the second on a smaller batch (needs an MI355X)."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from paper_2408_12525_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def _diameters(gpu, static, parts_log2=-1):
    dev = torch.device("cuda", 0)
    out = torch.full((gpu.B,), -7, dtype=torch.int32, device=dev)
    st = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    if static:
        rc = gpu.L.pcgrl_exact_diameter_static(gpu.h, C.c_void_p(out.data_ptr()), parts_log2, st)
    else:
        rc = gpu.L.pcgrl_exact_diameter(gpu.h, C.c_void_p(out.data_ptr()), st)
    assert rc == 0, rc
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_static_scratch_variant_equals_the_allocating_entry_point():
    dev = torch.device("cuda", 0)
    # first call: 700 levels, sources of a level shared out over 4 workgroups (2800 partial results);
    # second call: 45 larger levels over 32 workgroups each (1440): its partial results land on
    # words that still hold the first call's
    cases = [("binary16", 700, -1), ("dungeon32", 45, 5), ("maze64", 3, 6), ("binary16", 9000, 0)]
    envs = []
    for name, batch, lg in cases:
        cfg = wl.workload(name, batch=batch, max_steps=10**6, autoreset=0)
        gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
        gpu.pcgrl_reset(11)
        cpu.reset(11, want_obs=False)
        acts = wl.random_actions(cfg, 12, 30)
        for a in acts:
            gpu.pcgrl_step(torch.from_numpy(a).to(dev))
            cpu.step(a, want_obs=False)
        envs.append((gpu, cpu, lg, name))
    # the static calls back to back, nothing in between
    got = [_diameters(gpu, True, lg) for gpu, _, lg, _ in envs]
    for (gpu, cpu, lg, name), g in zip(envs, got):
        want = _diameters(gpu, False)
        assert np.array_equal(g, want), name
        assert np.array_equal(g, cpu.exact_diameters()), name
    # again in reverse order (large after small), and with every split the buffer size allows
    for gpu, cpu, lg, name in reversed(envs):
        side = 16 if max(gpu.Hm, gpu.Wm) <= 16 else 32 if max(gpu.Hm, gpu.Wm) <= 32 else 64
        for p in range(0, side.bit_length()):
            if (gpu.B << p) > (1 << 18) and p > 0:
                break
            assert np.array_equal(_diameters(gpu, True, p), cpu.exact_diameters()), (name, p)
    for gpu, *_ in envs:
        gpu.close()


def test_static_scratch_variant_rejects_what_does_not_fit():
    dev = torch.device("cuda", 0)
    cfg = wl.workload("binary16", batch=40000, max_steps=10**6, autoreset=0)
    gpu = binding.Pcgrl(cfg, 0)
    out = torch.empty((gpu.B,), dtype=torch.int32, device=dev)
    st = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    call = lambda lg: gpu.L.pcgrl_exact_diameter_static(gpu.h, C.c_void_p(out.data_ptr()), lg, st)
    assert call(3) == -6                       # 40 000 levels x 8 parts = 320 000 > 262 144 partial results
    assert call(2) == 0                        # 160 000 fit
    assert call(5) == -2 and call(-2) == -2    # more parts than rows / no such code
    assert gpu.L.pcgrl_exact_diameter_static(None, C.c_void_p(out.data_ptr()), 0, st) == -1
    assert b"static scratch" in gpu.L.pcgrl_strerror(-6)
    torch.cuda.synchronize()
    gpu.close()
