"""GPU library vs CPU oracle, through the C ABI, on the same seeded inputs (needs an MI355X)."""
import numpy as np
import pytest
import torch

import levels
import oracle
from parity import assert_same, check_obs, compare_state, expected_obs, run_parity
from paper_2408_12525_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def test_lane_exchange_selftest():
    assert binding.pcgrl_selftest(0) == 0


@pytest.mark.parametrize("mode", [1, 2, 3], ids=["cached", "non-temporal", "write-through"])
def test_store_rate_kernel_writes_every_byte_it_is_asked_to(mode):
    """The store-only measurement kernel: every 16-byte piece of the regions is written (first
    word 0x01010101), nothing after them is touched; regions pattern and linear sweep."""
    dev = torch.device("cuda", 0)
    for n_regions, region, order in ((37, 4816, 0), (5, 16, 0), (70000, 1936, 0), (9, 3072, 1), (37, 4816, 2),
                                     (70001, 1936, 2)):
        buf = torch.full((n_regions * region + 64,), 0xEE, dtype=torch.uint8, device=dev)
        binding.pcgrl_store_rate(buf, n_regions, region, mode, order)
        torch.cuda.synchronize()
        words = buf[:n_regions * region].view(torch.int32).view(-1, 4)
        assert bool((words[:, 0] == 0x01010101).all()), (n_regions, region, order)
        assert bool((buf[n_regions * region:] == 0xEE).all())
    with pytest.raises(binding.PcgrlError):
        binding.pcgrl_store_rate(buf, 4, 24, mode, 0)          # not a multiple of 16
    with pytest.raises(binding.PcgrlError):
        binding.pcgrl_store_rate(buf, 4, 2048 + 16, mode, 1)   # the linear order wants whole KiB pieces
    with pytest.raises(binding.PcgrlError):
        binding.pcgrl_store_rate(buf, 4, 1024, mode, 3)        # no such order


SMALL = [
    # label, config, steps, extra
    ("binary16 walls-pad", wl.workload("binary16", batch=67, max_steps=40), 130, {}),
    ("binary16 recount", wl.workload("binary16", batch=33, max_steps=50, regions_mode=wl.REGIONS_RECOUNT), 120, {}),
    ("maze16", wl.workload("maze16", batch=130, max_steps=60), 150, {}),
    ("maze16 scan+budget", wl.workload("maze16", batch=21, max_steps=300, pos_mode=wl.POS_SCAN, max_changes=25), 320, {}),
    ("maze16 empty start, pinpoints", wl.make_config(wl.MAZE, 19, 16, 31, probs="empty", n_frozen=2, max_steps=70), 150, {}),
    ("dungeon16 ow5", wl.make_config(wl.DUNGEON, 26, 13, 5, min_size=5, max_steps=45, n_frozen=3,
                                      probs=[.40, .40, .04, .04, .04, .04, .04]), 140, {}),
    ("binary32 rand ow3", wl.workload("binary32_rand_ow3", batch=75, max_steps=50), 130, {}),
    ("binary32 rand ow15", wl.workload("binary32_rand_ow15", batch=41, max_steps=50), 110, {}),
    ("binary32 rand ow63", wl.workload("binary32_rand_ow63", batch=23, max_steps=50), 110, {}),
    ("binary32 rand ow63 recount, bad actions", wl.workload("binary32_rand_ow63", batch=9, max_steps=50,
                                                              regions_mode=wl.REGIONS_RECOUNT), 110, dict(bad_fraction=0.1)),
    ("maze32 even window", wl.make_config(wl.MAZE, 37, 24, 8, min_size=9, max_w=31, min_w=9, max_steps=64,
                                          probs=[.45, .45, .05, .05]), 140, {}),
    ("dungeon32", wl.workload("dungeon32", batch=45, max_steps=60), 130, {}),
    ("dungeon32 uniform tiles, wall pad", wl.make_config(wl.DUNGEON, 18, 32, 15, pad_mode=wl.PAD_WALL, max_steps=80), 120, {}),
    ("maze64", wl.workload("maze64", batch=19, max_steps=60), 130, {}),
    ("maze64 uniform tiles scan", wl.make_config(wl.MAZE, 5, 64, 31, pos_mode=wl.POS_SCAN, max_steps=200), 210, {}),
    ("binary64 rand ow63", wl.make_config(wl.BINARY, 7, 64, 63, min_size=33, n_frozen=8, max_steps=90, probs=[.65, .35]), 200, {}),
    ("binary64 sparse walls", wl.make_config(wl.BINARY, 6, 64, 31, max_steps=90, probs=[.8, .2]), 120, {}),
    ("dungeon64 ow1", wl.make_config(wl.DUNGEON, 4, 40, 1, max_w=64, max_steps=90), 100, {}),
    ("batch of one", wl.make_config(wl.MAZE, 1, 16, 31, max_steps=30), 70, {}),
    ("maze16 bit-packed obs", wl.workload("maze16", batch=77, max_steps=40, obs_format=1), 100, {}),
    ("maze16 pinpoint channel", wl.workload("maze16_pinpoint", batch=60, max_steps=33, obs_frozen_channel=1, obs_w=31), 100, {}),
    ("binary32 pinpoint channel ow63 wall pad packed", wl.workload("binary32_rand_ow63", batch=11, max_steps=25, pad_mode=wl.PAD_WALL,
                                                                   obs_frozen_channel=1, obs_format=1), 60, {}),
    ("dungeon64 pinpoint channel, nothing frozen", wl.make_config(wl.DUNGEON, 5, 64, 15, max_steps=30, obs_frozen_channel=1), 50, {}),
    ("binary32 rand ow63 bit-packed", wl.workload("binary32_rand_ow63", batch=13, max_steps=30, obs_format=1), 70, {}),
    ("dungeon64 ow5 bit-packed", wl.make_config(wl.DUNGEON, 7, 64, 5, min_size=20, max_steps=30, obs_format=1), 70, {}),
    ("binary16 ow1 bit-packed", wl.make_config(wl.BINARY, 40, 16, 1, max_steps=30, obs_format=1, pad_mode=wl.PAD_WALL), 50, {}),
    ("maze16 pinpointed player and door", wl.workload("maze16_pinpoint", batch=90, max_steps=33), 120, {}),
    ("dungeon16 control targets", wl.workload("dungeon16_ctrl", batch=50, max_steps=27), 120, {}),
    ("maze32 pinpoints + control, scan", wl.make_config(wl.MAZE, 30, 32, 16, min_size=3, probs="empty", n_frozen=4,
                                                         pinpoint_tile=[2, 3, -1, 1], ctrl={1: (5, 40), 0: (1, 3)},
                                                         pos_mode=wl.POS_SCAN, max_steps=41), 130, {}),
    ("no autoreset", wl.make_config(wl.BINARY, 10, 16, 7, max_steps=20, autoreset=0), 50, {}),
]


SHAPES = [(0, 0, 0, "auto"), (2, 1, 0, "lpw2-unsplit"), (4, 2, 0, "lpw4-split"), (1, 1, 0, "lpw1-unsplit"),
          (4, 2, 2, "lpw4-split-obs2"), (4, 2, 1, "lpw4-split-obs1"), (2, 2, 1, "lpw2-split-obs1")]


def _applies(cfg, lpw, olv):
    """A 64-row level fills the wavefront (no packing to choose), and for 32-row levels a request
    for four levels per wavefront is the same launch shape as one for two."""
    side = max(cfg["max_h"], cfg["max_w"])
    return not (lpw > 1 and side > 32) and not (olv and lpw > 2 and side > 16)


SMALL_CASES = [pytest.param(label, cfg, steps, extra, lpw, split, olv, id=f"{label}-{sid}")
               for (label, cfg, steps, extra) in SMALL for (lpw, split, olv, sid) in SHAPES
               if _applies(cfg, lpw, olv)]


@pytest.mark.parametrize("label,cfg,steps,extra,lpw,split,olv", SMALL_CASES)
def test_small_configs_every_step(label, cfg, steps, extra, lpw, split, olv):
    """lpw = levels packed into one wavefront (automatic = 1 at these batch sizes, 2, as many as
    the size class takes); split = one wavefront per level group, or a metrics wavefront and
    observation wavefronts (automatic = split at these batch sizes); olv = levels per observation
    wavefront of a split step (0 = as many as the metrics wavefront holds).  Only the launch shapes
    that exist for a configuration's size class are listed."""
    run_parity(dict(cfg, levels_per_wave=lpw, split_step=split, split_obs_levels=olv), steps,
               label=f"{label} lpw={lpw} split={split} obs levels={olv}", **extra)


@pytest.mark.parametrize("mode", [1, 2, 3], ids=["cached", "non-temporal", "write-through"])
@pytest.mark.parametrize("name,batch,split", [("maze16", 70, 2), ("binary32_rand_ow63", 9, 1), ("maze64", 5, 1)])
def test_every_way_of_storing_the_observation(name, batch, split, mode):
    """The three store instructions the library chooses between by the size of a step's output,
    each forced on a small batch: steps (split and unsplit kernel) and a rollout."""
    cfg = wl.workload(name, batch=batch, max_steps=30, obs_store_mode=mode, split_step=split)
    run_parity(cfg, 45, label=f"{name} store mode {mode}")
    dev = torch.device("cuda", 0)
    T = 37
    acts_np = wl.random_actions(cfg, 5, T)
    gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
    gpu.pcgrl_reset(3)
    cpu.reset(3)
    obs = torch.zeros((2,) + gpu.obs_shape, dtype=torch.uint8, device=dev)
    gpu.pcgrl_rollout(torch.from_numpy(acts_np).to(dev), obs)
    want = {}
    for t in range(T):
        want[t % 2] = cpu.step(acts_np[t])[0]
    for k, o in want.items():
        assert_same("obs", obs[k], o, f"rollout slot {k}, store mode {mode}")
    gpu.close()


PITCHED = [
    ("maze16 lines", wl.workload("maze16", batch=70, max_steps=30, obs_pitch=-1), 4864),
    ("binary16 lines", wl.workload("binary16", batch=67, max_steps=30, obs_pitch=-1), 2048),
    ("binary32 ow3, 16-byte pitch", wl.workload("binary32_rand_ow3", batch=41, max_steps=30, obs_pitch=32), 32),
    ("binary32 ow63 lines", wl.workload("binary32_rand_ow63", batch=9, max_steps=30, obs_pitch=-1), 12032),
    ("dungeon32 lines", wl.workload("dungeon32", batch=21, max_steps=30, obs_pitch=-1), 1920),
    ("maze64 lines", wl.workload("maze64", batch=5, max_steps=30, obs_pitch=-1), 4864),
    ("maze64 wide pitch", wl.workload("maze64", batch=3, max_steps=30, obs_pitch=4805 // 16 * 16 + 48), 4848),
    ("maze16 bit-packed lines", wl.workload("maze16", batch=33, max_steps=30, obs_format=1, obs_pitch=-1), 640),
    ("dungeon64 ow5 bit-packed, pitch 32", wl.make_config(wl.DUNGEON, 7, 64, 5, min_size=20, max_steps=30, obs_format=1,
                                                           obs_pitch=32), 32),
    ("exact multiple of a line stays dense", wl.make_config(wl.BINARY, 10, 16, 8, max_steps=20, pad_mode=wl.PAD_WALL,
                                                             obs_pitch=-1), 128),
]


@pytest.mark.parametrize("mode", [0, 1, 2, 3], ids=["auto", "cached", "non-temporal", "write-through"])
@pytest.mark.parametrize("split", [1, 2], ids=["unsplit", "split"])
@pytest.mark.parametrize("label,cfg,stride", PITCHED, ids=[c[0] for c in PITCHED])
def test_pitched_observation_layout(label, cfg, stride, split, mode):
    """obs_pitch: every level's observation starts a fixed number of bytes after the one before
    (here mostly a whole number of 128-byte lines); the observation itself is unchanged and the
    bytes in between are zeros.  Steps, reset and observe in both launch shapes and every store
    kind, then a rollout into a ring of such buffers, all against the oracle's dense bytes."""
    cfg = dict(cfg, obs_store_mode=mode, split_step=split)
    dev = torch.device("cuda", 0)
    gpu = binding.Pcgrl(cfg, 0)
    assert gpu.obs_stride == stride
    if stride != gpu.obs_bytes:
        assert gpu.obs_shape == (cfg["batch"], stride)
    gpu.close()
    run_parity(cfg, 45, label=f"{label} split={split} store={mode}")
    gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
    gpu.pcgrl_reset(3)
    cpu.reset(3)
    check_obs(gpu, gpu.pcgrl_observe(), cpu.observe(), "pcgrl_observe")
    T = 37
    acts_np = wl.random_actions(cfg, 5, T)
    obs = torch.full((3,) + gpu.obs_shape, 0xAB, dtype=torch.uint8, device=dev)
    gpu.pcgrl_rollout(torch.from_numpy(acts_np).to(dev), obs)
    want = {}
    for t in range(T):
        want[t % 3] = cpu.step(acts_np[t])[0]
    for k, o in want.items():
        check_obs(gpu, obs[k], o, f"rollout slot {k}")
    gpu.close()


UNPACK = [
    ("maze16", wl.workload("maze16", batch=37, max_steps=30, obs_format=1)),
    ("maze64 lines", wl.workload("maze64", batch=5, max_steps=30, obs_format=1, obs_pitch=-1)),
    ("binary32 ow63 pinpoint channel", wl.workload("binary32_rand_ow63", batch=11, max_steps=25, obs_frozen_channel=1, obs_format=1)),
    ("dungeon32 ow15", wl.workload("dungeon32", batch=23, max_steps=30, obs_format=1, obs_pitch=240)),
    ("binary16 ow1", wl.make_config(wl.BINARY, 40, 16, 1, max_steps=30, obs_format=1, pad_mode=wl.PAD_WALL)),
    ("binary32 ow3", wl.workload("binary32_rand_ow3", batch=70, max_steps=30, obs_format=1)),
]


@pytest.mark.parametrize("label,cfg", UNPACK, ids=[c[0] for c in UNPACK])
def test_unpack_packed_observations(label, cfg):
    """The consumer's side of the bit-packed format: pcgrl_unpack_obs must give back the oracle's
    one-hot cells as uint8 0/1 and as 0.0/1.0 in float16, bfloat16 and float32, also into an output
    that starts at an odd element (its first and last few elements are then written one by one)."""
    dev = torch.device("cuda", 0)
    gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
    obs = gpu.new_obs()
    gpu.pcgrl_reset(9, obs)
    want = cpu.reset(9)
    acts = wl.random_actions(cfg, 10, 12)
    for t in range(13):
        for dt in (torch.uint8, torch.float16, torch.bfloat16, torch.float32):
            got = gpu.pcgrl_unpack_obs(obs, dtype=dt)
            assert got.dtype == dt and tuple(got.shape) == want.shape
            assert torch.equal(got.cpu().to(torch.float32), torch.from_numpy(want).to(torch.float32)), (label, t, dt)
            n = got.numel()
            big = torch.full((n + 3,), 7, dtype=dt, device=dev)      # one element further on: misaligned chunks
            view = big[1:n + 1].view(got.shape)
            gpu.pcgrl_unpack_obs(obs, out=view)
            assert torch.equal(view, got) and float(big[0]) == 7 and float(big[n + 1]) == 7, (label, t, dt)
        if t < 12:
            gpu.pcgrl_step(torch.from_numpy(acts[t]).to(dev), obs)
            want = cpu.step(acts[t])[0]
    with pytest.raises(binding.PcgrlError):
        plain = binding.Pcgrl(dict(cfg, obs_format=0), 0)
        plain.pcgrl_unpack_obs(plain.new_obs())
    gpu.close()


def test_obs_pitch_is_validated():
    for bad in (-2, 24, 4800, 100):           # unknown code, not a multiple of 16, smaller than the observation
        with pytest.raises(binding.PcgrlError):
            binding.Pcgrl(wl.workload("maze16", batch=4, obs_pitch=bad), 0)


@pytest.mark.parametrize("name,batch", [("binary16", 300), ("maze16", 130), ("binary32_rand_ow3", 90),
                                        ("dungeon32", 40), ("maze64", 6)])
def test_exact_diameter_query(name, batch):
    """All-sources BFS on the GPU against the oracle's, on fresh and on edited levels; the cached
    two-sweep estimate of the binary problem must never exceed it."""
    dev = torch.device("cuda", 0)
    cfg = wl.workload(name, batch=batch, max_steps=10**6, autoreset=0)
    gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
    gpu.pcgrl_reset(31)
    cpu.reset(31, want_obs=False)
    acts = wl.random_actions(cfg, 32, 60)
    for rnd in range(3):
        exact = gpu.pcgrl_exact_diameter().cpu().numpy()
        assert np.array_equal(exact, cpu.exact_diameters()), f"round {rnd}"
        if cfg["problem"] == wl.BINARY:
            est = gpu.pcgrl_metrics().cpu().numpy()[:, 1]
            assert (est <= exact).all()
        for t in range(20):
            a = acts[rnd * 20 + t]
            gpu.pcgrl_step(torch.from_numpy(a).to(dev))
            cpu.step(a, want_obs=False)
    gpu.close()


def test_pinpoint_channel_after_set_state():
    dev = torch.device("cuda", 0)
    cfg = wl.make_config(wl.MAZE, 4, 16, 15, autoreset=0, obs_frozen_channel=1)
    gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
    gpu.pcgrl_reset(2)
    cpu.reset(2)
    rng = np.random.default_rng(0)
    tiles = rng.integers(0, 4, size=(4, 16, 16)).astype(np.int8)
    fro = (rng.random((4, 16, 16)) < 0.2).astype(np.uint8)
    hw = np.full((4, 2), 16, np.int16)
    pos = rng.integers(0, 16, size=(4, 2)).astype(np.int16)
    gpu.pcgrl_set_state(*(torch.from_numpy(a).to(dev) for a in (tiles, fro, hw, pos)))
    cpu.set_state(tiles, fro, hw, pos)
    assert_same("obs", gpu.pcgrl_observe(), cpu.observe(), "after set_state")
    obs = gpu.new_obs()
    acts = wl.random_actions(cfg, 3, 40)
    for t in range(40):
        gpu.pcgrl_step(torch.from_numpy(acts[t]).to(dev), obs)
        o, _, _ = cpu.step(acts[t])
        assert_same("obs", obs, o, f"step {t}")
    compare_state(gpu, cpu, "end")
    gpu.close()


def test_control_targets_and_fractional_weights():
    # per-env target ranges and non-integer weights (products that round): rewards must still be equal
    cfg = wl.make_config(wl.DUNGEON, 32, 16, 9, max_steps=10**6, autoreset=0,
                         weights=[0.37, 1.13, 0.71, 0.0, 0.05, 2.9, 3.3, 1.7, 0.9, 0.11])
    rng = np.random.default_rng(0)
    lo = rng.integers(0, 20, size=(32, 10))
    hi = lo + rng.integers(0, 30, size=(32, 10))
    run_parity(cfg, 200, targets=np.stack([lo, hi], axis=2).astype(np.int32), label="control targets")


def test_set_state_with_hand_built_levels():
    dev = torch.device("cuda", 0)
    for name in levels.all_fixtures():
        problem, tiles, expect = levels.load(name)
        pid = levels.PROBLEM_ID[problem]
        h, w = tiles.shape
        size = max(h, w)
        cfg = wl.make_config(pid, 3, size, 5, min_size=1, autoreset=0)
        gpu = binding.Pcgrl(cfg, 0)
        cpu = oracle.Oracle(cfg)
        gpu.pcgrl_reset(5)
        cpu.reset(5)
        buf = np.full((3, size, size), -1, np.int8)
        buf[:, :h, :w] = tiles
        fro = np.zeros((3, size, size), np.uint8)
        fro[1, 0, 0] = 1
        hw = np.array([[h, w]] * 3, np.int16)
        pos = np.array([[0, 0], [0, 0], [h - 1, w - 1]], np.int16)
        gpu.pcgrl_set_state(*(torch.from_numpy(a).to(dev) for a in (buf, fro, hw, pos)))
        cpu.set_state(buf, fro, hw, pos)
        m = gpu.pcgrl_metrics().cpu().numpy()
        got = dict(zip(wl.metric_names(pid), (int(v) for v in m[0])))
        exact = gpu.pcgrl_exact_diameter().cpu().numpy()
        assert np.array_equal(exact, cpu.exact_diameters()), name
        if "exact_diameter" in expect:
            assert exact[0] == expect.pop("exact_diameter"), name
        for k, v in expect.items():
            assert got[k] == v, (name, k, got)
        assert_same("metrics", m, cpu.metrics(), name)
        assert_same("obs", gpu.pcgrl_observe(), cpu.observe(), name)
        compare_state(gpu, cpu, name)
        # a few edits on top, including one on the frozen cell of env 1
        K = wl.NUM_TILES[pid]
        rew = torch.empty(3, dtype=torch.float32, device=dev)
        for t in range(6):
            a = np.array([(t + 1) % K, (t + 1) % K, t % K], np.int32)
            gpu.pcgrl_step(torch.from_numpy(a).to(dev), None, rew, None)
            _, r, _ = cpu.step(a, want_obs=False)
            assert np.array_equal(rew.cpu().numpy(), r), (name, t)
            assert_same("metrics", gpu.pcgrl_metrics(), cpu.metrics(), (name, t))
        gpu.close()


FULL = [
    ("binary16", 64, 60, None),
    ("maze16", 4096, 24, None),
    ("binary32_rand_ow3", 16384, 12, None),
    ("binary32_rand_ow15", 16384, 12, None),
    ("binary32_rand_ow63", 16384, 8, slice(0, 16384, 7)),
    ("maze64", 8192, 8, None),
    ("dungeon32", 16384, 10, None),
]


@pytest.mark.parametrize("name,batch,steps,sl", FULL, ids=[f[0] for f in FULL])
def test_full_size_workloads(name, batch, steps, sl):
    """The benchmark's launch configuration (full batch, default modes), compared with the oracle
    on every env for a few steps."""
    cfg = wl.workload(name, batch=batch)
    run_parity(cfg, steps, seed=0, aseed=1, env_slice=sl, state_every=steps, label=name + " full size")


def test_results_do_not_depend_on_batch_partition():
    dev = torch.device("cuda", 0)
    cfg = wl.workload("maze16", batch=64, max_steps=30)
    acts = torch.from_numpy(wl.random_actions(cfg, 3, 70)).to(dev)
    big = binding.Pcgrl(cfg, 0)
    small = binding.Pcgrl(dict(cfg, batch=13), 0)
    ob, os_ = big.new_obs(), small.new_obs()
    big.pcgrl_reset(9, ob)
    small.pcgrl_reset(9, os_)
    for t in range(70):
        big.pcgrl_step(acts[t], ob)
        small.pcgrl_step(acts[t, :13].contiguous(), os_)
        assert torch.equal(ob[:13], os_)
    assert torch.equal(big.pcgrl_metrics()[:13], small.pcgrl_metrics())
    big.close()
    small.close()


def test_argument_errors_are_reported_not_raised_by_the_gpu():
    bad = wl.workload("maze16", batch=4)
    for field, val in (("obs_w", 64), ("max_h", 65), ("batch", 0), ("problem", 3), ("n_frozen", 9),
                       ("min_h", 17), ("max_steps", 0), ("pad_mode", 2), ("levels_per_wave", 5),
                       ("split_step", 3), ("obs_store_mode", 4), ("split_obs_levels", 5),
                       ("rollout_turns", 3)):
        with pytest.raises(binding.PcgrlError):
            binding.Pcgrl(dict(bad, **{field: val}), 0)
    env = binding.Pcgrl(bad, 0)
    with pytest.raises(binding.PcgrlError):
        env.pcgrl_step(torch.zeros(5, dtype=torch.int32, device="cuda"))
    with pytest.raises(binding.PcgrlError):
        env.pcgrl_step(torch.zeros(4, dtype=torch.int64, device="cuda"))
    assert env.L.pcgrl_step(env.h, None, None, None, None, None) == -1
    assert env.L.pcgrl_step(None, None, None, None, None, None) == -1
    env.close()


def test_steps_captured_in_a_hip_graph_replay_like_eager_calls():
    """pcgrl_step only launches a kernel, so a caller may capture it.  Replays (with eager work and
    synchronisation between them, and an auto-reset falling inside the graph) must give what the
    same calls give eagerly, and what the oracle gives."""
    dev = torch.device("cuda", 0)
    n, reps = 20, 4
    cfg = wl.workload("maze16", batch=300, max_steps=35)
    acts_np = wl.random_actions(cfg, 5, n)
    acts = torch.from_numpy(acts_np).to(dev)
    B = cfg["batch"]
    eager, graphed, cpu = binding.Pcgrl(cfg, 0), binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
    obs_e = eager.new_obs()
    rew_e = torch.empty(B, dtype=torch.float32, device=dev)
    done_e = torch.empty(B, dtype=torch.uint8, device=dev)
    obs_g = torch.empty((n,) + graphed.obs_shape, dtype=torch.uint8, device=dev)
    rew_g = torch.empty((n, B), dtype=torch.float32, device=dev)
    done_g = torch.empty((n, B), dtype=torch.uint8, device=dev)
    eager.pcgrl_reset(11, obs_e)
    cpu.reset(11)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graphed.pcgrl_reset(11)
        with torch.cuda.graph(g, stream=side):
            for t in range(n):
                graphed.pcgrl_step(acts[t], obs_g[t], rew_g[t], done_g[t])
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graphed.pcgrl_reset(11)          # capture does not execute; start both from the same state
    for rep in range(reps):
        g.replay()
        torch.cuda.synchronize()
        for t in range(n):
            eager.pcgrl_step(acts[t], obs_e, rew_e, done_e)
            o, r, d = cpu.step(acts_np[t])
            ctx = f"replay {rep} step {t}"
            assert torch.equal(obs_g[t], obs_e), ctx
            assert torch.equal(rew_g[t], rew_e) and torch.equal(done_g[t], done_e), ctx
            assert_same("obs", obs_g[t], o, ctx)
            assert np.array_equal(rew_g[t].cpu().numpy(), r) and np.array_equal(done_g[t].cpu().numpy(), d), ctx
        assert torch.equal(graphed.pcgrl_metrics(), eager.pcgrl_metrics())
        assert_same("metrics", graphed.pcgrl_metrics(), cpu.metrics(), f"replay {rep}")
        compare_state(graphed, cpu, f"replay {rep}")
        (obs_e.float().sum() + 1).item()      # unrelated eager work between replays
    for e in (eager, graphed):
        e.close()


ROLLOUTS = [
    ("binary16", wl.workload("binary16", batch=37, max_steps=23), 60, 60),
    ("maze16 ring of 7 obs slots", wl.workload("maze16", batch=70, max_steps=31), 50, 7),
    ("maze16 lpw4 pinpoints scan", wl.make_config(wl.MAZE, 50, 16, 9, n_frozen=4, max_steps=29, pos_mode=wl.POS_SCAN,
                                                  levels_per_wave=4, probs=[.45, .45, .05, .05]), 64, 64),
    ("binary32 rand ow15 pinpoints", wl.workload("binary32_rand_ow15", batch=33, max_steps=20), 45, 45),
    ("dungeon32 lpw2", wl.workload("dungeon32", batch=21, max_steps=26, levels_per_wave=2), 40, 1),
    ("maze64", wl.workload("maze64", batch=9, max_steps=17), 40, 40),
    ("binary64 budget", wl.make_config(wl.BINARY, 5, 64, 63, min_size=40, n_frozen=5, max_changes=9, max_steps=100), 60, 3),
    ("dungeon16 control targets", wl.workload("dungeon16_ctrl", batch=40, max_steps=13), 60, 2),
    ("maze16 pinpointed", wl.workload("maze16_pinpoint", batch=40, max_steps=19), 60, 60),
    ("maze16 bit-packed", wl.workload("maze16", batch=40, max_steps=19, obs_format=1), 40, 5),
    ("dungeon16 pinpoint channel", wl.workload("dungeon16_ctrl", batch=30, max_steps=17, obs_frozen_channel=1), 40, 40),
]


@pytest.mark.parametrize("split,olv,turns", [(1, 0, 0), (2, 0, 1), (2, 0, 0), (2, 1, 2)],
                         ids=["one-wavefront", "split-one-turn", "split", "split-obs1-two-turns"])
@pytest.mark.parametrize("label,cfg,T,slots", ROLLOUTS, ids=[r[0] for r in ROLLOUTS])
def test_rollout_equals_the_same_steps_one_by_one(label, cfg, T, slots, split, olv, turns):
    """pcgrl_rollout against the oracle stepped T times (every observation slot that survives,
    every reward and done flag, final state and metrics), with auto-resets inside the rollout, and
    against T calls of pcgrl_step.  split: the levels stay in one wavefront for the whole rollout,
    or in a metrics wavefront and observation wavefronts that each carry their own copy; turns:
    how many observation wavefronts take the steps in turn (0: the library's choice, which at
    these batches is as many as a workgroup holds)."""
    cfg = dict(cfg, split_step=split, split_obs_levels=olv, rollout_turns=turns)
    print(f"[rollout] {label} T={T} slots={slots} split={split} obs levels={olv} turns={turns}", flush=True)
    dev = torch.device("cuda", 0)
    B = cfg["batch"]
    acts_np = wl.random_actions(cfg, 8, T, bad_fraction=0.03)
    acts = torch.from_numpy(acts_np).to(dev)
    roll, single, cpu = binding.Pcgrl(cfg, 0), binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
    for e in (roll, single):
        e.pcgrl_reset(21)
    cpu.reset(21)
    obs = torch.zeros((slots,) + roll.obs_shape, dtype=torch.uint8, device=dev)
    rew = torch.empty((T, B), dtype=torch.float32, device=dev)
    done = torch.empty((T, B), dtype=torch.uint8, device=dev)
    roll.pcgrl_rollout(acts, obs, rew, done)
    want_obs = {}
    o1 = single.new_obs()
    r1 = torch.empty(B, dtype=torch.float32, device=dev)
    d1 = torch.empty(B, dtype=torch.uint8, device=dev)
    for t in range(T):
        o, r, d = cpu.step(acts_np[t])
        want_obs[t % slots] = expected_obs(cfg, o)
        assert np.array_equal(rew[t].cpu().numpy(), r), f"reward step {t}"
        assert np.array_equal(done[t].cpu().numpy(), d), f"done step {t}"
        single.pcgrl_step(acts[t], o1, r1, d1)
        assert torch.equal(r1, rew[t]) and torch.equal(d1, done[t])
    for k, o in want_obs.items():
        assert_same("obs", obs[k], o, f"slot {k}")
    assert torch.equal(o1, obs[(T - 1) % slots])
    assert_same("metrics", roll.pcgrl_metrics(), cpu.metrics(), "after rollout")
    compare_state(roll, cpu, "after rollout")
    assert roll.pcgrl_bad_action_count() == int(((acts_np < 0) | (acts_np >= roll.K)).sum())
    # a second rollout continues from the stored state, and single steps continue after a rollout
    acts2_np = wl.random_actions(cfg, 9, 11)
    roll.pcgrl_rollout(torch.from_numpy(acts2_np).to(dev), None, None, None)
    for t in range(11):
        cpu.step(acts2_np[t], want_obs=False)
    compare_state(roll, cpu, "after second rollout")
    a3 = wl.random_actions(cfg, 10, 1)[0]
    roll.pcgrl_step(torch.from_numpy(a3).to(dev), o1, r1, d1)
    o, r, d = cpu.step(a3)
    assert_same("obs", o1, expected_obs(cfg, o), "step after rollout")
    assert np.array_equal(r1.cpu().numpy(), r)
    assert_same("metrics", roll.pcgrl_metrics(), cpu.metrics(), "step after rollout")
    for e in (roll, single):
        e.close()


def test_rollout_argument_errors():
    env = binding.Pcgrl(wl.workload("maze16", batch=4), 0)
    acts = torch.zeros((5, 4), dtype=torch.int32, device="cuda")
    obs = torch.zeros((6,) + env.obs_shape, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.PcgrlError):
        env.pcgrl_rollout(acts, obs)                      # more slots than steps
    with pytest.raises(binding.PcgrlError):
        env.pcgrl_rollout(acts[0])                        # not [T, B]
    assert env.L.pcgrl_rollout(env.h, None, 5, None, 1, None, None, None) == -1
    assert env.L.pcgrl_rollout(env.h, acts.data_ptr(), 0, None, 1, None, None, None) == -2
    env.close()


def _serpentine(n):
    """n x n binary level: open even rows joined by single cells at alternating ends."""
    t = np.ones((n, n), np.int8)
    t[0::2, :] = 0
    for k, y in enumerate(range(1, n - 1, 2)):
        t[y, n - 1 if k % 2 == 0 else 0] = 0
    return t


@pytest.mark.parametrize("n", [16, 32, 64])
def test_degenerate_and_extreme_levels(n):
    """All-wall, all-empty, one-cell and one-row / one-column maps, and the longest possible
    shortest path in an n x n buffer (a serpentine: 2078 edges for n = 64, so the sweeps and, once
    the scanning agent cuts it, the region searches run hundreds of trips: the long-flood code of
    every lane layout)."""
    dev = torch.device("cuda", 0)
    cases = []
    cases.append(("all wall", np.ones((n, n), np.int8), (n, n)))
    cases.append(("all empty", np.zeros((n, n), np.int8), (n, n)))
    cases.append(("serpentine", _serpentine(n), (n, n)))
    one = np.full((n, n), -1, np.int8); one[0, 0] = 0
    cases.append(("single cell", one, (1, 1)))
    row = np.full((n, n), -1, np.int8); row[0, :] = 0; row[0, n // 2 - 1] = 1
    cases.append(("one row", row, (1, n)))
    col = np.full((n, n), -1, np.int8); col[:, 0] = 0
    cases.append(("one column", col, (n, 1)))
    checker = ((np.add.outer(np.arange(n), np.arange(n)) % 2) == 1).astype(np.int8)
    cases.append(("checkerboard", checker, (n, n)))
    B = len(cases)
    cfg = wl.make_config(wl.BINARY, B, n, min(63, 2 * n - 1), min_size=1, autoreset=0, max_steps=10**6,
                         pos_mode=wl.POS_SCAN)
    for lpw, rmode in ((0, wl.REGIONS_INCREMENTAL), (0, wl.REGIONS_RECOUNT)):
        gpu = binding.Pcgrl(dict(cfg, regions_mode=rmode, levels_per_wave=lpw), 0)
        cpu = oracle.Oracle(cfg)
        tiles = np.stack([c[1] for c in cases])
        hw = np.array([c[2] for c in cases], np.int16)
        pos = np.zeros((B, 2), np.int16)
        gpu.pcgrl_reset(1)
        cpu.reset(1)
        gpu.pcgrl_set_state(torch.from_numpy(tiles).to(dev), None, torch.from_numpy(hw).to(dev),
                            torch.from_numpy(pos).to(dev))
        cpu.set_state(tiles, None, hw, pos)
        m = gpu.pcgrl_metrics().cpu().numpy()
        assert_same("metrics", m, cpu.metrics(), "degenerate levels")
        assert list(m[:3, 0]) == [0, 1, 1] and list(m[:3, 1]) == [0, 2 * (n - 1), n * n // 2 + n // 2 - 2]
        assert m[3, 0] == 1 and m[3, 1] == 0 and m[6, 0] == n * n // 2 and m[6, 1] == 0
        assert_same("obs", gpu.pcgrl_observe(), cpu.observe(), "degenerate levels")
        rew = torch.empty(B, dtype=torch.float32, device=dev)
        obs = gpu.new_obs()
        for t in range(n + 6):                   # flip the cell under the scanning agent
            st = cpu.get_state()
            cur = st["tiles"][np.arange(B), st["pos"][:, 0], st["pos"][:, 1]]
            a = (1 - cur).astype(np.int32)
            gpu.pcgrl_step(torch.from_numpy(a).to(dev), obs, rew, None)
            o, r, _ = cpu.step(a)
            assert_same("metrics", gpu.pcgrl_metrics(), cpu.metrics(), f"flip {t}")
            assert np.array_equal(rew.cpu().numpy(), r), f"flip {t}"
            assert_same("obs", obs, o, f"flip {t}")
        compare_state(gpu, cpu, "after flips")
        gpu.close()


def _rings(n):
    """Concentric square rings of open cells, one cell wide, one wall cell apart: n // 4 components
    nested in each other (plus a single centre cell when n % 4 is 1 or 2)."""
    t = np.ones((n, n), np.int8)
    for k in range(0, (n + 1) // 2, 2):
        t[k, k:n - k] = 0
        t[n - 1 - k, k:n - k] = 0
        t[k:n - k, k] = 0
        t[k:n - k, n - 1 - k] = 0
    return t


@pytest.mark.parametrize("n", [16, 32, 64])
def test_full_region_count_on_nested_mirrored_and_random_levels(n):
    """The from-scratch region count (reset, pcgrl_set_state, recount mode) on shapes that a
    shrinking or a flooding count could get wrong in different ways: components nested inside each
    other, the same shapes mirrored in both axes (a directional operator must not care), their
    complements, and random maps from sparse to full, in square and ragged active areas; then
    random edits with the count redone from scratch every step."""
    dev = torch.device("cuda", 0)
    rng = np.random.default_rng(1000 + n)
    cases = []
    rings = _rings(n)
    for name, t in (("rings", rings), ("rings complement", 1 - rings), ("serpentine", _serpentine(n)),
                    ("serpentine complement", 1 - _serpentine(n))):
        for flip_name, f in (("", t), (" ud", t[::-1]), (" lr", t[:, ::-1]), (" T", t.T)):
            cases.append((name + flip_name, np.ascontiguousarray(f).astype(np.int8), (n, n)))
    for dens in (0.05, 0.3, 0.45, 0.55, 0.6, 0.75, 0.95, 1.0):
        for h, w in ((n, n), (n, max(1, n // 3)), (max(1, n // 2 - 1), n), (int(rng.integers(1, n + 1)), int(rng.integers(1, n + 1)))):
            t = np.full((n, n), -1, np.int8)
            t[:h, :w] = (rng.random((h, w)) >= dens).astype(np.int8)   # 0 = open with probability dens
            cases.append((f"random {dens} {h}x{w}", t, (h, w)))
    B = len(cases)
    cfg = wl.make_config(wl.BINARY, B, n, 5, min_size=1, autoreset=0, max_steps=10**6, pos_mode=wl.POS_RANDOM)
    tiles = np.stack([c[1] for c in cases])
    hw = np.array([c[2] for c in cases], np.int16)
    pos = np.zeros((B, 2), np.int16)
    for lpw in (0, 1):
        gpu = binding.Pcgrl(dict(cfg, regions_mode=wl.REGIONS_RECOUNT, levels_per_wave=lpw), 0)
        cpu = oracle.Oracle(cfg)
        gpu.pcgrl_reset(7)
        cpu.reset(7)
        gpu.pcgrl_set_state(torch.from_numpy(tiles).to(dev), None, torch.from_numpy(hw).to(dev),
                            torch.from_numpy(pos).to(dev))
        cpu.set_state(tiles, None, hw, pos)
        m = gpu.pcgrl_metrics().cpu().numpy()
        assert_same("metrics", m, cpu.metrics(), "set_state")
        nested = (n + 3) // 4                      # rings at k = 0, 2, 4, ... < (n + 1) // 2
        assert list(m[:4, 0]) == [nested] * 4, "nested rings and their mirror images"
        assert list(m[8:12, 0]) == [1] * 4, "a serpentine is one component however it is turned"
        acts = wl.random_actions(cfg, 11, 3 * n, bad_fraction=0.0)
        rew = torch.empty(B, dtype=torch.float32, device=dev)
        for t in range(acts.shape[0]):
            gpu.pcgrl_step(torch.from_numpy(acts[t]).to(dev), None, rew, None)
            _, r, _ = cpu.step(acts[t])
            assert np.array_equal(rew.cpu().numpy(), r), f"step {t}"
        assert_same("metrics", gpu.pcgrl_metrics(), cpu.metrics(), "after edits")
        compare_state(gpu, cpu, "after edits")
        gpu.close()


@pytest.mark.parametrize("problem,n", [(wl.MAZE, 16), (wl.BINARY, 16), (wl.DUNGEON, 32), (wl.BINARY, 32), (wl.MAZE, 64)])
def test_episodes_that_end_at_different_steps(problem, n):
    """A small change limit ends every level's episode at a step of its own, so that in most
    steps one level of a wavefront restarts while its neighbours go on (a restarting level's cells
    are then drawn by all the lane groups of its wavefront together), now and then two or all of
    them at once; every launch shape, random shapes and pinpoints, single steps and a rollout."""
    base = wl.make_config(problem, 150, n, 9, min_size=max(3, n // 3), n_frozen=2, max_changes=4,
                          max_steps=37, pos_mode=wl.POS_RANDOM)
    shapes = [dict(levels_per_wave=0, split_step=0), dict(levels_per_wave=1, split_step=1),
              dict(levels_per_wave=2, split_step=2), dict(levels_per_wave=4, split_step=2, split_obs_levels=1),
              dict(levels_per_wave=4, split_step=1)]
    for k, shape in enumerate(shapes):
        cfg = dict(base, **shape)
        run_parity(cfg, 45, seed=50 + k, aseed=60 + k, label=f"staggered {shape}")
        _rollout_against_oracle(cfg, 45, 45, 70 + k)


@pytest.mark.parametrize("n", [16, 32, 64])
def test_long_corridors_in_maze_and_dungeon(n):
    """Player and door (and key, enemy) far apart along a serpentine corridor: path searches of
    hundreds of layers, cut and re-joined by edits on the corridor."""
    dev = torch.device("cuda", 0)
    corridor = _serpentine(n)
    ys, xs = np.nonzero(corridor == 0)
    far_y = n - 2 if (n - 1) % 2 else n - 1           # the last open row
    end_x = 0 if ((far_y // 2) % 2 == 1) else n - 1   # the corridor's far end in that row
    path_len = n * n // 2 + n // 2 - 2
    for pid in (wl.MAZE, wl.DUNGEON):
        t = corridor.copy()
        t[0, 0] = 2                                   # player at the start
        if pid == wl.MAZE:
            t[far_y, end_x] = 3                       # door at the far end
        else:
            t[far_y, end_x] = 4                       # door at the far end
            t[(n // 2) & ~1, n // 2] = 3              # a key half way (an open row)
            t[2, n // 2] = 5                          # an enemy near the start
        B = 4
        tiles = np.stack([t] * B)
        hw = np.full((B, 2), n, np.int16)
        # agents on the corridor: near the start, in the middle, near the end, and on the player
        mid = len(ys) // 2
        pos = np.array([[0, 3], [ys[mid], xs[mid]], [far_y, n // 2], [0, 0]], np.int16)
        cfg = wl.make_config(pid, B, n, 5, min_size=1, autoreset=0, max_steps=10**6)
        gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
        gpu.pcgrl_reset(2)
        cpu.reset(2)
        gpu.pcgrl_set_state(torch.from_numpy(tiles).to(dev), None, torch.from_numpy(hw).to(dev),
                            torch.from_numpy(pos).to(dev))
        cpu.set_state(tiles, None, hw, pos)
        m = gpu.pcgrl_metrics().cpu().numpy()
        assert_same("metrics", m, cpu.metrics(), f"corridor {n}")
        if pid == wl.MAZE:
            assert m[0, 0] == 1 and m[0, 1] == path_len, m[0]
        rew = torch.empty(B, dtype=torch.float32, device=dev)
        K = wl.NUM_TILES[pid]
        for step in range(24):                        # wall / re-open / other tiles under the agents
            a = np.array([(1, 0, 1, 0)[step % 4], (1, 0)[step % 2], (step + 1) % K, (step * 3 + 1) % K], np.int32)
            gpu.pcgrl_step(torch.from_numpy(a).to(dev), None, rew, None)
            _, r, _ = cpu.step(a, want_obs=False)
            assert_same("metrics", gpu.pcgrl_metrics(), cpu.metrics(), f"corridor {n} step {step}")
            assert np.array_equal(rew.cpu().numpy(), r), f"corridor {n} step {step}"
        compare_state(gpu, cpu, f"corridor {n}")
        gpu.close()


def _rollout_against_oracle(cfg, T, slots, seed):
    dev = torch.device("cuda", 0)
    B = cfg["batch"]
    acts_np = wl.random_actions(cfg, seed, T, bad_fraction=0.02)
    roll, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
    roll.pcgrl_reset(seed)
    cpu.reset(seed)
    obs = torch.zeros((slots,) + roll.obs_shape, dtype=torch.uint8, device=dev)
    rew = torch.empty((T, B), dtype=torch.float32, device=dev)
    done = torch.empty((T, B), dtype=torch.uint8, device=dev)
    roll.pcgrl_rollout(torch.from_numpy(acts_np).to(dev), obs, rew, done)
    want = {}
    for t in range(T):
        o, r, d = cpu.step(acts_np[t])
        want[t % slots] = o
        assert np.array_equal(rew[t].cpu().numpy(), r), f"reward step {t}"
        assert np.array_equal(done[t].cpu().numpy(), d), f"done step {t}"
    for k, o in want.items():
        check_obs(roll, obs[k], o, f"slot {k}")
    assert_same("metrics", roll.pcgrl_metrics(), cpu.metrics(), "after rollout")
    compare_state(roll, cpu, "after rollout")
    roll.close()


def test_random_configurations_and_launch_shapes():
    """Seeded random draws over everything a configuration has - problem, buffer and minimum size,
    window, padding, position mode, pinpoints, step and change budgets, auto-reset, real-valued
    weights, a controlled target, output format - and over every tuning knob (levels per
    wavefront, split, store mode, observation wavefronts), at batches on both sides of every
    automatic launch rule: single steps and a rollout against the oracle, rewards equal."""
    rng = np.random.default_rng(5)
    for n in range(48):
        problem = int(rng.integers(0, 3))
        size = int(rng.choice([5, 9, 16, 16, 23, 32, 32, 47, 64]))
        ow = int(rng.choice([1, 3, 5, 8, 15, 22, 31, 33, 47, 63]))
        batch = int(rng.choice([1, 3, 37, 64, 130, 513, 1000, 2049, 4100, 9001]))
        if size > 32:
            batch = min(batch, 2049)
        ms = int(rng.integers(1, size + 1)) if rng.random() < 0.6 else None
        nf = min(int(rng.choice([0, 0, 1, 3])), (ms if ms is not None else size) ** 2)
        cfg = wl.make_config(
            problem, batch, size, ow, min_size=ms, pad_mode=int(rng.integers(0, 2)),
            pos_mode=int(rng.integers(0, 2)), n_frozen=nf, max_steps=int(rng.choice([7, 19, 1000])),
            max_changes=int(rng.choice([0, 0, 5])), autoreset=int(rng.integers(0, 2)),
            levels_per_wave=int(rng.choice([0, 0, 1, 2, 4])), split_step=int(rng.choice([0, 0, 1, 2])),
            obs_store_mode=int(rng.choice([0, 0, 1, 2, 3])), obs_format=int(rng.choice([0, 0, 1])),
            obs_frozen_channel=int(rng.integers(0, 2)), split_obs_levels=int(rng.choice([0, 0, 1, 2])),
            rollout_turns=int(rng.choice([0, 1, 2, 4])),
            weights=[float(v) for v in rng.uniform(-2, 4, size=16).astype(np.float32)] if rng.random() < 0.5 else None,
            ctrl={1: (3, 40)} if rng.random() < 0.3 else None)
        steps = 20 if batch * size * size < 3e6 else 8
        run_parity(cfg, steps, seed=int(rng.integers(1, 1000)), aseed=int(rng.integers(1, 1000)),
                   bad_fraction=0.02, state_every=steps, label=f"random configuration {n}")
        _rollout_against_oracle(cfg, steps, int(rng.choice([1, 2, steps])), int(rng.integers(1, 1000)))


def test_random_configurations_with_pitched_observations():
    """The same kind of draws with an observation pitch on top: whole lines, or a random multiple of
    16 bytes at or above the observation's size; steps and a rollout against the oracle."""
    rng = np.random.default_rng(17)
    for n in range(24):
        problem = int(rng.integers(0, 3))
        size = int(rng.choice([7, 16, 16, 29, 32, 64]))
        ow = int(rng.choice([1, 3, 8, 15, 31, 40, 63]))
        batch = int(rng.choice([2, 37, 130, 1000, 2049, 4100]))
        if size > 32:
            batch = min(batch, 1000)
        packed = int(rng.choice([0, 0, 1]))
        fzc = int(rng.integers(0, 2))
        pad = int(rng.integers(0, 2))
        C = wl.NUM_TILES[problem] + (1 - pad) + fzc
        cells = C * ow * ow
        nbytes = (cells + 7) // 8 if packed else cells
        pitch = -1 if rng.random() < 0.5 else (nbytes + 15) // 16 * 16 + 16 * int(rng.integers(0, 9))
        cfg = wl.make_config(
            problem, batch, size, ow, min_size=int(rng.integers(1, size + 1)) if rng.random() < 0.5 else None,
            pad_mode=pad, pos_mode=int(rng.integers(0, 2)), n_frozen=int(rng.choice([0, 0, 1])),
            max_steps=int(rng.choice([9, 1000])), autoreset=int(rng.integers(0, 2)),
            levels_per_wave=int(rng.choice([0, 0, 1, 2, 4])), split_step=int(rng.choice([0, 1, 2])),
            obs_store_mode=int(rng.choice([0, 1, 2, 3])), obs_format=packed, obs_frozen_channel=fzc,
            split_obs_levels=int(rng.choice([0, 0, 1, 2])), obs_pitch=pitch,
            rollout_turns=int(rng.choice([0, 1, 2, 4])))
        steps = 16 if batch * size * size < 3e6 else 8
        run_parity(cfg, steps, seed=int(rng.integers(1, 1000)), aseed=int(rng.integers(1, 1000)),
                   state_every=steps, label=f"random pitched configuration {n} (pitch {pitch}, {nbytes} bytes)")
        _rollout_against_oracle(cfg, steps, int(rng.choice([1, 2, steps])), int(rng.integers(1, 1000)))


@pytest.mark.parametrize("split", [1, 2], ids=["unsplit", "split"])
@pytest.mark.parametrize("problem,size,ow,batch", [
    (wl.MAZE, 47, 33, 2049), (wl.BINARY, 64, 63, 2049), (wl.DUNGEON, 64, 47, 2049),
    (wl.BINARY, 32, 33, 4100), (wl.MAZE, 32, 47, 4100), (wl.DUNGEON, 23, 63, 4100), (wl.MAZE, 16, 33, 6000)])
def test_wide_windows_with_every_simd_shared(problem, size, ow, batch, split):
    """Windows wider than 32 cells run kernels of their own; at these batches several wavefronts
    share every SIMD from the first launch on, which is the condition under which a kernel with a
    register allocation the hardware mishandles gives wrong observations in a few percent of the
    levels (the build checks for the instruction pattern; this checks the result)."""
    cfg = wl.make_config(problem, batch, size, ow, pad_mode=wl.PAD_BORDER, n_frozen=1, max_steps=1000,
                         split_step=split, obs_store_mode=1)
    run_parity(cfg, 4, seed=132, aseed=546, state_every=4, label=f"wide window {ow} on {size}x{size}, batch {batch}")


def test_pinpoints_installed_later_are_respected():
    """A context created without pinpoints runs the step kernels that carry no pinpoint code; once
    pcgrl_set_state installs a frozen mask, steps (and a rollout) must leave those cells alone."""
    dev = torch.device("cuda", 0)
    for name, batch, split in (("maze16", 50, 2), ("maze64", 5, 1), ("dungeon32", 20, 1)):
        cfg = wl.workload(name, batch=batch, max_steps=10**6, autoreset=0, split_step=split)
        gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
        obs = gpu.new_obs()
        rew = torch.empty(batch, dtype=torch.float32, device=dev)
        gpu.pcgrl_reset(4, obs)
        cpu.reset(4)
        acts = wl.random_actions(cfg, 5, 60)
        for t in range(10):                                        # steps before any pinpoint exists
            gpu.pcgrl_step(torch.from_numpy(acts[t]).to(dev), obs, rew)
            o, r, _ = cpu.step(acts[t])
            assert_same("obs", obs, o, f"{name} step {t}")
        st = cpu.get_state()
        rng = np.random.default_rng(3)
        fro = (rng.random(st["tiles"].shape) < 0.4).astype(np.uint8)
        gpu.pcgrl_set_state(*(torch.from_numpy(a).to(dev) for a in (st["tiles"], fro, st["hw"], st["pos"])))
        cpu.set_state(st["tiles"], fro, st["hw"], st["pos"])
        for t in range(10, 40):
            gpu.pcgrl_step(torch.from_numpy(acts[t]).to(dev), obs, rew)
            o, r, _ = cpu.step(acts[t])
            assert_same("obs", obs, o, f"{name} step {t}")
            assert np.array_equal(rew.cpu().numpy(), r), f"{name} step {t}"
        compare_state(gpu, cpu, f"{name} after frozen steps")
        gpu.pcgrl_rollout(torch.from_numpy(acts[40:]).to(dev))
        for t in range(40, 60):
            cpu.step(acts[t], want_obs=False)
        compare_state(gpu, cpu, f"{name} after the rollout")
        assert (cpu.get_state()["tiles"][fro.astype(bool)] == st["tiles"][fro.astype(bool)]).all()
        gpu.close()


def test_small_buffers_and_every_window_size():
    """Buffers smaller than a lane group (5x3, 1x1) and every window size 1..63 on a 16x16 maze."""
    run_parity(wl.make_config(wl.MAZE, 9, 5, 7, max_w=3, min_size=1, min_w=1, max_steps=11), 40, label="5x3 buffer")
    run_parity(wl.make_config(wl.DUNGEON, 3, 1, 3, max_steps=5), 12, label="1x1 buffer")
    dev = torch.device("cuda", 0)
    for ow in range(1, 64):
        cfg = wl.make_config(wl.MAZE, 6, 16, ow, min_size=9, max_steps=4, pad_mode=ow % 2,
                             levels_per_wave=(0, 2, 4)[ow % 3])
        gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
        obs = gpu.new_obs()
        gpu.pcgrl_reset(ow, obs)
        assert_same("obs", obs, cpu.reset(ow), f"ow={ow} reset")
        acts = wl.random_actions(cfg, ow, 6)
        for t in range(6):
            gpu.pcgrl_step(torch.from_numpy(acts[t]).to(dev), obs)
            o, _, _ = cpu.step(acts[t])
            assert_same("obs", obs, o, f"ow={ow} step {t}")
        gpu.close()


def test_largest_batch_spot_check():
    """2^20 binary levels: one reset and two steps; everything compared on a strided sample of
    environments (the oracle takes the same global environment indices through set_state)."""
    dev = torch.device("cuda", 0)
    B = 1 << 20
    cfg = wl.workload("binary16", batch=B, max_steps=50)
    gpu = binding.Pcgrl(cfg, 0)
    obs = gpu.new_obs()
    rew = torch.empty(B, dtype=torch.float32, device=dev)
    done = torch.empty(B, dtype=torch.uint8, device=dev)
    gpu.pcgrl_reset(3, obs)
    idx = np.arange(0, B, 4099)
    idx = np.concatenate([idx, [B - 3, B - 2, B - 1]])
    st0 = {k: v[torch.from_numpy(idx).to(dev)].cpu().numpy() for k, v in gpu.pcgrl_get_state().items()}
    cpu = oracle.Oracle(dict(cfg, batch=len(idx)))
    cpu.reset(0)
    cpu.set_state(st0["tiles"], st0["frozen"], st0["hw"], st0["pos"])
    tidx = torch.from_numpy(idx).to(dev)
    assert_same("metrics", gpu.pcgrl_metrics()[tidx], cpu.metrics(), "2^20 after reset")
    assert_same("obs", obs[tidx], cpu.observe(), "2^20 after reset")
    acts = wl.random_actions(cfg, 1, 1)[0]
    gpu.pcgrl_step(torch.from_numpy(acts).to(dev), obs, rew, done)
    _, r, d = cpu.step(acts[idx], want_obs=False)
    assert np.array_equal(rew[tidx].cpu().numpy(), r)
    assert_same("metrics", gpu.pcgrl_metrics()[tidx], cpu.metrics(), "2^20 after a step")
    g = gpu.pcgrl_get_state()
    assert_same("tiles", g["tiles"][tidx], cpu.get_state()["tiles"], "2^20 after a step")
    # the observation is centred on the GPU's own (seeded) next position: check it structurally
    o = obs[tidx].cpu().numpy()
    assert (o.sum(axis=1) == 1).all()
    pos = g["pos"][tidx].cpu().numpy()
    t = g["tiles"][tidx].cpu().numpy()
    assert (o[np.arange(len(idx)), t[np.arange(len(idx)), pos[:, 0], pos[:, 1]], 15, 15] == 1).all()
    gpu.close()


@pytest.mark.parametrize("pos_mode", [wl.POS_SCAN, wl.POS_RANDOM], ids=["scan", "random"])
def test_split_step_at_full_batch_for_thousands_of_steps(pos_mode):
    """The step split into a metrics wavefront and an observation wavefront per workgroup, at the
    benchmark batch, for 2000 steps: the observation wavefront reads the level that the metrics
    wavefront of the same step overwrites, so every observation has to show the state after
    exactly the edits so far.  Rewards, done flags and metrics of every step (all levels),
    observations and the whole state every 50th step; the oracle is sharded over host threads."""
    from concurrent.futures import ThreadPoolExecutor
    dev = torch.device("cuda", 0)
    steps, B, chunk, shards = 2000, 4096, 50, 8
    cfg = wl.workload("maze16", batch=B, max_steps=700, pos_mode=pos_mode, split_step=2)
    print(f"[split long] pos_mode={pos_mode} batch={B} steps={steps}", flush=True)
    gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
    obs = gpu.new_obs()
    gpu.pcgrl_reset(5, obs)
    cpu.reset(5, want_obs=False)
    acts_np = wl.random_actions(cfg, 6, steps)
    acts = torch.from_numpy(acts_np).to(dev)
    rew = torch.empty((chunk, B), dtype=torch.float32, device=dev)
    done = torch.empty((chunk, B), dtype=torch.uint8, device=dev)
    met = torch.empty((chunk, B, gpu.M), dtype=torch.int32, device=dev)
    c_obs = cpu.new_obs()
    c_rew = np.zeros((chunk, B), np.float32)
    c_done = np.zeros((chunk, B), np.uint8)
    c_met = np.zeros((chunk, B, gpu.M), np.int32)
    bounds = [(i * B // shards, (i + 1) * B // shards) for i in range(shards)]
    with ThreadPoolExecutor(shards) as pool:
        for t0 in range(0, steps, chunk):
            for k in range(chunk):
                gpu.pcgrl_step(acts[t0 + k], obs, rew[k], done[k])
                gpu.pcgrl_metrics(met[k])
            for k in range(chunk):
                o = c_obs if k == chunk - 1 else None      # the oracle writes the window only where it is compared
                list(pool.map(lambda b: cpu.step_range(b[0], b[1], acts_np[t0 + k], o, c_rew[k], c_done[k]), bounds))
                c_met[k] = cpu.metrics()
            ctx = f"steps {t0}..{t0 + chunk - 1}"
            assert np.array_equal(rew.cpu().numpy(), c_rew), "reward " + ctx
            assert np.array_equal(done.cpu().numpy(), c_done), "done " + ctx
            assert np.array_equal(met.cpu().numpy(), c_met), "metrics " + ctx
            assert_same("obs", obs, c_obs, f"step {t0 + chunk - 1}")
            compare_state(gpu, cpu, f"step {t0 + chunk - 1}")
            print(f"[split long] {ctx} ok", flush=True)
    gpu.close()


LONG = [
    ("maze16", wl.workload("maze16", batch=96, max_steps=3000), 4000),
    ("binary16", wl.workload("binary16", batch=64, max_steps=1000), 2500),
    ("dungeon32", wl.workload("dungeon32", batch=48, max_steps=1500), 2000),
    ("binary32 rand", wl.workload("binary32_rand_ow15", batch=48, max_steps=1000), 2000),
    ("maze64", wl.workload("maze64", batch=12, max_steps=1000), 1500),
    ("binary64 dense", wl.make_config(wl.BINARY, 8, 64, 31, max_steps=2000, probs=[.62, .38]), 1500),
]


@pytest.mark.parametrize("label,cfg,steps", LONG, ids=[l[0] for l in LONG])
def test_long_runs_do_not_drift(label, cfg, steps):
    """Thousands of steps in a row (the map drifts from its initial tile mix towards uniform, the
    incrementally maintained region and tile counts never get a fresh start inside an episode):
    rewards, done flags and metrics every step, observations and state now and then."""
    print(f"[long] {label} steps={steps}", flush=True)
    dev = torch.device("cuda", 0)
    B = cfg["batch"]
    gpu, cpu = binding.Pcgrl(cfg, 0), oracle.Oracle(cfg)
    obs = gpu.new_obs()
    gpu.pcgrl_reset(77, obs)
    cpu.reset(77, want_obs=False)
    acts_np = wl.random_actions(cfg, 78, steps)
    acts = torch.from_numpy(acts_np).to(dev)
    chunk = 50
    rew = torch.empty((chunk, B), dtype=torch.float32, device=dev)
    done = torch.empty((chunk, B), dtype=torch.uint8, device=dev)
    met = torch.empty((chunk, B, gpu.M), dtype=torch.int32, device=dev)
    for t0 in range(0, steps, chunk):
        n = min(chunk, steps - t0)
        for k in range(n):
            gpu.pcgrl_step(acts[t0 + k], obs, rew[k], done[k])
            gpu.pcgrl_metrics(met[k])
        g_r, g_d, g_m = rew.cpu().numpy(), done.cpu().numpy(), met.cpu().numpy()
        for k in range(n):
            last = k == n - 1
            o, r, d = cpu.step(acts_np[t0 + k], want_obs=last)
            ctx = f"step {t0 + k}"
            assert np.array_equal(g_r[k], r), "reward " + ctx
            assert np.array_equal(g_d[k], d), "done " + ctx
            assert np.array_equal(g_m[k], cpu.metrics()), "metrics " + ctx
        assert_same("obs", obs, o, f"step {t0 + n - 1}")
        if (t0 // chunk) % 8 == 0:
            compare_state(gpu, cpu, f"step {t0 + n - 1}")
    compare_state(gpu, cpu, "end")
    gpu.close()
