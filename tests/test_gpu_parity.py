"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle element by
element on the same seeded inputs.  Bit-exact where the work is selection and copying;
within 1e-6 (float32) / 1e-2 (bfloat16 parameters) of the terms' magnitude on values."""

import numpy as np
import pytest
import torch

from oracle import dadam_oracle as O
from paper_2410_11998_amd import binding as B
from paper_2410_11998_amd import workloads as WL

import harness as H

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
MODES = {"tile": B.DADAM_FORCE_TILE, "direct": B.DADAM_FORCE_DIRECT, "auto": 0}


def flat_layout(d):
    return WL.pack([("flat", (d,))])


def say(*a):
    print(*a, flush=True)


# ---------------------------------------------------------------------------------------------
# neighbour selection: permutation matrices copy bit-exactly
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("mode", ["tile", "direct"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout_name", ["flat", "odd"])
def test_permutation_mixing_is_a_bit_exact_copy(mode, dtype, layout_name):
    say("case", mode, dtype, layout_name)
    n = 7
    layout = flat_layout(5000) if layout_name == "flat" else WL.pack(WL.odd_shapes())
    perm = [3, 0, 6, 1, 5, 2, 4]
    sim = H.GpuSim(n, n, layout, H.HyperF32(s=2), [WL.permutation(perm)], dtype, dtype, pad_fill=None)
    d = layout.d
    # every element carries a code of (source, position) that is exact in the storage type
    for c in range(n):
        if dtype == "f32":
            code = torch.arange(d, dtype=torch.float32) + float(c) * 16384.0
            code[::7] = -0.0
        else:
            code = ((torch.arange(d) % 128).to(torch.float32) + 128.0) * float(2 ** c)   # 8 significant bits
        sim.x_src[c].copy_(code.to(H.TORCH_DT[dtype]))
    for i in range(n):
        sim.x_dst[i].fill_(-1.0)
    sim.mix(0, MODES[mode])
    torch.cuda.synchronize()
    mask = torch.from_numpy(H.valid_mask(layout)).to(DEV)
    view = torch.int32 if dtype == "f32" else torch.int16
    for i in range(n):
        got = sim.x_dst[i].view(view)[mask]
        want = sim.x_src[perm[i]].view(view)[mask]
        assert torch.equal(got, want), f"row {i} is not a bit copy of source {perm[i]}"
        if layout_name == "odd":
            assert bool(torch.all(sim.x_dst[i][~mask] == -1.0)), "padding was written"
    sim.close()


@pytest.mark.parametrize("mode", ["tile", "direct"])
def test_step_with_permutation_and_zero_direction_copies_bit_exact(mode):
    """The fused kernels select neighbours the same way: zero gradient and zero moments give a
    zero direction, so x_dst must again be a bit copy."""
    say("case", mode)
    n = 5
    perm = [4, 2, 0, 1, 3]
    layout = flat_layout(3001)
    d = layout.d
    sim = H.GpuSim(n, n, layout, H.HyperF32(s=2), [WL.permutation(perm)], pad_fill=None)
    for c in range(n):
        sim.x_src[c].copy_(torch.arange(d, dtype=torch.float32) * 0.25 + 1000.0 * c)
    zeros = [torch.zeros(d, device=DEV) for _ in range(n)]
    sim.step(zeros, 1, 0, B.DADAM_FUSE_ACCUM | MODES[mode])
    torch.cuda.synchronize()
    for i in range(n):
        assert torch.equal(sim.x_dst[i][:3001].view(torch.int32), sim.x_src[perm[i]][:3001].view(torch.int32))
        assert bool(torch.all(sim.x_dst[i][3001:] == 0)), "padding was written"
        assert bool(torch.all(sim.b[i] == 0)) and bool(torch.all(sim.m[i] == 0))
    sim.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_mix_matches_oracle_rectangular_random_rows(dtype):
    say("case", dtype)
    rng = np.random.default_rng(5)
    R, C = 3, 9
    layout = flat_layout(4099)
    d = layout.d
    row_ptr, col, w = [0], [], []
    for i in range(R):
        deg = [1, 9, 4][i]
        cols = rng.permutation(C)[:deg]
        ww = rng.random(deg).astype(np.float32) + np.float32(0.1)
        ww = (ww / ww.sum(dtype=np.float32)).astype(np.float32)
        col += list(cols); w += list(ww); row_ptr.append(len(col))
    t3 = (np.array(row_ptr, np.int32), np.array(col, np.int32), np.array(w, np.float32))
    sim = H.GpuSim(R, C, layout, H.HyperF32(s=1), [t3], dtype, dtype)
    for c in range(C):
        sim.x_src[c].copy_(H.to_device(WL.normal_np(100 + c, d, 1.0), dtype, DEV))
    sim.mix()
    torch.cuda.synchronize()
    xs = sim._get(sim.x_src, None)
    csr = H.csr_oracle(t3)
    ref = O.mix_only(xs, csr, "O32m", dtype)
    got = sim._get(sim.x_dst, None)
    for i in range(R):
        scale = sum(abs(csr.w[k]) * np.abs(xs[csr.col[k]]) for k in range(csr.row_ptr[i], csr.row_ptr[i + 1]))
        ok = H.valid_mask(layout)
        assert np.all(np.abs(got[i] - ref[i])[ok] <= (H.RTOL[dtype] * scale)[ok])
    sim.close()


# ---------------------------------------------------------------------------------------------
# configuration 1 whole, and small copies of configurations 2-5 whole
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("mode", ["tile", "direct"])
def test_config1_every_element_every_step(mode):
    say("case", mode)
    wl = WL.workload(1)
    hp = H.HyperF32(wl.lr, wl.beta1, wl.beta2, wl.eps, wl.s)
    worst = H.run_parity(wl.name, wl.n_rows, wl.n_cols, wl.layout(), hp, [wl.csr()], lambda t: 0, wl.steps,
                         seed=wl.cfg, grad_std=wl.grad_std, flags=B.DADAM_FUSE_ACCUM | MODES[mode])
    say("worst error / tolerance:", worst)


@pytest.mark.parametrize("cfg,div,mode,full", [(2, 16, "auto", True), (2, 16, "direct", False), (3, 16, "auto", True),
                                              (3, 16, "tile", False), (4, 16, "auto", True), (4, 8, "auto", False),
                                              (4, 8, "direct", False), (5, 32, "auto", True), (5, 16, "auto", False),
                                              (5, 16, "direct", False)])
def test_scaled_configs_every_element(cfg, div, mode, full):
    """Small copies of configurations 2-5 (same tensor lists, dimensions divided), every element checked
    at every iteration, teacher-forced and against a free-running oracle; `full` runs the configuration's
    whole step count (20, 50, 30, 10 iterations), the others two accumulation loops and a step."""
    say("case", cfg, div, mode, full)
    wl = WL.workload(cfg, scale_div=div)
    hp = H.HyperF32(wl.lr, wl.beta1, wl.beta2, wl.eps, wl.s)
    csrs = [wl.csr(k) for k in range(wl.n_slots())]
    T = wl.steps if full else min(wl.steps, 2 * wl.s + 1)
    worst = H.run_parity(wl.name, wl.n_rows, wl.n_cols, wl.layout(), hp, csrs, lambda t: wl.slot_of_step(t), T,
                         seed=10 + cfg, param_dtype=wl.param_dtype, grad_dtype=wl.grad_dtype, grad_std=wl.grad_std,
                         flags=B.DADAM_FUSE_ACCUM | MODES[mode], refresh_extra_sources=(cfg == 3),
                         inplace=(cfg == 3), pad_fill=None)
    say("worst error / tolerance:", worst)


# ---------------------------------------------------------------------------------------------
# ragged layouts, every phase, both modes, all dtype pairs
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("mode", ["tile", "direct"])
@pytest.mark.parametrize("pd,gd", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32"), ("f32", "bf16")])
@pytest.mark.parametrize("s", [1, 3])
def test_odd_layout_all_phases(mode, pd, gd, s):
    say("case", mode, pd, gd, s)
    n = 3
    layout = WL.pack(WL.odd_shapes())
    hp = H.HyperF32(lr=2e-3, s=s)
    worst = H.run_parity("odd", n, n, layout, hp, [WL.ring(n)], lambda t: 0, 2 * s + 1, seed=77, param_dtype=pd,
                         grad_dtype=gd, grad_std=1e-2, flags=B.DADAM_FUSE_ACCUM | MODES[mode])
    say("worst error / tolerance:", worst)


@pytest.mark.parametrize("mode", ["tile", "direct"])
def test_unfused_sequence_matches_oracle_and_fused_bitwise(mode):
    say("case", mode)
    n, s, T = 4, 2, 5
    layout = WL.pack(WL.odd_shapes())
    hp = H.HyperF32(s=s)
    H.run_parity("unfused", n, n, layout, hp, [WL.ring(n)], lambda t: 0, T, seed=78, unfused=True,
                 flags=B.DADAM_FUSE_ACCUM | MODES[mode])
    # and the two call sequences give identical bits
    sims = [H.GpuSim(n, n, layout, hp, [WL.ring(n)], pad_fill=None) for _ in range(2)]
    for sim in sims:
        for c in range(n):
            sim.x_src[c].copy_(H.to_device(WL.normal_np(900 + c, layout.d, 0.02), "f32", DEV))
    for t in range(1, T + 1):
        grads = [H.to_device(WL.normal_np(1000 + t * 8 + i, layout.d, 1e-2), "f32", DEV) for i in range(n)]
        sims[0].step(grads, t, 0, B.DADAM_FUSE_ACCUM | MODES[mode])
        sims[1].step(grads, t, 0, MODES[mode])
        sims[1].accumulate(grads, t)
        torch.cuda.synchronize()
        for a, b in zip(sims[0].x_dst + sims[0].m + sims[0].v + sims[0].b, sims[1].x_dst + sims[1].m + sims[1].v + sims[1].b):
            assert torch.equal(a, b)
        for sim in sims:
            sim.swap()
    for sim in sims:
        sim.close()


def test_in_place_tile_mode_equals_ping_pong_bitwise():
    n, T = 8, 4
    wl = WL.workload(2, scale_div=32)
    layout = wl.layout()
    hp = H.HyperF32(s=2)
    csr = WL.static_exponential(n)
    a = H.GpuSim(n, n, layout, hp, [csr], inplace=False)
    b = H.GpuSim(n, n, layout, hp, [csr], inplace=True)
    assert B.dadam_slot_uses_tile_mode(b.h, 0)
    for c in range(n):
        x0 = H.to_device(WL.normal_np(300 + c, layout.d, 0.02), "f32", DEV)
        a.x_src[c].copy_(x0); b.x_src[c].copy_(x0)
    for t in range(1, T + 1):
        grads = [H.to_device(WL.normal_np(400 + t * 8 + i, layout.d, 1e-3), "f32", DEV) for i in range(n)]
        a.step(grads, t); b.step(grads, t)
        torch.cuda.synchronize()
        for i in range(n):
            assert torch.equal(a.x_dst[i], b.x_dst[i])
        a.swap()
    with pytest.raises(B.DadamError) as e:
        b.step(grads, T + 1, 0, B.DADAM_FUSE_ACCUM | B.DADAM_FORCE_DIRECT)
    assert e.value.code == B.DADAM_EALIAS
    a.close(); b.close()


def test_bucket_ranges_compose_to_the_whole_step():
    """Stepping tensor ranges one after the other (buckets) gives the bits of one whole step."""
    n = 4
    layout = WL.pack(WL.odd_shapes() + [("big", (70001,))])
    hp = H.HyperF32(s=2)
    nt = len(layout.names)
    for mode in ("tile", "direct"):
        say("case", mode)
        a = H.GpuSim(n, n, layout, hp, [WL.ring(n)])
        b = H.GpuSim(n, n, layout, hp, [WL.ring(n)])
        for c in range(n):
            x0 = H.to_device(WL.normal_np(500 + c, layout.d, 0.02), "f32", DEV)
            a.x_src[c].copy_(x0); b.x_src[c].copy_(x0)
        for t in (1, 2, 3):
            grads = [H.to_device(WL.normal_np(600 + t * 8 + i, layout.d, 1e-2), "f32", DEV) for i in range(n)]
            a.step(grads, t, 0, B.DADAM_FUSE_ACCUM | MODES[mode])
            for tb, te in ((nt - 1, nt), (5, nt - 1), (0, 2), (2, 5), (3, 3)):
                b.step_range(grads, t, tb, te, 0, B.DADAM_FUSE_ACCUM | MODES[mode])
            torch.cuda.synchronize()
            for u, v in zip(a.x_dst + a.m + a.v + a.b, b.x_dst + b.m + b.v + b.b):
                assert torch.equal(u, v)
            a.swap(); b.swap()
        a.close(); b.close()


def test_resume_from_saved_buffers_is_bit_identical():
    n, T, T1 = 4, 7, 3
    layout = flat_layout(10007)
    hp = H.HyperF32(s=4)
    def fresh():
        s = H.GpuSim(n, n, layout, hp, [WL.ring(n)], pad_fill=None)
        return s
    grads_of = lambda t: [H.to_device(WL.normal_np(700 + t * 8 + i, layout.d, 1e-2), "f32", DEV) for i in range(n)]
    a = fresh()
    for c in range(n):
        a.x_src[c].copy_(H.to_device(WL.normal_np(650 + c, layout.d, 0.02), "f32", DEV))
    x0 = [x.clone() for x in a.x_src]
    for t in range(1, T + 1):
        a.step(grads_of(t), t); a.swap()
    b = fresh()
    for c in range(n):
        b.x_src[c].copy_(x0[c])
    for t in range(1, T1 + 1):
        b.step(grads_of(t), t); b.swap()
    torch.cuda.synchronize()
    saved = [[x.clone() for x in grp] for grp in (b.x_src, b.m, b.v, b.b)]
    b.close()
    c_ = fresh()
    for grp, src in zip((c_.x_src, c_.m, c_.v, c_.b), saved):
        for dst, s_ in zip(grp, src):
            dst.copy_(s_)
    for t in range(T1 + 1, T + 1):
        c_.step(grads_of(t), t); c_.swap()
    torch.cuda.synchronize()
    for u, v in zip(a.x_src + a.m + a.v + a.b, c_.x_src + c_.m + c_.v + c_.b):
        assert torch.equal(u, v)
    a.close(); c_.close()


def test_zero_gradient_zero_state_is_pure_mixing_without_nan():
    n = 4
    layout = flat_layout(2049)
    d = layout.d
    sim = H.GpuSim(n, n, layout, H.HyperF32(s=2), [WL.ring(n)], pad_fill=None)
    for c in range(n):
        sim.x_src[c].copy_(H.to_device(WL.normal_np(800 + c, d, 0.02), "f32", DEV))
    zeros = [torch.zeros(d, device=DEV) for _ in range(n)]
    sim.step(zeros, 1)
    torch.cuda.synchronize()
    stepped = [x.clone() for x in sim.x_dst]
    sim.mix()
    torch.cuda.synchronize()
    for i in range(n):
        assert bool(torch.all(torch.isfinite(stepped[i]))) and torch.equal(stepped[i], sim.x_dst[i])
    sim.close()


def test_max_rows_complete_graph_and_lr_change():
    """64 rows x 64 sources, every row of full degree: the largest neighbour list the
    library takes; then a change of step size through dadam_set_lr."""
    n = 64
    hp = H.HyperF32(s=1)
    layout = flat_layout(1500)
    d = layout.d
    for mode in ("tile", "direct"):
        say("case", mode)
        H.run_parity("complete64", n, n, layout, hp, [WL.complete(n)], lambda t: 0, 2, seed=91,
                     flags=B.DADAM_FUSE_ACCUM | MODES[mode], pad_fill=None)
    sim = H.GpuSim(2, 2, layout, hp, [WL.identity(2)], pad_fill=None)
    g = [torch.full((d,), 0.5, device=DEV) for _ in range(2)]
    sim.step(g, 1)
    B.dadam_set_lr(sim.h, 0.25)
    sim.swap()
    sim.step(g, 2)
    torch.cuda.synchronize()
    # constant gradient: every iteration moves by lr * c / (|c| + eps)
    want = -(np.float32(1e-3) + np.float32(0.25)) * 0.5 / (0.5 + 1e-8)
    np.testing.assert_allclose(sim.x_dst[0][:1500].cpu().numpy(), want, rtol=1e-6)
    sim.close()


def test_literal_beta1_fold_selectable():
    n, d, s = 2, 1000, 2
    hp = H.HyperF32(s=s, beta_vhat=0.9)
    H.run_parity("literal", n, n, flat_layout(d), hp, [WL.ring(n)], lambda t: 0, 4, seed=92, pad_fill=None)


# ---------------------------------------------------------------------------------------------
# full-size configurations in the benchmark's launch configuration, sampled coordinates
# ---------------------------------------------------------------------------------------------

def sample_coordinates(layout, rng, n_random, info):
    """The coordinates the full-size tests check: the first and last 4096, 64 either side of every tensor
    boundary, of the boundaries between the dies' shares of the tiles and of 1024 randomly chosen tile
    boundaries of each kernel's grid, and n_random seeded uniform ones."""
    d = layout.d
    pick = [np.arange(0, min(4096, d)), np.arange(max(0, d - 4096), d)]
    near = lambda edge: np.arange(max(0, edge - 64), min(d, edge + 64))
    for o, n in zip(layout.offsets, layout.numels):
        for edge in (int(o), int(o) + int(n)):
            pick.append(near(edge))
    for tile, n_tiles in ((int(info.tile_elems), int(info.n_tiles_tile)), (int(info.direct_elems), int(info.n_tiles_direct)),
                          (int(info.mix_tile_elems), int(info.n_tiles_mix))):
        if tile == 0 or n_tiles < 2:
            continue
        share = n_tiles // int(info.n_xcds)
        for k in range(1, int(info.n_xcds)):
            pick.append(near(k * share * tile))
        for b in rng.integers(1, n_tiles, size=1024):
            pick.append(near(int(b) * tile))
    pick.append(rng.integers(0, d, size=n_random))
    return np.unique(np.concatenate(pick))


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_configs_sampled(cfg):
    say("case", cfg)
    wl = WL.workload(cfg)
    layout = wl.layout()
    hp = H.HyperF32(wl.lr, wl.beta1, wl.beta2, wl.eps, wl.s)
    ohp = hp.oracle()
    csrs = [wl.csr(k) for k in range(wl.n_slots())]
    dev = torch.device(DEV)
    sim = H.GpuSim(wl.n_rows, wl.n_cols, layout, hp, csrs, wl.param_dtype, wl.grad_dtype, inplace=(cfg == 3), pad_fill=None,
                   spread=True)     # the layout bench.py times
    rng = np.random.default_rng(cfg)
    # 2^20 random coordinates per row (2^18 with 64 rows: the same 2^24 values a step, the oracle's minute)
    idx_np = sample_coordinates(layout, rng, 1 << (18 if wl.n_rows > 16 else 20), B.dadam_get_plan_info(sim.h))
    say("coordinates checked per row", len(idx_np))
    idx = torch.from_numpy(idx_np).to(dev)
    x0 = WL.normal_torch(WL.seed_for(cfg, 0), (layout.d,), wl.param_std, dev, H.TORCH_DT[wl.param_dtype])
    for c in range(wl.n_rows):
        sim.x_src[c].copy_(x0)
        # replicas start equal (Algorithm 1 line 1); perturb so that mixing is visible at once
        sim.x_src[c].add_(WL.normal_torch(WL.seed_for(cfg, 500 + c), (layout.d,), 1e-3, dev, H.TORCH_DT[wl.param_dtype]))
    del x0
    T = wl.steps                                   # the configuration's own number of iterations
    grads = [torch.empty(layout.d, dtype=H.TORCH_DT[wl.grad_dtype], device=dev) for _ in range(wl.n_rows)]
    gen = torch.Generator(device=dev)
    import time
    started = time.time()
    for t in range(1, T + 1):
        for c in range(wl.n_rows, wl.n_cols):
            sim.x_src[c].copy_(WL.normal_torch(WL.seed_for(cfg, 1) + 7 * t + c, (layout.d,), wl.param_std, dev, H.TORCH_DT[wl.param_dtype]))
        gen.manual_seed(WL.seed_for(cfg, 2 + t))
        for g in grads:
            if wl.grad_dtype == "f32":
                g.normal_(0.0, wl.grad_std, generator=gen)
            else:
                g.copy_(torch.empty(layout.d, dtype=torch.float32, device=dev).normal_(0.0, wl.grad_std, generator=gen))
        slot = wl.slot_of_step(t)
        prev = sim.snapshot(idx)
        g64 = [g[idx].to(torch.float64).cpu().numpy() for g in grads]
        sim.step(grads, t, slot)
        torch.cuda.synchronize()
        got = sim.outputs(idx)
        ref_state = O.State(prev.x_src, list(prev.m_hat), list(prev.v_hat), list(prev.b))
        csr = H.csr_oracle(csrs[slot])
        ref_x = O.dadam_step(ref_state, g64, csr, t, ohp, "O32m", wl.param_dtype)
        w = H.compare_step(prev, ref_x, ref_state, got, g64, csr, t, ohp, wl.param_dtype, None, f"{wl.name} t={t}")
        say(f"t={t} ({time.time() - started:.0f} s) worst error / tolerance: {w}")
        H.assert_within(w, f"{wl.name} full size t={t}")
        sim.swap()
    # a property that holds at any size: with a doubly stochastic W the replica mean moves only
    # by the mean direction, so mixing alone leaves it where it was (checked on a slice)
    if wl.n_rows == wl.n_cols:
        sl = slice(0, 1 << 20)
        before = torch.stack([x[sl].to(torch.float64) for x in sim.x_src]).mean(0)
        sim.mix(0)
        torch.cuda.synchronize()
        after = torch.stack([x[sl].to(torch.float64) for x in sim.x_dst]).mean(0)
        tol = 1e-6 if wl.param_dtype == "f32" else 1e-2
        assert float((after - before).abs().max()) <= tol * float(before.abs().max())
    sim.close()
    del sim, grads
    torch.cuda.empty_cache()


def test_spread_arena_layout_matches_oracle():
    """Buffers carved from one arena at the offsets dadam_spread_offsets gives (the layout the
    benchmark uses) behave like separate allocations."""
    from paper_2410_11998_amd.arena import SpreadArena
    n, T = 4, 3
    layout = WL.pack(WL.odd_shapes() + [("big", (300001,))])
    d = layout.d
    hp = H.HyperF32(s=2)
    for dtype in ("f32", "bf16"):
        say("case", dtype)
        sim = H.GpuSim(n, n, layout, hp, [WL.ring(n)], dtype, dtype, pad_fill=None)
        px = 2 if dtype == "bf16" else 4
        dts = [H.TORCH_DT[dtype]] * (2 * n) + [torch.float32] * (3 * n) + [H.TORCH_DT[dtype]] * n
        arena = SpreadArena([d * px] * (2 * n) + [d * 4] * (3 * n) + [d * px] * n, DEV, span_bytes=256 << 20)
        v = arena.views(dts)
        assert all(t.numel() == d and t.data_ptr() % (2 << 20) == 0 for t in v)
        sim.x_src, sim.x_dst, sim.m, sim.v, sim.b, grads = v[:n], v[n:2 * n], v[2 * n:3 * n], v[3 * n:4 * n], v[4 * n:5 * n], v[5 * n:]
        for t_ in sim.x_dst + sim.m + sim.v + sim.b:
            t_.zero_()
        for c in range(n):
            sim.x_src[c].copy_(H.to_device(WL.normal_np(1200 + c, d, 0.02), dtype, DEV))
        sim.bind()
        ohp = hp.oracle()
        csr = H.csr_oracle(WL.ring(n))
        mask = H.valid_mask(layout)
        for t in range(1, T + 1):
            for i in range(n):
                grads[i].copy_(H.to_device(WL.normal_np(1300 + 8 * t + i, d, 1e-2), dtype, DEV))
            g64 = [g.to(torch.float64).cpu().numpy() for g in grads]
            prev = sim.snapshot()
            sim.step(grads, t)
            torch.cuda.synchronize()
            ref_state = O.State(prev.x_src, list(prev.m_hat), list(prev.v_hat), list(prev.b))
            ref_x = O.dadam_step(ref_state, g64, csr, t, ohp, "O32m", dtype)
            H.assert_within(H.compare_step(prev, ref_x, ref_state, sim.outputs(), g64, csr, t, ohp, dtype, mask), f"arena {dtype} t={t}")
            sim.swap()
        sim.close()


def test_arena_finds_stretches_in_different_thirds_by_timing():
    """The arena's timing probe on the real memory: on a device with most of its memory free the arena reaches
    into at least two thirds, the buffers are dealt over two stretches the probe told apart, and a pass with its
    buffers split over the two regions runs at the rate that made the probe tell them apart - also when 40 GiB
    were allocated first (which moves the boundaries inside the arena)."""
    from paper_2410_11998_amd import arena as A
    free, total = torch.cuda.mem_get_info(DEV)
    if free < (200 << 30):
        pytest.skip("needs a device with 200 GiB free")
    sizes = [48 << 20] * 40 + [24 << 20] * 24
    for first_gib in (0, 40):
        say("case", f"{first_gib} GiB allocated first")
        first = torch.empty(first_gib << 30, dtype=torch.uint8, device=DEV) if first_gib else None
        ar = A.SpreadArena(sizes, DEV)
        say("layout", ar.describe())
        H.record("arena_calibration", dict(first_gib=first_gib, stretches=[[t, lo >> 30, hi >> 30] for t, lo, hi in ar.stretches],
                                           regions=[[lo >> 30, hi >> 30] for lo, hi in ar.regions_used], policy=ar.policy))
        if ar.report.note != 0:
            # what the probe sees is a property of the machine and of what else holds its memory; the placement
            # it falls back to is still checked by every test that carves its buffers from an arena
            pytest.skip("the timing probe found nothing usable on this device: " + ar.describe())
        assert len(ar.stretches) >= 2 and len({t for t, _lo, _hi in ar.stretches}) >= 2
        assert ar.policy.startswith("two regions found by timing") and ar.advice == B.DADAM_PLACE_TWO_REGIONS
        (lo0, hi0), (lo1, hi1) = ar.regions_used
        if ar.policy.startswith("two regions found by timing"):
            owner = lambda off: next(t for t, lo, hi in ar.stretches if lo <= off < hi)
            assert owner(lo0) == owner(hi0 - 1) != owner(lo1) == owner(hi1 - 1)
        for k, (o, n) in enumerate(zip(ar.offsets, sizes)):
            lo, hi = ar.regions_used[k % 2]
            assert lo <= o and o + n <= hi
        # boundaries between thirds are 96 GiB apart wherever the arena starts
        cuts = [hi for _t, _lo, hi in ar.stretches[:-1]]
        if len(cuts) == 2:
            assert abs((cuts[1] - cuts[0]) - (96 << 30)) <= 2 * B.PROBE_STEP_BYTES
        across, within = float(ar.report.rate_across), [float(r) for r in ar.report.rate_inside]
        H.record("arena_calibration_rates", dict(first_gib=first_gib, across=across, within=within))
        say("rates", f"across {across:.3f} within {within}")
        assert across >= 0.75 and all(0 < r < 0.95 * across for r in within) and ar.probe_launches > 500
        del ar, first
        import gc
        gc.collect()
        torch.cuda.empty_cache()


def test_time_varying_loops_alternating_exponential_ring():
    """16 replicas cycling through the four AER phases (rows of degree 4 and 8) and, on a second
    handle, through the two one-peer-ring matchings."""
    n = 16
    layout = WL.pack([("a", (70001,)), ("b", (333,))])
    hp = H.HyperF32(s=2)
    aer = [WL.aer(4, ph) for ph in range(4)]
    w = H.run_parity("aer", n, n, layout, hp, aer, lambda t: (t - 1) % 4, 6, seed=55, grad_std=1e-2)
    say("aer worst error / tolerance:", w)
    opr = [WL.one_peer_ring(n, k) for k in range(2)]
    w = H.run_parity("one-peer-ring", n, n, layout, hp, opr, lambda t: (t - 1) % 2, 5, seed=56, grad_std=1e-2)
    say("one-peer ring worst error / tolerance:", w)


@pytest.mark.parametrize("mode", ["tile", "direct"])
@pytest.mark.parametrize("dtype,s", [("f32", 1), ("f32", 2), ("bf16", 2)])
def test_per_tensor_weight_decay(mode, dtype, s):
    """AdamW-style decoupled decay on some tensors only (as in the paper's ResNet-50 recipe, which
    exempts normalisation parameters), ragged layout, both kernels, including the unfused sequence."""
    say("case", mode, dtype, s)
    n = 4
    layout = WL.pack(WL.odd_shapes() + [("big", (50001,))])
    wds = [0.0 if k % 3 == 0 else (3e-2 if k % 3 == 1 else 0.5) for k in range(len(layout.names))]
    hp = H.HyperF32(lr=1e-2, s=s)
    for unfused in (False, True):
        w = H.run_parity("decay", n, n, layout, hp, [WL.ring(n)], lambda t: 0, 2 * s + 1, seed=88, param_dtype=dtype,
                         grad_dtype=dtype, grad_std=1e-2, flags=B.DADAM_FUSE_ACCUM | MODES[mode], weight_decay=wds,
                         unfused=unfused)
        say("worst error / tolerance:", w)


def test_weight_decay_node_share_in_place():
    """One row with receive buffers, updated in place: the decay uses source buffer 0, the row's own."""
    layout = WL.pack([("w", (30000,)), ("norm", (257,))])
    w = H.run_parity("decay-node", 1, 3, layout, H.HyperF32(lr=1e-2, s=2), [WL.node_share_ring()], lambda t: 0, 4, seed=89,
                     inplace=True, refresh_extra_sources=True, weight_decay=[0.1, 0.0], pad_fill=None)
    say("worst error / tolerance:", w)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("topo", ["ring4", "exp16", "onepeer64"])
def test_consensus_error_by_product_of_mixing(dtype, topo):
    """dadam_mix_consensus writes the same x_dst bits as dadam_mix and reports the squared distance
    of the sources from their mean; over repeated gossip rounds on the 4-ring it shrinks by 1/9 per
    round (the lambda^2 rate of the consensus lemma)."""
    say("case", dtype, topo)
    n, csr3 = {"ring4": (4, WL.ring(4)), "exp16": (16, WL.static_exponential(16)), "onepeer64": (64, WL.one_peer_exponential(64, 3))}[topo]
    layout = WL.pack(WL.odd_shapes() + [("big", (40003,))])
    d = layout.d
    sim = H.GpuSim(n, n, layout, H.HyperF32(s=1), [csr3], dtype, dtype, pad_fill=None)
    for c in range(n):
        sim.x_src[c].copy_(H.to_device(WL.normal_np(2000 + c, d, 0.02) + 0.5, dtype, DEV))   # deviations << values
    mask = H.valid_mask(layout)
    out = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    prev_err = None
    for rnd in range(4):
        xs = [x[mask] for x in sim._get(sim.x_src, None)]
        want = O.consensus_error(xs)
        sim.mix()
        torch.cuda.synchronize()
        plain = [x.clone() for x in sim.x_dst]
        sim.mix_consensus(out)
        torch.cuda.synchronize()
        got = float(out.item())
        for a_, b_ in zip(plain, sim.x_dst):
            assert torch.equal(a_, b_)
        assert abs(got - want) <= 2e-5 * want + 1e-30, (rnd, got, want)
        if topo == "ring4" and dtype == "f32" and prev_err is not None:
            assert abs(got / prev_err - 1.0 / 9.0) < 1e-4
        prev_err = got
        sim.swap()
    # the by-product needs the tile kernel
    with pytest.raises(B.DadamError) as e:
        sim.mix_consensus(out, 0, B.DADAM_FORCE_DIRECT)
    assert e.value.code == B.DADAM_ESTATE
    sim.close()


def test_empty_layouts_and_single_replica():
    """Degenerate shapes: a layout whose tensors are all empty launches nothing and touches nothing;
    a single replica (n = 1, W = [1]) is plain Adam in either kernel."""
    layout = WL.PackedLayout(["e0", "e1"], np.array([0, 8], np.uint64), np.array([0, 0], np.uint64), 16)
    sim = H.GpuSim(2, 2, layout, H.HyperF32(s=2), [WL.ring(2)], pad_fill=None)
    for t_ in sim.x_src + sim.x_dst + sim.m + sim.v + sim.b:
        t_.fill_(3.0)
    g = [torch.ones(16, device=DEV) for _ in range(2)]
    for flags in (B.DADAM_FUSE_ACCUM, B.DADAM_FUSE_ACCUM | B.DADAM_FORCE_DIRECT, 0):
        sim.step(g, 2, 0, flags)
    sim.accumulate(g, 2)
    sim.mix()
    out = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    sim.mix_consensus(out)
    torch.cuda.synchronize()
    assert float(out.item()) == 0.0
    for t_ in sim.x_src + sim.x_dst + sim.m + sim.v + sim.b:
        assert bool(torch.all(t_ == 3.0))
    sim.close()
    for mode in ("tile", "direct"):
        H.run_parity("single", 1, 1, flat_layout(5003), H.HyperF32(s=3), [WL.ring(1)], lambda t: 0, 7, seed=93,
                     flags=B.DADAM_FUSE_ACCUM | MODES[mode])


def test_late_iteration_bias_correction():
    """t = 10^6 + k: the bias corrections are 1 to float32 precision; iteration numbers are 64-bit."""
    n, d = 2, 4099
    layout = flat_layout(d)
    hp = H.HyperF32(s=4)
    sim = H.GpuSim(n, n, layout, hp, [WL.ring(n)], pad_fill=None)
    ohp = hp.oracle()
    csr = H.csr_oracle(WL.ring(n))
    mask = H.valid_mask(layout)
    for c in range(n):
        sim.x_src[c].copy_(H.to_device(WL.normal_np(940 + c, layout.d, 0.02), "f32", DEV))
        sim.m[c].copy_(H.to_device(WL.normal_np(950 + c, layout.d, 1e-3), "f32", DEV))
        sim.v[c].copy_(H.to_device(np.abs(WL.normal_np(960 + c, layout.d, 1e-6)), "f32", DEV))
        sim.b[c].copy_(H.to_device(WL.normal_np(970 + c, layout.d, 1e-3), "f32", DEV))
    for t in (10 ** 6 + 2, 10 ** 6 + 3, 10 ** 6 + 4, (1 << 33) + 4):
        grads = [H.to_device(WL.normal_np(980 + (t % 97) * 4 + i, layout.d, 1e-2), "f32", DEV) for i in range(n)]
        g64 = [g.to(torch.float64).cpu().numpy() for g in grads]
        prev = sim.snapshot()
        sim.step(grads, t)
        torch.cuda.synchronize()
        ref_state = O.State(prev.x_src, list(prev.m_hat), list(prev.v_hat), list(prev.b))
        ref_x = O.dadam_step(ref_state, g64, csr, t, ohp, "O32m", "f32")
        H.assert_within(H.compare_step(prev, ref_x, ref_state, sim.outputs(), g64, csr, t, ohp, "f32", mask), f"late t={t}")
        sim.swap()
    sim.close()


@pytest.mark.parametrize("mode", ["tile", "direct"])
def test_buffers_beyond_4_gib_use_64_bit_offsets(mode):
    """1.34 G elements per buffer (5.4 GB of float32): byte offsets pass 2^32; checked on sampled
    coordinates including the last elements."""
    say("case", mode)
    d_real = (1 << 30) + (1 << 28) + 1001
    layout = WL.pack([("a", (1 << 30,)), ("b", ((1 << 28) + 1001,))])
    assert layout.d >= d_real
    n = 2
    hp = H.HyperF32(s=2)
    sim = H.GpuSim(n, n, layout, hp, [WL.ring(n)], pad_fill=None)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(4242)
    for c in range(n):
        sim.x_src[c].normal_(0.0, 0.02, generator=gen)
        sim.x_src[c][d_real:] = 0.0          # padding after the last tensor: must stay as it is
    grads = [torch.empty(layout.d, device=DEV).normal_(0.0, 1e-2, generator=gen) for _ in range(n)]
    rng = np.random.default_rng(5)
    idx_np = np.unique(np.concatenate([np.arange(0, 2048), np.arange(d_real - 4096, d_real), np.arange((1 << 30) - 512, (1 << 30) + 512),
                                       rng.integers(0, d_real, size=1 << 15), rng.integers((1 << 30), d_real, size=1 << 14)]))
    idx = torch.from_numpy(idx_np).to(DEV)
    ohp = hp.oracle()
    csr = H.csr_oracle(WL.ring(n))
    for t in (1, 2):
        prev = sim.snapshot(idx)
        g64 = [g[idx].to(torch.float64).cpu().numpy() for g in grads]
        sim.step(grads, t, 0, B.DADAM_FUSE_ACCUM | MODES[mode])
        torch.cuda.synchronize()
        ref_state = O.State(prev.x_src, list(prev.m_hat), list(prev.v_hat), list(prev.b))
        ref_x = O.dadam_step(ref_state, g64, csr, t, ohp, "O32m", "f32")
        H.assert_within(H.compare_step(prev, ref_x, ref_state, sim.outputs(idx), g64, csr, t, ohp, "f32", None), f"big t={t}")
        # nothing beyond the last tensor was written
        assert bool(torch.all(sim.x_dst[0][d_real:] == 0)) and bool(torch.all(sim.m[1][d_real:] == 0))
        sim.swap()
    sim.close()
    del sim, grads
    torch.cuda.empty_cache()


def test_random_rectangular_topologies_and_layouts():
    """Seeded random cases: rows and sources of different counts, random degrees and weights in
    shuffled order, ragged tensor lists with gaps, every dtype pair, s in 1..3, both kernels."""
    rng = np.random.default_rng(20241011)
    for case in range(14):
        R = int(rng.integers(1, 13))
        C = int(rng.integers(R, R + 8))
        row_ptr, col, w = [0], [], []
        for i in range(R):
            deg = int(rng.integers(1, min(C, 9) + 1))
            cols = rng.permutation(C)[:deg]
            ww = (rng.random(deg) + 0.05).astype(np.float32)
            ww = (ww / ww.sum(dtype=np.float32)).astype(np.float32)
            col += list(cols); w += list(ww); row_ptr.append(len(col))
        t3 = (np.array(row_ptr, np.int32), np.array(col, np.int32), np.array(w, np.float32))
        shapes = [(f"t{k}", (int(rng.choice([1, 7, 64, 255, 256, 257, 1000, 3333, 5000])),)) for k in range(int(rng.integers(1, 9)))]
        layout = WL.pack(shapes, align_elems=int(rng.choice([8, 16, 24])))
        pd, gd = [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32"), ("f32", "bf16")][case % 4]
        s = int(rng.integers(1, 4))
        mode = ["tile", "direct"][case % 2]
        say("case", case, "R", R, "C", C, "nnz", len(col), "d", layout.d, pd, gd, "s", s, mode)
        H.run_parity(f"random{case}", R, C, layout, H.HyperF32(lr=3e-3, s=s), [t3], lambda t: 0, s + 2, seed=300 + case,
                     param_dtype=pd, grad_dtype=gd, grad_std=1e-2, flags=B.DADAM_FUSE_ACCUM | MODES[mode],
                     refresh_extra_sources=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_free_running_distance_from_the_unrounded_iteration(dtype):
    """The device run against the iteration carried in double precision with nothing rounded (not the
    oracle convention that rounds stored state): after T iterations the distance is reported and must
    stay below T times the per-iteration tolerance times the largest magnitude the element's terms
    have had so far - rounding differences add up at most linearly, the mixing never amplifies
    them, and what was committed while an element was large stays when it shrinks."""
    say("case", dtype)
    n, d, s, T = 8, 1 << 15, 2, 40
    layout = flat_layout(d)
    hp = H.HyperF32(lr=1e-3, s=s)
    ohp = hp.oracle()
    t3 = WL.ring(n)
    csr = H.csr_oracle(t3)
    sim = H.GpuSim(n, n, layout, hp, [t3], dtype, "f32")
    dev = torch.device(DEV)
    for c in range(n):
        sim.x_src[c].copy_(H.to_device(WL.normal_np(9100 + c, layout.d, 0.02), dtype, dev))
    exact = sim.snapshot()                      # starts from the stored (rounded) initial parameters
    worst = 0.0
    smax = [np.zeros(layout.d) for _ in range(n)]
    for t in range(1, T + 1):
        g64 = [WL.normal_np(9200 + t * 16 + i, layout.d, 1e-2).astype(np.float32).astype(np.float64) for i in range(n)]
        grads = [H.to_device(g, "f32", dev) for g in g64]
        prev = O.State(list(exact.x_src), list(exact.m_hat), list(exact.v_hat), list(exact.b))
        scale = O.magnitude_scale(prev, g64, csr, t, ohp)
        ex = O.dadam_step(exact, g64, csr, t, ohp, "O64", dtype)
        for i in range(n):
            exact.x_src[i] = ex[i]
        sim.step(grads, t)
        torch.cuda.synchronize()
        gx = sim.outputs()[0]
        for i in range(n):            # a mixed element inherits from its neighbours: take the rows' common maximum
            smax[i] = np.maximum(smax[i], scale[i])
        common = np.max(np.stack(smax), axis=0)
        ratio = max(float((np.abs(gx[i] - ex[i]) / common).max()) for i in range(n))
        worst = max(worst, ratio / (t * H.H_RTOL(dtype)))
        sim.swap()
    say(f"{dtype}: after {T} iterations max |x - exact| = {ratio:.3e} x largest term magnitude so far; worst ratio to t x tolerance {worst:.3f}")
    assert worst <= 1.0
    sim.close()


@pytest.mark.parametrize("consensus", ["handle", "static"])
def test_step_sequence_can_be_captured_in_a_graph_and_replayed(consensus):
    """Callers that capture their loop: the library's calls are kernel launches only (no allocation, no
    synchronisation, no memset), so an accumulation loop and a mixing pass with the consensus error
    can be recorded once and replayed.  Every replay (with eager work and synchronisations between
    them) must reproduce the eager results bit for bit.  The consensus pass once with the handle's own
    partial sums and once through the entry point that keeps them in the library's device image."""
    n, s = 8, 2
    layout = WL.pack(WL.odd_shapes())
    d = layout.d
    hp = H.HyperF32(lr=2e-3, s=s)
    t3 = WL.ring(n)
    sim = H.GpuSim(n, n, layout, hp, [t3], "f32", "f32")
    dev = torch.device(DEV)
    x0 = [H.to_device(WL.normal_np(7700 + c, d, 0.02), "f32", dev) for c in range(n)]
    grads = [[H.to_device(WL.normal_np(7800 + t * 16 + i, d, 1e-2), "f32", dev) for i in range(n)] for t in range(s)]
    cons = torch.zeros(1, dtype=torch.float64, device=dev)
    state = sim.x_src + sim.x_dst + sim.m + sim.v + sim.b

    def reset():
        for t_ in state:
            t_.zero_()
        for c in range(n):
            sim.x_src[c].copy_(x0[c])
        cons.zero_()

    def sequence():
        for t in range(1, s + 1):
            sim.step(grads[t - 1], t)
            sim.swap()
        if consensus == "handle":        # reads the loop's result, writes the other buffer set
            sim.mix_consensus(cons)
        else:
            B.dadam_mix_consensus_static(sim.h, 0, cons, 0, sim.stream())
        # an even number of exchanges: the handle's tables are back where they were

    def results():
        torch.cuda.synchronize()
        return [t_.clone() for t_ in state] + [cons.clone()]

    assert s % 2 == 0
    reset()
    sequence()
    eager = results()

    reset()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sequence()
    for replay in range(3):
        reset()
        junk = torch.randn(1 << 16, device=dev).sum()      # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        got = results()
        for k, (a, b) in enumerate(zip(eager, got)):
            assert torch.equal(a, b), f"replay {replay}: buffer {k} differs from the eager run"
        del junk
    say("consensus error after the captured sequence:", float(cons.item()))
    sim.close()


@pytest.mark.parametrize("mode,inplace", [("tile", False), ("tile", True), ("direct", False)])
def test_buckets_on_concurrent_streams_give_the_bits_of_the_whole_step(mode, inplace):
    """Tensor ranges are independent work: issued on two streams at once (ranges that share a tile at
    their ragged edges included, and with the parameters updated in place) they give the whole step."""
    say("case", mode, inplace)
    n = 6
    layout = WL.pack(WL.odd_shapes() + [("big", (70001,)), ("tail", (333,))])
    hp = H.HyperF32(s=2)
    nt = len(layout.names)
    t3 = WL.ring(n)
    a = H.GpuSim(n, n, layout, hp, [t3])
    b = H.GpuSim(n, n, layout, hp, [t3], inplace=inplace)
    for c in range(n):
        x0 = H.to_device(WL.normal_np(8500 + c, layout.d, 0.02), "f32", DEV)
        a.x_src[c].copy_(x0); b.x_src[c].copy_(x0)
    side = [torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)]
    valid = torch.from_numpy(H.valid_mask(layout)).to(DEV)
    cuts = [0, 1, 2, 5, nt - 2, nt - 1, nt]
    for t in (1, 2, 3, 4):
        grads = [H.to_device(WL.normal_np(8600 + t * 8 + i, layout.d, 1e-2), "f32", DEV) for i in range(n)]
        a.step(grads, t, 0, B.DADAM_FUSE_ACCUM | MODES[mode])
        torch.cuda.synchronize()                      # inputs are ready before the side streams start
        for k in range(len(cuts) - 1):
            B.dadam_gossip_step_range(b.h, 0, grads, t, B.DADAM_FUSE_ACCUM | MODES[mode], cuts[k], cuts[k + 1],
                                      side[k % 2].cuda_stream)
        torch.cuda.synchronize()
        for u, v in zip(a.x_dst + a.m + a.v + a.b, b.x_dst + b.m + b.v + b.b):
            assert torch.equal(u[valid], v[valid])     # (padding differs by construction when b works in place)
        a.swap(); b.swap()
    a.close(); b.close()


def test_gossip_rounds_in_place_and_ring_contraction_on_the_device():
    """Repeated mixing x <- W x (the gossip of the consensus lemma with zero direction) on a ring of
    four with weights 1/3: in-place mixing gives the bits of ping-pong mixing, and the consensus error
    the device reports falls by the square of the second eigenvalue, 1/9, every round."""
    n = 4
    layout = WL.pack(WL.odd_shapes() + [("big", (50001,))])
    t3 = WL.ring(n)
    hp = H.HyperF32(s=1)
    a = H.GpuSim(n, n, layout, hp, [t3])
    b = H.GpuSim(n, n, layout, hp, [t3], inplace=True)
    valid = torch.from_numpy(H.valid_mask(layout)).to(DEV)
    for c in range(n):
        x0 = H.to_device(WL.normal_np(8800 + c, layout.d, 1.0), "f32", DEV)
        x0[~valid] = 0.0                      # padding takes no part; keep it out of the device's sum
        a.x_src[c].copy_(x0); b.x_src[c].copy_(x0)
    ca = torch.zeros(1, dtype=torch.float64, device=DEV)
    cb = torch.zeros(1, dtype=torch.float64, device=DEV)
    errs = []
    for r in range(6):
        a.mix_consensus(ca, 0, B.DADAM_FORCE_TILE)
        b.mix_consensus(cb, 0, B.DADAM_FORCE_TILE)
        torch.cuda.synchronize()
        assert float(ca.item()) == float(cb.item())
        for u, v in zip(a.x_dst, b.x_dst):
            assert torch.equal(u[valid], v[valid])
        errs.append(float(ca.item()))          # consensus error of the round's sources
        a.swap()
    say("consensus errors:", errs)
    for e0, e1 in zip(errs, errs[1:]):
        assert abs(e1 / e0 - 1.0 / 9.0) < 1e-5 * (1.0 / 9.0) * 10
    a.close(); b.close()


# ---------------------------------------------------------------------------------------------
# the per-bucket update against the oracle
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("mode,topo,inplace,streams,dtype", [
    ("tile", "ring6", False, 1, "f32"), ("tile", "ring6", True, 2, "f32"), ("tile", "ring6", False, 2, "bf16"),
    ("direct", "ring6", False, 1, "f32"), ("direct", "ring6", False, 2, "f32"),
    ("direct", "node_share", True, 1, "f32"), ("direct", "node_share", True, 2, "bf16"), ("tile", "node_share", True, 2, "f32")])
def test_bucket_by_bucket_update_matches_oracle(mode, topo, inplace, streams, dtype):
    """The paper updates (and communicates) parameters bucket by bucket (section on overlapping
    communication and computation); an iteration issued as tensor ranges - in shuffled order, with an
    empty range, ranges that meet inside a tile of either kernel, on one stream or dealt over two, ping-pong
    or in place - is compared with the oracle's whole iteration (Algorithm 3 lines 4-13) element by element."""
    say("case", mode, topo, inplace, streams, dtype)
    layout = WL.pack(WL.odd_shapes() + [("big", (70001,)), ("mid", (4099,)), ("tail", (333,))])
    nt = len(layout.names)
    cuts = [0, 1, 2, 5, 9, nt - 3, nt - 2, nt - 1, nt]
    ranges = [(cuts[k], cuts[k + 1]) for k in range(len(cuts) - 1)] + [(4, 4)]
    order = np.random.default_rng(12).permutation(len(ranges))
    ranges = [ranges[k] for k in order]
    if topo == "ring6":
        R, C, csr3 = 6, 6, WL.ring(6)
    else:
        R, C, csr3 = 1, 3, WL.node_share_ring()
    s = 3
    w = H.run_parity(f"buckets-{mode}-{topo}-{'inplace' if inplace else 'pingpong'}-{streams}streams-{dtype}", R, C, layout,
                     H.HyperF32(lr=2e-3, s=s), [csr3], lambda t: 0, 2 * s + 1, seed=120, param_dtype=dtype, grad_dtype=dtype,
                     grad_std=1e-2, flags=B.DADAM_FUSE_ACCUM | MODES[mode], inplace=inplace,
                     refresh_extra_sources=(topo == "node_share"), ranges=ranges, range_streams=streams,
                     pad_fill=None if inplace else 777.0)
    say("worst error / tolerance:", w)


# ---------------------------------------------------------------------------------------------
# exact arithmetic: inputs on which every intermediate is representable, so the bits must agree
# ---------------------------------------------------------------------------------------------

def dyadic_case(rng, n, d):
    """Inputs for which every operation of iterations t = 1..4 with s = 4 (group index 1 throughout) is exact in
    float32: beta1 = 1/2, beta2 = 3/4 (bias corrections 1/2 and 1/4), eps = u = 2^-6, lr = 2^-7, weights 1/2
    and 1/4.  With v_hat = w u^2 and g = a u the root is sqrt(3 w + a^2) u, an integer q times u for the pairs
    below, and q + 1 is a power of two, so the division is exact as well."""
    u = 2.0 ** -6
    classes = [(0, (1, 3, 7)), (16, (1,)), (15, (2,)), (11, (4,)), (8, (5,)), (3, (0,))]      # w, |a| allowed
    cls = rng.integers(0, len(classes), size=(n, d))
    v_hat = np.zeros((n, d))
    for k, (w, _) in enumerate(classes):
        v_hat[cls == k] = w * u * u
    def grads():
        g = np.zeros((n, d))
        for k, (_, allowed) in enumerate(classes):
            sel = cls == k
            g[sel] = rng.choice(allowed, size=int(sel.sum())) * rng.choice([-1.0, 1.0], size=int(sel.sum())) * u
        return g
    m_hat = rng.integers(-8, 9, size=(n, d)) * u
    x0 = rng.integers(-255, 256, size=(n, d)) * 2.0 ** -7          # 8 significant bits: exact in bfloat16 too
    return u, x0, m_hat, v_hat, grads


def dyadic_rows(n, offsets, weights):
    """CSR rows i <- {(i + o) mod n} with the given (dyadic) weights."""
    k = len(offsets)
    col = np.array([(i + o) % n for i in range(n) for o in offsets], np.int32)
    return np.arange(0, k * n + 1, k, dtype=np.int32), col, np.array(list(weights) * n, np.float32)


@pytest.mark.parametrize("mode", ["tile", "direct"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [4, 68])
def test_dyadic_inputs_give_the_oracles_bits(mode, dtype, n):
    """Sums of two, three and four neighbours with weights 1/2 and 1/4, the moment and update arithmetic,
    accumulation, fold and the bfloat16 store (round to nearest even, ties included) on inputs where
    nothing is rounded before the final store: the device's bits must equal the oracle's, for every
    element of a ragged layout, over a whole accumulation loop that ends in a fold."""
    say("case", mode, dtype, n)
    s = 4
    layout = WL.pack(WL.odd_shapes() + [("big", (60001,))])
    d = layout.d
    rng = np.random.default_rng(99)
    u, x0, m0, v0, grads = dyadic_case(rng, n, d)
    hp = H.HyperF32(lr=2.0 ** -7, beta1=0.5, beta2=0.75, eps=u, s=s)
    ohp = hp.oracle()
    half, quarter = np.float32(0.5), np.float32(0.25)
    rows = (np.array([0, 3, 6, 9, 12], np.int32), np.array([0, 1, 2, 1, 2, 3, 2, 3, 0, 3, 0, 1], np.int32),
            np.array([half, quarter, quarter] * 4, np.float32))                       # 1/2 self, 1/4 to two neighbours
    csrs = [WL.one_peer_exponential(n, 0), WL.complete(n), rows, WL.one_peer_exponential(n, 1)]
    if n != 4:      # the same degrees and weights for any number of replicas (68: the kernels of large handles)
        csrs = [dyadic_rows(n, (0, 1), (half, half)), dyadic_rows(n, (0, 1, 2, 3), (quarter,) * 4),
                dyadic_rows(n, (0, 1, 2), (half, quarter, quarter)), dyadic_rows(n, (0, 2), (half, half))]
    sim = H.GpuSim(n, n, layout, hp, csrs, dtype, dtype, pad_fill=None)
    dev = torch.device(DEV)
    for i in range(n):
        sim.x_src[i].copy_(H.to_device(x0[i], dtype, dev))
        sim.m[i].copy_(H.to_device(m0[i], "f32", dev))
        sim.v[i].copy_(H.to_device(v0[i], "f32", dev))
    state = sim.snapshot()
    assert all(np.array_equal(state.x_src[i], x0[i]) for i in range(n)), "inputs are not exact in the storage type"
    mask = H.valid_mask(layout)
    ties = 0
    bits = (lambda t_: t_.view(torch.int32)) if dtype == "f32" else (lambda t_: t_.view(torch.int16))
    for t in range(1, s + 1):
        g = grads()
        gd = [H.to_device(g[i], dtype, dev) for i in range(n)]
        csr = H.csr_oracle(csrs[t - 1])
        exact = O.dadam_step(O.State(list(state.x_src), list(state.m_hat), list(state.v_hat), list(state.b)),
                             list(g), csr, t, ohp, "O64", dtype)                  # nothing rounded
        ref_x = O.dadam_step(state, list(g), csr, t, ohp, "O32m", dtype)
        if dtype == "f32":
            assert all(np.array_equal(exact[i], ref_x[i]) for i in range(n)), "the case is not exact in float32"
        else:
            for i in range(n):                                                       # exact halves of a bfloat16 step
                f = exact[i][mask]
                e = np.floor(np.log2(np.maximum(np.abs(f), 1e-30)))
                ties += int(np.sum((f != 0) & (np.mod(np.abs(f) / 2.0 ** (e - 7), 1.0) == 0.5)))
        sim.step(gd, t, t - 1, B.DADAM_FUSE_ACCUM | MODES[mode])
        torch.cuda.synchronize()
        for name, got, want, dt in (("x", sim.x_dst, ref_x, dtype), ("m_hat", sim.m, state.m_hat, "f32"),
                                    ("v_hat", sim.v, state.v_hat, "f32"), ("b", sim.b, state.b, "f32")):
            view = (lambda t_: t_.view(torch.int16)) if dt == "bf16" else (lambda t_: t_.view(torch.int32))
            for i in range(n):
                w_ = H.to_device(want[i], dt, dev)
                vm = torch.from_numpy(mask).to(dev)
                same = view(got[i])[vm] == view(w_)[vm]
                both_zero = (got[i][vm] == 0) & (w_[vm] == 0)                         # +0 and -0 are the same value
                assert bool(torch.all(same | both_zero)), \
                    f"t={t} {name}[{i}]: {int((~(same | both_zero)).sum())} elements differ in their bits"
        state.x_src = ref_x
        sim.swap()
    assert bool(np.all(state.b[0] == 0)) and float(np.abs(state.m_hat[0]).max()) > 0       # the loop ended in a fold
    if dtype == "bf16":
        say("bfloat16 stores that were exact ties:", ties)
        assert ties >= 8, "the case does not exercise ties of the bfloat16 store"
    sim.close()


# ---------------------------------------------------------------------------------------------
# 64 sources: the tile the device's LDS allows, and the direct kernel when it does not fit
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("lds_limit", [0, 32768])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_64_sources_with_and_without_room_for_the_tile(lds_limit, dtype):
    """The planner works from the LDS size the device reports (160 KB per workgroup on an MI355X): 64
    sources need a 64 KB tile, which fits; a handle limited to 32 KB cannot stage them.  Rows of two sources
    stream directly by choice either way (the dies take them in the sharing order), and the tile is there on
    request.  Mixing and the fused step in every mode there is, against the oracle, on a one-peer exponential
    graph of 64 replicas."""
    say("case", lds_limit, dtype)
    n = 64
    layout = WL.pack([("a", (9001,)), ("b", (257,)), ("c", (1030,))])
    d = layout.d
    csrs = [WL.one_peer_exponential(n, k) for k in (0, 3, 5)]
    sim = H.GpuSim(n, n, layout, H.HyperF32(s=2), csrs, dtype, dtype, pad_fill=None, lds_limit_bytes=lds_limit)
    info = B.dadam_get_plan_info(sim.h)
    say("plan: lds limit", info.lds_limit_bytes, "dies", info.n_xcds, "tile LDS", info.lds_bytes_tile, "tile mode", info.tile_mode_possible)
    if lds_limit == 0:
        assert info.lds_limit_bytes >= 65536 and info.n_xcds >= 1 and info.tile_mode_possible == 1
        assert B.dadam_slot_uses_tile_mode(sim.h, 0) is (info.n_xcds < 2 or n % info.n_xcds != 0)
        order, used = B.dadam_get_row_order(sim.h, 0, n)
        assert sorted(order) == list(range(n)) and used is (info.n_xcds > 1 and n % info.n_xcds == 0)
    else:
        assert info.lds_limit_bytes == 32768 and info.tile_mode_possible == 0
        assert not B.dadam_slot_uses_tile_mode(sim.h, 0)
        with pytest.raises(B.DadamError):
            sim.mix(0, B.DADAM_FORCE_TILE)
    for c in range(n):
        sim.x_src[c].copy_(H.to_device(WL.normal_np(4100 + c, d, 0.5), dtype, DEV))
    mask = H.valid_mask(layout)
    modes = [0, B.DADAM_FORCE_DIRECT] + ([B.DADAM_FORCE_TILE] if lds_limit == 0 else [])
    for slot, mode in [(s_, m_) for m_ in modes for s_ in range(3)]:
        sim.mix(slot, mode)
        torch.cuda.synchronize()
        xs = sim._get(sim.x_src, None)
        csr = H.csr_oracle(csrs[slot])
        ref = O.mix_only(xs, csr, "O32m", dtype)
        got = sim._get(sim.x_dst, None)
        for i in range(n):
            scale = sum(abs(csr.w[k]) * np.abs(xs[csr.col[k]]) for k in range(csr.row_ptr[i], csr.row_ptr[i + 1]))
            assert np.all(np.abs(got[i] - ref[i])[mask] <= (H.RTOL[dtype] * scale)[mask]), f"slot {slot} mode {mode} row {i}"
        sim.swap()
    sim.close()
    for mode in modes:
        w = H.run_parity(f"onepeer64-lds{lds_limit}-mode{mode}-{dtype}", n, n, layout, H.HyperF32(s=2), csrs, lambda t: (t - 1) % 3, 3,
                         seed=130, param_dtype=dtype, grad_dtype=dtype, flags=B.DADAM_FUSE_ACCUM | mode, pad_fill=None,
                         lds_limit_bytes=lds_limit)
    say("worst error / tolerance:", w)


# ---------------------------------------------------------------------------------------------
# more than 64 rows / sources: pointer tables in device memory, neighbour lists longer than a wavefront
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("case", ["aer96-tile", "aer96-direct", "complete96-tile", "complete96-direct", "ring160-tile-bf16",
                                  "share-1x100-direct", "rect-70x130-tile", "ring100-auto", "pairs100-auto-bf16"])
def test_more_than_64_rows_or_sources(case):
    """Beyond 64 rows or sources the tables of the bound buffers live in device memory (one immutable copy
    per binding) and a row may list more neighbours than a wavefront has lanes.  An Alternating
    Exponential Ring over 4 nodes of 24 (loops of 24 and 48), the complete graph of 96 (rows of 96 entries),
    a ring of 160 in tile mode (160 KB of LDS, all the device has), one row with 99 receive buffers, and a
    70 x 130 rectangular case with random rows, all against the oracle, ping-pong with dadam_swap_x."""
    say("case", case)
    layout = WL.pack([("a", (3001,)), ("b", (7,)), ("c", (515,))])
    rng = np.random.default_rng(77)
    dtype, mode, inplace, refresh = "f32", "tile" if "tile" in case else "auto" if "auto" in case else "direct", False, False
    slot_of_t = lambda t: 0
    if case.startswith("aer96"):
        R = C = 96
        csrs = [WL.aer(24, ph) for ph in range(4)]
        slot_of_t = lambda t: (t - 1) % 4
    elif case.startswith("complete96"):
        R = C = 96
        csrs = [WL.complete(96)]
    elif case.startswith("ring160"):
        R = C = 160
        csrs, dtype = [WL.ring(160)], "bf16"
    elif case.startswith("ring100") or case.startswith("pairs100"):
        # 100 rows over 8 dies: the planner streams them (a CU would hold one workgroup of the 100 KB tile), the
        # dies take groups of 12 and 13 rows of the sharing order and four workgroups per tile stay idle
        R = C = 100
        csrs = [WL.ring(100)] if case.startswith("ring") else [dyadic_rows(100, (0, 1), (0.5, 0.5)), dyadic_rows(100, (0, 7), (0.5, 0.5))]
        dtype = "bf16" if case.endswith("bf16") else "f32"
        slot_of_t = lambda t: (t - 1) % len(csrs)
    elif case.startswith("share"):
        R, C = 1, 100
        csrs, inplace, refresh = [WL._uniform_rows([list(range(100))])], True, True
    else:
        R, C = 70, 130
        row_ptr, col, w = [0], [], []
        for i in range(R):
            deg = int(rng.integers(1, 100))
            cols = rng.permutation(C)[:deg]
            ww = (rng.random(deg) + 0.05).astype(np.float32)
            ww = (ww / ww.sum(dtype=np.float32)).astype(np.float32)
            col += list(cols); w += list(ww); row_ptr.append(len(col))
        csrs, refresh = [(np.array(row_ptr, np.int32), np.array(col, np.int32), np.array(w, np.float32))], True
    T = 5 if len(csrs) > 1 else 3
    if mode == "auto":
        hh = B.dadam_init(R, C, layout.d, layout.offsets, layout.numels, device=0)
        B.dadam_set_topology(hh, 0, *csrs[0])
        order, used = B.dadam_get_row_order(hh, 0, R)
        assert B.dadam_slot_uses_tile_mode(hh, 0) is False and used and sorted(order) == list(range(R))
        B.dadam_destroy(hh)
    w_ = H.run_parity(case, R, C, layout, H.HyperF32(lr=2e-3, s=2), csrs, slot_of_t, T, seed=140, param_dtype=dtype,
                      grad_dtype=dtype, grad_std=1e-2, flags=B.DADAM_FUSE_ACCUM | MODES[mode], inplace=inplace,
                      refresh_extra_sources=refresh, pad_fill=None)
    say("worst error / tolerance:", w_)


def test_bindings_of_a_large_handle_are_kept_while_work_is_in_flight():
    """A handle with more than 64 rows keeps the device copies of its last DADAM_BINDINGS_KEPT bindings: a step
    launched under one binding is not disturbed by rebinding other buffers right behind it, the consensus
    by-product and the mixing-only pass work with the device tables, and selection stays bit-exact."""
    n = 80
    layout = flat_layout(2500)
    d = layout.d
    perm = list(np.random.default_rng(5).permutation(n))
    sim = H.GpuSim(n, n, layout, H.HyperF32(s=1), [WL.permutation(perm), WL.ring(n)], pad_fill=None)
    other = [torch.full((d,), -7.0, device=DEV) for _ in range(n)]
    for c in range(n):
        sim.x_src[c].copy_(torch.arange(d, dtype=torch.float32, device=DEV) + 4096.0 * c)
    keep_dst = list(sim.x_dst)
    sim.mix(0)                                   # launched under the first binding
    for k in range(3):                           # three further bindings right behind it, outputs elsewhere
        B.dadam_bind(sim.h, sim.x_src, other, sim.m, sim.v, None)
    torch.cuda.synchronize()
    for i in range(n):
        assert torch.equal(keep_dst[i][:2500].view(torch.int32), sim.x_src[perm[i]][:2500].view(torch.int32))
        assert bool(torch.all(other[i] == -7.0)), "a later binding's buffers were written by the earlier launch"
    sim.mix(0)                                   # now under the last binding
    torch.cuda.synchronize()
    for i in range(n):
        assert torch.equal(other[i][:2500].view(torch.int32), sim.x_src[perm[i]][:2500].view(torch.int32))
    # consensus error through the device tables
    out = torch.zeros(1, dtype=torch.float64, device=DEV)
    B.dadam_bind(sim.h, sim.x_src, keep_dst, sim.m, sim.v, None)
    sim.mix_consensus(out, 1)
    torch.cuda.synchronize()
    want = O.consensus_error([x[:2500] for x in sim._get(sim.x_src, None)])
    assert abs(float(out.item()) - want) <= 2e-5 * want
    sim.close()
