"""Host-side tests of the C ABI that need no GPU: the library loads and exports every symbol the
header declares; argument validation, neighbour-list validation, aliasing rules and the planner
are exercised through a host-only handle (device = DADAM_DEVICE_NONE).  No kernel is launched."""

import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2410_11998_amd import binding as B
from paper_2410_11998_amd import workloads as WL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    txt = open(os.path.join(ROOT, "include", "dadam.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(dadam_[a-z_0-9]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    names = header_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(B.lib, n), f"{n} declared in include/dadam.h but not exported"
    assert sorted(B.EXPORTS) == names


def test_constants_match_header():
    txt = open(os.path.join(ROOT, "include", "dadam.h")).read()
    def macro(name):
        m = re.search(r"#define\s+" + name + r"\s+\(?(-?\d+)u?\)?", txt)
        assert m, name
        return int(m.group(1))
    for name in ("DADAM_ABI_VERSION", "DADAM_MAX_ROWS", "DADAM_MAX_SLOTS", "DADAM_DEVICE_NONE", "DADAM_F32", "DADAM_BF16",
                 "DADAM_EINVAL", "DADAM_EALIGN", "DADAM_ETOPO", "DADAM_EALIAS", "DADAM_ESTATE", "DADAM_EHIP",
                 "DADAM_FUSE_ACCUM", "DADAM_FORCE_DIRECT", "DADAM_FORCE_TILE"):
        assert getattr(B, name) == macro(name), name


def host_handle(n_rows=4, n_cols=4, shapes=None, **kw):
    L = WL.pack(shapes or [("flat", (10000,))])
    return B.dadam_init(n_rows, n_cols, L.d, L.offsets, L.numels, device=B.DADAM_DEVICE_NONE, **kw), L


def expect(code, fn, *a, **kw):
    with pytest.raises(B.DadamError) as e:
        fn(*a, **kw)
    assert e.value.code == code, str(e.value)
    return str(e.value)


def test_init_rejects_bad_configurations():
    L = WL.pack([("a", (100,)), ("b", (50,))])
    ok = dict(n_rows=2, n_cols=2, d=L.d, offsets=L.offsets, numels=L.numels, device=B.DADAM_DEVICE_NONE)
    B.dadam_destroy(B.dadam_init(**ok))
    for bad in (dict(n_rows=0), dict(n_rows=161), dict(n_cols=0), dict(n_cols=161), dict(d=0), dict(accum_s=0),
                dict(param_dtype=2), dict(grad_dtype=7), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=-1.0),
                dict(lr=float("inf")), dict(abi_version=99), dict(beta_vhat=1.5), dict(device=-3),
                dict(offsets=[0, 50]), dict(offsets=[104, 0]), dict(d=120), dict(offsets=[], numels=[]),
                dict(weight_decay=[0.0, -0.1]), dict(weight_decay=[float("nan"), 0.0]), dict(tensor_flags=[1, 0]),
                dict(n_rows=2, n_cols=1, weight_decay=[0.0, 0.1])):
        expect(B.DADAM_EINVAL, B.dadam_init, **{**ok, **bad})
    assert "weight decay" in B.dadam_last_error(None)      # the text of the last failure of this thread


def test_planner_segments_and_tiles():
    # contiguous tensors merge into one segment, a gap starts a new one, empty tensors are skipped
    h = B.dadam_init(2, 2, 5000, [0, 100, 300, 300, 1000], [100, 200, 0, 10, 4000], device=B.DADAM_DEVICE_NONE)
    info = B.dadam_get_plan_info(h)
    assert info.n_segments == 2       # [0,310) [1000,5000)
    assert info.tile_elems == 64 * 4 and info.lds_bytes_tile == 2 * 64 * 16     # 16 bytes per lane and source
    assert info.direct_elems == 256 * 4 * 2
    T = info.tile_elems
    want = sum((hi - 1) // T - lo // T + 1 for lo, hi in ((0, 310), (1000, 5000)))
    assert info.n_tiles_tile == want
    D = info.direct_elems
    assert info.n_tiles_direct == sum((hi - 1) // D - lo // D + 1 for lo, hi in ((0, 310), (1000, 5000)))
    B.dadam_destroy(h)
    # tensors with different weight decay do not merge even when contiguous
    h = B.dadam_init(2, 2, 5000, [0, 100, 300, 1000], [100, 200, 700, 4000], device=B.DADAM_DEVICE_NONE,
                     weight_decay=[0.0, 0.0, 0.1, 0.1])
    assert B.dadam_get_plan_info(h).n_segments == 2       # [0,300) and [300,5000)
    B.dadam_destroy(h)
    for cfg, segs in ((2, 1), (3, 1), (4, 1), (5, 1)):
        wl = WL.workload(cfg)
        L = wl.layout()
        h = B.dadam_init(wl.n_rows, wl.n_cols, L.d, L.offsets, L.numels, B.DADAM_BF16 if wl.param_dtype == "bf16" else 0,
                         B.DADAM_BF16 if wl.grad_dtype == "bf16" else 0, accum_s=wl.s, device=B.DADAM_DEVICE_NONE)
        info = B.dadam_get_plan_info(h)
        assert info.n_segments == segs and info.tile_mode_possible == 1
        assert info.n_tiles_tile == -(-L.d // info.tile_elems)
        assert info.lds_bytes_tile <= 65536
        B.dadam_destroy(h)


def test_planner_uses_the_lds_and_die_count_it_is_given():
    """A host-only handle plans for 64 KB of LDS per workgroup and 8 dies unless the configuration says
    otherwise (a device handle asks the device).  The mixing pass takes its two-vector tile only while
    that stays within 32 KB (16 sources); a tile that does not fit the limit rules tile mode out."""
    L = WL.pack([("flat", (100000,))])
    mk = lambda n, **kw: B.dadam_init(n, n, L.d, L.offsets, L.numels, device=B.DADAM_DEVICE_NONE, **kw)
    h = mk(64)
    i = B.dadam_get_plan_info(h)
    assert (i.lds_limit_bytes, i.n_xcds) == (65536, 8)
    assert i.tile_mode_possible == 1 and i.lds_bytes_tile == 65536 and (i.mix_vectors, i.lds_bytes_mix) == (1, 65536)
    B.dadam_destroy(h)
    h = mk(64, lds_limit_bytes=160 * 1024, n_xcds=4)
    i = B.dadam_get_plan_info(h)
    assert (i.lds_limit_bytes, i.n_xcds) == (160 * 1024, 4)
    assert (i.mix_vectors, i.lds_bytes_mix, i.mix_tile_elems) == (1, 65536, 256)
    B.dadam_destroy(h)
    h = mk(16)
    i = B.dadam_get_plan_info(h)
    assert (i.mix_waves, i.mix_vectors, i.lds_bytes_mix, i.mix_tile_elems) == (4, 2, 32768, 512)
    assert i.n_tiles_mix == -(-L.d // 512) and i.n_tiles_tile == -(-L.d // 256)
    B.dadam_destroy(h)
    h = mk(32, lds_limit_bytes=16 * 1024)            # 32 sources need 32 KB: no tile mode
    i = B.dadam_get_plan_info(h)
    assert i.tile_mode_possible == 0
    B.dadam_set_topology(h, 0, *WL.ring(32))
    assert B.dadam_slot_uses_tile_mode(h, 0) is False
    B.dadam_destroy(h)
    expect(B.DADAM_EINVAL, mk, 4, n_xcds=1000)


def test_pack_offsets_matches_workload_packer():
    L = WL.pack(WL.odd_shapes(), align_elems=8)
    off, d = B.dadam_pack_offsets([int(n) for n in L.numels], 8)
    assert np.array_equal(off, L.offsets) and d == L.d
    off, d = B.dadam_pack_offsets([5, 1, 8], 4)
    assert list(off) == [0, 8, 12] and d == 20


def test_set_topology_validation():
    h, _ = host_handle(4, 4)
    rp, col, w = WL.ring(4)
    assert B.dadam_set_topology(h, 0, rp, col, w) == 0
    assert B.dadam_slot_uses_tile_mode(h, 0) is True          # ring: sources are shared
    assert B.dadam_set_topology(h, 1, *WL.identity(4)) == 0
    assert B.dadam_slot_uses_tile_mode(h, 1) is False         # nothing shared: stream directly
    expect(B.DADAM_EINVAL, B.dadam_set_topology, h, 16, rp, col, w)
    expect(B.DADAM_ESTATE, B.dadam_slot_uses_tile_mode, h, 5)
    # rows of two sources over more than 16 sources stream directly (the dies take them in the sharing order);
    # three sources a row or few sources: the tile
    for n, csr, want in ((64, WL.one_peer_exponential(64, 0), False), (64, WL.one_peer_exponential(64, 5), False),
                         (16, WL.one_peer_exponential(16, 1), True), (64, WL.ring(64), True)):
        hh, _ = host_handle(n, n, lds_limit_bytes=160 * 1024)        # the device's figure (a host-only handle assumes 64 KB)
        B.dadam_set_topology(hh, 0, *csr)
        assert B.dadam_slot_uses_tile_mode(hh, 0) is want, (n, want)
        B.dadam_destroy(hh)
    hh, _ = host_handle(24, 24)                                   # 24 rows of two sources: direct
    pair24 = (np.arange(0, 49, 2, dtype=np.int32), np.array([(i + o) % 24 for i in range(24) for o in (0, 1)], np.int32), np.full(48, 0.5, np.float32))
    B.dadam_set_topology(hh, 0, *pair24)
    assert B.dadam_slot_uses_tile_mode(hh, 0) is False
    B.dadam_destroy(hh)
    hh, _ = host_handle(20, 20)                                   # 20 rows over 8 dies (groups of 2 and 3): direct as well
    pair20 = (np.arange(0, 41, 2, dtype=np.int32), np.array([(i + o) % 20 for i in range(20) for o in (0, 1)], np.int32), np.full(40, 0.5, np.float32))
    B.dadam_set_topology(hh, 0, *pair20)
    assert B.dadam_slot_uses_tile_mode(hh, 0) is False
    B.dadam_destroy(hh)
    # a tile of which a CU holds one workgroup (more than half of the LDS): rows of up to eight sources stream
    for n, csr, lds, want in ((100, WL.ring(100), 160 * 1024, False), (80, WL.ring(80), 160 * 1024, True),
                              (100, WL.complete(100), 160 * 1024, True), (40, WL.ring(40), 64 * 1024, False)):
        hh, _ = host_handle(n, n, lds_limit_bytes=lds)
        B.dadam_set_topology(hh, 0, *csr)
        assert B.dadam_slot_uses_tile_mode(hh, 0) is want, (n, lds, want)
        B.dadam_destroy(hh)
    bad = rp.copy(); bad[0] = 1
    expect(B.DADAM_ETOPO, B.dadam_set_topology, h, 2, bad, col, w)
    bad = rp.copy(); bad[2] = bad[1]
    expect(B.DADAM_ETOPO, B.dadam_set_topology, h, 2, bad, col, w)           # empty row
    bad = col.copy(); bad[1] = 4
    expect(B.DADAM_ETOPO, B.dadam_set_topology, h, 2, rp, bad, w)            # column out of range
    bad = col.copy(); bad[1] = -1
    expect(B.DADAM_ETOPO, B.dadam_set_topology, h, 2, rp, bad, w)
    bad = col.copy(); bad[1] = bad[0]
    expect(B.DADAM_ETOPO, B.dadam_set_topology, h, 2, rp, bad, w)            # duplicate in a row
    for val in (0.0, -0.5, float("nan"), float("inf")):
        bad = w.copy(); bad[3] = val
        expect(B.DADAM_ETOPO, B.dadam_set_topology, h, 2, rp, col, bad)
    bad = w.copy(); bad[:3] = 0.3
    assert "sums" in expect(B.DADAM_ETOPO, B.dadam_set_topology, h, 2, rp, col, bad)
    # rows fine, columns not: a warning, not an error
    rp2 = np.array([0, 1, 2, 3, 4], np.int32)
    assert B.dadam_set_topology(h, 2, rp2, np.array([0, 0, 1, 2], np.int32), np.ones(4, np.float32)) == B.DADAM_WARN_NOT_COLUMN_STOCHASTIC
    assert B.dadam_set_topology(h, 3, *WL.one_peer_exponential(4, 1)) == 0
    B.dadam_destroy(h)


def test_bind_alignment_and_aliasing_rules():
    h, L = host_handle(2, 3, accum_s=2)
    nb = L.d * 4
    base = 1 << 20
    P = lambda k: base + k * (nb + 256)       # disjoint, 16-byte aligned fake device addresses
    good = dict(x_src=[P(0), P(1), P(2)], x_dst=[P(3), P(4)], m_hat=[P(5), P(6)], v_hat=[P(7), P(8)], acc=[P(9), P(10)])
    B.dadam_bind(h, **good)
    expect(B.DADAM_EALIGN, B.dadam_bind, h, **{**good, "x_dst": [P(3) + 4, P(4)]})
    expect(B.DADAM_EALIGN, B.dadam_bind, h, **{**good, "acc": [P(9), P(10) + 8]})
    expect(B.DADAM_EINVAL, B.dadam_bind, h, **{**good, "m_hat": [0, P(6)]})
    expect(B.DADAM_EINVAL, B.dadam_bind, h, **{**good, "acc": None})
    # partial overlap of an output with a source
    expect(B.DADAM_EALIAS, B.dadam_bind, h, **{**good, "x_dst": [P(0) + 16, P(4)]})
    # two outputs on the same memory
    expect(B.DADAM_EALIAS, B.dadam_bind, h, **{**good, "x_dst": [P(3), P(3)]})
    # state on top of parameters
    expect(B.DADAM_EALIAS, B.dadam_bind, h, **{**good, "v_hat": [P(7), P(1)]})
    expect(B.DADAM_EALIAS, B.dadam_bind, h, **{**good, "acc": [P(9), P(5)]})
    # exact in-place is accepted; whether a step may run depends on the neighbour list
    B.dadam_bind(h, **{**good, "x_dst": [P(0), P(1)]})
    rp = np.array([0, 2, 4], np.int32)
    w = np.full(4, 0.5, np.float32)
    B.dadam_set_topology(h, 0, rp, np.array([0, 2, 1, 2], np.int32), w)   # sources 0 and 1 each read by their own row only
    assert B.dadam_slot_uses_tile_mode(h, 0) is True                       # source 2 is shared -> tile mode
    B.dadam_set_topology(h, 1, np.array([0, 1, 2], np.int32), np.array([0, 1], np.int32), np.ones(2, np.float32))
    assert B.dadam_slot_uses_tile_mode(h, 1) is False                      # in place, nothing shared: direct is legal
    B.dadam_set_topology(h, 2, np.array([0, 1, 2], np.int32), np.array([1, 0], np.int32), np.ones(2, np.float32))
    assert B.dadam_slot_uses_tile_mode(h, 2) is True                       # rows read each other's buffer: needs the tile
    # a host-only handle validates a call like a device handle and then refuses to launch
    assert "host-only" in expect(B.DADAM_ESTATE, B.dadam_gossip_step, h, 0, [P(11), P(12)], 1)
    assert "host-only" in expect(B.DADAM_ESTATE, B.dadam_accumulate, h, [P(11), P(12)], 1)
    assert "host-only" in expect(B.DADAM_ESTATE, B.dadam_mix, h, 0)
    assert "host-only" in expect(B.DADAM_ESTATE, B.dadam_mix_consensus, h, 0, P(13))
    expect(B.DADAM_EINVAL, B.dadam_mix_consensus, h, 0, 0)
    expect(B.DADAM_EINVAL, B.dadam_mix_consensus, h, 0, P(13) + 4)
    expect(B.DADAM_EINVAL, B.dadam_gossip_step, h, 0, [P(11), P(12)], 0)                 # iterations start at 1
    expect(B.DADAM_EINVAL, B.dadam_gossip_step, h, 0, [P(11), P(12)], 1, 64)             # unknown flag
    expect(B.DADAM_EINVAL, B.dadam_gossip_step, h, 0, [P(11), P(12)], 1, B.DADAM_FORCE_TILE | B.DADAM_FORCE_DIRECT)
    expect(B.DADAM_ESTATE, B.dadam_gossip_step, h, 7, [P(11), P(12)], 1)                 # empty slot
    expect(B.DADAM_EALIAS, B.dadam_gossip_step, h, 2, [P(11), P(12)], 1, B.DADAM_FUSE_ACCUM | B.DADAM_FORCE_DIRECT)
    expect(B.DADAM_EINVAL, B.dadam_gossip_step_range, h, 0, [P(11), P(12)], 1, B.DADAM_FUSE_ACCUM, 1, 5)
    B.dadam_destroy(h)


def test_in_place_row_whose_buffer_is_listed_as_two_sources():
    """Two source entries may name one buffer.  A row updated in place then overwrites both, so the
    direct kernel is legal only if nobody else reads either of them (update template of eq. (2): every
    row reads the PREVIOUS iterate)."""
    h, L = host_handle(2, 3, accum_s=2)
    nb = L.d * 4
    P = lambda k: (1 << 20) + k * (nb + 256)
    # x_src[2] is the same buffer as x_src[0], and row 0 is updated in place in it
    B.dadam_bind(h, x_src=[P(0), P(1), P(0)], x_dst=[P(0), P(3)], m_hat=[P(5), P(6)], v_hat=[P(7), P(8)], acc=[P(9), P(10)])
    half = np.full(4, 0.5, np.float32)
    # row 1 reads source 2, i.e. row 0's buffer: the direct kernel would let it see a new value
    B.dadam_set_topology(h, 0, np.array([0, 2, 4], np.int32), np.array([0, 1, 1, 2], np.int32), half)
    assert B.dadam_slot_uses_tile_mode(h, 0) is True
    expect(B.DADAM_EALIAS, B.dadam_gossip_step, h, 0, [P(11), P(12)], 1, B.DADAM_FUSE_ACCUM | B.DADAM_FORCE_DIRECT)
    # the same with the entries the other way round (row 1 reads source 0)
    B.dadam_set_topology(h, 1, np.array([0, 2, 4], np.int32), np.array([2, 1, 1, 0], np.int32), half)
    assert B.dadam_slot_uses_tile_mode(h, 1) is True
    expect(B.DADAM_EALIAS, B.dadam_gossip_step, h, 1, [P(11), P(12)], 1, B.DADAM_FUSE_ACCUM | B.DADAM_FORCE_DIRECT)
    # only row 0 reads its own buffer, under either name: direct is fine
    B.dadam_set_topology(h, 2, np.array([0, 2, 3], np.int32), np.array([0, 2, 1], np.int32), np.array([0.5, 0.5, 1.0], np.float32))
    assert B.dadam_slot_uses_tile_mode(h, 2) is False
    assert "host-only" in expect(B.DADAM_ESTATE, B.dadam_gossip_step, h, 2, [P(11), P(12)], 1, B.DADAM_FUSE_ACCUM | B.DADAM_FORCE_DIRECT)
    B.dadam_destroy(h)


def test_gradient_tables_are_checked_against_the_outputs_and_remembered():
    """Gradients may not overlap anything a call writes.  A table that passed is remembered, but only
    for the outputs it was checked against: binding other buffers or exchanging x_src and x_dst makes
    the library look again."""
    h, L = host_handle(2, 2, accum_s=2)
    nb = L.d * 4
    P = lambda k: (1 << 20) + k * (nb + 256)
    B.dadam_set_topology(h, 0, *WL.ring(2))
    bufs = dict(x_src=[P(0), P(1)], x_dst=[P(2), P(3)], m_hat=[P(4), P(5)], v_hat=[P(6), P(7)], acc=[P(8), P(9)])
    B.dadam_bind(h, **bufs)
    ok = lambda g, fn=B.dadam_gossip_step: "host-only" in expect(B.DADAM_ESTATE, fn, h, 0, g, 1)
    for _ in range(3):
        assert ok([P(10), P(11)])                     # checked once, then found in the cache
    assert ok([P(0), P(1)])                           # gradients on top of the SOURCES: read-only, harmless
    for k in (2, 3, 4, 5, 6, 7, 8, 9):                # on top of any output: refused
        expect(B.DADAM_EALIAS, B.dadam_gossip_step, h, 0, [P(10), P(k)], 1)
        expect(B.DADAM_EALIAS, B.dadam_gossip_step, h, 0, [P(k) + nb - 16, P(11)], 1)      # last 16 bytes overlap
        expect(B.DADAM_EALIAS, B.dadam_accumulate, h, [P(10), P(k)], 1)
    assert ok([P(9) + nb, P(11)])                     # starting exactly where an output ends is fine
    expect(B.DADAM_EALIGN, B.dadam_gossip_step, h, 0, [P(10) + 8, P(11)], 1)
    expect(B.DADAM_EINVAL, B.dadam_gossip_step, h, 0, [P(10), 0], 1)
    # after the exchange the old sources are outputs: the remembered table [P(0), P(1)] must be refused
    B.dadam_swap_x(h)
    expect(B.DADAM_EALIAS, B.dadam_gossip_step, h, 0, [P(0), P(1)], 1)
    assert ok([P(2), P(3)]) and ok([P(10), P(11)])
    B.dadam_swap_x(h)
    assert ok([P(0), P(1)])
    expect(B.DADAM_EALIAS, B.dadam_gossip_step, h, 0, [P(2), P(3)], 1)
    # many different tables: the memory of checked tables is bounded and stays correct
    for k in range(40):
        assert ok([P(20 + k), P(70 + k)])
    assert ok([P(10), P(11)])
    # new outputs on top of a remembered gradient table
    B.dadam_bind(h, **{**bufs, "m_hat": [P(10), P(5)]})
    expect(B.DADAM_EALIAS, B.dadam_gossip_step, h, 0, [P(10), P(11)], 1)
    B.dadam_destroy(h)


def test_swap_needs_square_and_bound():
    h, L = host_handle(2, 3)
    expect(B.DADAM_ESTATE, B.dadam_swap_x, h)
    B.dadam_destroy(h)
    h, L = host_handle(2, 2)
    expect(B.DADAM_ESTATE, B.dadam_swap_x, h)     # nothing bound yet
    nb = L.d * 4 + 256
    B.dadam_bind(h, [4096, 4096 + nb], [4096 + 2 * nb, 4096 + 3 * nb], [4096 + 4 * nb, 4096 + 5 * nb],
                 [4096 + 6 * nb, 4096 + 7 * nb], None)
    B.dadam_swap_x(h)
    B.dadam_set_lr(h, 0.5)
    expect(B.DADAM_EINVAL, B.dadam_set_lr, h, float("nan"))
    B.dadam_destroy(h)


def test_null_handle_is_an_error_not_a_crash():
    null = C.c_void_p(None)
    assert B.lib.dadam_swap_x(null) == B.DADAM_EINVAL
    assert B.lib.dadam_set_lr(null, 0.1) == B.DADAM_EINVAL
    assert B.lib.dadam_mix(null, 0, 0, None) == B.DADAM_EINVAL
    assert B.lib.dadam_accumulate(null, None, 1, None) == B.DADAM_EINVAL
    assert B.lib.dadam_gossip_step(null, 0, None, 1, 1, None) == B.DADAM_EINVAL
    assert B.lib.dadam_init(None, None) == B.DADAM_EINVAL
    B.lib.dadam_destroy(null)


def test_binding_rejects_short_or_mistyped_tensors():
    """The library cannot know how large a caller's buffer is; the binding can when it is handed
    tensors, and must refuse a buffer shorter than d before any kernel could overrun it."""
    import torch
    h, L = host_handle(2, 2, accum_s=2)
    full = lambda dt=torch.float32: torch.zeros(L.d, dtype=dt)
    short = torch.zeros(L.d - 8)
    good = dict(x_src=[full(), full()], x_dst=[full(), full()], m_hat=[full(), full()], v_hat=[full(), full()], acc=[full(), full()])
    B.dadam_bind(h, **good)
    for key in good:
        bad = dict(good); bad[key] = [good[key][0], short]
        with pytest.raises(ValueError):
            B.dadam_bind(h, **bad)
    with pytest.raises(ValueError):
        B.dadam_bind(h, **{**good, "x_src": [full(torch.bfloat16), full()]})
    with pytest.raises(ValueError):
        B.dadam_bind(h, **{**good, "m_hat": [full()[::2], full()]})
    with pytest.raises(ValueError):
        B.dadam_gossip_step(h, 0, [full(), short], 1)
    with pytest.raises(ValueError):
        B.dadam_accumulate(h, [short, full()], 1)
    B.dadam_destroy(h)


def test_spread_offsets_properties():
    unit = 2 << 20
    rng = np.random.default_rng(3)
    for _ in range(50):
        n = int(rng.integers(1, 40))
        sizes = [int(x) for x in rng.integers(1, 50 << 20, size=n)]
        packed = sum(-(-s // unit) * unit for s in sizes)
        arena = packed + int(rng.integers(0, 3 << 30))
        off = B.dadam_spread_offsets(sizes, arena)
        assert off[0] == 0 and all(o % unit == 0 for o in off)
        for k in range(1, n):
            assert off[k] >= off[k - 1] + sizes[k - 1]
        assert off[-1] + sizes[-1] <= arena
        if n > 2:
            gaps = {off[k + 1] - off[k] - (-(-sizes[k] // unit) * unit) for k in range(n - 1)}
            assert len(gaps) == 1                                   # equal gaps
            assert arena - (off[-1] + -(-sizes[-1] // unit) * unit) < (n - 1) * unit   # nothing much left over
    with pytest.raises(B.DadamError):
        B.dadam_spread_offsets([5 << 20, 5 << 20], 8 << 20)
    assert B.lib.dadam_spread_offsets(None, 1, 100, None) == B.DADAM_EINVAL


def test_kernels_use_no_scratch_memory_and_load_neighbour_lists_with_all_lanes(tmp_path):
    """Five properties of the compiled device code, read from the compiler's own output.

    (1) Every kernel keeps its state in registers: a struct copied to private memory once cost 8 %
    of the step's bandwidth without any test noticing (resource-usage remarks, scratch size 0).

    (2) A row's neighbour list sits one entry per lane and is handed out with readlane, so its load
    must run with every lane active.  The direct kernel once let threads of a clipped tile return
    early; a later build sank the list's load below that exit and rows whose leading lanes lay before
    the segment read indices from lanes that had never loaded.  The source must have no early exit
    in device code, and in the direct kernels' assembly no register that readlane reads may be
    loaded between a narrowing of the exec mask and its restoration."""
    import shutil
    import subprocess
    from concurrent.futures import ThreadPoolExecutor
    from paper_2410_11998_amd import build as bld
    if shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"):
        pytest.skip("hipcc not available")
    src = open(os.path.join(bld.CSRC, "dadam_device.h")).read()
    device_code = src[:src.index("// dispatch tables")]
    assert not re.search(r"\breturn\s*;", device_code), "an early exit in device code: see the docstring"
    flags = [f for f in bld.FLAGS if f not in ("-shared", "-fPIC")]

    def compile_unit(unit):
        name, source, defs = unit
        asm = tmp_path / (name + ".s")
        cmd = [bld.hipcc()] + flags + defs + ["--cuda-device-only", "-S", os.path.join(bld.CSRC, source),
                                              "-o", str(asm), "-Rpass-analysis=kernel-resource-usage"]
        r = subprocess.run(cmd, capture_output=True, text=True, timeout=1500)
        assert r.returncode == 0, r.stderr[-2000:]
        return name, str(asm), r.stderr

    units = [u for u in bld.UNITS if u[1].endswith(".hip")]
    with ThreadPoolExecutor(max_workers=bld.jobs()) as pool:
        done = list(pool.map(compile_unit, units))
    remarks = "".join(d[2] for d in done)
    sizes = [int(x) for x in re.findall(r"ScratchSize \[bytes/lane\]: (\d+)", remarks)]
    assert len(sizes) > 100, "no resource remarks found"
    assert max(sizes) == 0, f"{sum(1 for s in sizes if s)} kernels spill or copy to scratch"
    asm_text = "".join(open(d[1]).read() for d in done)
    asm = tmp_path / "all.s"
    asm.write_text(asm_text)

    # (3) the scratch array of the entry point that does not allocate is looked up by name at run time: the
    # code object must export it (a symbol left local makes the runtime abort in dadam_init)
    assert re.search(r"^\s*\.globl\s+_ZL7scratch\s*$", asm_text, flags=re.M), "static scratch array is not visible to the runtime"
    assert re.search(r"^_ZL7scratch:", asm_text, flags=re.M) and ".local\t_ZL7scratch" not in asm_text

    # (4) every pointer the kernels dereference is known to be global memory: a pointer rebuilt from an
    # integer without its address space turns all accesses through it into flat ones (5 % slower with 64 rows)
    assert not re.search(r"^\s*flat_(load|store|atomic)", asm_text, flags=re.M), "flat memory instructions in the kernels"

    import asm_checks
    # (5) kernels built for streaming carry the non-temporal hint on every vector store and on the vector loads
    # of sources, gradients and state (the few plain ones read the neighbour-list bounds, the segment table
    # and, in the kernels of large handles, the pointer tables).  The hint is metadata the optimiser may drop when it re-creates an access: a loop that ran once
    # around the stores of the one-vector bfloat16 tile kernels lost it, and 1.2 % of the step with it.
    hints = asm_checks.streaming_hints(str(asm))
    import subprocess as sp
    names = sorted(hints)
    plain_names = sp.run(["c++filt"], input="\n".join(names), capture_output=True, text=True).stdout.split("\n")
    streaming, other = 0, 0
    for mangled, plain in zip(names, plain_names):
        st_nt, st_plain, ld_nt, ld_plain = hints[mangled]
        m = re.search(r"\b(k_tile|k_direct|k_acc)<(.*)>\(", plain)
        if not m:
            continue
        targs = [x.strip() for x in m.group(2).split(",")]
        nt, ext = targs[-2] in ("true", "1", "2"), targs[-1] == "true"     # <..., hints, tables in device memory>
        if targs[-2] == "2":               # direct kernel for rows that share sources: source loads stay plain
            streaming += 1
            assert st_plain == 0 and st_nt > 0 and ld_plain > 0, f"{plain}: stores {st_nt}/{st_plain}, loads {ld_nt}/{ld_plain}"
            continue
        if nt:
            streaming += 1
            assert st_plain == 0 and st_nt > 0, f"{plain}: {st_plain} vector stores without the hint"
            assert ld_plain <= (60 if ext else 8) and ld_nt >= (1 if ext else 4) * ld_plain, \
                f"{plain}: {ld_plain} vector loads without the hint, {ld_nt} with"
        else:
            other += 1
            assert st_nt == 0 and ld_nt == 0, f"{plain}: hints in a kernel built without them"
    assert streaming > 150 and other > 150, (streaming, other)

    checked, bad = asm_checks.readlanes_of_loads_under_narrowed_exec(str(asm))
    assert checked > 1000, "no readlane of a loaded register found in the direct kernels"
    assert not bad, f"neighbour list loaded under a narrowed exec mask in {len(set(bad))} kernels, e.g. {bad[0]}"


def test_bench_byte_accounting_matches_the_workload_table():
    """bench.py's per-phase algorithmic bytes, averaged over one accumulation loop, are the
    per-element figures of the workload module (28 + 4/s, 36 + 4/s, 22 + 4/s)."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    want = {1: 30.0, 2: 29.0, 3: 36.5, 4: 30.0, 5: 23.0}
    for cfg in range(1, 6):
        wl = WL.workload(cfg)
        loop = [bench.phase_of(t, wl.s) for t in range(1, wl.s + 1)]
        avg = sum(bench.algorithmic_bytes_per_replica_param(wl, p) for p in loop) / wl.s
        assert abs(avg - want[cfg]) < 1e-12 and abs(wl.bytes_per_replica_param() - want[cfg]) < 1e-12
        assert loop[0] == "loopstart" and loop[-1] == "fold"
        for p in loop:
            assert bench.path_bytes_per_replica_param(wl, p, "fused") == bench.algorithmic_bytes_per_replica_param(wl, p)
            assert bench.path_bytes_per_replica_param(wl, p, "unfused") > bench.algorithmic_bytes_per_replica_param(wl, p)


def test_host_code_under_address_and_ub_sanitizers(tmp_path):
    """Builds the host side of the library with ASan + UBSan (kernel launchers stubbed out) together
    with tests/host_sanitizer_driver.cpp and runs a few thousand random, partly malformed call
    sequences through init / set_topology / bind / step validation / planner."""
    import subprocess
    clang = "/opt/rocm/lib/llvm/bin/clang++"
    if not os.path.exists(clang):
        pytest.skip("clang++ of the ROCm toolchain not available")
    exe = str(tmp_path / "san_driver")
    cmd = [clang, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2410_11998_amd", "csrc"),
           "-I", "/opt/rocm/include", os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"),
           os.path.join(ROOT, "paper_2410_11998_amd", "csrc", "dadam_host.cpp"),
           os.path.join(ROOT, "paper_2410_11998_amd", "csrc", "dadam_place.cpp"),
           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "sanitizer driver finished" in r.stdout, (r.stdout[-500:], r.stderr[-3000:])
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]


def _model_plan(offsets, numels, wds, tile, direct):
    """Python model of the planner: maximal runs of contiguous tensors with equal weight decay, and the
    number of tiles of a grid anchored at element 0 that each run touches."""
    segs = []
    for o, n, w in zip(offsets, numels, wds):
        if n == 0:
            continue
        if segs and segs[-1][1] == o and segs[-1][2] == w:
            segs[-1][1] = o + n
        else:
            segs.append([o, o + n, w])
    count = lambda T: sum((hi - 1) // T - lo // T + 1 for lo, hi, _ in segs)
    return len(segs), count(tile), count(direct)


def test_planner_against_python_model_random_layouts():
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=150, deadline=None)
    @given(st.lists(st.tuples(st.integers(0, 40), st.integers(0, 5000), st.sampled_from([0.0, 0.0, 0.01])), min_size=1, max_size=30),
           st.sampled_from([B.DADAM_F32, B.DADAM_BF16]), st.integers(1, 64))
    def check(items, dtype, n):
        offsets, numels, wds, cur = [], [], [], 0
        for gap, numel, wd in items:
            cur += gap
            offsets.append(cur); numels.append(numel); wds.append(wd)
            cur += numel
        d = cur + 1
        h = B.dadam_init(n, n, d, offsets, numels, dtype, dtype, accum_s=2, device=B.DADAM_DEVICE_NONE, weight_decay=wds)
        info = B.dadam_get_plan_info(h)
        vec = 8 if dtype == B.DADAM_BF16 else 4
        assert info.tile_elems == 64 * vec and info.direct_elems == 256 * vec * 2
        want = _model_plan(offsets, numels, [float(np.float32(w)) for w in wds], info.tile_elems, info.direct_elems)
        assert (info.n_segments, info.n_tiles_tile, info.n_tiles_direct) == want
        assert info.lds_bytes_tile == n * 64 * 16 and info.tile_mode_possible == 1
        B.dadam_destroy(h)

    check()


def test_c99_client_compiles_links_and_agrees_with_the_binding(tmp_path):
    """The header is plain C (gcc -std=c99 -pedantic -Werror), a C program links against the library,
    and what it is told (packing, plan, status codes) is what the Python binding is told."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    libdir = os.path.dirname(B.LIB_PATH)
    exe = str(tmp_path / "abi_client")
    rocm_lib = "/opt/rocm/lib"
    cmd = [gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "abi_client.c"), "-o", exe, "-L", libdir, "-ldadam",
           f"-Wl,-rpath,{libdir}", f"-Wl,-rpath,{rocm_lib}", f"-Wl,-rpath-link,{rocm_lib}"]
    subprocess.run(cmd, check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    got = dict(line.split(" ", 1) for line in out.strip().splitlines())

    numel = [1000, 24, 5001]
    offsets, d = B.dadam_pack_offsets(numel, 8)
    assert int(got["pack_rc"]) == 0 and int(got["d"]) == d
    assert [int(got[f"offset{i}"]) for i in range(3)] == [int(o) for o in offsets]
    h = B.dadam_init(4, 4, d, offsets, numel, accum_s=2, device=B.DADAM_DEVICE_NONE)
    info = B.dadam_get_plan_info(h)
    B.dadam_destroy(h)
    assert int(got["init_rc"]) == 0 and int(got["topology_rc"]) == 0 and int(got["warn"]) == 0
    assert int(got["bad_topology_rc"]) == B.DADAM_ETOPO and int(got["bad_topology_has_message"]) == 1
    assert int(got["plan_rc"]) == 0
    for key in ("n_segments", "tile_elems", "n_tiles_tile", "n_tiles_direct", "lds_bytes_tile"):
        assert int(got[key]) == int(getattr(info, key)), key
    assert int(got["row_order_rc"]) == 1 and sorted(got["row_order"]) == list("0123")
    assert int(got["stretches_rc"]) == 0 and int(got["n_stretches"]) == 3 and int(got["regions_found"]) == 1
    assert int(got["every"]) == 2 and int(got["deal_rc"]) == 0
    assert int(got["first_in_region0"]) == 1 and int(got["second_in_region1"]) == 1
    assert int(got["mix_on_host_only_handle_rc"]) == B.DADAM_ESTATE
    assert int(got["set_lr_rc"]) == 0 and int(got["done"]) == 1


def test_two_region_placement_policy():
    """Placement advice for device buffers (memory management, no GPU needed): two regions either
    side of the boundary between the first two thirds of the device memory, buffers dealt alternately
    and staggered inside their gaps; the flag says when the advice could not be applied."""
    GIB = 1 << 30
    total = 288 * GIB - (20 << 20)
    sizes = [476 << 20] * 112                                   # configuration 2 with two gradient sets
    off, regs, advice = B.dadam_place_offsets(sizes, 275 * GIB, total)
    assert advice == B.DADAM_PLACE_TWO_REGIONS and regs == [(30 * GIB, 94 * GIB), (98 * GIB, 162 * GIB)]
    assert (off, regs, advice) == B.dadam_place_offsets(sizes, 275 * GIB, total)      # deterministic
    even = [0] * len(sizes)                                     # the same regions at equal distances
    for r, (lo, hi) in enumerate(regs):
        for k, o in zip(range(r, len(sizes), 2), B.dadam_spread_offsets(sizes[r::2], hi - lo)):
            even[k] = lo + o
    for k, o in enumerate(off):
        lo, hi = regs[k % 2]
        assert lo <= o and o + sizes[k] <= hi and o % (2 << 20) == 0
        assert even[k] <= o and (k + 2 >= len(off) or o + sizes[k] <= even[k + 2]), "a buffer left its own gap"
    spans = sorted((o, o + n) for o, n in zip(off, sizes))
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
    # the bases of a region do not form an arithmetic progression
    below = [o for k, o in enumerate(off) if k % 2 == 0]
    assert len({b - a for a, b in zip(below, below[1:])}) > len(below) // 2
    # any run of consecutive buffers is split evenly over the two sides
    for start, count in ((0, 16), (16, 16), (0, 32), (80, 32)):
        n_below = sum(1 for k in range(start, start + count) if off[k] < 96 * GIB)
        assert n_below == count // 2
    # large buffers widen the regions up to the room there is
    off4, regs4, advice = B.dadam_place_offsets([3 * GIB] * 56, 275 * GIB, total)
    assert advice == B.DADAM_PLACE_TWO_REGIONS and regs4 == [(0, 94 * GIB), (98 * GIB, 190 * GIB)]
    # what cannot fit either side of the boundary, or an arena that does not cover the device (its offsets
    # are no physical positions): equal distances over the whole arena, and the flag says which
    placed, used, advice = B.dadam_place_offsets([4 * GIB] * 56, 275 * GIB, total)
    assert advice == B.DADAM_PLACE_TOO_LARGE and used == [(0, 275 * GIB)] and placed == B.dadam_spread_offsets([4 * GIB] * 56, 275 * GIB)
    for arena_bytes in (90 * GIB, 200 * GIB, 234 * GIB, 271 * GIB):
        placed, used, advice = B.dadam_place_offsets(sizes, arena_bytes, total)
        assert advice == B.DADAM_PLACE_ARENA_ELSEWHERE and used == [(0, arena_bytes)]
        assert placed == B.dadam_spread_offsets(sizes, arena_bytes)
    assert B.dadam_place_offsets(sizes, 272 * GIB, total)[2] == B.DADAM_PLACE_TWO_REGIONS
    assert B.dadam_place_offsets([1 << 30], 275 * GIB, total)[2] == 0          # one buffer: nothing to deal
    assert B.lib.dadam_place_offsets(None, 1, 100, 100, None, None, None) == B.DADAM_EINVAL
    with pytest.raises(B.DadamError):
        B.dadam_place_offsets([5 << 20, 5 << 20], 8 << 20, 288 * GIB)


def test_rows_that_share_sources_are_neighbours_in_direct_modes_row_order():
    """Direct mode hands contiguous groups of a row order to the device's dies; in that order rows that share a
    source follow each other, so that one die's L2 serves the second reader.  The order is a permutation, used
    only when rows share sources and there is more than one die, and follows the chains of a one-peer graph."""
    def order_of(n, csr, **kw):
        L = WL.pack([("flat", (1000,))])
        h = B.dadam_init(n, n, L.d, L.offsets, L.numels, device=B.DADAM_DEVICE_NONE, **kw)
        B.dadam_set_topology(h, 0, *csr)
        out = B.dadam_get_row_order(h, 0, n)
        B.dadam_destroy(h)
        return out
    def shared(csr, i, j):
        rp, col, _w = csr
        return len(set(col[rp[i]:rp[i + 1]]) & set(col[rp[j]:rp[j + 1]]))
    for k in range(6):                                               # hop 2^k on 64 replicas: chains 0, h, 2h, ...
        csr = WL.one_peer_exponential(64, k)
        order, used = order_of(64, csr)
        assert used and sorted(order) == list(range(64))
        hop = 1 << k
        chain = 64 // hop
        assert order[:chain] == [(j * hop) % 64 for j in range(chain)]
        breaks = sum(1 for a, b in zip(order, order[1:]) if shared(csr, a, b) == 0)
        assert breaks == hop - 1                                     # only where one chain ends and the next begins
        # within every group of 8 (one die's share) at most the group's first row lacks a sharing predecessor
        inside = sum(1 for g in range(8) for a, b in zip(order[8 * g:8 * g + 8], order[8 * g + 1:8 * g + 8]) if shared(csr, a, b))
        assert inside >= 56 - max(0, hop - 8) - 7 * (hop >= 8) - 7 and inside >= 28
    order, used = order_of(16, WL.ring(16))
    assert used and sorted(order) == list(range(16)) and all(shared(WL.ring(16), a, b) >= 1 for a, b in zip(order, order[1:]))
    assert order_of(16, WL.identity(16)) == (list(range(16)), False)     # nothing shared
    order, used = order_of(12, WL.ring(12))                              # 12 rows over 8 dies: groups of 1 or 2
    assert used and sorted(order) == list(range(12))
    assert order_of(12, WL.ring(12), n_xcds=1) == (list(range(12)), False)   # one die: nothing to deal
    rng = np.random.default_rng(3)
    for n in (8, 40, 160):                                               # random rows: still a permutation
        rp, col, w = [0], [], []
        for i in range(n):
            deg = int(rng.integers(1, 6))
            cs = rng.choice(n, size=deg, replace=False)
            col += [int(c) for c in cs]; w += [1.0 / deg] * deg; rp.append(len(col))
        order, _used = order_of(n, (np.array(rp, np.int32), np.array(col, np.int32), np.array(w, np.float32)))
        assert sorted(order) == list(range(n))
    h, _ = host_handle(4, 4)
    expect(B.DADAM_ESTATE, B.dadam_get_row_order, h, 3, 4)
    B.dadam_destroy(h)


def test_dealing_buffers_over_two_given_regions():
    """dadam_deal_offsets: even-numbered buffers in the first region, odd-numbered in the second, inside them,
    apart from each other, on 2 MiB marks, whichever region lies lower; bad regions are refused."""
    GIB, MIB = 1 << 30, 1 << 20
    sizes = [(100 + 7 * k) * MIB + 12345 for k in range(37)]
    for r0, r1 in (((10 * GIB, 40 * GIB), (130 * GIB, 150 * GIB)), ((130 * GIB, 150 * GIB), (10 * GIB, 40 * GIB)),
                   ((0, 6 * GIB), (6 * GIB, 12 * GIB))):
        off = B.dadam_deal_offsets(sizes, r0, r1)
        assert off == B.dadam_deal_offsets(sizes, r0, r1)
        for k, (o, n) in enumerate(zip(off, sizes)):
            lo, hi = (r0, r1)[k % 2]
            assert lo <= o and o + n <= hi and o % (2 * MIB) == 0, (k, o)
        spans = sorted((o, o + n) for o, n in zip(off, sizes))
        assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
        for r in (0, 1):                                             # order inside a region follows the buffers' order
            side = off[r::2]
            assert side == sorted(side)
    assert B.dadam_deal_offsets([5 * MIB], (0, 6 * MIB), (0, 0)) == [0]
    for bad in (((0, 2 * GIB), (1 * GIB, 3 * GIB)),                  # overlapping
                ((0, 1 * GIB), (2 * GIB, 2 * GIB + 200 * MIB)),      # second too small for its 18 buffers
                ((MIB, 1 * GIB), (2 * GIB, 40 * GIB)),               # not on a 2 MiB mark
                ((2 * GIB, 1 * GIB), (4 * GIB, 40 * GIB))):          # ends before it starts
        with pytest.raises(B.DadamError):
            B.dadam_deal_offsets(sizes, *bad)


def test_thirds_are_found_from_timings_of_a_modelled_memory():
    """The library's search for stretches in different thirds of the memory (dadam_find_stretches,
    dadam_regions_from_stretches), run against a model of the device in place of its timing probe:
    physical position = arena offset + a base, a pass over two chunks sustains 0.79 of peak across thirds and
    0.73 or 0.65 (alternating 8 GiB bands) inside one, with 1 % noise.  Whatever the base, the stretches found
    are those of the model, and the two regions chosen lie in different thirds with room for the buffers."""
    CHUNK = B.PROBE_CHUNK_BYTES
    GIB = 1 << 30
    rng = np.random.default_rng(5)

    def model(base):
        def third(off):
            return ((off + base) // (96 * GIB)) % 3, (off + base) % (96 * GIB) + CHUNK > 96 * GIB
        def rate(a, b):
            (ta, sa), (tb, sb) = third(a), third(b)
            r = 0.79 if ta != tb else (0.73 if ((a + base) // (8 * GIB) + (b + base) // (8 * GIB)) % 2 == 0 else 0.65)
            if sa or sb:                                             # a chunk across a boundary: in between
                r = 0.76
            return r * (1 + 0.01 * rng.uniform(-1, 1))
        return rate

    sizes = [476 << 20] * 112                                        # configuration 2 with two gradient sets: 26 GiB a side
    half = sum(sizes) // 2
    third_of = lambda off, base: (off + base) // (96 * GIB)
    seen_every = set()
    for base_gib, span_gib in ((0, 275), (40, 235), (70, 200), (100, 170), (190, 90), (3, 60), (50, 100), (75, 60), (20, 90)):
        base, span = base_gib * GIB, span_gib * GIB
        runs = B.dadam_find_stretches(span, model(base))
        assert runs and runs[0][1] == 0
        for t, lo, hi in runs:                                       # each stretch lies in one third (up to one chunk of overlap)
            assert third_of(lo, base) == third_of(hi - 1 - CHUNK, base), (base_gib, runs)
        firsts = {third_of(lo, base) for _t, lo, _hi in runs}
        assert len(runs) == len(firsts) == third_of(span - CHUNK, base) - third_of(0, base) + 1, (base_gib, runs)
        assert len({t for t, _lo, _hi in runs}) == len(runs)
        found = B.dadam_regions_from_stretches(runs, sizes)
        room = sorted(hi - lo for _t, lo, hi in runs)
        if len(runs) >= 2 and room[-1] >= sum(sizes) * 7 // 8 + (1 << 30) and room[-2] >= sum(sizes) // 8 + (1 << 30):
            (lo0, hi0), (lo1, hi1), every = found
            seen_every.add(every)
            off = B.dadam_deal_offsets(sizes, (lo0, hi0), (lo1, hi1), every)      # fits
            assert third_of(lo0, base) == third_of(hi0 - 1 - CHUNK, base) if lo0 < lo1 else third_of(lo0 + CHUNK, base) == third_of(hi0 - 1, base)
            assert third_of(lo1 + CHUNK, base) == third_of(hi1 - 1, base) if lo0 < lo1 else third_of(lo1, base) == third_of(hi1 - 1 - CHUNK, base)
            assert third_of((lo0 + hi0) // 2, base) != third_of((lo1 + hi1) // 2, base)
            assert hi0 - lo0 <= 64 * GIB and hi1 - lo1 <= 64 * GIB
            assert min(hi0, hi1) <= max(lo0, lo1)
            if every == 2:
                assert hi0 - lo0 >= half and hi1 - lo1 >= half
            else:                                                    # the even split did not fit anywhere
                assert room[-2] < half + (2 << 20) * len(sizes)
        elif len(runs) < 2 or room[-2] < sum(sizes) // 8:
            assert found is None
    assert seen_every >= {2} and len(seen_every) >= 2, seen_every
    # a memory with no fast pairing at all: one stretch, no regions
    runs = B.dadam_find_stretches(100 * GIB, lambda a, b: 0.66)
    assert len(runs) == 1 and B.dadam_regions_from_stretches(runs, sizes) is None
    assert B.dadam_find_stretches(5 * GIB, lambda a, b: 0.79) == []
    # timings that make no sense (a fast pairing here and there): nothing is believed
    noisy = np.random.default_rng(1)
    assert B.dadam_find_stretches(200 * GIB, lambda a, b: 0.79 if noisy.uniform() < 0.5 else 0.65) == []
    # a third that comes back later in the arena (an allocation pieced together from fragments) is accepted
    def fragments(a, b):
        piece = lambda off: 0 if off < 40 * GIB else 1 if off < 90 * GIB else 0
        return 0.79 if piece(a) != piece(b) else 0.66
    runs = B.dadam_find_stretches(130 * GIB, fragments)
    assert [t for t, _lo, _hi in runs] == [0, 1, 0] and B.dadam_regions_from_stretches(runs, sizes) is not None


def test_device_access_helpers_on_the_cpu_under_sanitizers(tmp_path):
    """The kernels' vector load / store helpers (the lane-to-element layout, clipping at segment
    edges, the two-group layout of 8-element lanes) and the maps from workgroup id to work item,
    compiled for the host from the kernel source's own text and run on exact-size buffers under
    ASan + UBSan."""
    import shutil
    import subprocess
    from paper_2410_11998_amd import build as bld
    clang = "/opt/rocm/llvm/bin/clang++" if os.path.exists("/opt/rocm/llvm/bin/clang++") else shutil.which("clang++")
    if clang is None:
        pytest.skip("no clang++ (the helpers use clang vector extensions)")
    src = open(os.path.join(bld.CSRC, "dadam_device.h")).read()
    a = src.index("typedef float f4 __attribute__((ext_vector_type(4)));")
    b = src.index("// Algorithm 3, lines 6-13, for one element.")
    b = src.rindex("// ----", a, b)
    (tmp_path / "helpers.inc").write_text(src[a:b])
    exe = str(tmp_path / "emulate")
    cmd = [clang, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-I", str(tmp_path), os.path.join(ROOT, "tests", "emulate_access_helpers.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = {k: v for k, v in os.environ.items()}
    env["ASAN_OPTIONS"] = "detect_leaks=0"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0 and "fails 0" in r.stdout, (r.stdout[-1500:], r.stderr[-1500:])
    assert r.stdout.count(" ok") == 11 and "work orders ok" in r.stdout
