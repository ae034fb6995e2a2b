"""Host-side checks of the C ABI: the library loads, exports what include/mdbf.h declares,
its host-only functions agree with the oracle, and every argument error is reported before
any HIP call (so these run on a host without a GPU)."""
import ctypes as C
import os
import re

import pytest

from oracle import mdbf_oracle as orc
from paper_2512_24545_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "mdbf.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(mdbf_[a-z_]+)\s*\(", hdr))
    assert {"mdbf_pack", "mdbf_unpack", "mdbf_forward", "mdbf_forward_batch", "mdbf_bpw"} <= declared
    L = mb.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(mb.EXPORTS)
    assert mb.mdbf_version() == 100


def test_bpw_and_rank_match_oracle():
    for (m, n, k, l) in [(256, 256, 128, 4), (4096, 4096, 2656, 16), (11008, 4096, 4096, 16), (4096, 11008, 4096, 16),
                         (100, 37, 11, 3)]:
        assert mb.mdbf_bpw(m, n, k, l) == orc.bits_per_weight(m, n, k, l)
    assert mb.mdbf_bpw(256, 256, 128, 4) == 1.75
    assert mb.mdbf_bpw(64, 48, 32, 1, merge_inner=True) == orc.bits_per_weight(64, 48, 32, 1, merge_inner=True)
    assert mb.mdbf_bpw(64, 48, 32, 2, merge_inner=True) < 0
    for (m, n, l, bpw) in [(4096, 4096, 16, 1.5), (11008, 4096, 16, 1.5), (4096, 4096, 8, 1.0), (11008, 4096, 8, 1.0),
                           (4096, 4096, 16, 2.0), (11008, 4096, 16, 2.0), (512, 384, 2, 1.25)]:
        for mult in (1, 32):
            assert mb.mdbf_rank_for_budget(m, n, l, bpw, 16, mult) == orc.rank_for_budget(m, n, l, bpw, 16, mult)


def test_packed_bytes():
    # 16-row tiles x 128-column blocks, 64 words each
    assert mb.mdbf_packed_bytes(16, 128) == 256
    assert mb.mdbf_packed_bytes(17, 129) == 4 * 256
    assert mb.mdbf_packed_bytes(4096, 2656) == 256 * 21 * 256
    out = C.c_size_t(0)
    assert mb.lib().mdbf_packed_bytes(0, 5, C.byref(out)) == -1
    assert mb.lib().mdbf_packed_bytes(5, 5, None) == -1


FAKE = 0x10000  # a non-null, 16-byte aligned address that is never dereferenced


def _call_forward(desc, SA=FAKE, SB=FAKE, env=None, X=FAKE, ldx=None, Y=FAKE, ldy=None, T=1, ws=FAKE, wsb=1 << 30):
    env = env if env is not None else mb.Env(FAKE, FAKE, FAKE, FAKE)
    ldx = desc.n if ldx is None else ldx
    ldy = desc.m if ldy is None else ldy
    return mb.lib().mdbf_forward(C.byref(desc), SA, SB, C.byref(env), X, ldx, Y, ldy, T, ws, wsb, None)


def test_forward_argument_errors_before_any_launch():
    good = lambda: mb.Desc(64, 48, 32, 4, 0, 0, 2, 0)
    d = good(); d.l = 17
    assert _call_forward(d) == -1
    d = good(); d.l = 0
    assert _call_forward(d) == -1
    d = good(); d.m = 0
    assert _call_forward(d) == -1
    d = good(); d.x_dtype = 7
    assert _call_forward(d) == -3
    d = good(); d.flags = 0x80
    assert _call_forward(d) == -5
    d = good()
    assert _call_forward(d, SA=None) == -1
    assert _call_forward(d, X=None) == -1
    assert _call_forward(d, env=mb.Env(FAKE, None, FAKE, FAKE)) == -1
    assert _call_forward(d, T=0) == -1
    assert _call_forward(d, ldx=47) == -1
    assert _call_forward(d, ldy=63) == -1
    assert _call_forward(d, SB=FAKE + 4) == -2
    assert _call_forward(d, Y=FAKE + 8) == -2
    assert _call_forward(d, ws=None) == -1
    assert _call_forward(d, wsb=16) == -4
    assert mb.lib().mdbf_forward(None, FAKE, FAKE, None, FAKE, 1, FAKE, 1, 1, FAKE, 0, None) == -1


def test_workspace_bytes():
    d = mb.Desc(4096, 4096, 2656, 16, 0, 0, 0, 0)
    assert mb.mdbf_workspace_bytes(d, 1) >= 2656 * 4
    assert mb.mdbf_workspace_bytes(d, 16) >= 16 * 2656 * 4
    out = C.c_size_t(0)
    assert mb.lib().mdbf_workspace_bytes(C.byref(d), 0, C.byref(out)) == -1


def test_workspace_of_a_one_token_call_holds_its_partial_sums():
    """A single one-token call of rank 16 / fp16 envelopes splits each factor's contraction across workgroups:
    its workspace has room for the partial sums (4096x4096, k = 2656: 21 tile groups x 8 splits of the first
    factor, 32 x 7 of the second) and the second factor's completion counters, on top of what the same layer
    needs with MDBF_FLAG_FP16_STAGED (no split).  Other token counts and the fp32 path are not affected."""
    split = mb.Desc(4096, 4096, 2656, 16, mb.MDBF_F16, mb.MDBF_F16, mb.MDBF_F32, 0)
    staged = mb.Desc(4096, 4096, 2656, 16, mb.MDBF_F16, mb.MDBF_F16, mb.MDBF_F32, mb.MDBF_FLAG_FP16_STAGED)
    extra = mb.mdbf_workspace_bytes(split, 1) - mb.mdbf_workspace_bytes(staged, 1)
    ld1, ld2 = 2688, 4096                      # k and m rounded up to 64 floats
    assert extra == 8 * ld1 * 4 + 7 * ld2 * 4 + 256
    assert mb.mdbf_workspace_bytes(split, 2) == mb.mdbf_workspace_bytes(staged, 2)
    precise = mb.Desc(4096, 4096, 2656, 16, mb.MDBF_F16, mb.MDBF_F16, mb.MDBF_F32, mb.MDBF_FLAG_PRECISE)
    f32env = mb.Desc(4096, 4096, 2656, 16, mb.MDBF_F16, mb.MDBF_F32, mb.MDBF_F32, 0)
    for d in (precise, f32env):
        assert mb.mdbf_workspace_bytes(d, 1) < mb.mdbf_workspace_bytes(split, 1)


def test_pack_argument_errors():
    L = mb.lib()
    assert L.mdbf_pack(None, 4, 4, 4, FAKE, 1 << 20, None) == -1
    assert L.mdbf_pack(FAKE, 4, 4, 3, FAKE, 1 << 20, None) == -1
    assert L.mdbf_pack(FAKE, 4, 4, 4, FAKE + 2, 1 << 20, None) == -2
    assert L.mdbf_pack(FAKE, 4, 4, 4, FAKE, 8, None) == -4
    assert L.mdbf_unpack(FAKE, 4, 0, FAKE, 4, None) == -1


def test_pad_envelope_argument_errors():
    L = mb.lib()
    assert L.mdbf_pad_envelope(None, 4, 2, 0, FAKE, 8, None) == -1
    assert L.mdbf_pad_envelope(FAKE, 4, 9, 0, FAKE, 8, None) == -1      # l_to < l
    assert L.mdbf_pad_envelope(FAKE, 4, 2, 0, FAKE, 17, None) == -1     # beyond the largest rank
    assert L.mdbf_pad_envelope(FAKE, 0, 2, 0, FAKE, 8, None) == -1
    assert L.mdbf_pad_envelope(FAKE, 4, 2, 7, FAKE, 8, None) == -3      # unknown element type
    assert L.mdbf_pad_envelope(FAKE + 2, 4, 2, 0, FAKE, 8, None) == -2


def test_stream_read_argument_errors():
    L = mb.lib()
    assert L.mdbf_stream_read(None, 1024, FAKE, 8, None) == -1
    assert L.mdbf_stream_read(FAKE, 1024, None, 8, None) == -1
    assert L.mdbf_stream_read(FAKE, 0, FAKE, 8, None) == -1
    assert L.mdbf_stream_read(FAKE, 1000, FAKE, 8, None) == -1          # not a multiple of 16 bytes
    assert L.mdbf_stream_read(FAKE, 1024, FAKE, 6, None) == -1          # whole workgroups only
    assert L.mdbf_stream_read(FAKE, 1024, FAKE, 0, None) == -1
    assert L.mdbf_stream_read(FAKE, 1024, FAKE, (1 << 20) + 4, None) == -1
    assert L.mdbf_stream_read(FAKE + 4, 1024, FAKE, 8, None) == -2


def test_batch_plan_errors_and_sizes():
    L = mb.lib()
    arr = (mb.Layer * 2)()
    for i in range(2):
        arr[i].desc = mb.Desc(64, 48, 32, 4, 0, 0, 2, 0)
        arr[i].SA_packed_dev = FAKE
        arr[i].SB_packed_dev = FAKE
        arr[i].env = mb.Env(FAKE, FAKE, FAKE, FAKE)
        arr[i].X_dev = FAKE
        arr[i].ldx = 48
        arr[i].Y_dev = FAKE
        arr[i].ldy = 64
        arr[i].T = 1
    pb, wb = C.c_size_t(0), C.c_size_t(0)
    assert L.mdbf_batch_plan_bytes(2, arr, C.byref(pb), C.byref(wb)) == 0
    assert pb.value > 0 and wb.value >= 2 * 32 * 4
    buf = C.create_string_buffer(pb.value)
    assert L.mdbf_batch_plan_build(2, arr, FAKE, wb.value, buf, pb.value) == 0
    assert L.mdbf_batch_plan_build(2, arr, FAKE, 8, buf, pb.value) == -4
    assert L.mdbf_batch_plan_build(2, arr, FAKE, wb.value, buf, 8) == -4
    arr[1].T = 0
    assert L.mdbf_batch_plan_bytes(2, arr, C.byref(pb), C.byref(wb)) == -1
    assert L.mdbf_batch_plan_bytes(0, arr, C.byref(pb), C.byref(wb)) == -1
    # a plan whose magic is wrong is rejected before any launch
    bad = C.create_string_buffer(4096)
    assert L.mdbf_forward_batch(bad, FAKE, 4096, None) == -1


class _StageProb(C.Structure):
    # mirror of the library's internal stage descriptor (white-box: the plan is a byte blob of the library)
    _fields_ = [("S", C.c_void_p), ("Ein", C.c_void_p), ("Eout", C.c_void_p), ("vin", C.c_void_p),
                ("out", C.c_void_p), ("xs", C.c_void_p), ("vin_ld", C.c_int64), ("out_ld", C.c_int64),
                ("rows", C.c_int32), ("K", C.c_int32), ("l", C.c_int32), ("T", C.c_int32),
                ("KB", C.c_int32), ("ntiles", C.c_int32), ("env_dt", C.c_int32), ("vin_dt", C.c_int32),
                ("out_dt", C.c_int32), ("flags", C.c_int32)]


class _WorkItem(C.Structure):
    _fields_ = [("p", _StageProb), ("tile0", C.c_int32), ("ntiles", C.c_int32), ("prob", C.c_int32),
                ("pad", C.c_int32), ("fill", C.c_uint8 * 8)]


class _PlanHeader(C.Structure):
    _fields_ = [("magic", C.c_uint32), ("count", C.c_int32), ("nitems", C.c_int32 * 2),
                ("tiles_per_item", C.c_int32 * 2), ("precise", C.c_int32), ("fast", C.c_int32 * 2),
                ("pre", C.c_int32 * 2), ("max_units", C.c_int32 * 2), ("mx", C.c_int32 * 2), ("gemm", C.c_int32),
                ("gemm_mode", C.c_int32 * 2), ("max_tokens", C.c_int32), ("max_units_mx", C.c_int32 * 2),
                ("probs_off", C.c_uint64 * 2), ("items_off", C.c_uint64 * 2), ("total_bytes", C.c_uint64)]


def _plan_items(shapes, T=1):
    """Builds a plan of rank-16 fp16 layers over placeholder pointers (plan building touches no device
    memory) and returns its header and the two work-item tables."""
    L = mb.lib()
    n = len(shapes)
    arr = (mb.Layer * n)()
    for i, (m, nn, k) in enumerate(shapes):
        arr[i].desc = mb.Desc(m, nn, k, 16, 0, 0, 0, 0)
        arr[i].SA_packed_dev = FAKE
        arr[i].SB_packed_dev = FAKE
        arr[i].env = mb.Env(FAKE, FAKE, FAKE, FAKE)
        arr[i].X_dev = FAKE
        arr[i].ldx = nn
        arr[i].Y_dev = FAKE
        arr[i].ldy = m
        arr[i].T = T
    pb, wb = C.c_size_t(0), C.c_size_t(0)
    assert L.mdbf_batch_plan_bytes(n, arr, C.byref(pb), C.byref(wb)) == 0
    buf = C.create_string_buffer(pb.value)
    assert L.mdbf_batch_plan_build(n, arr, FAKE, wb.value, buf, pb.value) == 0
    assert C.sizeof(_StageProb) == 104 and C.sizeof(_WorkItem) == 128
    h = _PlanHeader.from_buffer_copy(buf.raw[:C.sizeof(_PlanHeader)])
    tables = []
    for s in range(2):
        off = h.items_off[s]
        tables.append([_WorkItem.from_buffer_copy(buf.raw[off + 128 * i: off + 128 * (i + 1)])
                       for i in range(h.nitems[s])])
    return h, tables


def test_block_scaled_plan_schedule_is_a_balanced_permutation():
    """Host logic of mdbf_batch_plan_build for the block-scaled kernel: the work items of a stage are the
    64-tile cuts of every problem, each exactly once, and within each of the eight slices of the table the 32
    workgroups (entry j, j + 32, ...) carry stage counts that differ by at most one item's."""
    attn, down = (4096, 4096, 2656), (4096, 11008, 4096)
    shapes = [attn, down] * 40                       # contraction lengths of 32 and 86 blocks in stage 1
    h, tables = _plan_items(shapes)
    assert h.magic == 0x4D444246 and h.count == 80 and list(h.mx) == [16, 16] and h.gemm == 0
    for s, items in enumerate(tables):
        want = []
        for i, (m, nn, k) in enumerate(shapes):
            rows = k if s == 0 else m
            nt = (rows + 15) // 16
            want += [(i, t0, min(64, nt - t0)) for t0 in range(0, nt, 64)]
        got = [(w.prob, w.tile0, w.ntiles) for w in items]
        assert sorted(got) == sorted(want) and len(got) == len(want)
        n, stride = len(items), 32
        assert n >= 256
        cost = lambda w: w.p.T * ((w.p.KB + 1) // 2 + 1)
        for x in range(8):
            lo, hi = n * x // 8, n * (x + 1) // 8
            loads = [sum(cost(items[i]) for i in range(lo + j, hi, stride)) for j in range(stride)]
            assert max(loads) - min(loads) <= max(cost(w) for w in items[lo:hi])
    # stage 1 mixes 17-stage and 44-stage items: in problem order one workgroup would carry two long ones
    c1 = sorted({tables[0][i].p.KB for i in range(len(tables[0]))})
    assert c1 == [32, 86]


def test_block_scaled_plan_puts_long_items_where_fewer_items_go():
    """96 MLP projections: factor 1 has 384 items on 256 workgroups (48 per slice: the first 16 workgroups of
    a slice take two, the others one); 16 items of a slice are 44 stages long (contraction over 11008), 32 are
    17.  The long ones must go alone: no workgroup carries more than 44 stages."""
    shapes = [(11008, 4096, 4096), (11008, 4096, 4096), (4096, 11008, 4096)] * 32
    h, tables = _plan_items(shapes)
    assert list(h.mx) == [16, 16]
    items = tables[0]
    assert len(items) == 384
    cost = lambda w: w.p.T * ((w.p.KB + 1) // 2 + 1)
    assert sorted({cost(w) for w in items}) == [17, 44]
    for x in range(8):
        lo, hi = 48 * x, 48 * (x + 1)
        loads = [sum(cost(items[i]) for i in range(lo + j, hi, 32)) for j in range(32)]
        assert max(loads) == 44 and min(loads) == 34


def _covered_once(items, shapes, s):
    """Every row tile of every problem is in exactly one work item."""
    seen = {}
    for w in items:
        for t in range(w.tile0, w.tile0 + w.ntiles):
            assert (w.prob, t) not in seen
            seen[(w.prob, t)] = 1
    want = sum(((k if s == 0 else m) + 15) // 16 for (m, nn, k) in shapes)
    assert len(seen) == want
    for (prob, t) in seen:
        m, nn, k = shapes[prob]
        assert 0 <= t < ((k if s == 0 else m) + 15) // 16


def test_block_scaled_plan_of_equal_layers_keeps_problem_order():
    """Equal layers: nothing to balance; whole rounds keep the problem order (the layers' activation records
    are shared through one L2 by neighbouring workgroups)."""
    shapes = [(4096, 4096, 2656)] * 256                # 768 and 1024 items: 3 and 4 whole rounds of 256 workgroups
    h, tables = _plan_items(shapes)
    assert list(h.mx) == [16, 16]
    for s, items in enumerate(tables):
        got = [(w.prob, w.tile0) for w in items]
        assert got == sorted(got)
        _covered_once(items, shapes, s)


def test_block_scaled_plan_cuts_the_last_partial_round_into_pieces():
    """336 equal layers: the second factor has 1344 items = 5.25 rounds of 256 workgroups.  The 64 items of the
    last round are cut into four pieces of 16 row tiles each, one per workgroup, dealt to the ends of the eight
    slices of the table; every row tile is still covered exactly once."""
    shapes = [(4096, 4096, 2656)] * 336
    h, tables = _plan_items(shapes)
    assert list(h.mx) == [16, 16]
    items = tables[1]
    assert len(items) == 1280 + 256 and h.nitems[1] == len(items)
    _covered_once(items, shapes, 1)
    for x in range(8):
        sl = items[192 * x: 192 * (x + 1)]
        assert [w.ntiles for w in sl] == [64] * 160 + [16] * 32
        full = [(w.prob, w.tile0) for w in sl[:160]]
        assert full == sorted(full)
        assert all(w.tile0 % 8 == 0 for w in sl)
    # the first factor (166 row tiles: 1008 items, 3.94 rounds) has more than half a round left: not cut
    assert len(tables[0]) == 1008
    _covered_once(tables[0], shapes, 0)


def test_launches_per_plan():
    """Both factors on the block-scaled kernel: three launches (scale-in, product + the next factor's records,
    product); a small plan on the fp16-staged kernels: four; many tokens: two."""
    L = mb.lib()
    def launches(shapes, T=1):
        n = len(shapes)
        arr = (mb.Layer * n)()
        for i, (m, nn, k) in enumerate(shapes):
            arr[i].desc = mb.Desc(m, nn, k, 16, 0, 0, 0, 0)
            arr[i].SA_packed_dev = arr[i].SB_packed_dev = arr[i].X_dev = arr[i].Y_dev = FAKE
            arr[i].env = mb.Env(FAKE, FAKE, FAKE, FAKE)
            arr[i].ldx, arr[i].ldy, arr[i].T = nn, m, T
        pb, wb = C.c_size_t(0), C.c_size_t(0)
        assert L.mdbf_batch_plan_bytes(n, arr, C.byref(pb), C.byref(wb)) == 0
        buf = C.create_string_buffer(pb.value)
        assert L.mdbf_batch_plan_build(n, arr, FAKE, wb.value, buf, pb.value) == 0
        return L.mdbf_batch_plan_launches(buf, pb.value)
    assert launches([(4096, 4096, 2656)] * 336) == 3
    assert launches([(4096, 4096, 2656)] * 3) == 4
    assert launches([(4096, 4096, 2656)] * 8, T=8) == 2
    assert L.mdbf_batch_plan_launches(None, 0) == -1


def test_block_scaled_plan_picks_the_item_size_that_wastes_fewest_tile_slots():
    """166 row tiles are three items of 56 tiles (56 + 56 + 54), not 64 + 64 + 38: the same number of items, an
    eighth fewer sign words moved per item and no idle waves in the third.  256 row tiles stay four items of
    64; 176 row tiles (k = 2816) stay 64 + 64 + 48, because 56-tile items would be four."""
    h, tables = _plan_items([(4096, 4096, 2656)] * 336)
    assert list(h.tiles_per_item) == [56, 64]
    per_layer = [w.ntiles for w in tables[0] if w.prob == 5]
    assert sorted(per_layer, reverse=True) == [56, 56, 54]
    assert all(w.tile0 % 4 == 0 for w in tables[0])
    h, tables = _plan_items([(4096, 11008, 2816)] * 300)
    assert list(h.tiles_per_item) == [64, 64]
    # a launch is cut with ONE item size: here 166- and 256-tile first factors together
    h, tables = _plan_items([(4096, 4096, 2656)] * 200 + [(4096, 4096, 4096)] * 200)
    assert h.tiles_per_item[0] in (56, 64) and h.tiles_per_item[1] == 64
    for s in range(2):
        _covered_once(tables[s], [(4096, 4096, 2656)] * 200 + [(4096, 4096, 4096)] * 200, s)


def test_msvid_argument_checks_and_workspace():
    """mdbf_msvid: block sizes, shape limits and the workspace formula, all on the host."""
    L = mb.lib()
    assert [L.mdbf_msvid_block(l) for l in (1, 8, 9, 16)] == [16, 16, 24, 24]
    assert L.mdbf_msvid_block(0) == -1 and L.mdbf_msvid_block(17) == -1
    need = C.c_size_t(0)
    assert L.mdbf_msvid_workspace_bytes(4096, 2656, 16, C.byref(need)) == 0
    # at least the transposed copy of Z, the partial products of the wider orientation and three blocks
    b = 24
    assert need.value >= 4096 * 2656 * 4 + 32 * 2656 * b * 4 + (4096 + 2 * 2656) * b * 4
    assert need.value < 2 * 4096 * 2656 * 4
    assert L.mdbf_msvid_workspace_bytes(20, 2656, 16, C.byref(need)) == -5      # fewer rows than block columns
    assert L.mdbf_msvid_workspace_bytes(4096, 2656, 17, C.byref(need)) == -1
    call = lambda rows=512, cols=384, ld=384, l=4, iters=8, Z=FAKE, ws=FAKE, wsb=1 << 30: L.mdbf_msvid(
        Z, rows, cols, ld, l, iters, FAKE, FAKE, FAKE, FAKE, FAKE, ws, wsb, None)
    assert call(Z=None) == -1 and call(ld=383) == -1 and call(iters=65) == -1 and call(iters=-1) == -1
    assert call(l=0) == -1 and call(rows=10) == -5
    assert call(Z=FAKE + 4) == -2 and call(ws=FAKE + 8) == -2
    assert call(wsb=1024) == -4


def test_strerror():
    L = mb.lib()
    assert L.mdbf_strerror(0) == b"ok"
    assert b"aligned" in L.mdbf_strerror(-2)
    assert L.mdbf_last_hip_error() == b""


def test_static_scratch_call_checks_its_limit_on_the_host():
    """mdbf_forward_static: the same argument checks as mdbf_forward, and a request beyond the static array's
    16 MiB is refused before any HIP call (this host has no GPU)."""
    d = mb.Desc(4096, 4096, 2656, 16, mb.MDBF_F16, mb.MDBF_F16, mb.MDBF_F32, 0)
    env = mb.Env(FAKE, FAKE, FAKE, FAKE)
    need = C.c_size_t(0)
    assert mb.lib().mdbf_workspace_bytes(C.byref(d), 2048, C.byref(need)) == 0 and need.value > (16 << 20)
    call = lambda desc, T, X=FAKE: mb.lib().mdbf_forward_static(C.byref(desc), FAKE, FAKE, C.byref(env), X, desc.n,
                                                                FAKE, desc.m, T, None)
    assert call(d, 2048) == -4                      # MDBF_EWORKSPACE
    assert call(d, 0) == -1 and call(d, 1, None) == -1 and call(d, 1, FAKE + 4) == -2
    bad = mb.Desc(4096, 4096, 2656, 17, mb.MDBF_F16, mb.MDBF_F16, mb.MDBF_F32, 0)
    assert call(bad, 1) == -1
