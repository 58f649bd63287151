"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its schedule generator / simulator agree bit for bit with
the schedule oracle.  No compute call is made (there is no GPU here)."""
import ctypes as C
import os
import re

import pytest

from oracle import schedule_oracle as so
from paper_2107_06925_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "chimera.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(chimera_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 30
    raw = C.CDLL(b.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    # and the binding wraps each of them under the same name
    for n in names:
        assert n in b._SIGNATURES, n


ALGOS = [(b.DIRECT, so.chimera_schedule), (b.GPIPE, so.gpipe_schedule), (b.ONE_F_ONE_B, so.one_f_one_b_schedule)]
SHAPES = [(2, 2), (4, 4), (4, 8), (6, 6), (6, 18), (8, 8), (8, 32), (10, 20), (16, 64), (32, 32), (64, 64)]


@pytest.mark.parametrize("D,N", SHAPES)
@pytest.mark.parametrize("algo,make", ALGOS, ids=["chimera", "gpipe", "1f1b"])
def test_schedule_bit_exact(algo, make, D, N):
    want = make(D, N)
    ref = so.simulate(want, D, 1, 1)
    for rank in range(D):
        got = b.chimera_schedule(algo, D, N, rank)
        assert [o.astuple() for o in got] == want[rank]
        assert [o.start for o in got] == ref["start"][rank]
        # slots: a backward frees the slot its forward took; never two live in one slot
        live = {}
        for o in got:
            key = (o.pipe, o.slot)
            if o.kind == 0:
                assert key not in live
                live[key] = o.mb
            else:
                assert live.pop(key) == o.mb
        assert not live
        # the flagged op is the last backward of each pipe
        for pipe in {o.pipe for o in got}:
            bw = [o for o in got if o.kind == 1 and o.pipe == pipe]
            assert [o.last_of_stage for o in bw] == [0] * (len(bw) - 1) + [1]
    for cf, cb in ((1, 1), (1, 2), (2, 5)):
        ref = so.simulate(want, D, cf, cb)
        got = b.chimera_schedule_stats(algo, D, N, cf, cb)
        assert got["makespan"] == ref["makespan"]
        assert got["bubbles"] == ref["bubbles"]
        assert got["stash_peak"] == ref["stash_peak"]
        assert got["critical"] == ref["critical"]


def test_baselines_accept_odd_depth():
    for algo, make in ALGOS[1:]:
        want = make(5, 7)
        for rank in range(5):
            assert [o.astuple() for o in b.chimera_schedule(algo, 5, 7, rank)] == want[rank]


def test_stash_slots_per_stage():
    # worker 0 of D=4: down stage keeps 2 in flight, up stage 1; total peak 3 = D/2+1 (Table 2)
    assert b.stash_slots_needed(b.DIRECT, 4, 4, 0) == (2, 1)
    assert b.stash_slots_needed(b.DIRECT, 4, 4, 1) == (2, 2)
    for D in (4, 8, 32):
        for rank in range(D):
            d, u = b.stash_slots_needed(b.DIRECT, D, D, rank)
            assert max(d, u) <= D // 2 and d + u >= so.simulate(so.chimera_schedule(D, D), D)["stash_peak"][rank]


@pytest.mark.parametrize("args", [(b.DIRECT, 5, 5, 0), (b.DIRECT, 4, 6, 0), (b.DIRECT, 4, 2, 0), (b.DIRECT, 4, 4, 4),
                                  (b.DIRECT, 4, 4, -1), (b.DIRECT, 0, 4, 0), (b.GPIPE, 4, 0, 0), (7, 4, 4, 0)])
def test_schedule_errors(args):
    with pytest.raises(b.ChimeraError) as e:
        b.chimera_schedule(*args)
    assert e.value.code == b.EINVAL
    assert b.last_error()


def test_schedule_capacity():
    n = C.c_size_t(0)
    assert b.lib().chimera_schedule(b.DIRECT, 4, 4, 0, None, 0, C.byref(n)) == b.OK and n.value == 8
    buf = (b.chimera_op * 3)()
    assert b.lib().chimera_schedule(b.DIRECT, 4, 4, 0, buf, 3, C.byref(n)) == b.ENOMEM and n.value == 8
    assert b.lib().chimera_schedule_stats(b.DIRECT, 4, 4, 0, 1, None, None, None, None) == b.EINVAL


def test_stage_create_errors_and_sizes():
    L = b.lib()
    for bad in [(0, 128, 4, 64, 2, b.F32), (2, 130, 4, 64, 2, b.F32), (2, 128, 3, 64, 2, b.F32),
                (2, 128, 4, 0, 2, b.F32), (2, 128, 4, 64, 2, 9), (2, 100, 4, 64, 2, b.BF16)]:
        assert not L.chimera_stage_create(*bad)
        assert b.last_error()
    st = L.chimera_stage_create(2, 128, 4, 64, 2, b.F32)
    assert st
    H = 128
    per_layer = 12 * H * H + 13 * H
    assert L.chimera_stage_weight_bytes(st) == 2 * per_layer * 4
    assert L.chimera_stage_grad_bytes(st) == 2 * per_layer * 4
    M = 128
    assert L.chimera_stage_stash_slot_bytes(st) >= 2 * 15 * M * H * 4
    assert L.chimera_stage_workspace_bytes(st) > 0
    assert L.chimera_stage_set_option(st, b.OPT_CAUSAL, 0) == b.OK
    assert L.chimera_stage_set_option(st, b.OPT_CAUSAL, 2) == b.EINVAL
    assert L.chimera_stage_set_option(st, 99, 0) == b.EINVAL
    # protocol errors that need no device: unbound stage
    assert L.chimera_fwd(st, 0) == b.ESTATE
    assert L.chimera_bwd(st, 0) == b.ESTATE
    assert L.chimera_stage_zero_grads(st) == b.ESTATE
    assert L.chimera_stage_bind(st, None, None, None, 1, None, None) == b.EINVAL
    assert L.chimera_worker_bind(st, None) == b.ESTATE
    L.chimera_stage_destroy(st)
    st16 = L.chimera_stage_create(2, 128, 4, 64, 2, b.BF16)
    assert L.chimera_stage_weight_bytes(st16) == 2 * per_layer * 2
    assert L.chimera_stage_grad_bytes(st16) == 2 * per_layer * 4
    L.chimera_stage_destroy(st16)
