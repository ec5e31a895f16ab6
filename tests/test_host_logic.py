"""CPU-only checks of the library's host logic: the shared object loads, exports every symbol the header
declares, and its closed-form schedule arithmetic agrees with the oracle's real FIFO queues."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1909_02625_amd as D
from oracle import dsp_oracle as O
from tests.test_oracle_pins import PAPER_TUPLES, _run_counting

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "dsp.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dsp_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 30
    lib = ctypes.CDLL(D.lib_path())
    for n in names:
        assert hasattr(lib, n), "libdsp_hip.so does not export %s" % n
    assert sorted(D.EXPORTED_SYMBOLS) == names, "binding and header disagree"
    for n in names:  # the binding offers the same names
        assert hasattr(D, n), n


def test_loaded_library_was_built_from_these_sources():
    """The binary carries a hash of csrc/ and include/dsp.h; the binding refuses one built from other sources."""
    from paper_1909_02625_amd import build
    assert D.dsp_build_id() == build.source_hash() and len(D.dsp_build_id()) == 16


def test_strerror_and_status_codes():
    assert D.dsp_strerror(0) == "ok"
    assert "order" in D.dsp_strerror(2)
    with pytest.raises(D.DSPError) as e:
        D.dsp_schedule_validate((1, 1), (2, 0))   # p_{K-1} != 0
    assert e.value.status == 1 and "p_{K-1}" in str(e.value)


@pytest.mark.parametrize("p,m,q", PAPER_TUPLES)
def test_schedule_validate_matches_paper_tuples(p, m, q):
    assert D.dsp_schedule_validate(p, m) == list(q) == O.queue_lengths(p, m)


@pytest.mark.parametrize("p,m", [((1, 0), (1, 0)), ((2, 0), (2, 0)), ((1, 1, 0), (2, 2, 0)), ((0, 1, 0), (4, 2, 0)),
                                 ((1, 0), (0, 0)), ((1, 1, 0), (4, 4, 0)), ((1, 0), (2, -1)), ((0, 0, 0), (1, 1, 0)),
                                 ((0, 0, 0), (2, 0, 0))])
def test_schedule_rejects_what_the_oracle_rejects(p, m):
    with pytest.raises(ValueError):
        O.queue_lengths(p, m)
    with pytest.raises(D.DSPError):
        D.dsp_schedule_validate(p, m)


@pytest.mark.parametrize("p,m,_q", PAPER_TUPLES + [((1, 0), (2, 0), None), ((1, 1, 0), (7, 3, 1), None),
                                                   ((2, 1, 3, 0), (12, 8, 4, 0), None), ((0, 0, 0), (0, 0, 0), None),
                                                   ((0, 0, 0), (2, 1, 0), None), ((0, 0, 0, 0), (3, 2, 1, 0), None),
                                                   ((0, 0), (2, 0), None), ((0, 0, 0), (5, 2, 1), None)])
def test_closed_form_index_equals_fifo_simulation(p, m, _q):
    """Brute force: the oracle pushes tagged items through real queues for 64 ticks; the library's closed
    form must name the same forward batch, backward batch and update count for every block and tick, and
    its ring slots must never collide (a slot is not rewritten while a batch that still needs it lives there)."""
    K = len(p)
    _, orc = _run_counting(p, m, 64)
    q = D.dsp_schedule_validate(p, m)
    live = [dict() for _ in range(K)]     # ring slot -> batch held, per block
    for rec in orc.log:
        tau = rec["tau"]
        for k in range(K):
            ix = D.dsp_schedule_index(p, m, k, tau)
            assert ix["a"] == (rec["fwd"][k] if rec["fwd"][k] is not None else -1)
            assert ix["b"] == (rec["bwd"][k] if rec["bwd"][k] is not None else -1)
            assert ix["version"] == rec["version"][k]
            ring = 1 + m[k] + (p[k - 1] if k else 0)
            if ix["b"] >= 0:
                assert ix["slot_bwd"] == ix["b"] % ring
                assert ix["q_write"] == (ix["b"] % (1 + q[k]) if k > 0 else -1)
                assert ix["q_read"] == (ix["b"] % (1 + q[k + 1]) if k < K - 1 else -1)
            # the producer (block k-1, or the data source) fills slot of batch tau - P_{k-1} at this tick
            a_prod = tau - sum(p[:k - 1]) if k > 0 else tau
            if a_prod >= 0:
                slot = a_prod % ring
                old = live[k].get(slot)
                if old is not None:
                    # the batch being overwritten must already have had its backward in block k
                    assert old + sum(p[:k]) + m[k] <= tau - 1, (k, tau, old)
                live[k][slot] = a_prod


def test_queue_memory_formula():
    """Section 3.3: extra space O(sum_k m_k + p_k + q_k) -- rings hold (1+m_k+p_{k-1}) inputs and (1+q_k) gradients."""
    p, m = (1, 1, 0), (4, 2, 0)
    h = [100, 40, 20, 10]
    q = D.dsp_schedule_validate(p, m)
    want = (1 + 4) * 100 + (1 + 2 + 1) * 40 + (1 + 0 + 1) * 20 + (1 + q[1]) * 40 + (1 + q[2]) * 20
    assert D.dsp_schedule_queue_elems(p, m, h) == want
    # never more than the paper's three separate queues per block
    paper = sum((1 + m[k]) * h[k] + (1 + p[k]) * h[k + 1] + (1 + q[k]) * h[k] for k in range(3))
    assert want <= paper


def test_make_block_desc_marshalling():
    from workloads import get_config
    cfg = get_config("resnet20", batch=4, hw=8)
    desc, keep = D.make_block_desc(cfg["blocks"][1], (4, 16, 8, 8), D.DSP_FP32, 1, 3, 2, p_prev=1)
    assert desc.n_layers == len(cfg["blocks"][1]) and desc.m_k == 2 and desc.p_prev == 1
    ops = [keep[i].op for i in range(desc.n_layers)]
    assert ops[0] == 0 and ops[1] == 1
    res = [keep[i].in1 for i in range(desc.n_layers) if keep[i].op == 1]
    assert -2 in res and any(r >= -1 for r in res)


def _drift_simulation(p, m, spare, wait_dn, wait_up, label_slots, ticks, rng):
    """Lets K blocks run their ticks as intervals [start, end] on a common clock in a random order that only
    obeys "block k starts tick tau after block k-1 has ended tick tau - wait_dn[k] and block k+1 has ended
    tick tau - wait_up[k]" and its own stream order, with blocks stalling at random.  Every queue access of a
    tick may happen anywhere inside its interval.  Returns the list of hazards found: a read whose value was
    written by a tick that had not ended before the reader's tick started, or whose slot is rewritten by a
    tick that started before the reader's tick ended."""
    K = len(m)
    q = O.queue_lengths(p, m)
    P = [sum(p[:k]) for k in range(K)]
    ring = [1 + m[k] + (p[k - 1] + spare[k] if k else 0) for k in range(K)]
    qn = [1 + q[k] + spare[k] for k in range(K)]
    started, ended, clock = [0] * K, [0] * K, 0
    span = {}
    stall = [0] * K
    while min(ended) < ticks:
        moves = []
        for k in range(K):
            if started[k] > ended[k]:
                if stall[k] == 0:
                    moves.append(("end", k))
            elif started[k] < ticks:
                tau = started[k]
                dn_ok = k == 0 or wait_dn[k] == 0 or tau < wait_dn[k] or ended[k - 1] > tau - wait_dn[k]
                up_ok = k == K - 1 or wait_up[k] == 0 or tau < wait_up[k] or ended[k + 1] > tau - wait_up[k]
                if dn_ok and up_ok:
                    moves.append(("start", k))
        clock += 1
        if not moves:
            assert any(stall), "the waits deadlock: %r" % ((started, ended),)
        for k in range(K):
            stall[k] = max(0, stall[k] - 1)
        if not moves:
            continue
        kind, k = moves[rng.integers(len(moves))]
        if kind == "start":
            span[(k, started[k])] = [clock, None]
            started[k] += 1
            if rng.random() < 0.2:
                stall[k] = int(rng.integers(1, 12 * K))   # this tick takes many times longer than the others'
        else:
            span[(k, ended[k])][1] = clock
            ended[k] += 1
    # the accesses of every tick, per shared resource (a queue between two blocks, or the label ring)
    writes, reads = {}, []   # (resource, slot) -> [(batch, tick key)], and (resource, slot, batch, tick key)
    for k in range(K):
        for tau in range(ticks):
            a, key = tau - P[k], (k, tau)
            b = a - m[k] if a >= 0 else -1
            if k == 0:
                writes.setdefault(("labels", tau % label_slots), []).append((tau, key))
            if a >= 0:
                if k > 0:
                    reads.append((("act", k), a % ring[k], a, key))
                if k < K - 1:
                    writes.setdefault((("act", k + 1), a % ring[k + 1]), []).append((a, key))
                else:
                    reads.append(("labels", a % label_slots, a, key))
            if b >= 0:
                if k > 0:
                    reads.append((("act", k), b % ring[k], b, key))
                    writes.setdefault((("grad", k), b % qn[k]), []).append((b, key))
                if k < K - 1:
                    reads.append((("grad", k + 1), b % qn[k + 1], b, key))
    hazards = []
    for res, slot, batch, key in reads:
        ws = writes.get((res, slot), [])
        mine = [w for w in ws if w[0] == batch]
        if len(mine) != 1:
            hazards.append(("never written", res, batch, key))
            continue
        if not span[mine[0][1]][1] < span[key][0]:
            hazards.append(("read before written", res, batch, key))
        for wb, wkey in ws:
            if wb > batch and not span[wkey][0] > span[key][1]:
                hazards.append(("rewritten before read", res, batch, key, wb))
    return hazards


@pytest.mark.parametrize("p,m,spare", [
    ((1, 1, 0), (4, 2, 0), (0, 0, 0)), ((1, 1, 0), (4, 2, 0), (0, 2, 2)), ((2, 2, 0), (6, 3, 0), (0, 1, 3)),
    ((3, 3, 0), (10, 5, 0), (0, 4, 4)), ((3, 3, 0), (10, 5, 0), (0, 0, 1)), ((1, 1, 0), (7, 3, 1), (0, 2, 0)),
    ((2, 1, 3, 0), (12, 8, 4, 0), (0, 3, 0, 5)), ((1, 0), (2, 0), (0, 6)),
])
def test_wait_distances_keep_every_queue_access_ordered_however_the_blocks_drift(p, m, spare):
    """Section 3.3 / Section 6 (robustness): with spare queue entries the blocks may drift apart; the wait
    distances the library derives must still order every read after its write and before the slot's next
    write, never deadlock, and be the loosest that do (one tick more in either direction gives a hazard)."""
    K = len(m)
    q = O.queue_lengths(p, m)
    dn, up, labels = D.dsp_schedule_waits(p, m, spare)
    assert dn == [0] + [min(p[k - 1], 1 + spare[k]) for k in range(1, K)]
    assert up == [min(q[k + 1], 1 + spare[k + 1]) for k in range(K - 1)] + [0]
    rng = np.random.default_rng(99)
    for trial in range(12):
        assert _drift_simulation(p, m, spare, dn, up, labels, 60, rng) == []
    # teeth: looking one tick further back on any single edge lets some interleaving break an access
    for k in range(K):
        for which in ("dn", "up"):
            if (which == "dn" and k == 0) or (which == "up" and k == K - 1):
                continue
            d2, u2 = list(dn), list(up)
            (d2 if which == "dn" else u2)[k] += 1
            found = False
            for trial in range(40):
                try:
                    found = found or bool(_drift_simulation(p, m, spare, d2, u2, labels, 60, rng))
                except AssertionError:
                    found = True
                if found:
                    break
            assert found, (which, k)
    # the label ring (sufficient, not always the minimum) must at least span the forward lag of the last block
    assert sum(p) + 1 <= labels <= sum(p) + K + sum(spare)


def test_schedule_waits_arguments():
    assert D.dsp_schedule_waits((0, 0, 0), (0, 0, 0)) == ([0, 0, 0], [0, 0, 0], 3)
    assert D.dsp_schedule_waits((1, 1, 0), (4, 2, 0)) == ([0, 1, 1], [1, 1, 0], 5)
    with pytest.raises(D.DSPError):
        D.dsp_schedule_waits((1, 1, 0), (4, 2, 0), (1, 0, 0))    # block 0 has no queue below it
    with pytest.raises(D.DSPError):
        D.dsp_schedule_waits((1, 1, 0), (4, 2, 0), (0, 65, 0))
