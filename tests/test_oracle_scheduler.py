"""Pins for oracle/scheduler.py: a three-sample run worked out by hand, and brute-force
invariants on random workloads."""
import numpy as np
import pytest

from oracle.scheduler import SchedulerModel


def _hand_model():
    # page = 4 tokens, pool = 6 pages.  (P, max_new, L): s0 (5,3,3)  s1 (3,5,2)  s2 (6,6,4)
    # reservations ceil((P+max_new)/4) = 2, 2, 3  -> s2 must wait for a retirement.
    return SchedulerModel([5, 3, 6], [3, 5, 6], [3, 2, 4], pool_pages=6, page_tokens=4)


def test_hand_worked_three_samples():
    m = _hand_model()
    # step 0: admit s0, s1 (2+2 <= 6; s2 would make 7).  Prefill s0 writes 0..4 -> pages 0,1;
    # s1 writes 0..2 -> page 2.  Decode: s0 writes 5, s1 writes 3; both now have 2 tokens.
    i0 = m.generate_step()
    assert (i0.n_admitted, i0.n_prefill_tokens, i0.n_decoded, i0.n_active) == (2, 8, 2, 2)
    assert m.pages[:2] == [[0, 1], [2]] and m.ctx == [6, 4, 0] and m.gen_len == [2, 2, 0]
    assert m.retire() == [1]                       # s1 reached L = 2; page 2 returns
    assert m.free == [5, 4, 3, 2] and m.reserved == 2 and m.active == [0]
    # step 1: s2 fits now (2+3).  Its prompt 0..5 -> pages 2 (re-issued), 3.  Decode: s0
    # writes 6 (gen 3 = L), s2 writes 6.
    i1 = m.generate_step()
    assert (i1.n_admitted, i1.n_prefill_tokens, i1.n_decoded, i1.n_active) == (1, 6, 2, 2)
    assert m.pages[2] == [2, 3] and m.ctx == [7, 4, 7] and m.active == [0, 2]
    assert m.retire() == [0]                       # pages 1 then 0 go back: 0 is issued next
    assert m.free == [5, 4, 1, 0] and m.reserved == 3
    # step 2: s2 writes 7.  step 3: s2 writes 8 -> new page (0); gen 4 = L.
    assert m.generate_step().n_decoded == 1 and m.retire() == []
    assert m.generate_step().n_decoded == 1
    assert m.pages[2] == [2, 3, 0] and m.ctx[2] == 9
    assert m.retire() == [2]
    assert m.free == [5, 4, 1, 0, 3, 2] and m.reserved == 0
    assert m.retired == [1, 0, 2] and m.generation_done() and m.step == 4
    assert m.admit_step == [0, 0, 1]


@pytest.mark.parametrize("fused,R_t,chunk,want,want_steps", [
    # retire order 1 (5 tokens, step 0), 0 (8 tokens, step 1), 2 (10 tokens, step 3)
    (True, 4, 10, [[1], [0], [2]], [1, 3, 3]),   # 5 + 8 > 10: [1] closes when 0 arrives; 8 + 10 > 10: [0] when 2 arrives
    (True, 4, 13, [[1, 0], [2]], [3, 3]),        # 5 + 8 fits exactly and stays open until 2 (13 + 10 > 13) arrives
    (True, 2, 10, [[1], [0], [2]], [1, 3, 3]),   # remaining (1 waiting + 1 active) < 2 only after step 1
    (True, 1, 10, [[1], [0], [2]], [3, 3, 3]),   # remaining < 1 only when generation is over
    (False, 4, 13, [[1, 0], [2]], [3, 3]),       # sequential: same cut, all after the last step
    (True, 4, 1, [[1], [0], [2]], [1, 3, 3]),    # bound below every sample: each alone, closed by its successor
    (True, 4, 100, [[1, 0, 2]], [3]),            # everything fits: flushed at the end
])
def test_hand_worked_batches(fused, R_t, chunk, want, want_steps):
    m = _hand_model()
    trace = m.run_stage(fused, R_t, chunk)
    assert len(trace) == 4
    assert m.batches == want and m.batch_step == want_steps
    assert [len(t[2]) for t in trace].count(0) == 4 - len(set(want_steps))


@pytest.mark.parametrize("to_back", [False, True])
def test_hand_worked_migration(to_back):
    """Re-prefill migration (Section 4.2, second mechanism) worked by hand on the same three
    samples: after step 0 sample 0 (5 prompt tokens, 2 generated, pages 0 and 1) is migrated."""
    m = _hand_model()
    m.generate_step()
    assert m.retire() == [1]
    with pytest.raises(ValueError):
        m.migrate([1])                               # retired samples cannot move
    with pytest.raises(ValueError):
        m.migrate([2])                               # nor waiting ones
    m.migrate([0], to_back=to_back)
    # its pages return in reverse table order (1, then 0), its reservation is released
    assert m.free == [5, 4, 3, 2, 1, 0] and m.reserved == 0 and m.active == []
    assert m.waiting == ([2, 0] if to_back else [0, 2]) and m.ctx[0] == 0 and m.gen_len[0] == 2
    # step 1: both fit (2 + 3 <= 6).  Sample 0 rebuilds prompt + first generated token = 6
    # positions and emits nothing; sample 2 prefills its 6 prompt tokens.  Pages are issued
    # in admission order.  Then both decode: sample 0 feeds its second token (position 6).
    i1 = m.generate_step()
    assert (i1.n_admitted, i1.n_prefill_tokens, i1.n_decoded, i1.n_active) == (2, 12, 2, 2)
    if to_back:
        assert m.active == [2, 0] and m.pages[2] == [0, 1] and m.pages[0] == [2, 3]
    else:
        assert m.active == [0, 2] and m.pages[0] == [0, 1] and m.pages[2] == [2, 3]
    assert m.ctx == [7, 4, 7] and m.gen_len == [3, 2, 2]
    assert m.retire() == [0] and m.reserved == 3
    assert m.generate_step().n_decoded == 1 and m.retire() == []
    assert m.generate_step().n_decoded == 1 and m.retire() == [2]
    assert m.retired == [1, 0, 2] and m.generation_done() and m.step == 4
    assert sorted(m.free) == list(range(6)) and m.admit_step == [1, 0, 1]


def _check_invariants(m: SchedulerModel, ordered: bool = True):
    owned = [p for pl in m.pages for p in pl]
    assert len(owned) == len(set(owned))                         # a page has one owner
    assert sorted(owned + m.free) == list(range(m.pool_pages))   # free + owned = pool
    for i in range(m.N):
        assert len(m.pages[i]) == (-(-m.ctx[i] // m.page) if i in m.active else 0)
    assert not ordered or m.active == sorted(m.active)           # admission order = id order
    assert m.reserved == sum(m.reserve[i] for i in m.active)
    assert m.optimistic or m.reserved <= m.pool_pages
    assert len(m.active) <= m.max_active


@pytest.mark.parametrize("seed", range(6))
def test_invariants_random(seed):
    r = np.random.default_rng(seed)
    N = int(r.integers(1, 40))
    P = r.integers(1, 70, N)
    L = np.minimum(np.floor(4 * r.uniform(1e-3, 1, N) ** (-1 / 1.2)), 150).astype(int)
    max_new = L + r.integers(0, 20, N) if seed % 2 else np.full(N, 150)
    page = int(r.choice([4, 16]))
    need = max(-(-(int(p) + int(mn)) // page) for p, mn in zip(P, max_new))
    pool = int(need * r.choice([1, 2, 5]))
    m = SchedulerModel(P, max_new, L, pool, page, max_active=int(r.choice([3, N])))
    chunk = int(r.choice([1, 64, 400]))
    R_t = int(r.integers(0, N + 2))
    finish = {}
    while not m.generation_done():
        info = m.generate_step()
        _check_invariants(m)
        for i in m.retire():
            finish[i] = info.step
        _check_invariants(m)
        if len(m.waiting) + len(m.active) < R_t or m.generation_done():
            m.form_batches(chunk)
    assert sorted(m.retired) == list(range(N)) and len(m.free) == pool and m.reserved == 0
    for i in range(N):                    # prefill and the first decode share the admit step
        assert finish[i] == m.admit_step[i] + max(int(L[i]) - 2, 0)
        assert m.gen_len[i] == L[i] and m.ctx[i] == P[i] + L[i] - 1
    assert m.step == max(finish.values()) + 1
    assert [i for b in m.batches for i in b] == m.retired        # batches tile the FIFO in order
    flat = m.retired
    pos = 0
    for b in m.batches[:-1]:
        tok = sum(m.seq_tokens(i) for i in b)
        pos += len(b)
        assert tok <= chunk or len(b) == 1                       # bounded from above (one sample always goes)
        assert tok + m.seq_tokens(flat[pos]) > chunk             # and maximal: the next sample did not fit
    # waiting samples are admitted in order
    adm = [m.admit_step[i] for i in range(N)]
    assert adm == sorted(adm)


@pytest.mark.parametrize("seed", range(6))
def test_invariants_random_with_migrations(seed):
    """Random migrations of unfinished samples: pages and reservations stay consistent, every
    sample still ends with its own length, and a migrated sample costs exactly one more
    prefill over what it had cached."""
    r = np.random.default_rng(100 + seed)
    N = int(r.integers(2, 30))
    P = r.integers(1, 50, N)
    L = r.integers(1, 60, N)
    page = int(r.choice([4, 16]))
    need = max(-(-(int(p) + int(l)) // page) for p, l in zip(P, L))
    m = SchedulerModel(P, L, L, int(need * r.choice([1, 3])), page, max_active=int(r.choice([2, N])))
    decoded, prefilled, extra = 0, 0, 0
    while not m.generation_done():
        info = m.generate_step()
        decoded += info.n_decoded
        prefilled += info.n_prefill_tokens
        _check_invariants(m, ordered=False)
        m.retire()
        _check_invariants(m, ordered=False)
        movable = [i for i in m.active if m.gen_len[i] < m.target[i]]
        if movable and r.random() < 0.4:
            ids = [int(i) for i in r.permutation(movable)[:int(r.integers(1, len(movable) + 1))]]
            extra += sum(int(P[i]) + m.gen_len[i] - 1 for i in ids)
            m.migrate(ids, to_back=bool(r.integers(0, 2)))
            _check_invariants(m, ordered=False)
            assert all(m.ctx[i] == 0 and m.pages[i] == [] for i in ids)
        assert m.step < 100000
    assert sorted(m.retired) == list(range(N)) and len(m.free) == m.pool_pages and m.reserved == 0
    assert decoded == int(np.sum(L - 1)) and prefilled == int(np.sum(P)) + extra
    for i in range(N):
        assert m.gen_len[i] == L[i] and m.ctx[i] == P[i] + L[i] - 1


def test_hand_worked_optimistic_admission_and_preemption():
    """Admission on present need + preemption by re-prefill, worked by hand: page = 4 tokens, pool = 3
    pages, two samples (P, L) = (3, 9) and (3, 6) whose cap reservations (3 pages each) would run
    them one after the other."""
    m = SchedulerModel([3, 3], [9, 9], [9, 6], pool_pages=3, page_tokens=4, optimistic=True)
    # step 0: each needs ceil((3 + 1) / 4) = 1 page now; after sample 0, 2 pages are free and one
    # must stay free per running sample: 2 - 1 >= 1, so sample 1 is admitted too.
    i0 = m.generate_step()
    assert (i0.n_admitted, i0.n_prefill_tokens, i0.n_decoded) == (2, 6, 2)
    assert m.pages == [[0], [1]] and m.ctx == [4, 4] and m.free == [2]
    # step 1: both are about to write position 4 (a new page each) and one page is free: the
    # most recently admitted sample, 1, is preempted; its page comes back and sample 0 takes it.
    i1 = m.generate_step()
    assert (i1.n_admitted, i1.n_decoded, i1.n_active) == (0, 1, 1) and m.n_preempted == 1
    assert m.waiting == [1] and m.pages == [[0, 1], []] and m.ctx == [5, 0] and m.gen_len == [3, 2]
    assert m.free == [2]
    # steps 2-7: sample 1 would rebuild 3 + 1 rows and decode one more: 2 pages, only 1 (then 0)
    # free, so it waits; sample 0 takes the last page at position 8 and ends at step 7.
    for step in range(2, 8):
        info = m.generate_step()
        assert (info.n_admitted, info.n_decoded) == (0, 1)
        assert m.retire() == ([0] if step == 7 else [])
    assert m.free == [2, 1, 0] and m.ctx[0] == 11
    # step 8: sample 1 comes back: 4 rows rebuilt (page 0), nothing emitted, then it feeds its
    # second token at position 4 (page 1) in the same step.
    i8 = m.generate_step()
    assert (i8.step, i8.n_admitted, i8.n_prefill_tokens, i8.n_decoded) == (8, 1, 4, 1)
    assert m.pages[1] == [0, 1] and m.ctx[1] == 5 and m.gen_len[1] == 3
    while not m.generation_done():
        m.generate_step(); m.retire()
    assert m.step == 12 and m.retired == [0, 1] and sorted(m.free) == [0, 1, 2]


@pytest.mark.parametrize("seed", range(8))
def test_invariants_random_optimistic(seed):
    """Random workloads under optimistic admission, pools from barely one sample to ample: pages
    stay consistent, every step decodes something, everybody ends with their own length, prefill
    work is the prompts plus exactly the rows rebuilt after preemptions, and the run is never
    longer than under cap reservations."""
    r = np.random.default_rng(200 + seed)
    N = int(r.integers(2, 40))
    P = r.integers(1, 60, N)
    L = np.minimum(np.floor(3 * r.uniform(1e-3, 1, N) ** (-1 / 1.2)), 120).astype(int)
    cap = np.full(N, 120)
    page = int(r.choice([4, 16]))
    need = max(-(-(int(p) + 120) // page) for p in P)
    pool = int(need * r.choice([1, 1, 2, 6]))
    ma = int(r.choice([3, N]))
    m = SchedulerModel(P, cap, L, pool, page, max_active=ma, optimistic=True)
    decoded = prefilled = 0
    rebuilt = 0
    while not m.generation_done():
        before = {i: m.gen_len[i] for i in m.waiting}
        info = m.generate_step()
        decoded += info.n_decoded
        prefilled += info.n_prefill_tokens
        assert info.n_decoded >= 1 or all(m.gen_len[i] >= m.target[i] for i in m.active)
        _check_invariants(m, ordered=False)
        m.retire()
        _check_invariants(m, ordered=False)
        assert m.step < 200000
    assert sorted(m.retired) == list(range(N)) and len(m.free) == pool and m.reserved == 0
    assert decoded == int(np.sum(L - 1)) and prefilled >= int(np.sum(P))
    assert (prefilled == int(np.sum(P))) == (m.n_preempted == 0)
    for i in range(N):
        assert m.gen_len[i] == L[i] and m.ctx[i] == P[i] + L[i] - 1
    c = SchedulerModel(P, cap, L, pool, page, max_active=ma)
    while not c.generation_done():
        c.generate_step(); c.retire()
    assert m.step <= c.step


def test_oversized_sample_is_rejected():
    with pytest.raises(MemoryError):
        SchedulerModel([100], [100], [5], pool_pages=3, page_tokens=16)


def test_fused_and_sequential_score_the_same_samples():
    """Section 4.1: fusion re-times sample-level subtasks; the set of scored samples and each
    sample's own inputs do not change."""
    P, L = [7, 9, 30, 4, 4, 18], [3, 40, 2, 9, 1, 5]
    a = SchedulerModel(P, [40] * 6, L, 12, 16); a.run_stage(True, 7, 32)
    b = SchedulerModel(P, [40] * 6, L, 12, 16); b.run_stage(False, 0, 32)
    assert a.retired == b.retired and a.step == b.step
    assert sorted(i for x in a.batches for i in x) == sorted(i for x in b.batches for i in x)
    assert a.batch_step != b.batch_step
