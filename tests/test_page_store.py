"""Paged activation store (Sec. 3.4, Algorithm 3): the plain model in oracle/ against a
hand-worked example, invariants and brute force; then the C++ store (both index kinds)
against the model, decision by decision.  CPU only."""
import os
import random

import pytest

from oracle.page_store_oracle import ALLOCATED, EVICTED, PLANNED, RELEASED, PageStoreOracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
STATE_NAMES = {"planned": PLANNED, "allocated": ALLOCATED, "evicted": EVICTED, "released": RELEASED}


class OracleFace:
    """Gives the model the same face as the binding's Store."""

    def __init__(self, page, mem, time_ns, step, index_kind=None):
        self.o = PageStoreOracle(page, mem, time_ns, step)

    def add(self, *a):
        self.o.add(*a)

    def receive(self, i, imp):
        return self.o.receive(i, imp)

    def release(self, i):
        self.o.release(i)

    def reset(self):
        self.o.reset()

    def set_mem_budget(self, b):
        return self.o.set_mem_budget(b)

    def set_time_budget(self, b):
        self.o.set_time_budget(b)

    def query(self, i):
        return self.o.query(i)

    def pop_evicted(self):
        return self.o.pop_evicted()

    def capacity_bytes(self):
        return self.o.capacity_bytes()

    def used_bytes(self):
        return self.o.used_mem

    def used_time_ns(self):
        return self.o.used_time

    def validate(self):
        return True


def make_store(kind, *args):
    if kind == "oracle":
        return OracleFace(*args)
    from paper_2507_07149_amd import store
    return store.Store(*args, index_kind={"rbtree": store.INDEX_RBTREE, "sort": store.INDEX_SORT}[kind])


def ints(s):
    return [int(v) for v in s.split(",")]


def replay_golden(kind):
    st = None
    for raw in open(os.path.join(ROOT, "tests", "golden", "page_store_example.txt")):
        line = raw.strip()
        if not line or line.startswith("#"):
            continue
        lhs, _, rhs = line.partition("->")
        op, *a = lhs.split()
        want = rhs.split()
        if op == "create":
            st = make_store(kind, int(a[0]), int(a[1]), None if a[2] == "none" else int(a[2]), int(a[3]))
        elif op == "add":
            st.add(int(a[0]), ints(a[1]), ints(a[2]), ints(a[3]), float(a[4]))
        elif op == "receive":
            assert list(st.receive(int(a[0]), float(a[1]))) == [int(v) for v in want], line
        elif op == "release":
            st.release(int(a[0]))
        elif op == "set_mem_budget":
            moves = st.set_mem_budget(int(a[0]))
            assert [tuple(m) for m in moves] == [tuple(int(v) for v in m.split(":")) for m in want], line
        elif op == "query":
            got = st.query(int(a[0]))
            assert list(got) == [STATE_NAMES[want[0]]] + [int(v) for v in want[1:]], line
        elif op == "used":
            assert st.used_bytes() == int(want[0]), line
        elif op == "capacity":
            assert st.capacity_bytes() == int(want[0]), line
        elif op == "pop_evicted":
            assert st.pop_evicted() == [int(v) for v in want], line
        else:
            raise AssertionError(f"unknown operation in the fixture: {line}")
        assert st.validate(), line


@pytest.mark.parametrize("kind", ["oracle", "rbtree", "sort"])
def test_hand_worked_example(kind):
    replay_golden(kind)


# ---- the model against what the readings fix, independently of its own code -----------------

def check_model_invariants(o: PageStoreOracle):
    live = [a for a in o.acts.values() if a.state in (PLANNED, ALLOCATED)]
    pages = lambda a: -(-a.bytes[a.w] // o.P)
    assert o.used_mem == sum(pages(a) * o.P for a in live)
    assert o.used_time == sum(a.time[a.w] for a in live)
    over = o.used_mem > o.B_mem or (o.B_time is not None and o.used_time > o.B_time)
    assert not over or not live
    taken = [False] * o.capacity
    for a in o.acts.values():
        if a.state == ALLOCATED:
            assert a.pages == pages(a) and 0 <= a.offset and a.offset + a.pages <= o.capacity
            for p in range(a.offset, a.offset + a.pages):
                assert not taken[p], "two activations share a page"
                taken[p] = True
        else:
            assert a.offset == -1 and a.pages == 0
    assert o.capacity <= max(o.B_mem // o.P, 0) or o.capacity % o.step_pages == 0
    return taken


def lowest_fit(taken, need):
    run = 0
    for p, t in enumerate(taken):
        run = 0 if t else run + 1
        if run == need:
            return p - need + 1
    return None


def random_acts(rng, n, page):
    acts = []
    for i in range(n):
        base = rng.randint(1, 40) * page // 2 + rng.randint(0, page - 1)
        widths = [8, 4, 2, 1][:rng.randint(1, 4)]
        sizes = [max(1, base * w // 8) for w in widths]
        times = [rng.randint(100, 5000) for _ in widths]
        acts.append((i * 3 + 1, widths, sizes, times, round(rng.uniform(0.0, 10.0), 3)))
    return acts


@pytest.mark.parametrize("seed", range(12))
def test_model_invariants_and_first_fit_by_bitmap(seed):
    rng = random.Random(seed)
    page = 256
    o = PageStoreOracle(page, rng.randint(20, 120) * page, rng.choice([None, rng.randint(5000, 60000)]), 8 * page)
    acts = random_acts(rng, 24, page)
    for a in acts:
        o.add(*a)
        check_model_invariants(o)
    for a in acts:
        taken = check_model_invariants(o)
        cap0, evicted0 = o.capacity, sum(1 for x in o.acts.values() if x.state == EVICTED)
        bits, off, size = o.receive(a[0], a[4] * rng.uniform(0.2, 3.0))
        taken_after = check_model_invariants(o)
        if bits:
            assert off % page == 0 and size == a[2][a[1].index(bits)]
            evicted1 = sum(1 for x in o.acts.values() if x.state == EVICTED)
            if o.capacity == cap0 and evicted1 == evicted0:
                # nothing else moved: the run must be the lowest free one in the old bitmap
                assert off // page == lowest_fit(taken, -(-size // page))
        if rng.random() < 0.15:
            o.set_mem_budget(rng.randint(10, 120) * page)
            check_model_invariants(o)
        del taken_after


def test_model_victim_is_the_smallest_ratio_by_brute_force():
    # memory only; three planned activations, the budget forces exactly one step
    o = PageStoreOracle(100, 1000, None, 100)
    o.add(1, [8, 4], [400, 200], [1, 1], 4.0)      # 0.0100 per byte
    o.add(2, [8, 4], [400, 200], [1, 1], 2.0)      # 0.0050 per byte  <- goes first
    o.add(3, [8, 4], [400, 200], [1, 1], 3.0)      # 0.0075 per byte
    assert [o.query(i)[1] for i in (1, 2, 3)] == [8, 4, 8]
    # ties go to the smaller id
    o = PageStoreOracle(100, 700, None, 100)
    o.add(5, [8, 4], [400, 200], [1, 1], 2.0)
    o.add(4, [8, 4], [400, 200], [1, 1], 2.0)
    assert [o.query(i)[1] for i in (4, 5)] == [4, 8]


def test_model_time_constraint_evicts_and_tighter_rule():
    # memory plentiful; time budget 2500 ns, three activations of 1000 ns: the one with the smallest
    # importance per nanosecond is evicted (the time index never narrows)
    o = PageStoreOracle(100, 10 ** 6, 2500, 100)
    o.add(1, [8, 4], [400, 200], [1000, 900], 5.0)
    o.add(2, [8, 4], [400, 200], [1000, 900], 1.0)
    o.add(3, [8, 4], [400, 200], [1000, 900], 3.0)
    assert [o.query(i)[0] for i in (1, 2, 3)] == [PLANNED, EVICTED, PLANNED]
    # both over: remaining proportions decide.  memory (1000-1200)/1000 = -0.2, time (1000-1500)/1000 = -0.5
    o = PageStoreOracle(100, 1000, 1000, 100)
    o.add(1, [8, 4], [600, 300], [750, 750], 1.0)
    assert o.query(1)[0] == PLANNED
    o.add(2, [8, 4], [600, 300], [750, 750], 2.0)          # time is tighter: evict the smaller ratio, id 1
    assert [o.query(i)[0] for i in (1, 2)] == [EVICTED, PLANNED]


def test_model_unlimited_budgets_store_everything_back_to_back():
    o = PageStoreOracle(128, 10 ** 9, None, 128 * 1024)
    sizes = [1000, 129, 128, 5000, 1]
    for i, s in enumerate(sizes):
        o.add(i, [8, 2], [s, max(1, s // 4)], [10, 10], 1.0)
    pos = 0
    for i, s in enumerate(sizes):
        assert o.receive(i, 1.0) == (8, pos * 128, s)
        pos += -(-s // 128)
    assert o.capacity_bytes() == 128 * 1024 and o.pop_evicted() == []


@pytest.mark.parametrize("kind", ["oracle", "rbtree", "sort"])
def test_fragmentation_evicts_allocated_in_memory_order(kind):
    # arena of 6 pages: three runs of two pages; freeing the middle one leaves no room for a
    # three-page activation although three pages' worth of budget is free after a release
    o = make_store(kind, 100, 600, None, 600)
    for i, imp in ((1, 5.0), (2, 9.0), (3, 1.0)):
        o.add(i, [8], [200], [1], imp)
    for i, imp in ((1, 5.0), (2, 9.0), (3, 1.0)):
        o.receive(i, imp)
    o.release(2)                                    # pages 2..3 free, used 4 pages
    o.add(4, [8], [200], [1], 7.0)                  # fits the budget (6 pages) and the hole
    assert o.receive(4, 7.0) == (8, 200, 200)
    o.release(4)
    o.add(5, [8], [300], [1], 7.0)                  # 4 + 3 = 7 pages > 6: id 3 (smallest ratio) is evicted
    assert o.query(3)[0] == EVICTED and o.pop_evicted() == [3]
    assert o.receive(5, 7.0) == (8, 200, 300)       # pages 2..4 are now one free run
    assert o.pop_evicted() == []
    # budget allows it, the holes do not: pages 0..1 taken, 2..4 taken, page 5 free; release id 1
    # (pages 0..1 free) and ask for three pages -> no run of three; id 5 is the only allocated one left
    o.release(1)
    o.add(6, [8], [250], [1], 1.0)                  # 3 + 3 = 6 pages <= 6: within budget
    assert o.receive(6, 1.0) == (8, 0, 250)         # id 5 had to go: pages 0..5 are one run again
    assert o.pop_evicted() == [5] and o.validate()


# ---- the C++ store against the model --------------------------------------------------------------

def run_scenario(kind, seed, log):
    rng = random.Random(seed)
    page = rng.choice([64, 256, 4096])
    mem = rng.randint(8, 200) * page + rng.randint(0, page - 1)
    tb = rng.choice([None, None, rng.randint(3000, 200000)])
    step = rng.choice([1, 4, 16]) * page
    st = make_store(kind, page, mem, tb, step)
    for it in range(3):
        st.reset()
        acts = random_acts(rng, rng.randint(1, 60), page)
        for a in acts:
            st.add(*a)
            log.append(("add", a[0], st.used_bytes(), st.used_time_ns(), st.query(a[0])))
            assert st.validate()
        order = list(acts)
        stored = []
        for a in order:
            r = st.receive(a[0], max(0.0, a[4] * rng.uniform(0.0, 3.0)))
            log.append(("receive", a[0], r, st.capacity_bytes(), st.used_bytes(), st.pop_evicted()))
            assert st.validate()
            if r[0]:
                stored.append(a[0])
            roll = rng.random()
            if roll < 0.10:
                moves = st.set_mem_budget(rng.randint(4, 220) * page + rng.randint(0, page - 1))
                log.append(("mem_budget", moves, st.capacity_bytes(), st.used_bytes(), st.pop_evicted()))
                assert st.validate()
            elif roll < 0.15:
                st.set_time_budget(rng.choice([None, rng.randint(2000, 200000)]))
                log.append(("time_budget", st.used_time_ns(), st.pop_evicted()))
                assert st.validate()
        for i in reversed(stored):
            if st.query(i)[0] == ALLOCATED:
                st.release(i)
                log.append(("release", i, st.used_bytes()))
        log.append(("final", [st.query(a[0]) for a in acts]))
        assert st.validate()


@pytest.mark.parametrize("kind", ["rbtree", "sort"])
@pytest.mark.parametrize("seed", range(40))
def test_cpp_store_makes_the_models_decisions(kind, seed):
    want, got = [], []
    run_scenario("oracle", seed, want)
    run_scenario(kind, seed, got)
    assert len(want) == len(got)
    for w, g in zip(want, got):
        assert tuple(w) == tuple(g)


def test_cpp_store_rejects_bad_arguments():
    from paper_2507_07149_amd import DafError, store
    with pytest.raises(DafError):
        store.Store(0, 100, None, 100)
    with pytest.raises(DafError):
        store.Store(64, 100, None, 100)             # step not a multiple of the page
    st = store.Store(64, 6400, None, 640)
    st.add(1, [8, 4], [100, 50], [10, 10], 1.0)
    with pytest.raises(DafError):
        st.add(1, [8], [100], [10], 1.0)            # duplicate id
    with pytest.raises(DafError):
        st.add(2, [8], [0], [10], 1.0)              # empty size
    with pytest.raises(DafError):
        st.add(3, [8], [10], [10], float("nan"))
    with pytest.raises(DafError):
        st.receive(99, 1.0)
    with pytest.raises(DafError):
        st.release(1)                               # not allocated yet
    assert st.receive(1, 1.0) == (8, 0, 100)
    with pytest.raises(DafError):
        st.receive(1, 1.0)                          # already allocated
    st.release(1)
    assert st.query(1) == (store.RELEASED, 0, -1, 0) and st.validate()


def test_red_black_trees_stay_valid_under_churn():
    # many insert / re-key / erase cycles through the public calls; validate() checks the
    # search order, the colours and the black heights of both trees
    from paper_2507_07149_amd import store
    rng = random.Random(7)
    st = store.Store(64, 64 * 3000, 10 ** 7, 64 * 100)
    ids = list(range(1, 401))
    for i in ids:
        st.add(i, [8, 4, 2, 1], [64 * rng.randint(1, 40), 64 * rng.randint(1, 20), 64 * rng.randint(1, 10), 64],
               [rng.randint(1, 50000)] * 4, rng.uniform(0, 100))
        if i % 25 == 0:
            assert st.validate()
    rng.shuffle(ids)
    for n, i in enumerate(ids):
        st.receive(i, rng.uniform(0, 100))
        if n % 20 == 0:
            assert st.validate()
        if n % 50 == 49:
            st.set_mem_budget(64 * rng.randint(500, 3000))
            assert st.validate()
    assert st.validate()


@pytest.mark.parametrize("kind", ["rbtree", "sort"])
def test_batched_calls_equal_the_single_ones(kind):
    import numpy as np
    rng = random.Random(3)
    page = 512
    acts = random_acts(rng, 200, page)
    acts = [(i, [8, 4, 2, 1], [max(1, s[0] * w // 8) for w in (8, 4, 2, 1)], [t[0]] * 4, imp)
            for (i, _, s, t, imp) in acts]
    one = make_store(kind, page, 600 * page, 150000, 32 * page)
    many = make_store(kind, page, 600 * page, 150000, 32 * page)
    for a in acts:
        one.add(*a)
    many.add_many([a[0] for a in acts], [8, 4, 2, 1], np.array([a[2] for a in acts]),
                  np.array([a[3] for a in acts]), [a[4] for a in acts])
    imps = [a[4] * rng.uniform(0.1, 2.0) for a in acts]
    want = [one.receive(a[0], imp) for a, imp in zip(acts, imps)]
    bits, off, size = many.receive_many([a[0] for a in acts], imps)
    assert want == list(zip(bits.tolist(), off.tolist(), size.tolist()))
    assert one.pop_evicted() == many.pop_evicted() and many.validate()
    assert one.num_selections() == many.num_selections() > 0


def test_cpp_store_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """page_store.cpp is host-only code: build it with tests/page_store_churn.cpp under
    -fsanitize=address,undefined and run random call sequences on a red-black-tree store and a
    re-sorting store side by side (same decisions, daf_store_validate after every call)."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "page_store_churn")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I" + os.path.join(root, "include"), "-I" + os.path.join(root, "paper_2507_07149_amd", "csrc"),
           os.path.join(root, "tests", "page_store_churn.cpp"),
           os.path.join(root, "paper_2507_07149_amd", "csrc", "page_store.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "sanitize" in build.stderr and "cannot find" in build.stderr:
        pytest.skip("sanitizer runtimes are not installed")
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1")
    run = subprocess.run([exe, "12", "2500"], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.startswith("ok:")
