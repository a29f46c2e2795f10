"""The host-side plan of the split-K work list (no GPU needed): structure of the shares, the
capacity bound, and optimality against brute force on tiny lists."""
import itertools

import numpy as np
import pytest

import paper_2510_08525_amd as rl

ROUND, START = 2, 3          # the cost model stated in include/rlkv.h


def share_costs(rounds, wg_begin):
    """Cost of every share from the unit numbering: per pair one start unit, then its rounds."""
    kinds = []                                   # per unit: ('s', pair) or ('r', pair)
    for p, r in enumerate(rounds):
        if r:
            kinds += [("s", p)] + [("r", p)] * int(r)
    costs = []
    for w in range(len(wg_begin) - 1):
        seg = kinds[wg_begin[w]:wg_begin[w + 1]]
        costs.append(sum(START if k == "s" else ROUND for k, _ in seg))
    return costs, kinds


def check_plan(rounds, n_wg):
    used, wg_begin, seg_first, seg_count = rl.rlkv_plan_shares(rounds, n_wg)
    total = int(sum(r + 1 for r in rounds if r))
    assert wg_begin[0] == 0 and wg_begin[-1] == total
    assert (np.diff(wg_begin) >= 0).all()
    nonempty = int((np.diff(wg_begin) > 0).sum())
    assert nonempty == used <= n_wg or (total == 0 and used == 0)
    costs, kinds = share_costs(rounds, wg_begin)
    # no share ends on a start unit (a pair's start travels with its first round)
    for w in range(n_wg):
        if wg_begin[w + 1] > wg_begin[w] and wg_begin[w + 1] < total:
            assert kinds[wg_begin[w + 1] - 1][0] == "r"
    # the workgroups of a pair are the consecutive ones the records name
    for p, r in enumerate(rounds):
        holders = [w for w in range(n_wg) if any(k == ("r", p) or k == ("s", p) for k in kinds[wg_begin[w]:wg_begin[w + 1]])]
        if r == 0:
            assert seg_count[p] == 0
        else:
            assert holders == list(range(seg_first[p], seg_first[p] + seg_count[p]))
    return max(costs) if costs else 0, used


@pytest.mark.parametrize("seed", range(8))
def test_structure_on_random_lists(seed):
    rng = np.random.RandomState(seed)
    n_pairs = int(rng.randint(1, 200))
    rounds = rng.choice([0, 1, 3, 3, 3, 40, 129, 513], size=n_pairs)
    if not rounds.any():
        rounds[0] = 5
    n_wg = int(rng.choice([1, 7, 64, 256, 1024]))
    worst, used = check_plan(rounds, n_wg)
    avg = sum(ROUND * r + START for r in rounds if r) / n_wg
    assert worst >= avg - 1e-9
    # the greedy never needs more than the average plus one start and one round, unless a single
    # pair start plus a round is already more than that
    assert worst <= max(avg + START + ROUND, START + ROUND) + ROUND


def brute_force_best(rounds, n_wg):
    """Smallest possible maximum share cost over all ways to cut the unit sequence into at most n_wg
    contiguous shares that never end on a start unit."""
    kinds = []
    for p, r in enumerate(rounds):
        if r:
            kinds += ["s"] + ["r"] * int(r)
    n = len(kinds)
    cuts_allowed = [i for i in range(1, n) if kinds[i - 1] == "r"]
    best = None
    for k in range(0, min(n_wg - 1, len(cuts_allowed)) + 1):
        for cuts in itertools.combinations(cuts_allowed, k):
            edges = [0, *cuts, n]
            worst = max(sum(START if x == "s" else ROUND for x in kinds[a:b]) for a, b in zip(edges, edges[1:]))
            best = worst if best is None else min(best, worst)
    return best


@pytest.mark.parametrize("rounds,n_wg", [
    ([3], 1), ([3], 4), ([5, 1, 1], 2), ([5, 1, 1], 3), ([2, 2, 2, 2], 3), ([7, 0, 1], 4), ([1, 1, 1, 1, 1], 2),
    ([4, 3, 0, 2], 4), ([6, 1], 3), ([1, 6], 3), ([2, 5, 2], 5),
])
def test_greedy_capacity_is_optimal_on_tiny_lists(rounds, n_wg):
    worst, _ = check_plan(np.asarray(rounds), n_wg)
    assert worst == brute_force_best(rounds, n_wg)


def test_benchmark_shaped_list():
    """Qwen-shaped layer: 16 sequences x (2 full heads of 129 rounds + 2 compressed heads of 3)."""
    rounds = np.asarray(([129, 3, 129, 3]) * 16)
    worst, used = check_plan(rounds, 256)
    total_cost = sum(ROUND * r + START for r in rounds)
    assert used == 256 or worst * (256 - 1) < total_cost        # either every workgroup works or the tail is short
    assert worst <= total_cost / 256 + START + ROUND


def test_invalid_arguments():
    lib = rl.load_library()
    import ctypes
    a = (ctypes.c_int32 * 4)(1, 2, 3, 4)
    out = (ctypes.c_int32 * 8)()
    assert lib.rlkv_plan_shares(None, 4, 2, out, out, out) == -1
    assert lib.rlkv_plan_shares(a, 0, 2, out, out, out) == -1
    assert lib.rlkv_plan_shares(a, 4, 0, out, out, out) == -1
    bad = (ctypes.c_int32 * 4)(1, -2, 3, 4)
    assert lib.rlkv_plan_shares(bad, 4, 2, out, out, out) == -1


# ---- the form of a prefill chunk (host logic of rlkv_prefill_attention) ------------------------

def test_prefill_form_of_the_measured_cases():
    """Qwen shape (28 query / 4 KV heads: 36 chunk positions per workgroup, 57 workgroups per 2048-token
    chunk and full head), 256 compute units."""
    form = lambda n_full, tokens, cached, **kw: rl.rlkv_plan_prefill_form(256, 28, 4, n_full, tokens, cached, **kw)
    assert form(2, [2048], [131072 - 2048]) == (False, 2)        # 114 long workgroups -> 228
    assert form(1, [2048], [65536]) == (False, 4)                # 57 -> 228
    assert form(2, [2048, 2048], [8192, 8192]) == (False, 1)     # 228 already: neither divided nor narrowed
    assert form(2, [2048] * 16, [8192] * 16) == (False, 1)       # the batch-16 workload: untouched
    assert form(2, [2048], [0]) == (True, 1)                     # first chunk: nothing cached to divide
    assert form(2, [2048], [2 * 80 * 32 - 1]) == (True, 1)       # one key short of two shares of 80 tiles
    assert form(2, [2048], [2 * 80 * 32]) == (False, 2)
    assert form(2, [2048], [0], allow_narrow=False) == (False, 1)
    assert form(2, [2048], [4096], min_share_tiles=8) == (False, 2)
    assert form(1, [256], [100000]) == (False, 8)                # 8 long workgroups: the most shares there are
    # a sequence without a chunk counts for nothing, a short cached context among the active ones decides
    assert form(2, [2048, 0], [65536, 5]) == (False, 2)
    assert form(1, [1024, 1024], [65536, 100]) == (True, 1)


def test_prefill_form_bounds():
    """Shares never exceed the compute units in one round, the scratch slots (1024), or eight."""
    rng = np.random.default_rng(5)
    for _ in range(300):
        Hkv = int(rng.choice([1, 2, 4, 8])); G = int(rng.choice([1, 4, 7, 16])); n_full = int(rng.integers(0, Hkv + 1))
        B = int(rng.integers(1, 6)); n_cu = int(rng.choice([64, 256, 304]))
        tokens = rng.integers(0, 2049, size=B); cached = rng.integers(0, 200000, size=B)
        mst = int(rng.choice([8, 80]))
        if tokens.sum() == 0:
            tokens[0] = 1
        narrow, z = rl.rlkv_plan_prefill_form(n_cu, Hkv * G, Hkv, n_full, tokens, cached, min_share_tiles=mst)
        per_block = 256 // G
        blocks = int(sum(-(-int(t) // per_block) for t in tokens))
        long_wgs = blocks * (n_full if n_full else Hkv)
        assert 1 <= z <= 8 and not (narrow and z > 1)
        if z > 1:
            assert n_full > 0 and long_wgs * z <= n_cu
            rows = -(-int(tokens.max()) // per_block) * int((tokens > 0).sum()) * n_full
            assert rows * z <= 1024
            assert min(int(c) for c, t in zip(cached, tokens) if t > 0) // 32 // z >= mst
        if narrow:
            assert 2 * long_wgs <= n_cu
        if 2 * long_wgs > n_cu:
            assert (narrow, z) == (False, 1)


def test_prefill_form_rejects_bad_arguments():
    with pytest.raises(rl.RlkvError):
        rl.rlkv_plan_prefill_form(256, 28, 5, 1, [1], [0])
    with pytest.raises(rl.RlkvError):
        rl.rlkv_plan_prefill_form(0, 28, 4, 1, [1], [0])
    with pytest.raises(rl.RlkvError):
        rl.rlkv_plan_prefill_form(256, 28, 4, 5, [1], [0])
    with pytest.raises(rl.RlkvError):
        rl.rlkv_plan_prefill_form(256, 28, 4, 1, [-1], [0])


# ---- which grid rows of a prefill chunk go one row per XCD -------------------------------------

def test_prefill_rows_of_the_measured_cases():
    rows = rl.rlkv_plan_prefill_rows
    assert rows(2, [2048] * 16, [8192] * 16) == (32, 32)         # the batch-16 workload: every full row dealt by rows
    assert rows(1, [2048] * 16, [0] * 16) == (16, 16)
    assert rows(3, [2048] * 5, [4096] * 5) == (8, 15)            # 15 heavy rows: one group of 8, the other 7 one by one
    assert rows(0, [2048] * 4, [0] * 4) == (0, 0)                # no full head: nothing heavy
    assert rows(2, [0, 0, 7], [100, 100, 100]) == (0, 2)
    # a ragged late chunk (three sequences end at different lengths): the first group mixes a 1760-token row
    # with 412-token ones, so every heavy row is dealt workgroup by workgroup
    assert rows(4, [1760, 412, 278, 0], [30720] * 3 + [9000]) == (0, 12)
    # three whole chunks ahead of shorter ones: the first eight rows are alike, the second eight are not
    assert rows(4, [435, 1220, 2048, 2048, 2048, 1339], [28672] * 6) == (8, 24)


def test_prefill_rows_properties():
    """The dealt rows are whole groups of 8 leading heavy rows, each alike within 15 % by the stated work model,
    and the first group left out (if any heavy rows remain for one) is not."""
    rng = np.random.default_rng(11)
    for _ in range(400):
        B = int(rng.integers(1, 40)); n_full = int(rng.integers(0, 9))
        tokens = rng.integers(0, 2049, size=B) * (rng.random(B) < 0.8)
        if rng.random() < 0.5:
            tokens = np.where(tokens > 0, 2048, 0)
        cached = rng.integers(0, 70000, size=B) if rng.random() < 0.5 else np.full(B, int(rng.integers(0, 70000)))
        dealt, heavy = rl.rlkv_plan_prefill_rows(n_full, tokens, cached)
        active = [b for b in range(B) if tokens[b] > 0]
        assert heavy == len(active) * n_full and dealt % 8 == 0 and 0 <= dealt <= heavy
        order = sorted(active, key=lambda b: -(int(cached[b]) + int(tokens[b])))       # (sorted is stable)
        work = [float(tokens[b]) * (float(cached[b]) + 0.5 * float(tokens[b]) + 600.0) for b in order for _ in range(n_full)]
        for g in range(0, dealt, 8):
            assert work[g + 7] >= 0.85 * work[g]
        if dealt + 8 <= heavy:
            assert work[dealt + 7] < 0.85 * work[dealt]


def test_prefill_rows_rejects_bad_arguments():
    with pytest.raises(rl.RlkvError):
        rl.rlkv_plan_prefill_rows(-1, [1], [0])
    with pytest.raises(rl.RlkvError):
        rl.rlkv_plan_prefill_rows(1, [-1], [0])
    with pytest.raises(rl.RlkvError):
        rl.rlkv_plan_prefill_rows(1, [1], [-5])
    with pytest.raises(rl.RlkvError):
        rl.rlkv_plan_prefill_rows(1, [1, 2], [0])


def test_prefill_block_map_is_a_bijection_that_keeps_dealt_rows_on_one_xcd():
    """The hardware hands workgroup `lin` to XCD lin % 8.  Under the kernel's map every block of the grid is worked
    on exactly once; a dealt heavy row y and a light row of a whole group of 8 have all their blocks on one XCD
    (y % 8, resp. (y - heavy) % 8); the heavy rows not dealt are spread evenly; every XCD serves its blocks in row
    order (long rows first)."""
    rng = np.random.default_rng(3)
    cases = [(57, 64, 32, 32), (32, 256, 64, 65), (28, 256, 0, 12), (1, 1, 0, 0), (3, 7, 0, 5), (5, 8, 8, 8), (2, 9, 8, 9)]
    for _ in range(60):
        gx, gy = int(rng.integers(1, 40)), int(rng.integers(1, 80))
        heavy = int(rng.integers(0, gy + 4))
        dealt = 8 * int(rng.integers(0, heavy // 8 + 2))
        cases.append((gx, gy, dealt, heavy))
    for gx, gy, dealt, heavy in cases:
        F = min(max(heavy, 0), gy)
        A = min(max(dealt, 0), F) // 8 * 8
        seen = set()
        xcds_of_row = {}
        last_row = [-1] * 8
        for lin in range(gx * gy):
            bx, by = rl.rlkv_plan_prefill_block(lin, gx, gy, dealt, heavy)
            assert 0 <= bx < gx and 0 <= by < gy
            seen.add((bx, by))
            xcds_of_row.setdefault(by, set()).add(lin % 8)
            assert by >= last_row[lin % 8], (gx, gy, dealt, heavy, lin)           # rows in order on every XCD
            last_row[lin % 8] = by
        assert len(seen) == gx * gy, (gx, gy, dealt, heavy)
        light_whole = F + (gy - F) // 8 * 8
        for y, xs in xcds_of_row.items():
            if y < A:
                assert xs == {y % 8}
            elif F <= y < light_whole:
                assert xs == {(y - F) % 8}
        if F - A > 0 and (F - A) * gx >= 8:
            spread = [sum(1 for lin in range(gx * gy) if lin % 8 == k and A <= rl.rlkv_plan_prefill_block(lin, gx, gy, dealt, heavy)[1] < F)
                      for k in range(8)]
            assert max(spread) - min(spread) <= 1
    with pytest.raises(rl.RlkvError):
        rl.rlkv_plan_prefill_block(6, 2, 3, 0, 0)
    with pytest.raises(rl.RlkvError):
        rl.rlkv_plan_prefill_block(-1, 2, 3, 0, 0)
