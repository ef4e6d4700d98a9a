"""Pins for the discrete part of the oracle: the LRU expert cache and the speculative-prefetch
bookkeeping (Sec. 3.1-3.3).  The simulator is compared with a brute-force replay that keeps no
slots and no stamps: after any access sequence an LRU cache of k entries holds the k distinct
most recently accessed keys, found by scanning the history backwards."""
import itertools

import numpy as np

from oracle import moe_oracle as O


def most_recent_distinct(history, k):
    seen = []
    for e in reversed(history):
        if e not in seen:
            seen.append(e)
            if len(seen) == k:
                break
    return seen  # most recent first


class BruteCache:
    """History-replay model of one layer; access order inside a step: resident experts first,
    then absent ones, each in ascending id (the order the engine touches the cache in)."""

    def __init__(self, k):
        self.k, self.history = k, []

    def step(self, needed):
        before = most_recent_distinct(self.history, self.k)
        needed = sorted(set(needed))
        order = [e for e in needed if e in before] + [e for e in needed if e not in before]
        out = []
        for e in order:
            cur = most_recent_distinct(self.history, self.k)
            hit = e in cur
            victim = -1
            if not hit and len(cur) == self.k:
                victim = cur[-1]          # least recently used of the k
            out.append((e, hit, victim))
            self.history.append(e)
        return out

    def contents(self):
        return sorted(most_recent_distinct(self.history, self.k))


def test_lru_exhaustive_single_access_traces():
    for E in (2, 3, 4):
        for k in (1, 2, 3):
            for length in range(1, 7):
                for trace in itertools.product(range(E), repeat=length):
                    sim = O.ExpertCacheSim(1, E, k, b=0)
                    brute = BruteCache(k)
                    for e in trace:
                        acc, _ = sim.step(0, [[e]])
                        want = brute.step([e])
                        assert [(a.expert, a.status == O.HIT, a.victim) for a in acc] == want
                        assert sim.contents(0) == brute.contents()


def test_lru_random_top2_and_batched_steps():
    rng = np.random.default_rng(0)
    for E, k, B in [(8, 2, 1), (8, 4, 1), (8, 3, 1), (8, 4, 4), (8, 4, 16), (6, 2, 3)]:
        sim = O.ExpertCacheSim(1, E, k, b=0)
        brute = BruteCache(k)
        for _ in range(300):
            sel = [list(rng.choice(E, size=2, replace=False)) for _ in range(B)]
            acc, _ = sim.step(0, sel)
            want = brute.step([e for t in sel for e in t])
            assert [(a.expert, a.status == O.HIT, a.victim) for a in acc] == want
            assert sim.contents(0) == brute.contents()
            # slot bookkeeping is consistent: each access names the slot that now holds it (unless
            # a later access of the same step reused that slot)
            for a in acc:
                assert 0 <= a.slot < k
            for s, e in enumerate(sim.slot_expert[0]):
                if e >= 0:
                    assert [a.slot for a in acc if a.expert == e] in ([], [s])
        st = sim.stats[0]
        assert st.hits + st.misses == st.needed and st.prefetch_hits == 0


def test_lru_empty_slots_fill_in_index_order_before_any_eviction():
    sim = O.ExpertCacheSim(1, 8, 4, b=0)
    acc, _ = sim.step(0, [[5, 2]])
    assert [(a.expert, a.slot, a.victim) for a in acc] == [(2, 0, -1), (5, 1, -1)]
    acc, _ = sim.step(0, [[7, 5]])
    assert [(a.expert, a.status, a.slot, a.victim) for a in acc] == [(5, O.HIT, 1, -1), (7, O.MISS, 2, -1)]
    acc, _ = sim.step(0, [[0, 1]])
    assert [(a.expert, a.slot, a.victim) for a in acc] == [(0, 3, -1), (1, 0, 2)]
    assert sim.stats[0].evictions == 1


def test_lru_closed_form_k2_top2():
    """k = K = 2, batch 1: after every step the cache holds exactly that step's two experts, so an
    access hits iff the expert was selected at the previous token; hits = sum |S_t & S_{t-1}|."""
    rng = np.random.default_rng(1)
    E = 8
    sim = O.ExpertCacheSim(1, E, 2, b=0)
    prev, hits = set(), 0
    for _ in range(2000):
        S = set(int(e) for e in rng.choice(E, size=2, replace=False))
        acc, _ = sim.step(0, [sorted(S)])
        assert {a.expert for a in acc if a.status == O.HIT} == (S & prev)
        assert set(sim.contents(0)) == S
        hits += len(S & prev)
        prev = S
    st = sim.stats[0]
    assert st.hits == hits and st.needed == 4000
    # uniform i.i.d. routing: P(hit) = K/E = 0.25 (binomial std over 4000 draws ~ 0.007)
    assert abs(st.recall - 0.25) < 0.03


def test_cache_as_large_as_the_expert_set_only_misses_on_first_touch():
    rng = np.random.default_rng(2)
    sim = O.ExpertCacheSim(1, 8, 8, b=0)
    seen = set()
    for _ in range(200):
        S = [int(e) for e in rng.choice(8, size=2, replace=False)]
        acc, _ = sim.step(0, [S])
        for a in acc:
            assert (a.status == O.MISS) == (a.expert not in seen)
            seen.add(a.expert)
    assert sim.stats[0].misses == len(seen) == 8 and sim.stats[0].evictions == 0


def test_warm_start_holds_experts_zero_to_k_minus_one():
    sim = O.ExpertCacheSim(2, 8, 3, b=4, warm=True)
    assert sim.contents(0) == [0, 1, 2] and sim.contents(1) == [0, 1, 2]
    acc, _ = sim.step(0, [[1, 6]])
    assert [(a.expert, a.status, a.victim) for a in acc] == [(1, O.HIT, -1), (6, O.MISS, 0)]


# ------------------------------------------------------------------ speculative prefetch

def test_prefetch_guess_equals_selection_when_gates_coincide():
    rng = np.random.default_rng(3)
    E, H = 8, 64
    wg = rng.normal(size=(E, H)).astype(np.float32)
    for _ in range(100):
        h = rng.normal(size=H).astype(np.float16)
        idx, _, _ = O.route(wg, h, 2)
        assert O.prefetch_guess(O.prefetch_scores(wg, h), 2) == idx
    # batch: the score is the summed softmax mass, so a single token reduces to its own gate
    hb = rng.normal(size=(5, H)).astype(np.float16)
    s = O.prefetch_scores(wg, hb)
    assert np.allclose(s, sum(O.softmax(O.gate_logits(wg, hb[t])) for t in range(5)), atol=1e-14)
    assert abs(s.sum() - 5.0) < 1e-12


def test_prefetch_never_touches_the_cache_until_used():
    sim = O.ExpertCacheSim(3, 8, 2, b=4)
    sim.step(1, [[0, 1]])
    before = (list(sim.slot_expert[1]), list(sim.slot_stamp[1]))
    # guess {1 (resident: skipped), 5 (staged)} for layer 1 while running layer 0
    acc, dec = sim.step(0, [[2, 3]], guess=[1, 5])
    assert dec == [(1, False), (5, True)]
    assert (list(sim.slot_expert[1]), list(sim.slot_stamp[1])) == before
    assert sim.staged[1] == [5] and sim.stats[1].spec_issued == 1
    # layer 1 now needs 5 (a prefetch hit, which evicts the LRU entry 0) and 1 (a plain hit)
    acc, _ = sim.step(1, [[5, 1]])
    assert [(a.expert, a.status, a.victim) for a in acc] == [(1, O.HIT, -1), (5, O.PREFETCH_HIT, 0)]
    assert sim.staged[1] == [] and sim.stats[1].spec_wasted == 0 and sim.stats[1].prefetch_hits == 1


def test_unused_guesses_are_dropped_and_counted():
    sim = O.ExpertCacheSim(2, 8, 2, b=4)
    sim.step(0, [[0, 1]], guess=[6, 7])
    assert sim.staged[1] == [6, 7]
    acc, _ = sim.step(1, [[6, 2]])
    assert [(a.expert, a.status) for a in acc] == [(2, O.MISS), (6, O.PREFETCH_HIT)]
    assert sim.stats[1].spec_wasted == 1 and sim.staged_total() == 0
    # the last layer has no successor: its guess is ignored
    _, dec = sim.step(1, [[6, 2]], guess=[3, 4])
    assert dec == [] and sim.staged_total() == 0


def test_staging_buffers_are_a_shared_bounded_pool():
    sim = O.ExpertCacheSim(4, 8, 2, b=3)
    _, d0 = sim.step(0, [[0, 1]], guess=[4, 5])
    _, d2 = sim.step(2, [[0, 1]], guess=[6, 7])      # layer 1 has not run: its guesses still hold 2 buffers
    assert d0 == [(4, True), (5, True)] and d2 == [(6, True), (7, False)]
    assert sim.staged_total() == 3
    _, d0 = sim.step(0, [[0, 1]], guess=[4, 2])      # 4 already staged; pool full for 2
    assert d0 == [(4, False), (2, False)]


def test_prefetch_changes_labels_but_not_cache_contents_or_evictions():
    """Sec. 3.2: speculative loading does not change what the model computes; in cache terms the
    contents, slots, victims and order after every step are identical with and without it."""
    rng = np.random.default_rng(4)
    L, E, k = 4, 8, 2
    on = O.ExpertCacheSim(L, E, k, b=4)
    off = O.ExpertCacheSim(L, E, k, b=4)
    for _ in range(300):
        for l in range(L):
            sel = [[int(e) for e in rng.choice(E, size=2, replace=False)]]
            guess = [int(e) for e in rng.choice(E, size=2, replace=False)]
            a_on, _ = on.step(l, sel, guess)
            a_off, _ = off.step(l, sel, None)
            assert [(a.expert, a.slot, a.victim) for a in a_on] == [(a.expert, a.slot, a.victim) for a in a_off]
            assert [(a.status == O.HIT) for a in a_on] == [(a.status == O.HIT) for a in a_off]
            assert on.slot_expert[l] == off.slot_expert[l] and on.slot_stamp[l] == off.slot_stamp[l]
    for l in range(L):
        s_on, s_off = on.stats[l], off.stats[l]
        assert s_on.hits == s_off.hits and s_on.evictions == s_off.evictions
        assert s_on.misses + s_on.prefetch_hits == s_off.misses and s_off.prefetch_hits == 0
        assert s_on.spec_issued == s_on.prefetch_hits + s_on.spec_wasted + len(on.staged[l])
    assert sum(s.prefetch_hits for s in on.stats) > 0


def test_zero_experts_make_the_speculative_guess_exact():
    """If the experts output 0 the residual stream is unchanged, so the next layer's gate sees the
    same x; with equal norm gains its true selection equals the guess: speculative recall 1."""
    rng = np.random.default_rng(5)
    E, H, F, g = 8, 64, 64, 16
    zero_expert = [(np.zeros(s, np.uint8), np.ones((s[0], s[1] // g), np.float16), np.zeros((s[0], s[1] // g), np.float16))
                   for s in ((F, H), (F, H), (H, F))]
    gam = np.ones(H, np.float16)
    wg0 = rng.normal(size=(E, H)).astype(np.float32)
    wg1 = rng.normal(size=(E, H)).astype(np.float32)
    for _ in range(50):
        x = rng.normal(size=H).astype(np.float16)
        r0 = O.moe_block(x, wg0, [zero_expert] * E, g, 2, gam, 1e-5)
        assert (r0.x_out == x).all()
        guess = O.prefetch_guess(O.prefetch_scores(wg1, r0.h), 2)
        r1 = O.moe_block(r0.x_out, wg1, [zero_expert] * E, g, 2, gam, 1e-5)
        assert guess == r1.idx


def test_swap_placement_keeps_every_expert_in_exactly_one_buffer():
    """Sec. 3.3, hosts that cannot hold all experts: after any sequence of steps the experts on the device are
    exactly the cache contents, the E-k others occupy E-k distinct host buffers, the spare is the one remaining
    buffer, and there was one write-back per eviction (= per miss or used guess, the cache being full from the start).
    Brute force over random top-2 traces for several (E, k)."""
    rng = np.random.default_rng(11)
    for E, k, m in ((8, 2, 2), (8, 4, 1), (5, 3, 2), (3, 2, 0), (16, 4, 4)):
        sim = O.ExpertCacheSim(2, E, k, 4, warm=True)
        place = [O.SwapPlacement(E, k) for _ in range(2)]
        history = [[list(range(k))], [list(range(k))]]
        for t in range(200):
            for l in range(2):
                sel = [sorted(rng.choice(E, size=min(2, E), replace=False).tolist()) for _ in range(int(rng.integers(1, 3)))]
                guess = rng.permutation(E)[:m].tolist() if (l == 0 and m) else None
                acc, _ = sim.step(l, sel, guess)
                place[l].apply(acc)
                assert place[l].on_device() == sim.contents(l)
                host = [place[l].host_buf_of[e] for e in range(E) if place[l].host_buf_of[e] >= 0]
                assert len(host) == E - k and len(set(host)) == E - k
                assert sorted(host + [place[l].spare]) == list(range(E - k + 1))
        for l in range(2):
            assert place[l].writebacks == sim.stats[l].evictions == sim.stats[l].misses + sim.stats[l].prefetch_hits


def test_swap_placement_hand_worked_trace():
    """E=4, k=2: experts 0,1 on the device, 2 -> host buffer 0, 3 -> host buffer 1, spare = buffer 2.
    Need {2}: 0 (least recent) is evicted into the spare (2), buffer 0 becomes the spare.
    Need {3}: 1 is evicted into buffer 0, buffer 1 becomes the spare.  Need {0}: 2 leaves into buffer 1, spare = 2."""
    sim = O.ExpertCacheSim(1, 4, 2, 4, warm=True)
    p = O.SwapPlacement(4, 2)
    assert (p.host_buf_of, p.spare) == ([-1, -1, 0, 1], 2)
    p.apply(sim.step(0, [[2]])[0])
    assert (p.host_buf_of, p.spare) == ([2, -1, -1, 1], 0)
    p.apply(sim.step(0, [[3]])[0])
    assert (p.host_buf_of, p.spare) == ([2, 0, -1, -1], 1)
    p.apply(sim.step(0, [[0]])[0])
    assert (p.host_buf_of, p.spare) == ([-1, 0, 1, -1], 2)
    p.apply(sim.step(0, [[0, 3]])[0])          # both resident: nothing moves
    assert (p.host_buf_of, p.spare, p.writebacks) == ([-1, 0, 1, -1], 2, 3)


# ------------------------------------------------------------------ speculative recall in isolation (Sec. 4.1)

def test_speculative_recall_hand_worked_example():
    """Three experts, width 2, three layers, two tokens, top-2; every logit worked out by hand (ties go to the
    lower expert).  Guessing layer l+1 from layer l's input: the four guesses are, most likely first,
    (2,1,0) (0,1,2) (0,2,1) (0,2,1) against the needed sets {1,2} {0,2} {0,2} {0,1}; two layers ahead:
    (0,1,2) (2,1,0) against {0,2} {0,1}.  A routine that took the wrong layer's gate, the wrong layer's input
    or the wrong layer's selection gives other counts."""
    gates = [np.array(g, np.float32) for g in ([[1, 0], [0, 1], [-1, -1]], [[0, 1], [1, 0], [1, 1]], [[2, 0], [0, -1], [-1, 1]])]
    h = np.array([[[1, 0.5], [0.5, -1], [-1, 2]], [[-2, 1], [1, 1], [0.5, 0.25]]], np.float16)
    routing = [[O.route(gates[l], h[t][l], 2)[0] for l in range(3)] for t in range(2)]
    assert routing == [[[0, 1], [1, 2], [2, 0]], [[1, 2], [2, 0], [0, 1]]]
    assert O.speculative_recall(routing, h, gates, 1, 1) == (4, 8)
    assert O.speculative_recall(routing, h, gates, 1, 2) == (6, 8)
    assert O.speculative_recall(routing, h, gates, 1, 3) == (8, 8)
    assert O.speculative_recall(routing, h, gates, 2, 1) == (1, 4)
    assert O.speculative_recall(routing, h, gates, 2, 2) == (2, 4)
    assert O.speculative_recall(routing, h, gates, 3, 2) == (0, 0)       # no layer that far ahead


def test_speculative_recall_closed_forms():
    """(i) zero layers ahead a layer is guessed from its own input: min(m, K) of its K experts are found;
    (ii) guessing all E experts recalls everything at any distance; (iii) experts that output zero leave the
    residual stream unchanged, so with one gate matrix shared by all layers (and no norm) every layer selects the
    same experts and guessing K of them any number of layers ahead recalls everything."""
    rng = np.random.default_rng(17)
    T, L, E, H, K = 9, 5, 8, 32, 2
    gates = [rng.normal(size=(E, H)).astype(np.float32) for _ in range(L)]
    h = rng.normal(size=(T, L, H)).astype(np.float16)
    routing = [[O.route(gates[l], h[t][l], K)[0] for l in range(L)] for t in range(T)]
    for m in (1, 2, 3):
        assert O.speculative_recall(routing, h, gates, 0, m) == (min(m, K) * T * L, K * T * L)
    for a in (1, 2, 4):
        assert O.speculative_recall(routing, h, gates, a, E) == (K * T * (L - a), K * T * (L - a))
        got, need = O.speculative_recall(routing, h, gates, a, 2)
        assert need == K * T * (L - a) and 0 <= got < need          # unrelated random gates: far from perfect
        assert O.speculative_recall(routing, h, gates, a, 1)[0] <= got <= O.speculative_recall(routing, h, gates, a, 4)[0]
    shared = [gates[0]] * L
    x = rng.normal(size=(T, H)).astype(np.float16)
    h_same = np.repeat(x[:, None, :], L, axis=1)                      # x_{l+1} = x_l + 0
    routing_same = [[O.route(shared[l], h_same[t][l], K)[0] for l in range(L)] for t in range(T)]
    for a in (1, 2, 4):
        assert O.speculative_recall(routing_same, h_same, shared, a, K) == (K * T * (L - a), K * T * (L - a))
