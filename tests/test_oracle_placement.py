"""Pins for the placement oracle (Section 5.3: Eq. 5, 6, 7 and Algorithm 1): hand-computed values, closed forms,
brute force over explicit post-move states, and invariants on seeded clusters.  CPU only."""
import itertools

import pytest

from oracle import placement as P
from paper_2401_02669_amd import synth


def model(t_natn, n=10, T=100, g=1.0e6):
    return P.Model(n, T, g, t_natn)


# ---- hand-computed values (Eq. 5, Eq. 6, TPS, Eq. 7) ---------------------------------------------------
def test_layer_time_hand_value():
    m = model([0.0, 0.001, 0.002])
    # Eq. 5: 0.002 + (1000 + 3000) / 1e6 = 0.006
    assert P.layer_time(m, 2, 4000) == pytest.approx(0.006, rel=1e-15)


def test_instance_tps_hand_value():
    m = model([0.0, 0.001, 0.002])
    i = P.Instance([1000, 3000], capacity_blocks=100)
    # TPS = beta / (n T) = 2 / (10 * 0.006)
    assert P.instance_tps(m, i) == pytest.approx(33.0 + 1.0 / 3.0, rel=1e-14)
    assert P.instance_tps(m, P.Instance([], capacity_blocks=100)) == 0.0


def test_debtor_and_creditor_time_shift_hand_values():
    m = model([0.0, 0.001, 0.002])
    d = P.Instance([1000, 3000], capacity_blocks=40)     # 10 + 30 blocks: full
    c = P.Instance([500], capacity_blocks=100)
    # 5 blocks = 500 tokens leave: T_dbt = 0.006 - 500/1e6 = 0.0055; T_cdt = 0.001 + 500/1e6 + 500/1e6 = 0.002
    assert P.debtor_tps(m, d, 5) == pytest.approx(2 / (10 * 0.0055), rel=1e-14)
    assert P.creditor_tps(m, c, 5) == pytest.approx(1 / (10 * 0.002), rel=1e-14)
    assert P.pair_estimate(m, d, c, 5) == pytest.approx(2 / 0.055 + 1 / 0.02, rel=1e-14)
    # k = 0 is the state as it stands
    assert P.debtor_tps(m, d, 0) == P.instance_tps(m, d)
    assert P.creditor_tps(m, c, 0) == P.instance_tps(m, c)


def test_admission_raises_batch_hand_value():
    m = model([0.0, 0.001, 0.002, 0.003, 0.004])
    d = P.Instance([4000], capacity_blocks=40, waiting=5, admit_blocks=3)   # 40 blocks: full
    assert P.admit_count(m, d, 0) == 0
    assert P.admit_count(m, d, 2) == 0
    assert P.admit_count(m, d, 3) == 1
    assert P.admit_count(m, d, 7) == 2
    assert P.admit_count(m, d, 39) == 3          # table ends at batch 4: beta' <= 4
    # 7 blocks leave, two requests of 3 blocks (300 tokens) join: beta' = 3,
    # T = t[3] + (4000 + 600 - 700) / 1e6 = 0.003 + 0.0039 = 0.0069
    assert P.debtor_tps(m, d, 7) == pytest.approx(3 / (10 * 0.0069), rel=1e-14)
    d.waiting = 1
    assert P.admit_count(m, d, 39) == 1


def test_cluster_tps_is_the_sum():
    m = model([0.0, 0.001, 0.002])
    a, b = P.Instance([1000, 3000], 100), P.Instance([500], 100, hosted_blocks=5)
    assert P.cluster_tps(m, [a, b]) == pytest.approx(2 / 0.06 + 1 / (10 * 0.002), rel=1e-14)


def test_existing_remote_blocks_shorten_the_debtor():
    m = model([0.0, 0.001])
    d = P.Instance([5000], capacity_blocks=30, req_remote_blocks=[20])
    assert P.used_blocks(m, d) == 30
    # K^d = 2000 tokens: T = 0.001 + 5000/1e6 - 2000/1e6 = 0.004
    assert P.instance_tps(m, d) == pytest.approx(1 / (10 * 0.004), rel=1e-14)


def test_estimates_at_zero_blocks_are_the_present_state_whatever_the_role():
    m = model([0.0, 0.001, 0.002])
    i = P.Instance([1000, 3000], capacity_blocks=100, req_remote_blocks=[0, 10], hosted_blocks=7)
    # T = 0.002 + 4000/1e6 - 1000/1e6 + 700/1e6 = 0.0057
    assert P.instance_tps(m, i) == pytest.approx(2 / (10 * 0.0057), rel=1e-14)
    assert P.debtor_tps(m, i, 0) == P.instance_tps(m, i)
    assert P.creditor_tps(m, i, 0) == P.instance_tps(m, i)


def test_a_remote_last_block_counts_its_tokens_only():
    m = model([0.0, 0.001])
    d = P.Instance([250], capacity_blocks=30, req_remote_blocks=[3])     # 3 blocks of 100: the last holds 50
    assert P.remote_tokens(m, d) == 250
    assert P.instance_tps(m, d) == pytest.approx(1 / (10 * 0.001), rel=1e-14)


# ---- closed forms for the greedy choice --------------------------------------------------------------
def test_idle_creditor_takes_all_but_the_last_block():
    # with beta_c = 0 the creditor loses nothing and the debtor's time falls with every block: best k = Block_max - 1
    m = model([0.0, 0.001, 0.002])
    d = P.Instance([4000], capacity_blocks=40)
    c = P.Instance([], capacity_blocks=100)
    moves, after = P.schedule(m, [d, c], beta_thres=4, u_thres=0.5)
    assert moves == [(0, 0, 1, 39)]
    assert after[0].req_remote_blocks == [39] and after[1].hosted_blocks == 39


def test_idle_creditor_bounded_by_its_free_blocks_then_next_creditor():
    m = model([0.0, 0.001, 0.002])
    d = P.Instance([4000], capacity_blocks=40)
    c1 = P.Instance([], capacity_blocks=10)
    c2 = P.Instance([], capacity_blocks=12)
    moves, after = P.schedule(m, [d, c1, c2], beta_thres=4, u_thres=0.5)
    # both idle (utilisation 0): lower index first; 10 blocks fill c1, then c2 takes its 12
    assert moves == [(0, 0, 1, 10), (0, 0, 2, 12)]
    assert after[0].req_remote_blocks == [22]


def test_symmetric_pair_convexity():
    # identical debtor and creditor, constant non-attention time: 1/(a-x) + 1/(a+x) grows with x, so the
    # greedy choice is the largest k allowed
    m = model([0.0, 0.002, 0.002])
    d = P.Instance([4000], capacity_blocks=40)
    c = P.Instance([4000], capacity_blocks=100)
    moves, _ = P.schedule(m, [d, c], beta_thres=1, u_thres=0.5)
    assert moves == [(0, 0, 1, 39)]


def test_hosted_blocks_count_as_used():
    m = model([0.0, 0.001, 0.002])
    d = P.Instance([4000], capacity_blocks=40)
    c = P.Instance([], capacity_blocks=10, hosted_blocks=4)
    assert P.used_blocks(m, c) == 4 and P.utilisation(m, c) == pytest.approx(0.4)
    moves, after = P.schedule(m, [d, c], beta_thres=4, u_thres=0.5)
    assert moves == [(0, 0, 1, 6)]
    assert P.used_blocks(m, after[1]) == 10


def test_creditors_in_ascending_utilisation_and_resorted():
    m = model([0.0, 0.001, 0.002])
    d = P.Instance([4000], capacity_blocks=40)
    c1 = P.Instance([], capacity_blocks=20, hosted_blocks=8)    # 0.40
    c2 = P.Instance([], capacity_blocks=20, hosted_blocks=2)    # 0.10
    c3 = P.Instance([], capacity_blocks=20, hosted_blocks=4)    # 0.20
    moves, _ = P.schedule(m, [d, c1, c2, c3], beta_thres=4, u_thres=0.5)
    assert moves == [(0, 0, 2, 18), (0, 0, 3, 16), (0, 0, 1, 5)]


def test_equal_estimates_keep_the_blocks_at_home():
    # with an infinitely fast attention rate every k gives the same estimate: the smallest k (0) wins, no move
    m = P.Model(10, 100, float("inf"), [0.0, 0.001, 0.002])
    d = P.Instance([4000], capacity_blocks=40)
    c = P.Instance([100], capacity_blocks=100)
    assert P.schedule(m, [d, c], beta_thres=4, u_thres=0.5)[0] == []


def test_queue_drains_as_requests_are_admitted():
    m = model([0.0] + [0.001] * 8)
    d = P.Instance([4000], capacity_blocks=40, waiting=2, admit_blocks=5)
    c1 = P.Instance([], capacity_blocks=7)
    c2 = P.Instance([], capacity_blocks=30)
    moves, after = P.schedule(m, [d, c1, c2], beta_thres=4, u_thres=0.5)
    # 7 blocks to c1 admit one request (5 blocks); all but the last of the remaining 33 go to c2: the freed
    # space admits the second and last waiting request, no third although there is room for more
    assert moves == [(0, 0, 1, 7), (0, 0, 2, 30)]
    assert after[0].admitted == 2 and after[0].waiting == 0
    assert P.batch(after[0]) == 3
    assert P.used_blocks(m, after[0]) == 40 - 37 + 10


def first_step_gain_closed_form(beta_d, t_d, beta_c, t_c, x):
    # TPS_d(1) - TPS_d(0) + TPS_c(1) - TPS_c(0) with x = block_tokens / g, up to the common factor 1/n
    return beta_d * x / (t_d * (t_d - x)) - beta_c * x / (t_c * (t_c + x))


@pytest.mark.parametrize("t_two,expect_move", [(0.5, True), (0.0005, False)])
def test_no_gain_means_no_move(t_two, expect_move):
    # a debtor dominated by non-attention time gains little per block; a creditor with a short layer time loses
    # more than that, one with a long layer time loses less
    t = [0.0, 0.05, t_two]
    m = P.Model(10, 100, 1.0e6, t)
    d = P.Instance([4000], capacity_blocks=40)
    c = P.Instance([100, 100], capacity_blocks=1000)
    t_d = 0.05 + 4000 / 1e6
    t_c = t_two + 200 / 1e6
    gain = first_step_gain_closed_form(1, t_d, 2, t_c, 100 / 1e6)
    assert (gain > 0) == expect_move
    moves, _ = P.schedule(m, [d, c], beta_thres=1, u_thres=0.5)
    if expect_move:
        assert moves == [(0, 0, 1, 39)]     # the pair's sum is convex in k: once it rises it keeps rising
    else:
        assert moves == []


# ---- brute force over explicit post-move states -----------------------------------------------------------
def tps_from_state(n, T, g, t_natn, req_tokens, remote_blocks_total, hosted):
    beta = len(req_tokens)
    if beta == 0:
        return 0.0
    return beta / (n * (t_natn[beta] + (sum(req_tokens) - T * remote_blocks_total + T * hosted) / g))


def brute_force_best_k(n, T, g, t_natn, d, c, block_max):
    """Builds the two instances' states after moving k blocks, admitted requests written out as real requests."""
    best = (None, -1)
    d_used = sum(-(-s // T) for s in d["req_tokens"]) - sum(d["req_remote_blocks"]) + d["hosted_blocks"]
    c_used = sum(-(-s // T) for s in c["req_tokens"]) - sum(c["req_remote_blocks"]) + c["hosted_blocks"]
    for k in range(block_max):
        if k > c["capacity_blocks"] - c_used:
            break
        free = d["capacity_blocks"] - d_used + k
        admitted = 0
        while (d["admit_blocks"] > 0 and admitted < d["waiting"] and (admitted + 1) * d["admit_blocks"] <= free
               and len(d["req_tokens"]) + admitted + 1 <= len(t_natn) - 1):
            admitted += 1
        reqs = list(d["req_tokens"]) + [d["admit_blocks"] * T] * admitted
        total = tps_from_state(n, T, g, t_natn, reqs, sum(d["req_remote_blocks"]) + k, d["hosted_blocks"]) \
            + tps_from_state(n, T, g, t_natn, c["req_tokens"], sum(c["req_remote_blocks"]), c["hosted_blocks"] + k)
        if best[0] is None or total > best[0] * (1 + 1e-13):
            best = (total, k)
    return best[1]


@pytest.mark.parametrize("seed", range(12))
def test_pair_choice_equals_brute_force(seed):
    import numpy as np
    rng = np.random.default_rng(1000 + seed)
    T, n, g = 64, 8, 2.0e6
    t_natn = [0.0] + [2e-4 + 3e-5 * b ** 0.7 for b in range(1, 40)]
    d = dict(req_tokens=[int(rng.integers(3000, 9000))] + [int(x) for x in rng.integers(10, 500, size=int(rng.integers(0, 3)))],
             req_remote_blocks=None, hosted_blocks=0, capacity_blocks=0, waiting=int(rng.integers(0, 30)),
             admit_blocks=int(rng.integers(1, 6)))
    d["req_remote_blocks"] = [int(rng.integers(0, 10))] + [0] * (len(d["req_tokens"]) - 1)
    d["capacity_blocks"] = sum(-(-s // T) for s in d["req_tokens"]) - d["req_remote_blocks"][0] + int(rng.integers(0, 3))
    c = dict(req_tokens=[int(x) for x in rng.integers(50, 800, size=int(rng.integers(0, 30)))], req_remote_blocks=[],
             hosted_blocks=int(rng.integers(0, 20)), capacity_blocks=int(rng.integers(300, 600)), waiting=0, admit_blocks=0)
    c["req_remote_blocks"] = [0] * len(c["req_tokens"])
    m = P.Model(n, T, g, t_natn)
    moves, after = P.schedule(m, [P.Instance(**d), P.Instance(**c)], beta_thres=5, u_thres=0.9)
    block_max = -(-d["req_tokens"][0] // T) - d["req_remote_blocks"][0]
    want = brute_force_best_k(n, T, g, t_natn, d, c, block_max)
    got = moves[0][3] if moves else 0
    assert got == want
    if moves:
        # the state after the move, evaluated through Eq. 5 on written-out requests, is what the estimate promised
        D, C = after
        reqs = list(D.req_tokens) + [D.admit_blocks * T] * D.admitted
        total = tps_from_state(n, T, g, t_natn, reqs, sum(D.req_remote_blocks), 0) \
            + tps_from_state(n, T, g, t_natn, C.req_tokens, 0, C.hosted_blocks)
        assert P.cluster_tps(m, after) == pytest.approx(total, rel=1e-12)


# ---- Algorithm 1: order and invariants on seeded clusters ----------------------------------------------
def as_oracle(cluster):
    md, ins = cluster
    return P.Model(md["num_layers"], md["block_tokens"], md["attn_tokens_per_s"], md["t_natn"]), [P.Instance(**d) for d in ins]


@pytest.mark.parametrize("seed", range(8))
def test_schedule_invariants(seed):
    m, ins = as_oracle(synth.make_cluster(seed))
    beta_thres, u_thres = 8, 0.6
    before = P.cluster_tps(m, ins)
    moves, after = P.schedule(m, ins, beta_thres, u_thres)
    assert moves, "the seeded clusters always hold a long-request instance and a lender"
    debtors_seen = []
    for d, r, c, k in moves:
        assert k >= 1
        assert d != c
        # roles (Section 5.2: never both)
        assert P.batch(ins[d]) <= beta_thres and P.utilisation(m, ins[d]) > u_thres
        assert P.utilisation(m, ins[c]) <= u_thres and P.remote_blocks(ins[c]) == 0
        # the longest request of the debtor
        assert ins[d].req_tokens[r] == max(ins[d].req_tokens)
        if not debtors_seen or debtors_seen[-1] != d:
            debtors_seen.append(d)
    # each debtor once, in ascending batch-size order; a creditor at most once per debtor
    assert len(set(debtors_seen)) == len(debtors_seen)
    sizes = [P.batch(ins[d]) for d in debtors_seen]
    assert sizes == sorted(sizes)
    for d in debtors_seen:
        cs = [c for dd, _, c, _ in moves if dd == d]
        assert len(set(cs)) == len(cs)
    # blocks are conserved, capacities hold, the last block of a request stays at home
    moved_out = sum(P.remote_blocks(a) - P.remote_blocks(b) for a, b in zip(after, ins))
    moved_in = sum(a.hosted_blocks - b.hosted_blocks for a, b in zip(after, ins))
    assert moved_out == moved_in == sum(k for *_, k in moves)
    for a in after:
        assert 0 <= P.used_blocks(m, a) <= a.capacity_blocks
        for s, rb in zip(a.req_tokens, a.req_remote_blocks):
            assert rb <= P.blocks_of(m, s) - 1 or rb == 0 or s == 0 or rb <= P.blocks_of(m, s)
        assert a.waiting >= 0
    for (d, r, c, k) in moves:
        assert after[d].req_remote_blocks[r] <= P.blocks_of(m, after[d].req_tokens[r]) - 1
    # every move was chosen because the pair's estimate rose, and nobody else changed: the cluster gains
    assert P.cluster_tps(m, after) > before


def test_thresholds_select_nobody():
    m, ins = as_oracle(synth.make_cluster(3))
    assert P.schedule(m, ins, beta_thres=-1, u_thres=0.6)[0] == []
    assert P.schedule(m, ins, beta_thres=8, u_thres=-1.0)[0] == []


def test_search_space_formula_small_case():
    # Section 5.2, search-space size: distributing Y_i identical blocks of creditor i over N debtors or nobody
    # is bounded by (N+1)^sum(Y) / prod(Y_i!); check the count of distinct placements against brute force for
    # one creditor: multisets of size Y over N+1 choices never exceed the bound's numerator and the quotient
    # is a lower bound on them.
    import math
    N, Y = 3, 4
    distinct = len(set(tuple(sorted(x)) for x in itertools.product(range(N + 1), repeat=Y)))
    assert (N + 1) ** Y / math.factorial(Y) <= distinct <= (N + 1) ** Y
