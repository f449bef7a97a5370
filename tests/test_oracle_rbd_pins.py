"""Pins for the oracle's stage 0 of the Redundancy-Bypassing Dispatch (Section 4.2): a worked example done by hand,
the invariants the section states, the limits (one node, one expert per node), reconstruction of the plain
dispatch, and the closed-form expected redundancy under uniform routing.  No GPU is used."""
import numpy as np
import pytest

import oracle
import xmoe_inputs as xi


def _route(T, E, k, seed, std=1.0):
    logits = xi.make_logits(T, E, seed=seed, std=std)
    idx, w, _ = oracle.route(logits, k)
    return idx, w, oracle.build_eri(idx, w, E)


def test_worked_example_by_hand():
    """T=3, k=3, E=4, two experts per node (node 0 = experts 0,1; node 1 = experts 2,3).
    token 0 -> experts (0,1,2) keys (5,3,9): node 0 group {e0,e1}: pilot e1 (key 3); node 1 group {e2}: pilot e2
    token 1 -> experts (3,2,0) keys (7,7,1): node 1 group {e3,e2}: equal keys, lower flat entry wins: e3; node 0: e0
    token 2 -> experts (1,3,2) keys (4,8,2): node 0 {e1}: pilot; node 1 {e3,e2}: pilot e2 (key 2)
    PFT rows (sorted by expert, token ascending): e0:[t0,t1] e1:[t0,t2] e2:[t0,t1,t2] e3:[t1,t2] -> rows 0..8;
    the expected arrays below were worked out by hand from these."""
    topk = np.array([[0, 1, 2], [3, 2, 0], [1, 3, 2]], dtype=np.int32)
    keys = np.array([5, 3, 9, 7, 7, 1, 4, 8, 2], dtype=np.uint32)
    eri = oracle.build_eri(topk, np.ones((3, 3)), 4)
    assert eri["token_ids"].tolist() == [0, 1, 0, 2, 0, 1, 2, 1, 2]
    assert eri["expert_ids"].tolist() == [0, 0, 1, 1, 2, 2, 2, 3, 3]
    s0 = oracle.rbd_stage0(topk, keys, eri, 4, 2)
    # row: 0=(t0,e0) replica of (t0,e1)=row2; 1=(t1,e0) pilot; 2=(t0,e1) pilot; 3=(t2,e1) pilot; 4=(t0,e2) pilot;
    #      5=(t1,e2) replica of (t1,e3)=row7; 6=(t2,e2) pilot; 7=(t1,e3) pilot; 8=(t2,e3) replica of (t2,e2)=row6
    assert s0["is_pilot"].tolist() == [False, True, True, True, True, False, True, True, False]
    assert s0["pilot"]["token_ids"].tolist() == [1, 0, 2, 0, 2, 1]
    assert s0["pilot"]["expert_ids"].tolist() == [0, 1, 1, 2, 2, 3]
    assert s0["pilot"]["tokens_per_expert"].tolist() == [1, 2, 2, 1]
    assert s0["pilot"]["expert_offsets"].tolist() == [0, 1, 3, 5, 6]
    assert s0["replica"]["token_ids"].tolist() == [0, 1, 2]
    assert s0["replica"]["expert_ids"].tolist() == [0, 2, 3]
    assert s0["replica"]["tokens_per_expert"].tolist() == [1, 0, 1, 1]
    # replica (t0,e0): pilot (t0,e1) is the first pilot of expert 1 -> (expert 1, relative 0)
    # replica (t1,e2): pilot (t1,e3) is the first pilot of expert 3 -> (expert 3, relative 0)
    # replica (t2,e3): pilot (t2,e2) is the second pilot of expert 2 -> (expert 2, relative 1)
    assert s0["s1_mapping_experts"].tolist() == [1, 3, 2]
    assert s0["s1_mapping_indices"].tolist() == [0, 0, 1]
    assert oracle.rbd_absolute_index(s0["s1_mapping_indices"], s0["s1_mapping_experts"],
                                     s0["pilot"]["expert_offsets"]).tolist() == [1, 5, 4]
    assert s0["merge_src"].tolist() == [6, 0, 1, 2, 3, 7, 4, 5, 8]


@pytest.mark.parametrize("T,E,k,epn,seed", [(64, 8, 3, 2, 0), (200, 64, 6, 8, 1), (128, 256, 8, 8, 2), (50, 6, 6, 3, 3),
                                            (97, 12, 5, 4, 4)])
def test_invariants(T, E, k, epn, seed):
    idx, w, eri = _route(T, E, k, seed)
    keys = xi.make_rbd_keys(T * k, seed)
    s0 = oracle.rbd_stage0(idx, keys, eri, E, epn)
    B = T * k
    tok, ex = eri["token_ids"], eri["expert_ids"]
    pil = s0["is_pilot"]
    # exactly one pilot per (token, destination node) that the token visits
    pairs = set(zip(tok.tolist(), (ex // epn).tolist()))
    ppairs = list(zip(tok[pil].tolist(), (ex[pil] // epn).tolist()))
    assert len(ppairs) == len(set(ppairs)) == len(pairs) and set(ppairs) == pairs
    # the two sets of ERI-arrays partition the PFT, keep its order and are sorted by expert
    for part, rows in (("pilot", np.flatnonzero(pil)), ("replica", np.flatnonzero(~pil))):
        assert np.array_equal(s0[part]["token_ids"], tok[rows]) and np.array_equal(s0[part]["expert_ids"], ex[rows])
        assert (np.diff(s0[part]["expert_ids"]) >= 0).all()
        assert np.array_equal(s0[part]["tokens_per_expert"], np.bincount(ex[rows], minlength=E))
    assert s0["pilot"]["expert_offsets"][-1] + s0["replica"]["expert_offsets"][-1] == B
    assert np.array_equal(s0["pilot"]["tokens_per_expert"] + s0["replica"]["tokens_per_expert"],
                          eri["tokens_per_expert"])
    # every replica points at a pilot of the same token on the same node, and that pilot won the draw
    absolute = oracle.rbd_absolute_index(s0["s1_mapping_indices"], s0["s1_mapping_experts"],
                                         s0["pilot"]["expert_offsets"])
    assert np.array_equal(s0["pilot"]["token_ids"][absolute], s0["replica"]["token_ids"])
    assert np.array_equal(s0["pilot"]["expert_ids"][absolute] // epn, s0["replica"]["expert_ids"] // epn)
    assert np.array_equal(s0["pilot"]["expert_ids"][absolute], s0["s1_mapping_experts"])
    flat_of_row = np.empty(B, dtype=np.int64)
    flat_of_row[eri["row_of_slot"]] = np.arange(B)
    prow, rrow = np.flatnonzero(pil), np.flatnonzero(~pil)
    kp, kr = flat_of_row[prow][absolute], flat_of_row[rrow]
    assert all((int(keys[a]), a) < (int(keys[b]), b) for a, b in zip(kp.tolist(), kr.tolist()))
    # relative indices stay inside the pilot's segment
    assert (s0["s1_mapping_indices"] >= 0).all()
    assert (s0["s1_mapping_indices"] < s0["pilot"]["tokens_per_expert"][s0["s1_mapping_experts"]]).all()
    # merge_src is a permutation of 0..B-1
    assert np.array_equal(np.sort(s0["merge_src"]), np.arange(B))


@pytest.mark.parametrize("epn", [1, 2, 4, 8])
def test_reconstruction_equals_plain_dispatch(epn):
    T, E, k = 150, 8, 4
    idx, w, eri = _route(T, E, k, 7)
    x = np.random.default_rng(0).standard_normal((T, 16))
    s0 = oracle.rbd_stage0(idx, xi.make_rbd_keys(T * k, 5), eri, E, epn)
    assert np.array_equal(oracle.rbd_reconstruct(x, s0), oracle.dispatch(x, eri["token_ids"]))


def test_limits_one_node_and_one_expert_per_node():
    T, E, k = 90, 16, 5
    idx, w, eri = _route(T, E, k, 8)
    keys = xi.make_rbd_keys(T * k, 1)
    one_node = oracle.rbd_stage0(idx, keys, eri, E, E)          # everything on one node: one pilot per token
    assert one_node["is_pilot"].sum() == T and len(one_node["replica"]["token_ids"]) == T * (k - 1)
    assert sorted(one_node["pilot"]["token_ids"].tolist()) == list(range(T))
    alone = oracle.rbd_stage0(idx, keys, eri, E, 1)             # one expert per node: a token's experts are distinct
    assert alone["is_pilot"].all() and len(alone["s1_mapping_indices"]) == 0
    assert np.array_equal(alone["pilot"]["token_ids"], eri["token_ids"])


def test_equal_keys_fall_back_to_the_lower_flat_entry():
    T, E, k = 40, 8, 4
    idx, w, eri = _route(T, E, k, 9)
    s0 = oracle.rbd_stage0(idx, np.zeros(T * k, dtype=np.uint32), eri, E, 4)
    flat_of_row = np.empty(T * k, dtype=np.int64)
    flat_of_row[eri["row_of_slot"]] = np.arange(T * k)
    for t in range(T):
        for node in range(2):
            members = [t * k + j for j in range(k) if idx[t, j] // 4 == node]
            if members:
                prow = [r for r in np.flatnonzero(s0["is_pilot"]) if flat_of_row[r] in members]
                assert len(prow) == 1 and flat_of_row[prow[0]] == min(members)


def test_redundancy_matches_hypergeometric_expectation():
    """Uniform routing: the measured share of replicas agrees with 1 - E[distinct nodes]/k (here E=256, k=8 and 8
    experts per node, the Large model on 32 nodes of 8 devices with one expert each)."""
    T, E, k, epn = 4000, 256, 8, 8
    rng = np.random.default_rng(3)
    idx = np.stack([rng.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32)
    eri = oracle.build_eri(idx, np.ones((T, k)), E)
    s0 = oracle.rbd_stage0(idx, xi.make_rbd_keys(T * k, 2), eri, E, epn)
    measured = len(s0["replica"]["token_ids"]) / (T * k)
    want = oracle.rbd_expected_redundancy(E, k, epn)
    assert abs(measured - want) < 0.01, (measured, want)
    # brute force of the same expectation on a case small enough to enumerate: E=6, k=3, 2 experts per node
    import itertools
    tot = 0
    combos = list(itertools.combinations(range(6), 3))
    for c in combos:
        tot += 3 - len({e // 2 for e in c})
    assert abs(tot / (3 * len(combos)) - oracle.rbd_expected_redundancy(6, 3, 2)) < 1e-12


def test_random_pilots_spread_over_a_nodes_experts():
    """The section's reason for a random choice: always taking the smallest expert id of a node piles the pilots on
    that expert.  With random keys the pilots of a node spread over its experts."""
    T, E, k, epn = 3000, 16, 6, 8
    idx, w, eri = _route(T, E, k, 11)
    rnd = oracle.rbd_stage0(idx, xi.make_rbd_keys(T * k, 3), eri, E, epn)["pilot"]["tokens_per_expert"]
    # keys that order entries by expert id reproduce the biased rule
    biased = oracle.rbd_stage0(idx, idx.reshape(-1).astype(np.uint32), eri, E, epn)["pilot"]["tokens_per_expert"]
    for node in range(E // epn):
        seg = slice(node * epn, (node + 1) * epn)
        assert rnd[seg].max() < 1.6 * rnd[seg].mean()
        assert biased[seg].max() > 2.0 * biased[seg].mean()
