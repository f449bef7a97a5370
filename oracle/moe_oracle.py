"""CPU oracle for the padding-free MoE layer (X-MoE, arXiv 2508.13337).

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may
import this package.  It shares no code with the HIP library and never calls it.

Everything is written the slow, obvious way in float64 numpy, one step after the other in the order of the
paper's Listing 1 ("Padding-free MoE-layer": gating -> PFT_construction -> dispatch -> mlp -> combine) with the
notation of Section 4.1.1 (token_ids, expert_ids, tokens_per_expert, combine_weights = the ERI-arrays of a PFT).
numpy's matmul and stable argsort serve as library primitives; nothing is blocked, fused or reordered.

Readings of the paper that this oracle fixes (the paper is silent or garbled on each):
  * top_experts / combine_weights are [T, k] (Appendix B.3), not [S, E] as the listing's docstring says.
  * combine weights are the raw softmax-over-E probabilities of the selected experts, not renormalised.
  * top-k is taken on the logits (softmax is monotone), ties go to the lower expert index, slot j holds the
    j-th largest.
  * the sort of the flattened expert ids is stable, so rows of one expert stay in ascending token order.
  * token_ids holds the token index n // k of flat entry n (Section 4.1.1's "ti-th input token").
  * the hot path is dropless (max_token_count >= T): B = T*k and the ERI-arrays are a permutation.
  * the scatter of Section 4.1.2 / Appendix B.4 accumulates: out[token_ids[i]] += combine_weights[i]*Y[i].
  * expert i's segment is rows [sum(tpe[:i]), sum(tpe[:i+1])) (Appendix B.4 prints an off-by-one).
  * the expert is a SwiGLU FFN, Y = (silu(X Wg) * (X Wu)) Wd, no biases (the benchmark definition binds this;
    the paper's own expert is a two-matrix MLP).
  * a shared expert is one more SwiGLU expert applied to every token with weight 1, outside the gate.
  * the gate projection is evaluated in float32 in a fixed order (oracle/gate_order.c) so that routing is
    reproducible bit for bit; an all-float64 mode exists for finite-difference checks.
  * backward is not described in the paper beyond mirroring the forward; it is derived here by calculus with
    the top-k indices held constant.
  * the paper's own expert (Listing 1 mlp(): two sequential GeMMs w1, w2; Table 1 counts 2 h' h parameters per
    expert; Table 3's totals need two matrices per expert) is also provided: Y = act(X W1) W2.  The listing
    prints no activation between the two GeMMs while Section 3.2 (Table 2) speaks of two intermediate activations between
    the FFN sub-layers; act is therefore a parameter: "identity" (the listing as printed), "gelu" (x Phi(x), the
    exact erf form: the default of the Megatron-style MLP that the paper's framework trains) or "silu".
  * Redundancy-Bypassing Dispatch, stage 0 (Section 4.2): experts are laid out over nodes in contiguous blocks
    (node of expert e = e // experts_per_node); all tokens of this PFT share one source, so a group is the set of a
    token's flat entries whose experts live on one destination node; the random choice of the group's pilot is
    the entry with the smallest (rand_key[n], n), the keys being an input; pilot and replica ERI-arrays keep the
    PFT's order (sorted by expert, stable); a replica's s1_mapping_indices entry is its pilot's position inside
    the pilot segment of the pilot's expert ("relative index starting from 0 for each target expert"), and the
    pilot's expert is recorded beside it so that the index can be made absolute against any offsets table.
"""
from __future__ import annotations

import ctypes
from typing import Optional

import numpy as np

from . import build as _build

_gate_lib = None


def _load_gate_lib():
    global _gate_lib
    if _gate_lib is None:
        lib = ctypes.CDLL(_build.build())
        lib.xmoe_oracle_gate_logits_f32.restype = None
        lib.xmoe_oracle_gate_logits_f32.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 3
        _gate_lib = lib
    return _gate_lib


# ----------------------------------------------------------------------------------------------------------
# gating (Listing 1, gating(); Appendix B.3 "Padding-free Gating")
# ----------------------------------------------------------------------------------------------------------
def gate_logits_contract(x: np.ndarray, w_router: np.ndarray, bias: Optional[np.ndarray]) -> np.ndarray:
    """logits[t,e] = sum_i x[t,i] Wr[i,e] (+ bias[e]) in float32, in the fixed order of gate_order.c."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    w32 = np.ascontiguousarray(w_router, dtype=np.float32)
    T, d = x32.shape
    E = w32.shape[1]
    assert w32.shape[0] == d
    out = np.empty((T, E), dtype=np.float32)
    b32 = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    _load_gate_lib().xmoe_oracle_gate_logits_f32(
        x32.ctypes.data, w32.ctypes.data, None if b32 is None else b32.ctypes.data, out.ctypes.data, T, d, E)
    return out


def gate_logits_f64(x, w_router, bias) -> np.ndarray:
    """The same projection in float64 (for finite differences, where float32 rounding would drown the step)."""
    l = np.asarray(x, np.float64) @ np.asarray(w_router, np.float64)
    if bias is not None:
        l = l + np.asarray(bias, np.float64)[None, :]
    return l


def softmax(logits: np.ndarray) -> np.ndarray:
    """Row softmax over the E experts (Listing 1: softmax(FFN(tokens), axis=-1))."""
    l = np.asarray(logits, np.float64)
    z = l - l.max(axis=1, keepdims=True)
    ez = np.exp(z)
    return ez / ez.sum(axis=1, keepdims=True)


def route(logits: np.ndarray, k: int):
    """Top-k gate routing.  Returns (topk_idx [T,k] int32, topk_w [T,k] float64, p [T,E] float64).

    k times: pick the not yet picked expert with the largest logit, lowest index on ties."""
    l = np.array(logits, copy=True)
    T, E = l.shape
    assert 1 <= k <= E
    p = softmax(logits)
    idx = np.empty((T, k), dtype=np.int32)
    taken = np.zeros((T, E), dtype=bool)
    rows = np.arange(T)
    for j in range(k):
        masked = np.where(taken, -np.inf, l)
        pick = np.argmax(masked, axis=1)          # numpy returns the first (lowest-index) maximum
        idx[:, j] = pick
        taken[rows, pick] = True
    w = p[rows[:, None], idx]
    return idx, w, p


# ----------------------------------------------------------------------------------------------------------
# PFT construction (Listing 1, PFT_construction(), step 1 and the histogram; dropless)
# ----------------------------------------------------------------------------------------------------------
def build_eri(topk_idx: np.ndarray, topk_w: np.ndarray, E: int) -> dict:
    """ERI-arrays of the PFT (Section 4.1.1) for B = T*k rows.

    flat entry n = t*k + j; rows are the flat entries stably sorted by expert id."""
    T, k = topk_idx.shape
    flat_e = topk_idx.reshape(-1).astype(np.int64)
    order = np.argsort(flat_e, kind="stable")           # row i holds flat entry order[i]
    token_ids = (order // k).astype(np.int32)
    expert_ids = flat_e[order].astype(np.int32)
    combine_weights = np.asarray(topk_w).reshape(-1)[order]
    row_of_slot = np.empty(T * k, dtype=np.int32)
    row_of_slot[order] = np.arange(T * k, dtype=np.int32)
    tokens_per_expert = np.bincount(expert_ids, minlength=E).astype(np.int32)
    expert_offsets = np.zeros(E + 1, dtype=np.int32)
    expert_offsets[1:] = np.cumsum(tokens_per_expert)
    return {
        "token_ids": token_ids, "expert_ids": expert_ids, "tokens_per_expert": tokens_per_expert,
        "expert_offsets": expert_offsets, "combine_weights": combine_weights, "row_of_slot": row_of_slot,
    }


def build_eri_capped(topk_idx: np.ndarray, topk_w: np.ndarray, E: int, max_token_count: int) -> dict:
    """PFT construction with token dropping (Listing 1 PFT_construction(); Appendix B.2): every expert keeps at
    most max_token_count of the rows routed to it, the ones with the largest combine weights.

    The steps are the listing's, in its order: (1) sort the flat assignments by expert; (2) order the flat entries
    by combine weight, one-hot encode their experts, running count per expert down that order (rank_in_expert), keep
    an entry while its expert's count has not passed max_token_count; prune the arrays of step 1 to the retained
    entries; histogram.  Readings: the order by weight is descending (the largest weights are kept, Appendix B.2),
    entries of equal weight keep the lower flat index first, and the rank test is inclusive (rank <= max_token_count,
    as in the listing).  row_of_slot[n] is the retained row of flat entry n, or -1 if the entry was dropped."""
    T, k = topk_idx.shape
    B = T * k
    C = int(max_token_count)
    # step 1: expert ids and token ids of all entries, sorted by expert (stable)
    flat_top_experts = topk_idx.reshape(-1).astype(np.int64)
    by_expert = np.argsort(flat_top_experts, kind="stable")
    token_ids = (by_expert // k).astype(np.int32)
    expert_ids = flat_top_experts[by_expert].astype(np.int32)
    # step 2: which entries survive
    flat_combine_weights = np.asarray(topk_w).reshape(-1)
    sorted_indices = np.argsort(-flat_combine_weights, kind="stable")        # heaviest first, ties: lower index
    sorted_top_experts = flat_top_experts[sorted_indices]
    one_hot_enc = np.zeros((B, E), dtype=np.int64)
    one_hot_enc[np.arange(B), sorted_top_experts] = 1
    rank_in_expert = np.cumsum(one_hot_enc, axis=0)
    weight_mask = ((rank_in_expert <= C) & (one_hot_enc == 1)).any(axis=1)
    filtered_indices = sorted_indices[weight_mask]                           # retained flat entries
    retained = np.zeros(B, dtype=bool)
    retained[filtered_indices] = True
    retained_rows = retained[by_expert]                                      # in the order of step 1
    kept = by_expert[retained_rows]
    token_ids = token_ids[retained_rows]
    expert_ids = expert_ids[retained_rows]
    combine_weights = flat_combine_weights[kept]
    tokens_per_expert = np.bincount(expert_ids, minlength=E).astype(np.int32)
    expert_offsets = np.zeros(E + 1, dtype=np.int32)
    expert_offsets[1:] = np.cumsum(tokens_per_expert)
    row_of_slot = np.full(B, -1, dtype=np.int32)
    row_of_slot[kept] = np.arange(kept.size, dtype=np.int32)
    return {
        "token_ids": token_ids, "expert_ids": expert_ids, "tokens_per_expert": tokens_per_expert,
        "expert_offsets": expert_offsets, "combine_weights": combine_weights, "row_of_slot": row_of_slot,
    }


# ----------------------------------------------------------------------------------------------------------
# dispatch / mlp / combine (Listing 1; Section 4.1.2; Appendix B.4)
# ----------------------------------------------------------------------------------------------------------
def dispatch(x: np.ndarray, token_ids: np.ndarray) -> np.ndarray:
    """Gather kernel: dispatch_in[i,:] = gate_out[token_ids[i],:]."""
    return np.asarray(x)[token_ids]


def silu(g):
    return g / (1.0 + np.exp(-g))


def swiglu_ffn(X, wg, wu, wd):
    """One expert on its rows: Y = (silu(X Wg) * (X Wu)) Wd.  Returns (Y, G, U)."""
    G = X @ wg
    U = X @ wu
    A = silu(G) * U
    return A @ wd, G, U


def expert_ffn_fwd(Xd, expert_offsets, wg, wu, wd):
    """Sequential GeMM over the ragged segments: expert e multiplies rows [off[e], off[e+1])."""
    Xd = np.asarray(Xd, np.float64)
    B = Xd.shape[0]
    E, d, f = wg.shape
    Y = np.zeros((B, d))
    G = np.zeros((B, f))
    U = np.zeros((B, f))
    for e in range(E):
        lo, hi = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if hi == lo:
            continue
        Y[lo:hi], G[lo:hi], U[lo:hi] = swiglu_ffn(Xd[lo:hi], np.asarray(wg[e], np.float64),
                                                  np.asarray(wu[e], np.float64), np.asarray(wd[e], np.float64))
    return Y, G, U


def combine(Y, token_ids, combine_weights, T):
    """Scatter kernel, accumulating: out[token_ids[i],:] += combine_weights[i] * Y[i,:]."""
    out = np.zeros((T, Y.shape[1]))
    for i in range(Y.shape[0]):
        out[token_ids[i]] += combine_weights[i] * Y[i]
    return out


def shared_ffn_fwd(x, swg, swu, swd):
    """Sum over shared experts of FFN_s(x[t]) for every token (weight 1)."""
    x = np.asarray(x, np.float64)
    out = np.zeros_like(x)
    G, U = [], []
    for s in range(swg.shape[0]):
        y, g, u = swiglu_ffn(x, np.asarray(swg[s], np.float64), np.asarray(swu[s], np.float64),
                             np.asarray(swd[s], np.float64))
        out += y
        G.append(g)
        U.append(u)
    return out, G, U


# ----------------------------------------------------------------------------------------------------------
# the paper's own expert: two-matrix MLP (Listing 1 mlp(w1, w2); Tables 1 and 3)
# ----------------------------------------------------------------------------------------------------------
def activation(name: str, h):
    """act(h) for the two-matrix expert: identity | gelu (h * Phi(h), exact erf form) | silu."""
    h = np.asarray(h, np.float64)
    if name == "identity":
        return h
    if name == "gelu":
        from scipy.special import erf          # library primitive
        return 0.5 * h * (1.0 + erf(h / np.sqrt(2.0)))
    if name == "silu":
        return silu(h)
    raise ValueError(name)


def activation_grad(name: str, h):
    """d act(h) / dh."""
    h = np.asarray(h, np.float64)
    if name == "identity":
        return np.ones_like(h)
    if name == "gelu":
        from scipy.special import erf
        Phi = 0.5 * (1.0 + erf(h / np.sqrt(2.0)))
        phi = np.exp(-0.5 * h * h) / np.sqrt(2.0 * np.pi)
        return Phi + h * phi
    if name == "silu":
        sig = 1.0 / (1.0 + np.exp(-h))
        return sig * (1.0 + h * (1.0 - sig))
    raise ValueError(name)


def mlp2_ffn(X, w1, w2, act: str):
    """One two-matrix expert on its rows: H = X W1 (inter_activ of the listing), Y = act(H) W2.  Returns (Y, H)."""
    H = X @ w1
    return activation(act, H) @ w2, H


def expert_mlp2_fwd(Xd, expert_offsets, w1, w2, act: str):
    """Listing 1 mlp(): two sequential GeMMs over the ragged segments.  Returns (Y [B,d], H [B,f])."""
    Xd = np.asarray(Xd, np.float64)
    B = Xd.shape[0]
    E, d, f = w1.shape
    Y = np.zeros((B, d))
    H = np.zeros((B, f))
    for e in range(E):
        lo, hi = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if hi == lo:
            continue
        Y[lo:hi], H[lo:hi] = mlp2_ffn(Xd[lo:hi], np.asarray(w1[e], np.float64), np.asarray(w2[e], np.float64), act)
    return Y, H


def mlp2_ffn_bwd(X, H, dY, w1, w2, act: str):
    """Backward of one two-matrix expert.  Returns dX, dW1, dW2."""
    A = activation(act, H)
    dA = dY @ w2.T
    dW2 = A.T @ dY
    dH = dA * activation_grad(act, H)
    dX = dH @ w1.T
    dW1 = X.T @ dH
    return dX, dW1, dW2


def expert_mlp2_bwd(Xd, H, dY, expert_offsets, w1, w2, act: str):
    """Backward of the two sequential GeMMs; an empty expert gets zero weight gradients."""
    E, d, f = w1.shape
    dXd = np.zeros_like(np.asarray(Xd, np.float64))
    dW1 = np.zeros((E, d, f))
    dW2 = np.zeros((E, f, d))
    for e in range(E):
        lo, hi = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if hi == lo:
            continue
        dXd[lo:hi], dW1[e], dW2[e] = mlp2_ffn_bwd(np.asarray(Xd[lo:hi], np.float64), H[lo:hi], dY[lo:hi],
                                                  np.asarray(w1[e], np.float64), np.asarray(w2[e], np.float64), act)
    return dXd, dW1, dW2


def moe2_layer_fwd(inp: dict, k: int, act: str, logits_mode: str = "contract",
                   max_token_count: Optional[int] = None) -> dict:
    """Listing 1's call(tokens, k, max_token_count, w1, w2) with the paper's two-matrix expert.

    inp: x [T,d], w_router [d,E], bias [E]|None, w1 [E,d,f], w2 [E,f,d]."""
    x = np.asarray(inp["x"], np.float64)
    T = x.shape[0]
    E = inp["w1"].shape[0]
    if logits_mode == "contract":
        logits = gate_logits_contract(inp["x"], inp["w_router"], inp.get("bias"))
    else:
        logits = gate_logits_f64(inp["x"], inp["w_router"], inp.get("bias"))
    topk_idx, topk_w, p = route(logits, k)
    eri = build_eri(topk_idx, topk_w, E) if max_token_count is None else \
        build_eri_capped(topk_idx, topk_w, E, max_token_count)
    Xd = dispatch(x, eri["token_ids"])
    Y, H = expert_mlp2_fwd(Xd, eri["expert_offsets"], inp["w1"], inp["w2"], act)
    out = combine(Y, eri["token_ids"], eri["combine_weights"], T)
    return {"logits": logits, "p": p, "topk_idx": topk_idx, "topk_w": topk_w, "eri": eri,
            "Xd": Xd, "Y": Y, "H": H, "out": out}


def moe2_dense_definition(inp: dict, k: int, act: str, logits: np.ndarray) -> np.ndarray:
    """out[t] = sum_e [e in TopK(t)] p[t,e] act(x[t] W1_e) W2_e, looping over every (t, e); no ERI-arrays."""
    x = np.asarray(inp["x"], np.float64)
    T, d = x.shape
    E = inp["w1"].shape[0]
    p = softmax(logits)
    out = np.zeros((T, d))
    for t in range(T):
        chosen = sorted(range(E), key=lambda e: (-float(logits[t, e]), e))[:k]
        for e in chosen:
            y, _ = mlp2_ffn(x[t:t + 1], np.asarray(inp["w1"][e], np.float64), np.asarray(inp["w2"][e], np.float64),
                            act)
            out[t] += p[t, e] * y[0]
    return out


def moe2_layer_bwd(inp: dict, fwd: dict, k: int, act: str) -> dict:
    """Gradients of L = <dout, out> with respect to x, w_router, w1, w2."""
    x = np.asarray(inp["x"], np.float64)
    dout = np.asarray(inp["dout"], np.float64)
    T = x.shape[0]
    eri = fwd["eri"]
    dY, dw = combine_bwd(dout, fwd["Y"], eri["token_ids"], eri["combine_weights"], eri["row_of_slot"], k)
    dXd, dW1, dW2 = expert_mlp2_bwd(fwd["Xd"], fwd["H"], dY, eri["expert_offsets"], inp["w1"], inp["w2"], act)
    dx = dispatch_bwd(dXd, eri["row_of_slot"], T, k)
    dlogits = route_bwd(fwd["p"], fwd["topk_idx"], dw)
    dWr = x.T @ dlogits
    dx_gate = dlogits @ np.asarray(inp["w_router"], np.float64).T
    return {"dY": dY, "dw": dw, "dXd": dXd, "dw1": dW1, "dw2": dW2, "dx_routed": dx, "dlogits": dlogits,
            "dw_router": dWr, "dx_gate": dx_gate, "dx": dx + dx_gate}


def expert_param_count(E: int, d: int, f: int, matrices: int = 2) -> int:
    """Parameters of one MoE layer's experts: `matrices` matrices of d*f per expert (Table 1: 2 h' h per expert)."""
    return E * matrices * d * f


# ----------------------------------------------------------------------------------------------------------
# Redundancy-Bypassing Dispatch, stage 0: pilot selection and the two sets of ERI-arrays (Section 4.2)
# ----------------------------------------------------------------------------------------------------------
def rbd_stage0(topk_idx: np.ndarray, rand_key: np.ndarray, eri: dict, E: int, experts_per_node: int) -> dict:
    """Splits the rows of a PFT into pilot tokens (one per token and destination node, chosen at random) and local
    replicas (the token's other rows bound for the same node), with ERI-arrays for both and the mapping from every
    replica to its pilot.

    topk_idx [T,k]; rand_key [T*k] unsigned (one draw per flat entry n = t*k + j); eri: the dropless ERI-arrays."""
    T, k = topk_idx.shape
    B = T * k
    tok, exp_ids, ros = eri["token_ids"], eri["expert_ids"], eri["row_of_slot"]
    node_of = lambda e: int(e) // experts_per_node
    is_pilot = np.zeros(B, dtype=bool)            # per PFT row
    pilot_row_of = np.full(B, -1, dtype=np.int64)  # per PFT row: the PFT row of its group's pilot
    for t in range(T):
        groups = {}
        for j in range(k):
            groups.setdefault(node_of(topk_idx[t, j]), []).append(t * k + j)
        for members in groups.values():
            pilot = min(members, key=lambda n: (int(rand_key[n]), n))
            for n in members:
                pilot_row_of[ros[n]] = ros[pilot]
            is_pilot[ros[pilot]] = True
    pilot_rows = np.flatnonzero(is_pilot)          # PFT order: sorted by expert, ascending token inside an expert
    replica_rows = np.flatnonzero(~is_pilot)
    rank_in_class = np.empty(B, dtype=np.int64)
    rank_in_class[pilot_rows] = np.arange(pilot_rows.size)
    rank_in_class[replica_rows] = np.arange(replica_rows.size)

    def sub_eri(rows):
        tpe = np.bincount(exp_ids[rows], minlength=E).astype(np.int32)
        off = np.zeros(E + 1, dtype=np.int32)
        off[1:] = np.cumsum(tpe)
        return {"token_ids": tok[rows].astype(np.int32), "expert_ids": exp_ids[rows].astype(np.int32),
                "tokens_per_expert": tpe, "expert_offsets": off}

    pilot, replica = sub_eri(pilot_rows), sub_eri(replica_rows)
    # a replica records where its pilot sits inside the pilot segment of the pilot's expert
    s1_experts = exp_ids[pilot_row_of[replica_rows]].astype(np.int32)
    s1_indices = (rank_in_class[pilot_row_of[replica_rows]] - pilot["expert_offsets"][s1_experts]).astype(np.int32)
    merge_src = np.where(is_pilot, rank_in_class, pilot_rows.size + rank_in_class).astype(np.int32)
    return {"is_pilot": is_pilot, "pilot": pilot, "replica": replica, "s1_mapping_indices": s1_indices,
            "s1_mapping_experts": s1_experts, "merge_src": merge_src}


def rbd_absolute_index(s1_mapping_indices, s1_mapping_experts, pilot_offsets_at_destination):
    """Re-encodes the relative pilot indices to absolute rows of a pilot buffer whose expert segments start at the
    given offsets (after the uneven exchange these are the receiver's offsets; on one device, the sender's)."""
    return (np.asarray(pilot_offsets_at_destination)[s1_mapping_experts] + s1_mapping_indices).astype(np.int32)


def rbd_reconstruct(x, stage0: dict):
    """Stages 0-2 on one device (both exchanges are the identity): instantiate the pilot buffer with the gather
    kernel, rebuild the replicas from their pilots, merge the two groups into the experts' input order."""
    pilot_buf = dispatch(x, stage0["pilot"]["token_ids"])
    absolute = rbd_absolute_index(stage0["s1_mapping_indices"], stage0["s1_mapping_experts"],
                                  stage0["pilot"]["expert_offsets"])
    replica_buf = pilot_buf[absolute]
    both = np.concatenate([pilot_buf, replica_buf], axis=0)
    return both[stage0["merge_src"]]


def rbd_expected_redundancy(E: int, k: int, experts_per_node: int) -> float:
    """Expected share of replicas among the k rows of a token that picks k distinct experts uniformly at random:
    1 - E[number of distinct destination nodes] / k, with P(node untouched) = C(E - m, k) / C(E, k)."""
    from math import comb
    m = experts_per_node
    n_nodes = E // m
    distinct = n_nodes * (1.0 - comb(E - m, k) / comb(E, k))
    return 1.0 - distinct / k


# ----------------------------------------------------------------------------------------------------------
# whole layer
# ----------------------------------------------------------------------------------------------------------
def moe_layer_fwd(inp: dict, k: int, logits_mode: str = "contract", max_token_count: Optional[int] = None) -> dict:
    """Listing 1's call(): gating -> PFT_construction -> dispatch -> mlp -> combine (+ shared experts).

    inp: x [T,d], w_router [d,E], bias [E]|None, wg/wu [E,d,f], wd [E,f,d], shared_wg/wu/wd [E_s,...].
    max_token_count: None = dropless; else the per-expert capacity of the token-dropping PFT construction."""
    x = np.asarray(inp["x"], np.float64)
    T = x.shape[0]
    E = inp["wg"].shape[0]
    if logits_mode == "contract":
        logits = gate_logits_contract(inp["x"], inp["w_router"], inp.get("bias"))
    else:
        logits = gate_logits_f64(inp["x"], inp["w_router"], inp.get("bias"))
    topk_idx, topk_w, p = route(logits, k)
    eri = build_eri(topk_idx, topk_w, E) if max_token_count is None else \
        build_eri_capped(topk_idx, topk_w, E, max_token_count)
    Xd = dispatch(x, eri["token_ids"])
    Y, G, U = expert_ffn_fwd(Xd, eri["expert_offsets"], inp["wg"], inp["wu"], inp["wd"])
    out = combine(Y, eri["token_ids"], eri["combine_weights"], T)
    res = {"logits": logits, "p": p, "topk_idx": topk_idx, "topk_w": topk_w, "eri": eri,
           "Xd": Xd, "Y": Y, "G": G, "U": U, "out_routed": out}
    sh = inp.get("shared_wg")
    if sh is not None and sh.shape[0] > 0:
        so, sG, sU = shared_ffn_fwd(x, inp["shared_wg"], inp["shared_wu"], inp["shared_wd"])
        res["shared_out"], res["shared_G"], res["shared_U"] = so, sG, sU
        out = out + so
    res["out"] = out
    return res


def moe_dense_definition(inp: dict, k: int, logits: np.ndarray) -> np.ndarray:
    """The layer's plain definition with no ERI-arrays at all:
    out[t] = sum_e [e in TopK(t)] p[t,e] FFN_e(x[t]) + sum_s FFN_s(x[t]), looping over every (t, e)."""
    x = np.asarray(inp["x"], np.float64)
    T, d = x.shape
    E = inp["wg"].shape[0]
    p = softmax(logits)
    out = np.zeros((T, d))
    for t in range(T):
        # the k largest logits, lower index first among equals
        chosen = sorted(range(E), key=lambda e: (-float(logits[t, e]), e))[:k]
        for e in range(E):
            if e in chosen:
                y, _, _ = swiglu_ffn(x[t:t + 1], np.asarray(inp["wg"][e], np.float64),
                                     np.asarray(inp["wu"][e], np.float64), np.asarray(inp["wd"][e], np.float64))
                out[t] += p[t, e] * y[0]
        sh = inp.get("shared_wg")
        if sh is not None:
            for s in range(sh.shape[0]):
                y, _, _ = swiglu_ffn(x[t:t + 1], np.asarray(inp["shared_wg"][s], np.float64),
                                     np.asarray(inp["shared_wu"][s], np.float64),
                                     np.asarray(inp["shared_wd"][s], np.float64))
                out[t] += y[0]
    return out


# ----------------------------------------------------------------------------------------------------------
# backward (derived: the paper only says it mirrors the forward, Section 4.3)
# ----------------------------------------------------------------------------------------------------------
def combine_bwd(dout, Y, token_ids, combine_weights, row_of_slot, k):
    """dY[i] = combine_weights[i] * dOut[token_ids[i]];  dw[t,j] = <dOut[t], Y[row_of_slot[t*k+j]]>, and 0 for a
    dropped entry (row_of_slot < 0): the output does not depend on its weight."""
    dout = np.asarray(dout, np.float64)
    T = dout.shape[0]
    dY = combine_weights[:, None] * dout[token_ids]
    dw = np.zeros((T, k))
    for t in range(T):
        for j in range(k):
            r = row_of_slot[t * k + j]
            if r >= 0:
                dw[t, j] = np.dot(dout[t], Y[r])
    return dY, dw


def swiglu_ffn_bwd(X, G, U, dY, wg, wu, wd):
    """Backward of one expert.  Returns dX, dWg, dWu, dWd."""
    sig = 1.0 / (1.0 + np.exp(-G))
    S = G * sig
    A = S * U
    dA = dY @ wd.T
    dWd = A.T @ dY
    dG = dA * U * (sig * (1.0 + G * (1.0 - sig)))
    dU = dA * S
    dX = dG @ wg.T + dU @ wu.T
    dWg = X.T @ dG
    dWu = X.T @ dU
    return dX, dWg, dWu, dWd


def expert_ffn_bwd(Xd, G, U, dY, expert_offsets, wg, wu, wd):
    """Backward of the sequential GeMM; an empty expert gets zero weight gradients."""
    E, d, f = wg.shape
    dXd = np.zeros_like(np.asarray(Xd, np.float64))
    dWg = np.zeros((E, d, f))
    dWu = np.zeros((E, d, f))
    dWd = np.zeros((E, f, d))
    for e in range(E):
        lo, hi = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if hi == lo:
            continue
        dXd[lo:hi], dWg[e], dWu[e], dWd[e] = swiglu_ffn_bwd(
            np.asarray(Xd[lo:hi], np.float64), G[lo:hi], U[lo:hi], dY[lo:hi],
            np.asarray(wg[e], np.float64), np.asarray(wu[e], np.float64), np.asarray(wd[e], np.float64))
    return dXd, dWg, dWu, dWd


def dispatch_bwd(dXd, row_of_slot, T, k):
    """dx[t] = sum_j dXd[row_of_slot[t*k+j]] over the retained entries (transpose of the gather)."""
    dx = np.zeros((T, dXd.shape[1]))
    for t in range(T):
        for j in range(k):
            r = row_of_slot[t * k + j]
            if r >= 0:
                dx[t] += dXd[r]
    return dx


def route_bwd(p, topk_idx, dw):
    """Softmax Jacobian on the selected entries: dp[t,e_j] = dw[t,j], 0 elsewhere;
    dlogits = p * (dp - sum_e p*dp)."""
    T, E = p.shape
    dp = np.zeros((T, E))
    rows = np.arange(T)
    for j in range(topk_idx.shape[1]):
        dp[rows, topk_idx[:, j]] += dw[:, j]
    inner = (p * dp).sum(axis=1, keepdims=True)
    return p * (dp - inner)


def moe_layer_bwd(inp: dict, fwd: dict, k: int) -> dict:
    """Gradients of L = <dout, out> with respect to x, w_router, wg, wu, wd and the shared experts."""
    x = np.asarray(inp["x"], np.float64)
    dout = np.asarray(inp["dout"], np.float64)
    T = x.shape[0]
    eri = fwd["eri"]
    dY, dw = combine_bwd(dout, fwd["Y"], eri["token_ids"], eri["combine_weights"], eri["row_of_slot"], k)
    dXd, dWg, dWu, dWd = expert_ffn_bwd(fwd["Xd"], fwd["G"], fwd["U"], dY, eri["expert_offsets"],
                                        inp["wg"], inp["wu"], inp["wd"])
    dx = dispatch_bwd(dXd, eri["row_of_slot"], T, k)
    dlogits = route_bwd(fwd["p"], fwd["topk_idx"], dw)
    dWr = x.T @ dlogits
    dx_gate = dlogits @ np.asarray(inp["w_router"], np.float64).T
    res = {"dY": dY, "dw": dw, "dXd": dXd, "dwg": dWg, "dwu": dWu, "dwd": dWd, "dx_routed": dx,
           "dlogits": dlogits, "dw_router": dWr, "dx_gate": dx_gate}
    dx = dx + dx_gate
    sh = inp.get("shared_wg")
    if sh is not None and sh.shape[0] > 0:
        Es = sh.shape[0]
        dsx = np.zeros_like(x)
        dswg = np.zeros(np.shape(inp["shared_wg"]))
        dswu = np.zeros(np.shape(inp["shared_wu"]))
        dswd = np.zeros(np.shape(inp["shared_wd"]))
        for s in range(Es):
            dxs, dswg[s], dswu[s], dswd[s] = swiglu_ffn_bwd(
                x, fwd["shared_G"][s], fwd["shared_U"][s], dout, np.asarray(inp["shared_wg"][s], np.float64),
                np.asarray(inp["shared_wu"][s], np.float64), np.asarray(inp["shared_wd"][s], np.float64))
            dsx += dxs
        res.update({"dx_shared": dsx, "dshared_wg": dswg, "dshared_wu": dswu, "dshared_wd": dswd})
        dx = dx + dsx
    res["dx"] = dx
    return res


# ----------------------------------------------------------------------------------------------------------
# activation footprint (Section 3.2, Table 2; the paper's printed instance is Table 4's "Theoretical" row)
# ----------------------------------------------------------------------------------------------------------
def activation_bytes(T: int, k: int, d: int, f: int, bytes_per_el: int, c: float = 1.0) -> float:
    """A_dispatch + A_combine (k*T*d each) plus the two FFN intermediates (k*T*f each), times capacity c."""
    return c * bytes_per_el * T * k * (2 * d + 2 * f)
