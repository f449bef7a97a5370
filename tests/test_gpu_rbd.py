"""GPU parity of stage 0 of the Redundancy-Bypassing Dispatch (xmoe_rbd_stage0, xmoe_rbd_absolute_index) against
the CPU oracle: every index array bit for bit, and the single-device reconstruction (pilot buffer -> replicas ->
merge, all through the gather kernel) against the plain dispatch, bit for bit.  Through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import xmoe_inputs as xi

pytestmark = pytest.mark.gpu


def xm():
    import paper_2508_13337_amd as m
    return m


def i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def run_stage0(idx, keys, eri, E, epn):
    m = xm()
    T, k = idx.shape
    B = T * k
    out = {n: torch.full((B,), 12345, dtype=torch.int32, device="cuda")
           for n in ("pilot_token_ids", "pilot_expert_ids", "replica_token_ids", "replica_expert_ids",
                     "s1_mapping_indices", "s1_mapping_experts", "merge_src")}
    out.update({n: torch.empty(E, dtype=torch.int32, device="cuda")
                for n in ("pilot_tokens_per_expert", "replica_tokens_per_expert")})
    out.update({n: torch.empty(E + 1, dtype=torch.int32, device="cuda") for n in ("pilot_offsets", "replica_offsets")})
    ws = m.alloc_workspace(m.xmoe_workspace_bytes(m.WS_RBD_STAGE0, T, 0, E, k, 0, m.XMOE_BF16))
    key_bits = torch.from_numpy(keys.view(np.int32).copy()).cuda()
    m.xmoe_rbd_stage0(i32(idx), key_bits, i32(eri["token_ids"]), i32(eri["expert_ids"]), i32(eri["expert_offsets"]),
                      i32(eri["row_of_slot"]), epn, out, ws)
    torch.cuda.synchronize()
    return {n: v.cpu().numpy() for n, v in out.items()}, out


CASES = [(64, 8, 3, 2, 0, 1.0), (1000, 64, 6, 8, 1, 1.0), (513, 256, 8, 8, 2, 1.0), (77, 6, 6, 3, 3, 1.0),
         (2100, 12, 5, 4, 4, 3.0), (300, 16, 4, 16, 5, 1.0), (300, 16, 4, 1, 6, 1.0), (1, 4, 2, 2, 7, 1.0),
         (8192, 64, 6, 8, 8, 1.0), (4096, 256, 8, 8, 9, 1.0)]


@pytest.mark.parametrize("T,E,k,epn,seed,std", CASES)
def test_rbd_stage0_bit_exact(T, E, k, epn, seed, std):
    logits = xi.make_logits(T, E, seed=seed, std=std)
    idx, w, _ = oracle.route(logits, k)
    eri = oracle.build_eri(idx, w, E)
    keys = xi.make_rbd_keys(T * k, seed)
    if seed % 2 == 1:
        keys[::2] = 7          # many exact ties: the lower flat entry must win
    want = oracle.rbd_stage0(idx, keys, eri, E, epn)
    got, dev = run_stage0(idx, keys, eri, E, epn)
    B = T * k
    n_p, n_r = len(want["pilot"]["token_ids"]), len(want["replica"]["token_ids"])
    assert n_p + n_r == B
    for part, n in (("pilot", n_p), ("replica", n_r)):
        assert np.array_equal(got[part + "_token_ids"][:n], want[part]["token_ids"]), part
        assert np.array_equal(got[part + "_expert_ids"][:n], want[part]["expert_ids"]), part
        assert (got[part + "_token_ids"][n:] == -1).all() and (got[part + "_expert_ids"][n:] == E).all()
        assert np.array_equal(got[part + "_tokens_per_expert"], want[part]["tokens_per_expert"])
        assert np.array_equal(got[part + "_offsets"], want[part]["expert_offsets"])
    assert np.array_equal(got["s1_mapping_indices"][:n_r], want["s1_mapping_indices"])
    assert np.array_equal(got["s1_mapping_experts"][:n_r], want["s1_mapping_experts"])
    assert (got["s1_mapping_indices"][n_r:] == -1).all() and (got["s1_mapping_experts"][n_r:] == E).all()
    assert np.array_equal(got["merge_src"], want["merge_src"])

    # stages 0-2 on one device through the library's gather kernel, against the plain dispatch
    m = xm()
    d = 64
    x = torch.randn((T, d), dtype=torch.bfloat16, device="cuda", generator=torch.Generator("cuda").manual_seed(seed))
    absolute = torch.empty(B, dtype=torch.int32, device="cuda")
    m.xmoe_rbd_absolute_index(dev["s1_mapping_indices"], dev["s1_mapping_experts"], dev["pilot_offsets"], absolute)
    torch.cuda.synchronize()
    assert np.array_equal(absolute.cpu().numpy()[:n_r],
                          oracle.rbd_absolute_index(want["s1_mapping_indices"], want["s1_mapping_experts"],
                                                    want["pilot"]["expert_offsets"]))
    assert (absolute.cpu().numpy()[n_r:] == -1).all()
    both = torch.zeros((2 * B, d), dtype=torch.bfloat16, device="cuda")
    m.xmoe_dispatch(x, dev["pilot_token_ids"], both[:B])                 # pilot buffer (rows past n_pilot untouched)
    replica_buf = torch.zeros((B, d), dtype=torch.bfloat16, device="cuda")
    m.xmoe_dispatch(both[:B], absolute, replica_buf)                     # replicas copied from their pilots
    both[n_p:n_p + n_r].copy_(replica_buf[:n_r])                         # [pilot buffer ; replica buffer]
    merged = torch.empty((B, d), dtype=torch.bfloat16, device="cuda")
    m.xmoe_dispatch(both[:B], dev["merge_src"], merged)
    plain = torch.empty((B, d), dtype=torch.bfloat16, device="cuda")
    m.xmoe_dispatch(x, i32(eri["token_ids"]), plain)
    torch.cuda.synchronize()
    assert torch.equal(merged, plain)
    print(f"T={T} E={E} k={k} experts/node={epn}: redundancy {n_r / B:.3f}")


def test_rbd_stage0_rejects_bad_arguments():
    from paper_2508_13337_amd import _lib
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    p = t.data_ptr()
    args = [p] * 6 + [4, 8, 2, 0] + [p] * 11
    assert _lib.lib().xmoe_rbd_stage0(*args, p, 1 << 20, None) == 1          # experts_per_node < 1
    args = [p] * 6 + [4, 8, 2, 2] + [p] * 11
    assert _lib.lib().xmoe_rbd_stage0(*args, p, 16, None) == 3               # workspace too small
    torch.cuda.synchronize()
