"""The entry point that allocates nothing (xmoe_build_eri_static: the scratch is a static device array inside the
library) against the existing entry point (xmoe_build_eri with a caller-provided workspace): every output array bit
for bit, on two calls in a row, the second on a smaller input, so that whatever the first call left in the shared
array must not leak into the second."""
import numpy as np
import pytest
import torch

import oracle
import xmoe_inputs as xi

pytestmark = pytest.mark.gpu


def _run(m, idx, w, E, static):
    T, k = idx.shape
    B = T * k
    i32 = dict(dtype=torch.int32, device="cuda")
    out = {"tokens_per_expert": torch.full((E,), -7, **i32), "expert_offsets": torch.full((E + 1,), -7, **i32),
           "token_ids": torch.full((B,), -7, **i32), "expert_ids": torch.full((B,), -7, **i32),
           "combine_weights": torch.full((B,), -7.0, dtype=torch.float32, device="cuda"),
           "row_of_slot": torch.full((B,), -7, **i32)}
    args = (idx, w, E, out["tokens_per_expert"], out["expert_offsets"], out["token_ids"], out["expert_ids"],
            out["combine_weights"], out["row_of_slot"])
    if static:
        m.xmoe_build_eri_static(*args)
    else:
        ws = m.alloc_workspace(m.xmoe_workspace_bytes(m.WS_BUILD_ERI, T, 0, E, k, 0, 0))
        m.xmoe_build_eri(*args, ws)
    torch.cuda.synchronize()
    return out


def test_build_eri_static_matches_build_eri_twice_in_a_row():
    import paper_2508_13337_amd as m
    # first a large, skewed table (many chunks, every expert count differs), then a smaller one with other sizes
    for T, E, k, seed, skew in ((8192, 64, 6, 11, 1.5), (1000, 40, 3, 12, 0.0)):
        print(f"case T={T} E={E} k={k} seed={seed}", flush=True)
        logits = xi.make_logits(T, E, seed=seed)
        if skew:
            logits = logits - np.float32(skew) * np.log(np.arange(1, E + 1, dtype=np.float32))[None, :]
        idx_np, w_np, _ = oracle.route(logits, k)
        idx = torch.from_numpy(np.ascontiguousarray(idx_np, np.int32)).cuda()
        w = torch.from_numpy(np.ascontiguousarray(w_np, np.float32)).cuda()
        got = _run(m, idx, w, E, static=True)
        want = _run(m, idx, w, E, static=False)
        for key in want:
            assert torch.equal(got[key], want[key]), (T, key)
        ref = oracle.build_eri(idx_np, w_np.astype(np.float32), E)   # and both against the oracle
        for key in ("tokens_per_expert", "expert_offsets", "token_ids", "expert_ids", "row_of_slot"):
            assert np.array_equal(got[key].cpu().numpy(), ref[key]), key


def test_build_eri_static_rejects_sizes_beyond_its_array():
    import paper_2508_13337_amd as m
    T, E, k = 600_000, 512, 1          # ceil(T*k/1024) * E * 4 bytes = 1.2 MB > 1 MiB
    idx = torch.zeros((T, k), dtype=torch.int32, device="cuda")
    w = torch.zeros((T, k), dtype=torch.float32, device="cuda")
    i32 = dict(dtype=torch.int32, device="cuda")
    with pytest.raises(m.XMoEError) as err:
        m.xmoe_build_eri_static(idx, w, E, torch.empty(E, **i32), torch.empty(E + 1, **i32), torch.empty(T * k, **i32),
                                torch.empty(T * k, **i32), torch.empty(T * k, dtype=torch.float32, device="cuda"),
                                torch.empty(T * k, **i32))
    assert err.value.status == 3       # XMOE_ERR_WORKSPACE
