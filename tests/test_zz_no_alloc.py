"""The LayerNorm backward entry point that allocates nothing: same results as the entry point that
takes a workspace, on two calls in a row (the second smaller), and a clear refusal past its limit."""
import numpy as np
import pytest
import torch

import paper_2209_02478_amd as mi
from gpu_util import DEV, dev, host, sync

pytestmark = pytest.mark.gpu


def both(dtype, T, H, seed, wide):
    rng = np.random.default_rng(seed)
    tdt = torch.float32 if (dtype == 0 or wide) else torch.bfloat16
    x = torch.tensor(rng.standard_normal((T, H)).astype(np.float32)).to(tdt).to(DEV)
    dy = torch.tensor(rng.standard_normal((T, H)).astype(np.float32)).to(tdt).to(DEV)
    gamma = dev(rng.standard_normal(H).astype(np.float32), dtype)
    add = dev(rng.standard_normal((T, H)).astype(np.float32), dtype)
    out_dt = torch.float32 if dtype == 0 else torch.bfloat16
    res = []
    for noalloc in (False, True):
        dx = torch.full((T, H), 3.0, dtype=out_dt, device=DEV)
        dg = torch.full((H,), 5.0, dtype=torch.float32, device=DEV)
        db = torch.full((H,), 5.0, dtype=torch.float32, device=DEV)
        if noalloc:
            mi.mimose_op_layernorm_bwd_noalloc(dtype, dy, int(wide), x, int(wide), gamma, dx, add, dg, db, T, H, 1e-5)
        else:
            partial = torch.zeros(mi.mimose_op_partial_rows(T) * 2 * H, dtype=torch.float32, device=DEV)
            mi.mimose_op_layernorm_bwd(dtype, dy, int(wide), x, int(wide), gamma, dx, add, dg, db, partial, T, H, 1e-5)
        sync()
        res.append((host(dx), host(dg), host(db)))
    return res


@pytest.mark.parametrize("dtype,wide", [(1, 1), (1, 0), (0, 0)])
def test_noalloc_layernorm_bwd_matches_workspace_version(dtype, wide):
    # two calls in a row on the shared array, the second with a smaller input
    for T, H, seed in [(6400, 768, 1), (130, 768, 2), (37, 64, 3)]:
        (dx0, dg0, db0), (dx1, dg1, db1) = both(dtype, T, H, seed, wide)
        assert np.array_equal(dx0, dx1) and np.array_equal(dg0, dg1) and np.array_equal(db0, db1), (T, H)
        assert np.isfinite(dg1).all() and np.abs(dg1).max() > 0


def test_noalloc_layernorm_bwd_refuses_past_its_limit():
    limit = mi.mimose_op_layernorm_bwd_noalloc_max_floats()
    H = 1024
    T = 16 * (limit // (2 * H)) + 16                      # one partial row too many
    assert mi.mimose_op_partial_rows(T) * 2 * H > limit
    t = torch.zeros(8, dtype=torch.bfloat16, device=DEV)  # never touched: the size check comes first
    f = torch.zeros(H, dtype=torch.float32, device=DEV)
    with pytest.raises(mi.MimoseError) as e:
        mi.mimose_op_layernorm_bwd_noalloc(1, t, 0, t, 0, t, t, None, f, f, T, H, 1e-5)
    assert "scratch floats" in str(e.value)
    # the largest size that fits is accepted (BERT-base at B=32, L=512 fits with room to spare)
    assert mi.mimose_op_partial_rows(16384) * 2 * 768 <= limit
