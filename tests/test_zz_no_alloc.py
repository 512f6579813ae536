"""tppo_egae_static (the entry point that allocates nothing) against tppo_egae.

Both run the same kernels; the only difference is where the plan lives (the
library's fixed array instead of a caller's workspace), so the outputs must be
identical bit for bit.  Two calls in a row, the second on a smaller batch: the
array keeps the first call's contents, and nothing of them may leak into the
second.  Collected last on purpose (file name): the round's GPU run stops at the
first failure.
"""
import numpy as np
import pytest
import torch

from paper_2506_15050_amd import binding as tp
from paper_2506_15050_amd import synth

pytestmark = pytest.mark.gpu


def _case(name, seed_shift=0):
    cfg = dict(synth.CONFIGS[name])
    meta = synth._rng(cfg["seed"] + seed_shift, "meta")
    done = (meta.random(cfg["B"]) < cfg["p_done"]).astype(np.int32)
    win = synth._draw_lengths(meta, cfg, done)
    off = np.concatenate([[0], np.cumsum(win)]).astype(np.int32)
    n = int(off[-1])
    vals = np.random.default_rng(cfg["seed"] + 7919 + seed_shift)
    rewards = vals.standard_normal(n).astype(np.float32) * 0.1
    values = vals.standard_normal(n).astype(np.float32)
    boot = vals.standard_normal(cfg["B"]).astype(np.float32)
    return tuple(torch.from_numpy(x).cuda() for x in (rewards, values, off, done, boot))


@pytest.mark.parametrize("first,second", [("longcot", "small"), ("longcot5x", "longcot")])
def test_static_entry_point_matches_tppo_egae_twice_in_a_row(first, second):
    for i, name in enumerate((first, second)):                       # the second call is the smaller batch
        print(f"[gpu case] tppo_egae_static call {i}: layout {name}", flush=True)
        rewards, values, off, done, boot = _case(name, seed_shift=i)
        st_a, st_b = tp.new_status("cuda"), tp.new_status("cuda")
        want_adv, want_ret = tp.tppo_egae(rewards, values, off, done, 1.0, 0.95, bootstrap=boot, status=st_a)
        adv = torch.full_like(rewards, float("nan"))
        ret = torch.full_like(rewards, float("nan"))
        tp.tppo_egae_static(rewards, values, off, done, 1.0, 0.95, bootstrap=boot, status=st_b, out=(adv, ret))
        torch.cuda.synchronize()
        assert int(st_a.item()) == 0 and int(st_b.item()) == 0
        assert torch.equal(adv, want_adv), f"advantages differ on call {i} ({name})"
        assert torch.equal(ret, want_ret), f"returns differ on call {i} ({name})"


def test_static_entry_point_rejects_what_its_array_cannot_hold():
    lib = tp.load()
    limit = lib.tppo_egae_static_max_tiles()
    assert limit == 47872
    B = 8
    n_resp = (limit - B) * 1024                                        # n_resp / 1024 + B + 1 == limit + 1
    x = torch.zeros(8, device="cuda")
    off = torch.zeros(B + 1, dtype=torch.int32, device="cuda")
    done = torch.zeros(B, dtype=torch.int32, device="cuda")
    rc = lib.tppo_egae_static(x.data_ptr(), x.data_ptr(), off.data_ptr(), done.data_ptr(), None, B, n_resp,
                              1.0, 0.95, x.data_ptr(), x.data_ptr(), None, None)
    assert rc == -2                                      # refused on the host: nothing was launched
