"""Host-side successive-batching bookkeeping of the library against the oracle's
(same calls, same layouts), plus its error paths.  No GPU involved."""
import numpy as np
import pytest

from oracle import definitional as odef


@pytest.fixture(scope="module")
def tp():
    from paper_2506_15050_amd import binding
    binding.load()
    return binding


def test_batcher_follows_the_oracle(tp):
    rng = np.random.default_rng(61)
    K, l, L = 7, 8, 24
    nat, ref = tp.Batcher(K, l, L), odef.SuccessiveBatch(K, l, L)
    prompts = rng.integers(1, 12, size=K + 2)
    assert nat.refill(prompts) == ref.refill(prompts) == K
    for step in range(15):
        cu, ctx, prompt, done, ids = ref.layout()
        gen, eos = [], []
        for k in range(K):
            so_far = cu[k + 1] - cu[k] - prompt[k]
            room = min(l, L - so_far)
            stop = rng.random() < 0.35
            gen.append(int(rng.integers(0 if stop else 1, room + 1)) if stop else room)
            eos.append(1 if stop else 0)
        nat.advance(gen, eos)
        ref.advance(gen, eos)
        got, want = nat.layout(), ref.layout()
        for g, w in zip(got, want):
            assert np.array_equal(g, np.asarray(w))
        new = rng.integers(1, 12, size=int(sum(want[3])) + 1)
        assert nat.refill(new) == ref.refill(new)
        for g, w in zip(nat.layout(), ref.layout()):
            assert np.array_equal(g, np.asarray(w))
    nat.close()


def test_batcher_errors_change_nothing(tp):
    with pytest.raises(ValueError):
        tp.Batcher(0, 8, 24)
    with pytest.raises(ValueError):
        tp.Batcher(4, 8, 4)                                  # maximum response shorter than a window
    b = tp.Batcher(3, 8, 24)
    with pytest.raises(RuntimeError, match="TPPO_ERR_PARAM"):
        b.layout()                                           # empty slots
    assert b.refill([5, 6]) == 2
    with pytest.raises(RuntimeError, match="TPPO_ERR_PARAM"):
        b.advance([8, 8, 8], [0, 0, 0])                      # slot 2 is still empty
    b2 = tp.Batcher(2, 8, 12)
    with pytest.raises(RuntimeError, match="TPPO_ERR_PARAM"):
        b2.refill([3, 0])                                    # an empty prompt
    b2 = tp.Batcher(2, 8, 12)
    b2.refill([3, 4])
    before = [a.copy() for a in b2.layout()]
    with pytest.raises(RuntimeError, match="TPPO_ERR_SIZE"):
        b2.advance([8, 9], [0, 0])                           # longer than the window
    with pytest.raises(RuntimeError, match="TPPO_ERR_PARAM"):
        b2.advance([8, 5], [0, 0])                           # stops short without ending
    for x, y in zip(b2.layout(), before):
        assert np.array_equal(x, y)
    b2.advance([8, 5], [0, 1])
    cu, ctx, prompt, done, ids = b2.layout()
    assert list(done) == [0, 1] and list(cu) == [0, 11, 20]
    with pytest.raises(RuntimeError, match="TPPO_ERR_PARAM"):
        b2.advance([4, 1], [0, 0])                           # slot 1 has ended: refill first
    b2.refill([2])
    with pytest.raises(RuntimeError, match="TPPO_ERR_SIZE"):
        b2.advance([8, 8], [0, 0])                           # slot 0 would pass the maximum response length
    b2.advance([4, 8], [0, 0])                               # reaches the maximum: ends without eos
    assert list(b2.layout()[3]) == [1, 0]
