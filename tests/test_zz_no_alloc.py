"""ppo_permutation_static (the entry point that allocates nothing: its scratch is a static device array of the
library) against ppo_permutation of a context, bit for bit, through the C ABI: two calls in a row on the same
GPU array, the second with a smaller input, plus the size limit's error."""
import numpy as np
import pytest

from oracle import ppo_oracle as orc
from paper_2509_16434_amd import configs

pytestmark = pytest.mark.gpu


def _ctx_permutation(L, S, seed, upd, epoch):
    cfg = configs.get_config(0, num_envs=S // 8, horizon=8)
    lrn = L.Learner(cfg["net"], cfg["num_envs"], cfg["horizon"], cfg["obs_dtype"])
    out = lrn.permutation(seed, upd, epoch)
    lrn.close()
    return out


def test_static_permutation_matches_context_permutation():
    import torch
    from paper_2509_16434_amd import learner as L
    # 40 008 samples (ragged last block, 2048 buckets), then 1 000 (32 buckets: most of the array keeps the first call's data)
    for S, seed, upd, epoch in ((40008, 77, 3, 1), (1000, 5, 0, 2)):
        want = _ctx_permutation(L, S, seed, upd, epoch)
        got = L.permutation_static(S, seed, upd, epoch)
        torch.cuda.synchronize()
        got = got.cpu().numpy()
        np.testing.assert_array_equal(got, want)
        np.testing.assert_array_equal(got, orc.permutation(seed, upd, epoch, S))
    # on a side stream, into a caller-owned slice, twice (the second call finds the first one's counts)
    st = torch.cuda.Stream()
    buf = torch.full((3000,), -1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    for _ in range(2):
        L.permutation_static(2000, 9, 1, 0, out=buf[:2000], stream=st)
    st.synchronize()
    np.testing.assert_array_equal(buf[:2000].cpu().numpy(), orc.permutation(9, 1, 0, 2000))
    assert bool((buf[2000:] == -1).all())
    # limits
    assert L.permutation_static(0, 1, 1, 1).numel() == 0
    with pytest.raises(L.LearnerError) as e:
        L.permutation_static(L.STATIC_PERM_MAX + 1, 1, 1, 1, out=buf)
    assert e.value.code == L.PPO_ESHAPE
    with pytest.raises(L.LearnerError) as e:
        L.permutation_static(-1, 1, 1, 1, out=buf)
    assert e.value.code == L.PPO_EINVAL
