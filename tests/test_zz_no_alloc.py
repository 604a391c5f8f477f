"""The SDE step for callers that cannot allocate (`br_sde_step_static`: scratch built into the
library) against `br_sde_step` with a caller buffer: bit-identical latents and log-probs on two
calls in a row, the second on a smaller input; sizes beyond the built-in scratch are refused."""
import numpy as np
import pytest
import torch

from paper_2509_06040_amd import binding as br
from paper_2509_06040_amd import synth
from gpu_util import DEV, bytes_buffer, host

pytestmark = pytest.mark.gpu


def _both(T, splits, K, n_tree, D, step, seed):
    t = br.Tree(T, splits, K, n_tree=n_tree)
    sched = synth.schedule(T, 3.0, logp_mean=False)
    n = n_tree * t.n_nodes
    z0 = torch.from_numpy(synth.random_latents(n, D, seed)).to(DEV)
    v = torch.from_numpy(synth.random_latents(n_tree * int(t.width[step]), D, seed + 1)).to(DEV)
    za, zb = z0.clone(), z0.clone()
    la, lb = torch.full((n,), 7.0, device=DEV), torch.full((n,), 7.0, device=DEV)
    br.sde_step(t, sched, seed, step, D, v, za, la, bytes_buffer(br.sde_scratch_bytes(t, D)))
    br.sde_step_static(t, sched, seed, step, D, v, zb, lb)
    torch.cuda.synchronize()
    assert np.array_equal(host(za), host(zb))
    assert np.array_equal(host(la), host(lb))
    kids = slice(int(t.off[step + 1]), int(t.off[step + 2]))
    assert np.all(host(lb).reshape(n_tree, -1)[:, kids] != 7.0)          # every child of the step got a log-prob
    assert not np.array_equal(host(zb).reshape(n_tree, t.n_nodes, D)[:, kids], host(z0).reshape(n_tree, t.n_nodes, D)[:, kids])


def test_static_scratch_matches_caller_scratch_twice(lib):
    assert br.sde_static_scratch_limit() == 1 << 16
    # a split step of 3 trees x 4 parents at a latent size with a ragged tail, then a smaller plain step
    _both(6, (1, 3), 2, 3, 65536 + 4 * 37, 3, 11)
    _both(4, (0,), 2, 1, 4 * 1000, 2, 12)


def test_static_scratch_rejects_sizes_beyond_its_limit(lib):
    t = br.Tree(14, tuple(range(14)), 2, n_tree=1)          # 16384 leaves: 128 KiB of accumulator words
    D = 4096
    assert br.sde_scratch_bytes(t, D) > br.sde_static_scratch_limit()
    sched = synth.schedule(14, 3.0)
    z = torch.zeros(8, device=DEV)                          # never touched: the call is refused before any launch
    with pytest.raises(br.BranchRolloutError) as e:
        br.sde_step_static(t, sched, 1, 0, D, z, z, z)
    assert e.value.code == -4
