"""Random networks against the oracle, every output of every step bit for bit: group graphs
with several producers and consumers per group, kernel shapes from 1x1 to 95x90, flatten
multipliers, non-prunable tensors, gaps and odd offsets, value patterns with ties,
zeros, denormals and infinities, whole filters and input features scaled away.  Each net
goes through every selection path and the single-variant steps, the batched portfolio in
its four forms, and the liveness fixpoint."""
import numpy as np
import pytest

from oracle import shifter_oracle as O
from paper_2309_06973_amd import shifter as S
from paper_2309_06973_amd import synth
from test_gpu_parity import check_batch, check_fixpoint, run_config

pytestmark = pytest.mark.gpu

SEEDS = list(range(120))


def counts_for(spec, seed):
    n = spec.n_prunable
    rng = np.random.default_rng(seed)
    ps = {0, n, synth.prune_count(n, 0.5), synth.prune_count(n, 0.9)}
    ps.update(int(x) for x in rng.integers(0, n + 1, 3))
    return sorted(ps)


@pytest.mark.parametrize("seed", SEEDS)
def test_random_net(seed):
    big = seed % 8 == 3
    spec = synth.random_spec(seed, max_weights=3_000_000 if big else 250_000)
    w, v = synth.random_weights(spec, seed)
    ps = counts_for(spec, seed)
    flags = O.FLAG_FREEZE_RESIDUAL if seed % 3 == 1 else O.FLAG_JOINT
    print(f"seed {seed}: N={spec.n_prunable} tensors={len(spec.tensors)} groups={len(spec.groups)} "
          f"counts={ps} flags={flags}", flush=True)
    run_config(spec, w, v, ps, flags=flags, fused=seed % 2 == 0, check_every=2, single_every=3)
    order = np.random.default_rng(seed + 1).permutation(len(ps))
    check_batch(spec, w, v, [ps[i] for i in order], flags=flags)
    for p in (ps[len(ps) // 2], ps[-2]):
        check_fixpoint(spec, w, v, p, flags=flags)
