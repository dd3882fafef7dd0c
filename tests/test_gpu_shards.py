"""Sharded stepping (Section 3.4, "Distributed training"): a flat tensor cut into `world` shards by
flashoptim_shard_range and stepped shard by shard - as one list of shard descriptors, and as one call per
shard, the way `world` ranks would - gives the same bits as stepping the whole tensor, and as the oracle.
One GPU, no communication: the shards are pointer offsets into the same buffers."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_23349_amd as fo
import workloads as W
from helpers import upload_state, download, compare_state, assert_parity

pytestmark = pytest.mark.gpu

N = 1_000_000 + 37          # 3907 units of 256 elements, the last one ragged (and its last group short)


def _shards(buf, world):
    out, covered = [], 0
    for rank in range(world):
        begin, length = fo.shard_range(buf.numel, world, rank)
        assert begin == covered and begin % 256 == 0
        covered += length
        if length:
            out.append(buf.shard(begin, length))
    assert covered == buf.numel
    return out


@pytest.mark.parametrize("kind", ["adamw", "sgd"])
@pytest.mark.parametrize("world", [1, 7, 8])
def test_sharded_step_equals_whole_tensor_step_and_oracle(kind, world):
    spec = W.ParamSpec("flat", (N,), "matrix")
    st = oracle.TensorState(W.theta0(spec, 0, seed=3).numpy(), kind)
    lr, wd = (1e-3, 0.01) if kind == "adamw" else (1e-2, 5e-4)
    whole, as_list, per_rank = (upload_state(st) for _ in range(3))
    for b in (whole, as_list, per_rank):
        b.lr, b.weight_decay = lr, wd
    report = []
    for t in (1, 2, 3):
        g = W.grad_bf16(spec, 0, t, seed=3, scale=1e-3)
        for b in (whole, as_list, per_rank):
            b.grad.copy_(g)
        gbits = g.view(torch.int16).numpy().view(np.uint16)
        if kind == "adamw":
            oracle.adamw_step(st, gbits, lr, wd, 0.9, 0.999, 1e-8, t)
            fo.adamw_step_exact([whole], 0.9, 0.999, 1e-8, t)
            fo.adamw_step_exact(_shards(as_list, world), 0.9, 0.999, 1e-8, t)      # one list of shard descriptors
            for sh in _shards(per_rank, world):                                     # one call per "rank"
                fo.adamw_step_exact([sh], 0.9, 0.999, 1e-8, t)
        else:
            oracle.sgd_step(st, gbits, lr, wd, 0.9)
            fo.sgd_step([whole], 0.9)
            fo.sgd_step(_shards(as_list, world), 0.9)
            for sh in _shards(per_rank, world):
                fo.sgd_step([sh], 0.9)
        torch.cuda.synchronize()
        for name, b in (("whole", whole), ("shard list", as_list), ("per rank", per_rank)):
            compare_state(download(b), st, where=f"{kind} world={world} t={t} {name}", report=report)
    assert_parity(report, "exact", f"{kind}, {world} shards")
