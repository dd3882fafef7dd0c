"""GPU parity of the FlashSGD and FlashLion steps at full size: the Llama-3.1-8B parameter list (291 tensors,
8.03 G parameters) in one fused call per step, the launch configuration of the benchmark's SGD and Lion lines
(tiles of 4096 elements, launches of 2^28 elements).

Quantisation groups of 32 elements are independent of each other, so the oracle runs the same two steps on
SAMPLED groups of every tensor - first and last group, groups on both sides of the first tile boundaries and of
every boundary between two kernel launches of the call, random groups - fed with copies of the inputs the GPU
used.  The comparison is exact: every code, scale and BF16 weight of the sampled groups.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_23349_amd as fo
import workloads as W
from helpers import bits16, compare_state

pytestmark = pytest.mark.gpu

HP = {"sgd": dict(lr=1e-2, wd=5e-4, momentum=0.9), "lion": dict(lr=1e-4, wd=0.1, beta1=0.9, beta2=0.99)}
SEED = 3
GRAD_SCALE = 1e-4
N_RANDOM_GROUPS = 12
TILE = 4096                       # elements per workgroup of the SGD and Lion steps
LAUNCH_TILES = (1 << 28) // TILE  # workgroups per kernel launch of a fused call


def _sample_groups(numel, rng, first_tile):
    ng = (numel + 31) // 32
    pick = {0, ng - 1}
    edges = [TILE // 32, 2 * TILE // 32]
    n_tiles = (numel + TILE - 1) // TILE
    k = (first_tile + LAUNCH_TILES - 1) // LAUNCH_TILES
    while k * LAUNCH_TILES < first_tile + n_tiles:
        if k * LAUNCH_TILES > first_tile:
            edges.append((k * LAUNCH_TILES - first_tile) * TILE // 32)
        k += 1
    for edge in edges:
        for g in (edge - 1, edge):
            if 0 <= g < ng:
                pick.add(g)
    pick.update(int(x) for x in rng.integers(0, ng, size=min(N_RANDOM_GROUPS, ng)))
    return np.array(sorted(pick), dtype=np.int64), len(edges) - 2


def _download_sample(buf, eidx, gidx):
    return dict(thp=bits16(buf.param[eidx]), rho=buf.rho[eidx].cpu().numpy(), mq=buf.m_q[eidx].cpu().numpy(),
                ms=bits16(buf.m_scale[gidx]))


@pytest.mark.parametrize("kind", ["sgd", "lion"])
def test_llama_fused_sgd_and_lion_sampled_parity(kind):
    hp = HP[kind]
    specs = W.llama31_8b()
    assert sum(s.numel for s in specs) == 8_030_261_248 and len(specs) == 291
    assert fo.step_launch_count(kind, [s.numel for s in specs]) == 30
    rng = np.random.default_rng(99)
    bufs, states, eidx, gidx = [], [], [], []
    first, n_launch_edges = 0, 0
    for i, sp in enumerate(specs):
        groups, inside = _sample_groups(sp.numel, rng, first)
        n_launch_edges += inside + (1 if first > 0 and first % LAUNCH_TILES == 0 else 0)
        first += (sp.numel + TILE - 1) // TILE
        e = (torch.from_numpy(groups).cuda()[:, None] * 32 + torch.arange(32, device="cuda")[None, :]).reshape(-1)
        eidx.append(e[e < sp.numel])
        gidx.append(torch.from_numpy(groups).cuda())
        b = fo.ParamBuffers(sp.numel, kind, with_grad=True)
        th = W.theta0(sp, i, seed=SEED, device="cuda")
        fo.split_weights(th, b.param, b.rho)
        states.append(oracle.TensorState(th[eidx[i]].cpu().numpy(), kind))
        del th
        b.lr, b.weight_decay = hp["lr"], (hp["wd"] if sp.role == "matrix" else 0.0)
        bufs.append(b)
    # all 29 boundaries between the call's 30 launches are sampled on both sides (inside a tensor, or between
    # two tensors, whose last and first groups are always sampled)
    assert (first + LAUNCH_TILES - 1) // LAUNCH_TILES == 30 and n_launch_edges == 29
    tl = fo.TensorList(bufs)
    n_elements = 0
    for t in (1, 2):
        for i, (sp, b) in enumerate(zip(specs, bufs)):
            b.grad.copy_(W.grad_bf16(sp, i, t, seed=SEED, device="cuda", dist="normal", scale=GRAD_SCALE))
            g = bits16(b.grad[eidx[i]])
            if kind == "sgd":
                oracle.sgd_step(states[i], g, hp["lr"], b.weight_decay, hp["momentum"])
            else:
                oracle.lion_step(states[i], g, hp["lr"], b.weight_decay, hp["beta1"], hp["beta2"])
        if kind == "sgd":
            fo.sgd_step(tl, hp["momentum"])
        else:
            fo.lion_step(tl, hp["beta1"], hp["beta2"])
        torch.cuda.synchronize()
        for i, (sp, b) in enumerate(zip(specs, bufs)):
            rep = compare_state(_download_sample(b, eidx[i], gidx[i]), states[i], where=f"{kind} t={t} {sp.name}")
            assert sum(r[1] for r in rep) == 0, (kind, t, sp.name, rep)
            n_elements += int(eidx[i].numel())
    print(f"{kind}: {n_elements // 2} sampled elements of 291 tensors, steps 1-2: no difference")
    for b in bufs[:12]:
        assert int(b.m_q.min()) >= -127 and bool(b.m_q.any())
    del bufs, tl
    fo.release_cache()
    torch.cuda.empty_cache()
