"""GPU parity of the fused optimizer steps against the CPU oracle on the small and medium
workloads: flat 2^20 tensor (AdamW, 1 and 100 steps after 10 warm-up steps), the GPT-2 124M
list (SGD, Lion), the ResNet-50 list (AdamW, heavy-tailed gradients), ragged tensor sizes, and
hand-built edge cases.  All calls go through the C ABI via the Python binding."""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2602_23349_amd as fo
import workloads as W
from helpers import (ADAMW_MODES, adamw_step_fn, assert_parity, bits16, compare_state, download, grads_for,
                     to_dev_u16, total_mismatches, upload_state, weight_decay_for)

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

ADAMW = dict(lr=1e-3, wd=0.01, beta1=0.9, beta2=0.999, eps=1e-8)
SGD = dict(lr=1e-2, wd=5e-4, momentum=0.9)
LION = dict(lr=1e-4, wd=0.1, beta1=0.9, beta2=0.99)


def _g_bits(g):
    return g.view(torch.int16).numpy().view(np.uint16)


def _oracle_step(kind, st, g, lr, wd, hp, t):
    if kind == "adamw":
        oracle.adamw_step(st, g, lr, wd, hp["beta1"], hp["beta2"], hp["eps"], t)
    elif kind == "sgd":
        oracle.sgd_step(st, g, lr, wd, hp["momentum"])
    else:
        oracle.lion_step(st, g, lr, wd, hp["beta1"], hp["beta2"])


def _gpu_step(kind, tl, hp, t, mode="exact"):
    if kind == "adamw":
        adamw_step_fn(mode)(tl, hp["beta1"], hp["beta2"], hp["eps"], t)
    elif kind == "sgd":
        fo.sgd_step(tl, hp["momentum"])
    else:
        fo.lion_step(tl, hp["beta1"], hp["beta2"])


@pytest.mark.parametrize("mode", ADAMW_MODES)
def test_flat_tensor_adamw_1_and_100_steps(mode):
    # workload 1: 2^20 parameters, states from 10 warm-up steps (run by the oracle), then parity after
    # 1 and after 100 further steps
    spec = W.flat_tensor(1 << 20)[0]
    st = oracle.TensorState(W.theta0(spec, 0, seed=0).numpy(), "adamw")
    for t in range(1, 11):
        oracle.adamw_step(st, _g_bits(W.grad_bf16(spec, 0, t, seed=0)), ADAMW["lr"], ADAMW["wd"], 0.9, 0.999, 1e-8, t)
    buf = upload_state(st)
    buf.lr, buf.weight_decay = ADAMW["lr"], ADAMW["wd"]
    tl = fo.TensorList([buf])
    report = []
    for t in range(11, 111):
        g = W.grad_bf16(spec, 0, t, seed=0)
        buf.grad.copy_(g.cuda())
        adamw_step_fn(mode)(tl, 0.9, 0.999, 1e-8, t)
        oracle.adamw_step(st, _g_bits(g), ADAMW["lr"], ADAMW["wd"], 0.9, 0.999, 1e-8, t)
        if t in (11, 12, 20, 60, 110):
            compare_state(download(buf), st, where=f"flat t={t}", report=report)
    assert_parity(report, mode, "flat tensor")


@pytest.mark.parametrize("kind,hp,mode", [("adamw", ADAMW, "exact"), ("adamw", ADAMW, "default"), ("sgd", SGD, "exact"),
                                          ("lion", LION, "exact")])
def test_ragged_sizes_multi_tensor(kind, hp, mode):
    # tensors whose sizes straddle the group / vector / tile / chunk boundaries, in ONE launch
    specs = W.odd_sizes()
    states = [oracle.TensorState(W.theta0(sp, i, seed=3).numpy(), kind) for i, sp in enumerate(specs)]
    bufs = [upload_state(s) for s in states]
    for b, sp in zip(bufs, specs):
        b.lr, b.weight_decay = hp["lr"], weight_decay_for(sp, hp["wd"])
    tl = fo.TensorList(bufs)
    report = []
    for t in (1, 2, 3):
        grads = grads_for(specs, t, seed=3, per_tensor_sigma=True)
        for b, g in zip(bufs, grads):
            b.grad.copy_(g.cuda())
        _gpu_step(kind, tl, hp, t, mode)
        for i, (s, g, sp) in enumerate(zip(states, grads, specs)):
            _oracle_step(kind, s, _g_bits(g), hp["lr"], weight_decay_for(sp, hp["wd"]), hp, t)
            compare_state(download(bufs[i]), s, where=f"{kind} {sp.name} t={t}", report=report)
    assert_parity(report, mode, f"ragged {kind}")


@pytest.mark.parametrize("kind", ["adamw", "sgd", "lion"])
def test_stream_probe_changes_nothing(kind):
    # the measurement aid moves a step's bytes and must leave every array as it was, ragged ends
    # and single-tensor (table-free) lists included
    specs = W.odd_sizes()
    bufs = []
    for i, sp in enumerate(specs):
        st = W.random_state(sp.numel, i, seed=9, with_variance=(kind == "adamw"))
        b = fo.ParamBuffers(sp.numel, kind)
        b.param.copy_(st["thp"].cuda()); b.rho.copy_(st["rho"].cuda())
        b.m_q.copy_(st["mq"].cuda()); b.m_scale.copy_(st["ms"].cuda())
        if kind == "adamw":
            b.v_q.copy_(st["vq"].cuda()); b.v_scale.copy_(st["vs"].cuda())
        b.grad.copy_(W.grad_bf16(sp, i, 1, seed=9).cuda())
        bufs.append(b)
    before = [download(b) for b in bufs]
    fo.stream_probe(kind, fo.TensorList(bufs))
    fo.stream_probe(kind, fo.TensorList([bufs[3]]))
    torch.cuda.synchronize()
    for b, want in zip(bufs, before):
        got = download(b)
        for k in want:
            assert np.array_equal(got[k], want[k]), k
    L = fo.load_library()
    assert L.flashoptim_stream_probe(7, None, 0, None) == -1
    assert L.flashoptim_stream_probe(0, None, 0, None) == 0


@pytest.mark.parametrize("mode", ADAMW_MODES)
def test_single_tensor_direct_path_matches_list_path(mode):
    # a list of length one takes the table-free launch (the gradient-release call)
    spec = W.ParamSpec("x", (3 * 8192 + 4096 + 77,), "matrix")
    st = oracle.TensorState(W.theta0(spec, 0, seed=4).numpy(), "adamw")
    buf = upload_state(st)
    buf.lr, buf.weight_decay = ADAMW["lr"], ADAMW["wd"]
    tl = fo.TensorList([buf])
    for t in (1, 2):
        g = W.grad_bf16(spec, 0, t, seed=4)
        buf.grad.copy_(g.cuda())
        adamw_step_fn(mode)(tl, 0.9, 0.999, 1e-8, t)
        oracle.adamw_step(st, _g_bits(g), ADAMW["lr"], ADAMW["wd"], 0.9, 0.999, 1e-8, t)
    report = []
    compare_state(download(buf), st, where="direct", report=report)
    assert_parity(report, mode, "direct path")


def test_edge_values_in_one_step():
    # zero weights (theta' = 0 path), exact powers of two, BF16-subnormal weights, zero gradients,
    # huge and tiny gradients (scale saturation / underflow), zero state
    n = 32 * 12
    theta = np.zeros(n, np.float32)
    theta[32:64] = 1.0
    theta[64:96] = -2.0 ** -126
    theta[96:128] = np.float32(1e-40)
    theta[128:160] = 3.0e38
    theta[160:] = (np.random.default_rng(5).standard_normal(n - 160) * 0.02).astype(np.float32)
    g = np.zeros(n, np.float32)
    g[0:16] = 1e-3
    g[40:48] = -7.0
    g[192:224] = 1e-20      # v underflows towards subnormals, FP16 scale underflows
    g[224:256] = 3e4        # sqrt(v) fits, m scale near the FP16 maximum
    g[256:288] = 1e30       # g^2 overflows FP32: v = inf, both scales saturate at 65504
    g[288:] = np.random.default_rng(6).standard_normal(n - 288) * 1e-3
    gb = torch.from_numpy(g).to(torch.bfloat16)
    for kind, hp, mode in (("adamw", ADAMW, "exact"), ("adamw", ADAMW, "default"), ("sgd", SGD, "exact"),
                           ("lion", LION, "exact")):
        st = oracle.TensorState(theta, kind)
        buf = upload_state(st)
        buf.lr, buf.weight_decay = hp["lr"], hp["wd"]
        buf.grad.copy_(gb.cuda())
        tl = fo.TensorList([buf])
        for t in (1, 2):
            _gpu_step(kind, tl, hp, t, mode)
            _oracle_step(kind, st, _g_bits(gb), hp["lr"], hp["wd"], hp, t)
            rep = compare_state(download(buf), st, where=f"edge {kind} {mode} t={t}")
            assert sum(r[1] for r in rep) == 0      # a few hundred elements: a systematic difference, not a rare tie
            assert np.isfinite(oracle.bf16_to_f32(st.thp)).all()


@pytest.mark.parametrize("mode", ADAMW_MODES)
@pytest.mark.parametrize("eps", [1e-15, 1e-12, 1e-11, 1e-8])
def test_zero_variance_with_live_momentum_and_small_eps(eps, mode):
    # v_hat = 0 (variance codes 0, gradient 0) under a non-zero momentum: the update is m_hat / eps, and
    # sqrt(v_hat) + eps must round to eps whichever square-root sequence the kernel selects for this eps
    n = 2048 * 3 + 96
    rs = W.random_state(n, 0, seed=21, with_variance=True)
    st = oracle.TensorState(np.zeros(n, np.float32), "adamw")
    st.thp = bits16(rs["thp"]); st.rho = rs["rho"].numpy().copy()
    st.mq = rs["mq"].numpy().copy(); st.ms = bits16(rs["ms"])
    st.vq = np.zeros(n, np.uint8); st.vs = bits16(rs["vs"])
    st.vq[1::7] = rs["vq"].numpy()[1::7]                 # most elements have v = 0, some do not
    finite = np.isfinite(oracle.bf16_to_f32(st.thp))
    st.thp[~finite] = 0x3f80
    buf = upload_state(st)
    buf.lr, buf.weight_decay = 1e-9, 0.0                 # m_hat / eps is huge: keep the weights finite
    g = torch.zeros(n, dtype=torch.bfloat16)
    g[5::11] = 1e-4
    buf.grad.copy_(g.cuda())
    tl = fo.TensorList([buf])
    for t in (1, 2):
        adamw_step_fn(mode)(tl, 0.9, 0.999, eps, t)
        oracle.adamw_step(st, _g_bits(g), 1e-9, 0.0, 0.9, 0.999, eps, t)
        rep = compare_state(download(buf), st, where=f"zero variance eps={eps} {mode} t={t}")
        assert sum(r[1] for r in rep) == 0


@pytest.mark.parametrize("mode", ADAMW_MODES)
@pytest.mark.parametrize("scenario", ["v_hat around 2^60", "m_hat around 2^60", "tiny momentum under a live variance",
                                      "eps below 2^-60", "eps above 1", "mixed wavefronts"])
def test_operand_range_boundaries_of_the_short_sequences(scenario, mode):
    # The AdamW kernels take a short square root and a short division when one wave-uniform test finds every
    # operand of the wavefront inside their ranges (v_t in [2^-96, 2^60 / rbc2], |m_t| <= 2^60 / rbc1 and, for the
    # correctly rounded division, >= 2^-60; eps in [2^-60, 1]), and the general sequences otherwise.  Both must
    # give the oracle's bits: inputs on either side of each limit, alone and mixed within wavefronts.
    n = 2048 * 4 + 160
    rng = np.random.default_rng(len(scenario))
    rs = W.random_state(n, 3, seed=33, with_variance=True)
    st = oracle.TensorState(np.zeros(n, np.float32), "adamw")
    st.thp = bits16(rs["thp"]); st.rho = rs["rho"].numpy().copy()
    st.mq = rs["mq"].numpy().copy(); st.ms = bits16(rs["ms"])
    st.vq = rs["vq"].numpy().copy(); st.vs = bits16(rs["vs"])
    finite = np.isfinite(oracle.bf16_to_f32(st.thp))
    st.thp[~finite] = 0x3f80
    eps, lr = 1e-8, 1e-12                                 # a tiny learning rate keeps the weights finite
    g = (rng.standard_normal(n) * 1e-4).astype(np.float32)
    if scenario == "v_hat around 2^60":
        st.mq[:] = 0; st.vq[:] = 0                         # t = 1 from Q(0): v_hat = g^2 up to rounding
        g = (2.0 ** 30 * 10.0 ** rng.uniform(-0.3, 0.3, n) * rng.choice([-1.0, 1.0], n)).astype(np.float32)
    elif scenario == "m_hat around 2^60":
        st.mq[:] = 0; st.vq[:] = 0                         # m_hat = g; g^2 ~ 1e36 stays finite
        g = (2.0 ** 60 * 10.0 ** rng.uniform(-0.3, 0.3, n) * rng.choice([-1.0, 1.0], n)).astype(np.float32)
    elif scenario == "tiny momentum under a live variance":
        st.mq[:] = 0                                       # m_t = (1 - beta1) g below 2^-60, v_t = beta2 v well above 2^-96
        st.vq[st.vq == 0] = 1                              # (every element: a zero variance would send the wavefront
        st.vs[st.vs == 0] = 0x1400                         #  to the general sequences on its own)
        g = (2.0 ** -58 * 10.0 ** rng.uniform(-1.5, 0.5, n)).astype(np.float32)
    elif scenario == "eps below 2^-60":
        eps = 1e-20
    elif scenario == "eps above 1":
        eps = 2.5
    else:
        # ordinary values with, here and there, one element beyond a limit: the wavefronts that hold one take the
        # general sequences, their neighbours the short ones
        for pos, val in ((5, 3.0e9), (700, -1.0e19), (1500, 1e-30), (2049, 0.0), (4100, 2.0e18), (8200, -4.0e9)):
            g[pos] = val
    gb = torch.from_numpy(g).to(torch.bfloat16)
    buf = upload_state(st)
    buf.lr, buf.weight_decay = lr, 0.01
    buf.grad.copy_(gb.cuda())
    tl = fo.TensorList([buf])
    for t in (1, 2):
        adamw_step_fn(mode)(tl, 0.9, 0.999, eps, t)
        oracle.adamw_step(st, _g_bits(gb), lr, 0.01, 0.9, 0.999, eps, t)
        rep = compare_state(download(buf), st, where=f"{scenario} {mode} t={t}")
        assert sum(r[1] for r in rep) == 0


@pytest.mark.parametrize("kind,hp", [("adamw", ADAMW), ("sgd", SGD), ("lion", LION)])
def test_zero_element_tensors_and_empty_lists(kind, hp):
    # tensors without elements are skipped wherever they stand in the list; a list of nothing is a no-op
    specs = [W.ParamSpec("e0", (0,), "bias"), W.ParamSpec("a", (33,), "matrix"), W.ParamSpec("e1", (0,), "matrix"),
             W.ParamSpec("b", (4097,), "matrix"), W.ParamSpec("e2", (0,), "gain")]
    states = [oracle.TensorState(W.theta0(sp, i, seed=8).numpy(), kind) if sp.numel else None for i, sp in enumerate(specs)]
    bufs = [upload_state(s) if s is not None else fo.ParamBuffers(0, kind) for s in states]
    for b in bufs:
        b.lr, b.weight_decay = hp["lr"], hp["wd"]
    report = []
    for t in (1, 2):
        for i, (b, sp) in enumerate(zip(bufs, specs)):
            if sp.numel:
                g = W.grad_bf16(sp, i, t, seed=8)
                b.grad.copy_(g.cuda())
                _oracle_step(kind, states[i], _g_bits(g), hp["lr"], hp["wd"], hp, t)
        _gpu_step(kind, fo.TensorList(bufs), hp, t)
        _gpu_step(kind, fo.TensorList([bufs[0], bufs[2]]), hp, t)        # only empty tensors
        _gpu_step(kind, fo.TensorList([]), hp, t)                        # no tensors at all
        _gpu_step(kind, fo.TensorList([bufs[4]]), hp, t)                 # the single-tensor path with nothing in it
        for i, sp in enumerate(specs):
            if sp.numel:
                compare_state(download(bufs[i]), states[i], where=f"{kind} {sp.name} t={t}", report=report)
    assert_parity(report, "exact", f"{kind} with empty tensors")


def _run_list(kind, hp, specs, seed, dist, scale, per_tensor_sigma, steps, nthreads=0, mode="exact"):
    states = [oracle.TensorState(W.theta0(sp, i, seed=seed).numpy(), kind) for i, sp in enumerate(specs)]
    bufs = [upload_state(s) for s in states]
    for b, sp in zip(bufs, specs):
        b.lr, b.weight_decay = hp["lr"], weight_decay_for(sp, hp["wd"])
    tl = fo.TensorList(bufs)
    report = []
    subnormal_scales = 0
    for t in steps:
        grads = grads_for(specs, t, seed=seed, dist=dist, scale=scale, per_tensor_sigma=per_tensor_sigma)
        for b, g in zip(bufs, grads):
            b.grad.copy_(g.cuda(), non_blocking=False)
        _gpu_step(kind, tl, hp, t, mode)
        torch.cuda.synchronize()
        for i, (s, g, sp) in enumerate(zip(states, grads, specs)):
            _oracle_step(kind, s, _g_bits(g), hp["lr"], weight_decay_for(sp, hp["wd"]), hp, t)
            compare_state(download(bufs[i]), s, where=f"{kind} {sp.name} t={t}", report=report)
            subnormal_scales += int(((s.ms > 0) & (s.ms < 0x0400)).sum())
    bad = [r for r in report if r[2]]
    print(f"{kind}: {len(specs)} tensors, steps {list(steps)}: code mismatches {bad if bad else 'none'}; "
          f"groups with FP16-subnormal momentum scales: {subnormal_scales}")
    assert_parity(report, mode, f"{kind} list")


@pytest.mark.parametrize("kind,hp", [("adamw", ADAMW), ("sgd", SGD)])
def test_list_whose_tile_lookup_needs_several_steps(kind, hp):
    # More than 16 K tiles in one launch, so that one coarse-table entry stands for several tiles, with runs
    # of tiny tensors inside single buckets: workgroups there walk over several descriptors to find theirs.
    big = (2048 if kind == "adamw" else 4096) * 20000      # 20000 tiles of the kind's tile size
    sizes = [big + 77] + [1, 33, 2048, 2049, 4096, 100, 6000, 31, 2047, 5000] + [big // 2 + 5] + \
            [7, 2048 * 3 + 1, 64, 4097] + [big // 4]
    specs = [W.ParamSpec(f"t{i}", (n,), "matrix") for i, n in enumerate(sizes)]
    _run_list(kind, hp, specs, seed=21, dist="normal", scale=1e-3, per_tensor_sigma=False, steps=(1, 2), nthreads=0)


def test_list_that_spans_several_kernel_launches():
    # A call is issued as consecutive launches of 2^28 elements' worth of tiles: here the boundary between
    # the first two launches falls inside the second tensor, and the third tensor ends raggedly in the
    # second launch.  Every element of every tensor is compared.
    sizes = [(1 << 28) - 5000, 70000, (1 << 26) + 123]
    assert fo.step_launch_count("adamw", sizes) == 2
    specs = [W.ParamSpec(f"t{i}", (n,), "matrix") for i, n in enumerate(sizes)]
    _run_list("adamw", ADAMW, specs, seed=23, dist="normal", scale=1e-3, per_tensor_sigma=False, steps=(1, 2), nthreads=0)


def test_gpt2_list_sgd():
    # workload 2: GPT-2 124M parameter list, per-tensor gradient scale log-uniform in [1e-5, 1e-2]
    _run_list("sgd", SGD, W.gpt2_small(), seed=0, dist="normal", scale=None, per_tensor_sigma=True, steps=(1, 2, 3))


def test_gpt2_list_lion():
    _run_list("lion", LION, W.gpt2_small(), seed=0, dist="normal", scale=None, per_tensor_sigma=True, steps=(1, 2, 3))


@pytest.mark.parametrize("mode", ADAMW_MODES)
def test_resnet50_list_adamw_heavy_tailed(mode):
    # workload 3: ResNet-50 list (161 tensors, 107 of them under 4K elements), Student-t(3) gradients
    _run_list("adamw", ADAMW, W.resnet50(), seed=0, dist="student3", scale=1e-3, per_tensor_sigma=False, steps=(1, 2, 3),
              mode=mode)


def test_checkpoint_pack_unpack_small_lists():
    for kind in ("adamw", "sgd"):
        specs = W.odd_sizes()[:14]
        states = []
        for i, sp in enumerate(specs):
            s = oracle.TensorState(W.theta0(sp, i, seed=9).numpy(), kind)
            rs = W.random_state(sp.numel, i, seed=9, with_variance=(kind == "adamw"))
            s.rho = rs["rho"].numpy(); s.mq = rs["mq"].numpy()
            s.ms = rs["ms"].view(torch.int16).numpy().view(np.uint16)
            if kind == "adamw":
                s.vq = rs["vq"].numpy(); s.vs = rs["vs"].view(torch.int16).numpy().view(np.uint16)
            states.append(s)
        bufs = [upload_state(s, with_grad=False) for s in states]
        size = fo.checkpoint_size(kind, [s.n for s in states])
        blob = torch.full((size,), 0xAB, dtype=torch.uint8, device="cuda")
        fo.checkpoint_pack(kind, bufs, 4242, blob)
        want = oracle.checkpoint_pack(kind, states, 4242)
        assert np.array_equal(blob.cpu().numpy(), want)
        fresh = [fo.ParamBuffers(s.n, kind, with_grad=False) for s in states]
        assert fo.checkpoint_unpack(kind, blob, fresh) == 4242
        for f, s in zip(fresh, states):
            rep = compare_state(download(f), s, where="unpack")
            assert sum(r[1] for r in rep) == 0
        # a blob packed for another list is rejected and nothing is written
        with pytest.raises(fo.FlashOptimError):
            fo.checkpoint_unpack(kind, blob, fresh[:-1])
        blob2 = blob.clone(); blob2[0] = 0
        with pytest.raises(fo.FlashOptimError):
            fo.checkpoint_unpack(kind, blob2, fresh)
        # resume: the step after unpacking into new buffers is the step the oracle takes from the saved state
        hp = ADAMW if kind == "adamw" else SGD
        resumed = [fo.ParamBuffers(s.n, kind) for s in states]
        assert fo.checkpoint_unpack(kind, blob, resumed) == 4242
        grads = grads_for(specs, 4243, seed=9)
        for b, g, sp, st in zip(resumed, grads, specs, states):
            b.lr, b.weight_decay = hp["lr"], weight_decay_for(sp, hp["wd"])
            b.grad.copy_(g.cuda())
            _oracle_step(kind, st, _g_bits(g), hp["lr"], weight_decay_for(sp, hp["wd"]), hp, 4243)
        _gpu_step(kind, fo.TensorList(resumed), hp, 4243)
        for b, st in zip(resumed, states):
            rep = compare_state(download(b), st, where="resume")
            assert sum(r[1] for r in rep) == 0


def test_hyperparameters_and_gradient_buffers_may_change_between_steps():
    # lr follows a schedule, weight decay toggles, and gradients arrive in different buffers: the cached
    # device table of the list must follow (it is re-uploaded in stream order when its content changes)
    specs = W.odd_sizes()[8:20]
    states = [oracle.TensorState(W.theta0(sp, i, seed=11).numpy(), "adamw") for i, sp in enumerate(specs)]
    bufs = [upload_state(s) for s in states]
    alt = [torch.empty_like(b.grad) for b in bufs]
    tl = fo.TensorList(bufs)
    for t in range(1, 8):
        lr = 1e-3 * (0.5 + 0.1 * t)
        grads = grads_for(specs, t, seed=11, scale=1e-3)
        for i, (b, g, sp) in enumerate(zip(bufs, grads, specs)):
            wd = 0.01 if (sp.role == "matrix" and t % 2) else 0.0
            dst = b.grad if t % 3 else alt[i]
            dst.copy_(g.cuda())
            tl.set_grad(i, dst)
            tl.set_hyper(i, lr=lr, weight_decay=wd)
            oracle.adamw_step(states[i], _g_bits(g), lr, wd, 0.9, 0.999, 1e-8, t)
        fo.adamw_step_exact(tl, 0.9, 0.999, 1e-8, t)
        # no synchronisation between steps: uploads and kernels are ordered on the stream
    for i, s in enumerate(states):
        rep = compare_state(download(bufs[i]), s, where=f"schedule {specs[i].name}")
        assert sum(r[1] for r in rep) == 0


def test_non_default_stream_and_two_lists_interleaved():
    specs = W.odd_sizes()[10:16]
    st_a = [oracle.TensorState(W.theta0(sp, i, seed=12).numpy(), "sgd") for i, sp in enumerate(specs)]
    st_b = [oracle.TensorState(W.theta0(sp, i, seed=13).numpy(), "lion") for i, sp in enumerate(specs)]
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    ba = [upload_state(s) for s in st_a]
    bb = [upload_state(s) for s in st_b]
    for b in ba:
        b.lr, b.weight_decay = SGD["lr"], SGD["wd"]
    for b in bb:
        b.lr, b.weight_decay = LION["lr"], LION["wd"]
    tla, tlb = fo.TensorList(ba), fo.TensorList(bb)
    torch.cuda.synchronize()
    for t in (1, 2, 3):
        ga = grads_for(specs, t, seed=12)
        gb = grads_for(specs, t, seed=13)
        with torch.cuda.stream(s1):
            for b, g in zip(ba, ga):
                b.grad.copy_(g.cuda(), non_blocking=True)
            fo.sgd_step(tla, SGD["momentum"], stream=s1)
        with torch.cuda.stream(s2):
            for b, g in zip(bb, gb):
                b.grad.copy_(g.cuda(), non_blocking=True)
            fo.lion_step(tlb, LION["beta1"], LION["beta2"], stream=s2)
        for s, g in zip(st_a, ga):
            oracle.sgd_step(s, _g_bits(g), SGD["lr"], SGD["wd"], SGD["momentum"])
        for s, g in zip(st_b, gb):
            oracle.lion_step(s, _g_bits(g), LION["lr"], LION["wd"], LION["beta1"], LION["beta2"])
    s1.synchronize(); s2.synchronize()
    for b, s in zip(ba + bb, st_a + st_b):
        rep = compare_state(download(b), s, where="streams")
        assert sum(r[1] for r in rep) == 0


def test_two_host_threads_step_their_own_lists_at_once():
    # two host threads, each with its own list and stream, call the library concurrently (the foreign-function
    # call releases the interpreter lock): the cached tables and their staging are shared, locked state
    import threading
    specs = W.odd_sizes()[4:14]
    work = []
    for k, (kind, hp) in enumerate((("adamw", ADAMW), ("sgd", SGD))):
        states = [oracle.TensorState(W.theta0(sp, i, seed=40 + k).numpy(), kind) for i, sp in enumerate(specs)]
        bufs = [upload_state(s) for s in states]
        for b, sp in zip(bufs, specs):
            b.lr, b.weight_decay = hp["lr"], weight_decay_for(sp, hp["wd"])
        grads = {t: grads_for(specs, t, seed=40 + k) for t in range(1, 21)}
        dev = {t: [g.cuda() for g in gs] for t, gs in grads.items()}
        work.append((kind, hp, states, bufs, grads, dev, torch.cuda.Stream()))
    torch.cuda.synchronize()
    errors = []

    def run(kind, hp, states, bufs, grads, dev, stream):
        try:
            tl = fo.TensorList(bufs)
            for t in range(1, 21):
                with torch.cuda.stream(stream):
                    for i, b in enumerate(bufs):
                        b.grad.copy_(dev[t][i], non_blocking=True)
                        tl.set_hyper(i, lr=hp["lr"] * (1.0 + 0.01 * t))     # forces a table upload every step
                    if kind == "adamw":
                        fo.adamw_step_exact(tl, hp["beta1"], hp["beta2"], hp["eps"], t, stream=stream)
                    else:
                        fo.sgd_step(tl, hp["momentum"], stream=stream)
            stream.synchronize()
        except Exception as e:                                              # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=run, args=w) for w in work]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=120)
        assert not th.is_alive()
    assert not errors, errors
    for kind, hp, states, bufs, grads, dev, stream in work:
        for t in range(1, 21):
            for i, (s, sp) in enumerate(zip(states, specs)):
                _oracle_step(kind, s, _g_bits(grads[t][i]), float(np.float32(hp["lr"] * (1.0 + 0.01 * t))),
                             weight_decay_for(sp, hp["wd"]), hp, t)
        for i, s in enumerate(states):
            rep = compare_state(download(bufs[i]), s, where=f"threads {kind} {specs[i].name}")
            assert sum(r[1] for r in rep) == 0


def test_short_square_root_is_verified_on_this_device_before_use():
    # the library checks the short square-root sequence against sqrtf for every value of its range before the
    # first AdamW step on a device; the environment can tell it not to use the sequence at all
    b = fo.ParamBuffers(64, "adamw")
    b.lr = 1e-3
    fo.adamw_step([b], 0.9, 0.999, 1e-8, 1)
    torch.cuda.synchronize()
    forced = os.environ.get("FLASHOPTIM_FORCE_GENERAL_SQRT", "0") not in ("", "0")
    assert fo.short_sqrt_state() == (2 if forced else 1)


def test_adamw_parity_holds_with_the_general_square_root():
    # the same AdamW parity tests in a child process that tells the library not to trust the short sequence
    if os.environ.get("FLASHOPTIM_FORCE_GENERAL_SQRT"):
        pytest.skip("already inside that child process")
    env = dict(os.environ, FLASHOPTIM_FORCE_GENERAL_SQRT="1")
    r = subprocess.run([sys.executable, "-u", "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "gpu",
                        os.path.join(ROOT, "tests", "test_gpu_steps.py"), "--timeout", "200", "--timeout-method", "thread",
                        "-k", "short_square_root or flat_tensor or ragged or edge_values or zero_variance or resnet50"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "passed" in r.stdout


def test_clock_monitor_reports_a_plausible_shader_clock():
    # the measurement aid: a one-wavefront kernel on its own stream that samples cycles per fixed-rate tick
    mon = fo.ClockMonitor(n_samples=20, seconds_per_sample=5e-4)
    mon.start()
    ghz = mon.ghz()
    assert ghz.shape == (20,) and (ghz > 0.3).all() and (ghz < 3.5).all()
    L = fo.load_library()
    assert L.flashoptim_clock_monitor(None, 4, 1e-3, None, None) == -1


def test_many_distinct_lists_evict_cached_tables():
    # more distinct lists than the library keeps cached tables for; every call must still be right
    spec = W.ParamSpec("w", (3000,), "matrix")
    results = []
    for k in range(270):
        sts = [oracle.TensorState(W.theta0(spec, 100 * k + j, seed=14).numpy(), "sgd") for j in range(2)]
        bufs = [upload_state(s) for s in sts]
        for b in bufs:
            b.lr, b.weight_decay = SGD["lr"], SGD["wd"]
        gs = [W.grad_bf16(spec, 100 * k + j, 1, seed=14) for j in range(2)]
        for b, g in zip(bufs, gs):
            b.grad.copy_(g.cuda())
        fo.sgd_step(bufs, SGD["momentum"])
        for s, g in zip(sts, gs):
            oracle.sgd_step(s, _g_bits(g), SGD["lr"], SGD["wd"], SGD["momentum"])
        results.append((bufs, sts))
    torch.cuda.synchronize()
    for bufs, sts in results:
        for b, s in zip(bufs, sts):
            rep = compare_state(download(b), s, where="evict")
            assert sum(r[1] for r in rep) == 0
    fo.release_cache()


def test_single_tensor_beyond_2_to_31_elements():
    # 64-bit element offsets: one tensor of 2^31 + 2^20 + 77 elements (15.3 GB of AdamW state),
    # oracle on sampled groups at the start, around element 2^31, and at the ragged end
    n = (1 << 31) + (1 << 20) + 77
    spec = W.ParamSpec("huge", (n,), "matrix")
    ng = (n + 31) // 32
    groups = np.array(sorted({0, 1, ng - 1, ng - 2, (1 << 31) // 32 - 1, (1 << 31) // 32, (1 << 31) // 32 + 1,
                              (1 << 30) // 32, 3 * (1 << 29) // 32 + 5, ng // 3}), dtype=np.int64)
    idx = (torch.from_numpy(groups).cuda()[:, None] * 32 + torch.arange(32, device="cuda")[None, :]).reshape(-1)
    idx = idx[idx < n]
    gidx = torch.from_numpy(groups).cuda()
    b = fo.ParamBuffers(n, "adamw")
    th = W.theta0(spec, 0, seed=15, device="cuda")
    fo.split_weights(th, b.param, b.rho)
    st = oracle.TensorState(th[idx].cpu().numpy(), "adamw")
    del th
    b.lr, b.weight_decay = ADAMW["lr"], ADAMW["wd"]
    tl = fo.TensorList([b])
    for t in (1, 2):
        b.grad.copy_(W.grad_bf16(spec, 0, t, seed=15, device="cuda", scale=1e-3))
        g = b.grad[idx].view(torch.int16).cpu().numpy().view(np.uint16)
        fo.adamw_step_exact(tl, 0.9, 0.999, 1e-8, t)
        oracle.adamw_step(st, g, ADAMW["lr"], ADAMW["wd"], 0.9, 0.999, 1e-8, t)
    got = dict(thp=bits16(b.param[idx]), rho=b.rho[idx].cpu().numpy(), mq=b.m_q[idx].cpu().numpy(),
               ms=bits16(b.m_scale[gidx]), vq=b.v_q[idx].cpu().numpy(), vs=bits16(b.v_scale[gidx]))
    rep = compare_state(got, st, where="huge tensor")
    assert sum(r[1] for r in rep) == 0
    del b, tl
    torch.cuda.empty_cache()
