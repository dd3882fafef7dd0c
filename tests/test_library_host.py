"""Host-side checks of the HIP library that need no GPU: it loads, exports every symbol the
header declares, computes checkpoint sizes, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2602_23349_amd as fo
from paper_2602_23349_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "flashoptim.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(flashoptim_[a-z0-9_]+)\s*\(", header)))
    assert declared == sorted(fo.EXPORTED_SYMBOLS)
    L = fo.load_library()
    for name in declared:
        assert hasattr(L, name), name


def test_header_is_plain_c_and_a_c_program_links_against_the_library(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 with warnings as errors, the struct sizes seen
    # by a C compiler must be the ones the binding assumes, and a C program that takes the address of every
    # declared function must link against the shared library
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    header = open(os.path.join(ROOT, "include", "flashoptim.h")).read()
    names = sorted(set(re.findall(r"\b(flashoptim_[a-z0-9_]+)\s*\(", re.sub(r"/\*.*?\*/", "", header, flags=re.S))))
    src = tmp_path / "use_header.c"
    refs = "\n".join(f"    (void (*)(void))&{n}," for n in names)
    src.write_text(f"""#include <stdio.h>
#include "flashoptim.h"
typedef void (*fn_t)(void);
static const fn_t all_entry_points[] = {{
{refs}
}};
int main(void) {{
    printf("%zu %zu %zu %zu %zu\\n", sizeof(flashoptim_tensor), sizeof(flashoptim_tensor_ex), sizeof(flashoptim_adamw_hp),
           sizeof(all_entry_points) / sizeof(all_entry_points[0]), sizeof(flashoptim_lion_hp));
    return flashoptim_version() >= 1 ? 0 : 1;
}}
""")
    lib_dir = os.path.join(ROOT, "paper_2602_23349_amd")
    exe = tmp_path / "use_header"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", lib_dir, "-l:libflashoptim.so", "-Wl,-rpath," + lib_dir,
                    "-Wl,-rpath-link,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    t, tex, hp, n, lion = (int(x) for x in r.stdout.split())
    assert t == C.sizeof(B._Tensor) == 72 and hp == C.sizeof(B._AdamWHp) == 24 and n == len(names)
    assert tex == C.sizeof(B._TensorEx) and lion == 8


def test_struct_layout_matches_header():
    # flashoptim_tensor: 7 pointers, int64, 2 floats = 72 bytes on LP64
    assert C.sizeof(B._Tensor) == 72
    assert B._Tensor.numel.offset == 56 and B._Tensor.lr.offset == 64 and B._Tensor.weight_decay.offset == 68
    assert C.sizeof(B._AdamWHp) == 24 and B._AdamWHp.step.offset == 16


def test_checkpoint_size_matches_layout_definition():
    rng = np.random.default_rng(0)
    for kind in ("adamw", "sgd", "lion"):
        for _ in range(20):
            numels = [int(x) for x in rng.integers(0, 100000, size=rng.integers(0, 12))]
            assert fo.checkpoint_size(kind, numels) == oracle.checkpoint_size(kind, numels)
    # 2 + 1 + 1 + 1 bytes per parameter plus scales (Section 3.4), when 64 | n
    n = 1 << 20
    assert fo.checkpoint_size("adamw", [n]) - 128 == 5 * n + 2 * 2 * (n // 32)
    assert fo.checkpoint_size("lion", [n]) - 128 == 4 * n + 2 * (n // 32)
    with pytest.raises(fo.FlashOptimError):
        fo.checkpoint_size("adamw", [-1])


def _fake_tensor(**kw):
    t = B._Tensor()
    base = 0x10000
    for i, f in enumerate(("param", "rho", "grad", "m_q", "m_scale", "v_q", "v_scale")):
        setattr(t, f, base * (i + 1))
    t.numel, t.lr, t.weight_decay = 64, 1e-3, 0.0
    for k, v in kw.items():
        setattr(t, k, v)
    return t


def test_invalid_arguments_are_rejected_before_any_device_work():
    # pointers below are never dereferenced: validation fails first
    L = fo.load_library()
    arr = (B._Tensor * 1)(_fake_tensor())
    hp0 = B._AdamWHp(0.9, 0.999, 1e-8, 0)          # step must be >= 1
    assert L.flashoptim_adamw_step(arr, 1, C.byref(hp0), None) == -1
    hp = B._AdamWHp(0.9, 0.999, 1e-8, 1)
    assert L.flashoptim_adamw_step(arr, -1, C.byref(hp), None) == -1
    assert L.flashoptim_adamw_step(None, 1, C.byref(hp), None) == -1
    assert L.flashoptim_adamw_step(arr, 1, None, None) == -1
    arr[0] = _fake_tensor(rho=0x20008)              # misaligned
    assert L.flashoptim_adamw_step(arr, 1, C.byref(hp), None) == -2
    arr[0] = _fake_tensor(numel=-5)
    assert L.flashoptim_adamw_step(arr, 1, C.byref(hp), None) == -3
    arr[0] = _fake_tensor(numel=1 << 40)
    assert L.flashoptim_adamw_step(arr, 1, C.byref(hp), None) == -3
    arr[0] = _fake_tensor(v_q=None)                 # AdamW needs the variance buffers ...
    assert L.flashoptim_adamw_step(arr, 1, C.byref(hp), None) == -1
    shp = B._SgdHp(0.9)
    arr[0] = _fake_tensor(grad=None)
    assert L.flashoptim_sgd_step(arr, 1, C.byref(shp), None) == -1
    arr[0] = _fake_tensor(m_scale=0x50002)
    assert L.flashoptim_lion_step(arr, 1, C.byref(B._LionHp(0.9, 0.99)), None) == -2
    # empty lists and empty tensors are fine and launch nothing
    assert L.flashoptim_sgd_step(None, 0, C.byref(shp), None) == 0
    arr[0] = _fake_tensor(numel=0, param=None, rho=None, m_q=None)
    assert L.flashoptim_sgd_step(arr, 1, C.byref(shp), None) == 0
    # elementwise entry points
    assert L.flashoptim_split_weights(None, 0x1000, 0x2000, 16, None) == -1
    assert L.flashoptim_split_weights(0x1004, 0x1000, 0x2000, 16, None) == -2
    assert L.flashoptim_quantize_variance(0x1000, 0x2000, 0x3000, -1, None) == -3
    assert L.flashoptim_dequantize_momentum(None, None, None, 0, None) == 0
    # checkpoint: bad kind, short blob
    arr[0] = _fake_tensor()
    assert L.flashoptim_checkpoint_pack(7, arr, 1, 0, 0x100000, 1 << 20, None) == -1
    assert L.flashoptim_checkpoint_pack(0, arr, 1, 0, 0x100000, 64, None) == -5
    step = C.c_int64(0)
    assert L.flashoptim_checkpoint_unpack(0, 0x100000, 64, arr, 1, C.byref(step), None) == -5
    assert "aligned" in fo.strerror(-2) and fo.strerror(0) == "ok" and fo.strerror(-99) == "unknown status"
    assert fo.version() >= 1


def test_step_launch_count_is_one_launch_per_2_to_28_elements_of_whole_tiles():
    import workloads as W
    # a step call covers its list tile by tile (2048 elements for AdamW, 4096 for SGD and Lion, per tensor)
    # and issues one kernel launch per 2^28 elements' worth of tiles
    def expect(kind, numels):
        tile = 2048 if kind == "adamw" else 4096
        tiles = sum(-(-n // tile) for n in numels)
        per_launch = (1 << 28) // tile
        return -(-tiles // per_launch)
    cases = [[], [1], [1 << 28], [(1 << 28) + 1], [5, 0, 7], [s.numel for s in W.llama31_8b()],
             [s.numel for s in W.resnet50()], [(1 << 33) + 12345]]
    for kind in ("adamw", "sgd", "lion"):
        for numels in cases:
            assert fo.step_launch_count(kind, numels) == expect(kind, numels), (kind, numels[:3])
    assert fo.step_launch_count("adamw", [s.numel for s in W.llama31_8b()]) == 30
    L = fo.load_library()
    assert L.flashoptim_step_launch_count(3, None, 0) == -1
    assert L.flashoptim_step_launch_count(0, (C.c_int64 * 1)(-5), 1) == -3


def test_shard_range_arithmetic():
    # even split on multiples of 256, sizes differ by at most one unit, ragged end on the last non-empty shard
    for numel, world in ((0, 4), (1, 4), (255, 2), (256, 2), (257, 2), (1_000_037, 7), (1_000_037, 64), (8_030_261_248, 8), (1000, 16)):
        pieces = [fo.shard_range(numel, world, r) for r in range(world)]
        assert pieces[0][0] == 0 and sum(l for _, l in pieces) == numel
        for (b0, l0), (b1, _) in zip(pieces, pieces[1:]):
            assert b1 == b0 + l0
        sizes = [l for _, l in pieces if l]
        assert all(b % 256 == 0 for b, l in pieces if l)
        assert all(l % 256 == 0 for l in sizes[:-1])
        if sizes:
            assert max(sizes) - min(sizes[:-1] or sizes) <= 256
    for bad in ((10, 0, 0), (10, 2, 2), (10, 2, -1), (-1, 2, 0)):
        with pytest.raises(fo.FlashOptimError):
            fo.shard_range(*bad)
