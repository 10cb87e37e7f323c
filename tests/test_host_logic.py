"""CPU-only checks of the library's host side: it loads, exports the header's
symbols, validates arguments, and its work lists cover every element once."""
import os
import re

import numpy as np
import pytest

import oracle.lqsgd_oracle as orc
from paper_2506_17974_amd import binding as B
from paper_2506_17974_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "lqsgd.h")) as fh:
        text = fh.read()
    declared = set(re.findall(r"\b(lqsgd_[a-z_]+)\s*\(", text))
    assert declared == set(B.SYMBOLS), declared ^ set(B.SYMBOLS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_kernel_names():
    names = [B.kernel_name(k) for k in range(B.KERNEL_COUNT)]
    assert all(names) and B.kernel_name(99) == ""


@pytest.mark.parametrize("kw,code", [
    (dict(rank=0), B.EINVAL), (dict(rank=65), B.EUNSUPPORTED), (dict(bits_p=9), B.EINVAL),
    (dict(bits_q=-1), B.EINVAL), (dict(workers=0), B.EINVAL), (dict(workers=65), B.EINVAL),
    (dict(alpha=0.0), B.EINVAL), (dict(alpha=float("nan")), B.EINVAL),
    (dict(layers=[(0, 4, 0)]), B.ESHAPE), (dict(layers=[(4, -1, 0)]), B.ESHAPE),
    (dict(layers=[(65536, 65536, 0)]), B.ESHAPE), (dict(layers=[(8, 2, B.LAYER_VECTOR)]), B.ESHAPE),
    (dict(layers=[(8, 2, 4)]), B.EINVAL), (dict(flags=16), B.EINVAL),
])
def test_plan_rejects_bad_arguments(kw, code):
    args = dict(layers=[(16, 8, 0)], rank=2, bits_p=8, bits_q=8, workers=2, alpha=255.0)
    args.update(kw)
    with pytest.raises(B.LqsgdError) as ei:
        B.plan_query(**args)
    assert ei.value.code == code


def _coverage(layers, rank, W, sweep):
    tiles = B.plan_tiles(layers, rank, 8, 8, W, sweep)
    cover = {}
    for gidx, w, row0, nrows, col0, ncols in tiles.tolist():
        rows, cols = layers[gidx][0], layers[gidx][1]
        assert 0 <= row0 and nrows > 0 and row0 + nrows <= rows
        assert 0 <= col0 and ncols > 0 and col0 + ncols <= cols
        m = cover.setdefault((gidx, w), np.zeros((rows, cols), np.int32))
        m[row0:row0 + nrows, col0:col0 + ncols] += 1
    return cover


@pytest.mark.parametrize("rank", [4, 16, 32])
@pytest.mark.parametrize("sweep", [0, 1, 2])
def test_work_lists_cover_each_element_once(sweep, rank):
    w = wl.small_cnn()
    layers = B.layer_list(w.layers, w.vectors)
    layers += [(1, 1, 0), (3, 5000, 0), (2100, 132, 0), (64, 27, 0)]
    W = 3
    cover = _coverage(layers, rank, W, sweep)
    n_matrix = sum(1 for l in layers if l[2] == 0)
    assert len(cover) == n_matrix * W
    for key, m in cover.items():
        assert m.min() == 1 and m.max() == 1, key


@pytest.mark.parametrize("rank", [4, 16, 32])
def test_ghat_pass_covers_each_layer_once(rank):
    w = wl.small_cnn()
    layers = B.layer_list(w.layers, w.vectors)
    layers += [(1, 1, 0), (3, 5000, 0), (2100, 132, 0), (64, 27, 0)]
    cover = _coverage(layers, rank, 3, 3)
    assert sorted(cover) == [(i, 0) for i, l in enumerate(layers) if l[2] == 0]
    for key, m in cover.items():
        assert m.min() == 1 and m.max() == 1, key
    rn = wl.resnet18()
    big = _coverage(B.layer_list(rn.layers, rn.vectors), rank, 8, 3)
    assert all(m.min() == 1 and m.max() == 1 for m in big.values())
    assert sum(m.size for m in big.values()) == rn.elements_per_worker


def test_plan_sizes_resnet18():
    w = wl.resnet18()
    info = B.plan_query(B.layer_list(w.layers, w.vectors), 4, 8, 8, 8)
    assert info.matrix_elements == w.elements_per_worker == 11164352
    assert info.n_matrix == 21 and info.n_vector == len(w.vectors) and info.rank_pad == 4
    # the library's wire size equals the oracle's count (Section 4.3 + sign plane + scales)
    assert info.wire_bytes == orc.wire_bytes(list(w.layers), 4, 8, 8)
    for r, bp, bq in ((1, 8, 8), (2, 4, 8), (7, 0, 3), (32, 2, 0)):
        info = B.plan_query(B.layer_list(w.layers), r, bp, bq, 2)
        assert info.wire_bytes == orc.wire_bytes(list(w.layers), r, bp, bq)
    # state + scratch stays close to the residual itself (4 B per element per worker)
    info = B.plan_query(B.layer_list(w.layers, w.vectors), 4, 8, 8, 8)
    assert info.device_bytes < 1.2 * 4 * 8 * w.elements_per_worker


def test_plan_sizes_large_configs():
    w3 = wl.llm_stack()
    info = B.plan_query(B.layer_list(w3.layers), 4, 8, 8, 4)
    assert info.matrix_elements == 5033164800
    assert info.device_bytes < 1.02 * 4 * 4 * info.matrix_elements
    w4 = wl.sweep_8192(32, 8)
    info = B.plan_query(B.layer_list(w4.layers), 32, 8, 8, 16)
    assert info.rank_pad == 32


def test_compressor_refuses_to_run_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    with pytest.raises(RuntimeError):
        B.Compressor([(4, 4, 0)], 1)


@pytest.mark.parametrize("flags", [0, B.FLAG_EAGER_RESIDUAL, B.FLAG_AGGREGATE_FIRST, B.FLAG_BF16_GRADIENTS,
                                   B.FLAG_NO_COOPERATIVE_LAUNCH,
                                   B.FLAG_EAGER_RESIDUAL | B.FLAG_AGGREGATE_FIRST | B.FLAG_BF16_GRADIENTS | B.FLAG_NO_COOPERATIVE_LAUNCH])
def test_plan_accepts_every_flag_combination(flags):
    w = wl.small_cnn()
    info = B.plan_query(B.layer_list(w.layers, w.vectors), 4, 8, 8, 4, flags=flags)
    assert info.n_matrix == 4 and info.n_vector == 4 and info.rank_pad == 4


@pytest.mark.parametrize("rank,pad", [(1, 1), (3, 4), (7, 8), (12, 16), (30, 32), (33, 64), (50, 64), (64, 64)])
def test_rank_pad(rank, pad):
    info = B.plan_query([(128, 256, 0)], rank, 8, 8, 2)
    assert info.rank_pad == pad
    # the pad follows the largest EFFECTIVE rank: a 10-row layer clips rank 50 to 10
    assert B.plan_query([(10, 256, 0)], 50, 8, 8, 2).rank_pad == 16


@pytest.mark.parametrize("rank", [40, 64])
@pytest.mark.parametrize("sweep", [0, 1, 2, 3])
def test_work_lists_cover_each_element_once_at_rank_pad_64(sweep, rank):
    layers = [(96, 520, 0), (129, 131, 0), (2100, 132, 0), (64, 27, 0), (7, 1, B.LAYER_VECTOR)]
    W = 2
    cover = _coverage(layers, rank, W, sweep)
    want = [(i, w) for i, l in enumerate(layers) if l[2] == 0 for w in range(1 if sweep == 3 else W)]
    assert sorted(cover) == want
    for key, m in cover.items():
        assert m.min() == 1 and m.max() == 1, key


def test_empty_layer_list_is_rejected_and_vector_only_is_planned():
    with pytest.raises(B.LqsgdError) as ei:
        B.plan_query([], 4, 8, 8, 2)
    assert ei.value.code == B.EINVAL
    info = B.plan_query([(7, 1, B.LAYER_VECTOR), (1000, 1, B.LAYER_VECTOR)], 4, 8, 8, 2)
    assert info.n_matrix == 0 and info.n_vector == 2 and list(info.tiles) == [0, 0, 0] and info.matrix_elements == 0


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 with pedantic warnings as errors,
    and a C program can link against the library and call a host-only entry point."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_lqsgd.c"
    src.write_text(
        '#include <stdio.h>\n#include "lqsgd.h"\n'
        "int main(void) {\n"
        "  lqsgd_config cfg = {4, 8, 8, 2, 255.0f, LQSGD_FLAG_NONE};\n"
        "  lqsgd_layer layers[2] = {{64, 576, LQSGD_LAYER_MATRIX}, {10, 1, LQSGD_LAYER_VECTOR}};\n"
        "  lqsgd_plan_info info;\n"
        "  int rc = lqsgd_plan_query(&cfg, layers, 2, &info);\n"
        '  printf("%d %d %d %lld\\n", rc, (int)info.n_matrix, (int)info.n_vector, (long long)info.matrix_elements);\n'
        "  return rc;\n}\n")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(root, "include"),
                    "-fsyntax-only", str(src)], check=True)
    exe = tmp_path / "use_lqsgd"
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-I", os.path.join(root, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-l:" + os.path.basename(B.LIB_PATH), "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert out == ["0", "1", "1", str(64 * 576)]
