"""CPU-only checks of the boundary: the library loads, exports every symbol the
header declares, and the host-side argument checks work without a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "zeno.h")


@pytest.fixture(scope="module")
def B():
    from paper_1805_10032_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_1805_10032_amd import build
        build.build(verbose=False)
    binding.load_library()
    return binding


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zeno_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(B):
    names = _declared_functions()
    assert {"zeno_score", "zeno_aggregate", "zeno_mean", "zeno_median", "zeno_model_create"} <= set(names)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_model_create_validates(B):
    m = B.ZenoModel([3072, 512, 10], True, "softmax_ce", "fp32")
    assert m.num_params == 3072 * 512 + 512 + 512 * 10 + 10
    assert B.ZenoModel([64, 1], False, "squared", "fp32").num_params == 64
    assert B.ZenoModel([4096, 4096, 4096, 4096, 1000], True, "softmax_ce", "bf16").num_params == 54440936
    with pytest.raises(B.ZenoError):
        B.ZenoModel([4, 3], True, "squared", "fp32")          # squared loss needs width 1
    with pytest.raises(B.ZenoError):
        B.ZenoModel([4, 0, 3], True, "softmax_ce", "fp32")
    with pytest.raises(B.ZenoError):
        B.ZenoModel([4] * 11, True, "softmax_ce", "fp32")     # more than 8 layers


def test_workspace_query(B):
    m = B.ZenoModel([784, 10], True, "softmax_ce", "fp32")
    assert m.workspace_bytes(20, 32) > 0
    assert m.workspace_bytes(20, 32) % 256 == 0
    assert m.workspace_bytes(0, 32) == 0 and m.workspace_bytes(2000, 32) == 0 and m.workspace_bytes(20, 0) == 0
    big = B.ZenoModel([4096, 4096, 4096, 4096, 1000], True, "softmax_ce", "bf16")
    assert big.workspace_bytes(64, 128) < 1 << 30


def test_null_pointers_are_rejected_on_the_host(B):
    lib = B.load_library()
    assert lib.zeno_aggregate(None, 8, None, 4, 8, 1, None, None, None) == 1
    assert lib.zeno_mean(None, 8, 4, 8, None, None) == 1
    assert lib.zeno_median(None, 8, 4, 8, None, None) == 1
    assert lib.zeno_score(None, None, None, 8, 4, None, 0.1, 0.1, None, None, 0, None) == 1
    assert lib.zeno_status_string(0) == b"ok"
    assert lib.zeno_profile_collect(None, 0) == 0


def test_missing_library_fails_loudly(B, tmp_path):
    saved = B._lib
    B._lib = None
    try:
        with pytest.raises(FileNotFoundError):
            B.load_library(str(tmp_path / "nope.so"))
    finally:
        B._lib = saved


PLAN_SHAPES = [
    # dims, fwd
    ([3072, 2048, 2048, 10], "bf16"),          # a ten-class layer behind wide hidden layers
    ([3072, 2048, 2048, 10], "fp32"),
    ([4096, 4096, 4096, 4096, 1000], "bf16"),
    ([3072, 2048, 2048, 2048, 10], "bf16"),
    ([3072, 512, 10], "fp32"),
    ([784, 10], "fp32"),
    ([64, 1], "fp32"),
    ([300, 129, 65, 33, 7], "bf16"),           # widths that are not multiples of 32/64/128/256
    ([300, 129, 65, 33, 7], "fp32"),
    ([1024, 257, 385, 3], "bf16"),
    ([64, 128, 64, 32, 16, 8, 4, 3, 2], "fp32"),
]


@pytest.mark.parametrize("dims,fwd", PLAN_SHAPES)
def test_every_launch_stays_inside_its_workspace_slot(B, dims, fwd):
    """Host-only walk over the launch sequence of zeno_score: whatever workgroup width a launch takes
    (one, four or eight waves), the rows of W it copies in operand order, the activations, the
    pre-activations and the partial norms it writes lie inside their workspace slots."""
    loss = "squared" if dims[-1] == 1 else "softmax_ce"
    mdl = B.ZenoModel(dims, True, loss, fwd)
    for m in (1, 7, 60, 64, 100, 1024):
        for n_r in (1, 32, 33, 64, 128, 300):
            assert mdl.plan_check(m, n_r) == 0, (dims, fwd, m, n_r)
    assert mdl.plan_check(0, 4) == 1 and mdl.plan_check(4, 0) == 1


def test_library_sources_never_allocate_device_memory():
    """Every entry point runs on memory the caller hands over (or, for zeno_score_static, on the
    library's static device array): no source of the library calls a HIP allocation routine."""
    csrc = os.path.join(ROOT, "paper_1805_10032_amd", "csrc")
    pat = re.compile(r"\bhip(Malloc\w*|Free\w*|HostMalloc|HostAlloc|ExtMallocWithFlags|MemPool\w*)\s*\(")
    for name in sorted(os.listdir(csrc)):
        text = open(os.path.join(csrc, name)).read()
        text = re.sub(r"//[^\n]*|/\*.*?\*/", "", text, flags=re.S)
        assert not pat.search(text), name
