"""Host-side contracts that need no GPU: bench.py refuses more than one GPU with a message, the
product path fails loudly without the built library, nothing in the product path reaches for the
oracle, and argument checks of the C ABI that return before any device work."""
import ctypes
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr or "--gpus 1" in res.stderr
    assert res.stdout.strip() == ""                       # no JSON line for a run that did not happen


def test_bench_refuses_a_multi_rank_launch():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0")
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True,
                         timeout=120, env=env)
    assert res.returncode != 0 and res.stdout.strip() == ""


def test_product_path_never_mentions_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_07239_amd")
    for base, _, files in os.walk(pkg):
        if "_build" in base or "__pycache__" in base:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(base, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
    text = open(os.path.join(ROOT, "include", "comet_ring.h")).read()
    assert "oracle" not in text.lower()


def test_missing_library_raises(monkeypatch, tmp_path):
    import paper_2505_07239_amd.binding as binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libcomet_ring.so"))
    with pytest.raises(FileNotFoundError):
        binding.load_library()


def test_null_context_is_rejected_without_touching_a_device():
    lib_path = os.path.join(ROOT, "paper_2505_07239_amd", "libcomet_ring.so")
    if not os.path.exists(lib_path):
        pytest.skip("library not built")
    lib = ctypes.CDLL(lib_path)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    lib.comet_mask_share.argtypes = [vp, vp, vp, vp, sz]
    lib.comet_truncate_share.argtypes = [vp, i32, vp, vp, sz, i32]
    lib.comet_permute_mask.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32]
    assert lib.comet_mask_share(None, None, None, None, 16) == -1          # COMET_EINVAL
    assert lib.comet_truncate_share(None, 0, None, None, 16, 16) == -1
    assert lib.comet_permute_mask(None, None, None, None, None, 4, 4, 0, 1) == -1


def test_device_side_stream_equals_the_host_stream():
    """bench.py draws its large inputs with torch on the device; the words must be the ones the
    tests draw on the host from the same (seed, stream, index)."""
    import numpy as np
    torch = pytest.importorskip("torch")
    from workloads import rng
    for seed, stream, n, off in ((rng.BASE_SEED, 300005, 4099, 0), (1, 99999, 77, 12345),
                                 (rng.BASE_SEED, 7, 5, 1 << 40)):
        host = rng.uniform_u64(seed, stream, n, off)
        dev = rng.uniform_u64_torch(seed, stream, n, "cpu", off).numpy().view(np.uint64)
        assert np.array_equal(host, dev)
