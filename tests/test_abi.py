"""The C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2601_08743_amd", "libtablecache.so")


def _declared():
    src = open(os.path.join(ROOT, "include", "tablecache.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(tc_[a-z_0-9]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_four_path_calls():
    d = _declared()
    for name in ("tc_register_table_kv", "tc_stitch_kv", "tc_prefill_attn", "tc_load_async"):
        assert name in d


def test_every_declared_symbol_is_exported(lib):
    for name in _declared():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_names(lib):
    from paper_2601_08743_amd import binding
    assert sorted(binding.EXPORTS) == _declared()


def test_size_helpers_are_pure_host_functions(lib):
    from paper_2601_08743_amd import binding as B
    cfg = B.make_config(28, 28, 4, 128, B.TC_BF16, 4000, 40, 600)
    assert B.tc_block_bytes(cfg) == 2 * 4 * 16 * 128 * 2
    assert B.tc_pool_bytes(cfg) == 28 * 4000 * 32768
    assert B.tc_first_seq_block(cfg) == 40 * 38
    bad = B.make_config(28, 28, 5, 128, B.TC_BF16, 4000, 40, 600)       # Hq % Hkv != 0
    assert B.tc_pool_bytes(bad) == 0 and B.tc_first_seq_block(bad) == -1
    bad = B.make_config(28, 28, 4, 64, B.TC_BF16, 4000, 40, 600)        # bf16 needs D = 128
    assert B.tc_pool_bytes(bad) == 0
    bad = B.make_config(1, 8, 2, 64, B.TC_F32, 10, 4, 600)              # slots do not fit the pool
    assert B.tc_pool_bytes(bad) == 0
    assert "gfx950" in B.tc_version()


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message (nothing here uses a second GPU)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr


def test_binding_shares_the_hip_runtime_with_torch():
    """Importing the binding in a fresh interpreter, before anything else, must leave exactly one
    HIP runtime mapped into the process: the one torch ships.  (Loaded ahead of torch, the library
    would bring in the system's copy, and with two runtimes the second sees no device.)"""
    import subprocess
    import sys
    code = ("import paper_2601_08743_amd.binding, torch, os\n"
            "maps = {l.split()[-1] for l in open('/proc/self/maps') if 'libamdhip64' in l}\n"
            "print(sorted(maps))\n"
            "assert len(maps) == 1, maps\n"
            "assert os.path.dirname(torch.__file__) in next(iter(maps)), maps\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
