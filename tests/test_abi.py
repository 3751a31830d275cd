"""The C-ABI library loads, exports every function include/spin.h declares, and
its host-side argument checks work without a GPU (no kernel is launched here)."""
import ctypes as C
import os
import re

import pytest

from paper_2604_26837_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for header in ("spin.h", "spin_measure.h"):        # the method's calls; the measurement aids
        txt = open(os.path.join(ROOT, "include", header)).read()
        txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
        names |= set(re.findall(r"\b(spin_[a-z_0-9]+)\s*\(", txt))
    return sorted(names)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(build.LIB_PATH):
        build.build_library()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert len(names) >= 17
    for n in names:
        assert hasattr(lib, n), n
    assert set(binding.EXPORTS) == set(names)


def test_create_validates_and_sizes(lib):
    sp = binding.Spin(max_batch=16, num_q_heads=32, num_kv_heads=8, topk=128, sink_pages=4, recent_pages=8,
                      max_context=32768)
    assert sp.sel_stride == 128 and sp.page_stride == 128 and sp.dir_stride == 4
    assert sp.decode_splits == 2
    assert sp.workspace_bytes % 256 == 0 and sp.workspace_bytes > 0
    assert sp.summary_bytes(2048 * 16) == 2048 * 16 * 8 * 512
    # block partitions: 32 blocks on top of the forced ones, 8 pages each plus stand-alone forced pages
    sp3 = binding.Spin(max_batch=4, num_q_heads=32, num_kv_heads=8, partition_tokens=128, score_kind=2, topk=32,
                       topk_includes_forced=0, sink_pages=4, recent_pages=64, max_context=131072)
    assert sp3.sel_stride == 32 + 1 + 8 + 1 and sp3.page_stride == 42 * 8 + 68 and sp3.dir_stride == 16
    for bad in (dict(head_dim=64), dict(page_tokens=8), dict(partition_tokens=24), dict(num_q_heads=33),
                dict(num_q_heads=8 * 17), dict(score_kind=7), dict(decode_waves=3), dict(topk=-1)):
        cfg = dict(max_batch=1, num_q_heads=32, num_kv_heads=8, topk=8, max_context=1024)
        cfg.update(bad)
        with pytest.raises(binding.SpinError):
            binding.Spin(**cfg)


def test_stage_calls_reject_bad_arguments_before_launching(lib):
    sp = binding.Spin(max_batch=2, num_q_heads=8, num_kv_heads=2, topk=8, max_context=1024)
    h = sp.h
    null = None
    assert lib.spin_sparse_decode(h, 3, null, null, 1, null, null, null, null, null, null, null) == -1   # batch > max
    assert lib.spin_sparse_decode(h, 1, null, null, 1, null, null, null, null, null, null, null) == -1   # NULL pointers
    assert lib.spin_sparse_decode(h, 0, null, null, 1, null, null, null, null, null, null, null) == 0    # empty batch
    assert lib.spin_score_partitions(h, 1, null, null, null, null, null, null, null, null) == -1
    assert lib.spin_select_topk(h, 1, null, null, null, null, null, null, null) == -1
    assert lib.spin_workspace_init(h, null, null) == -3
    assert lib.spin_status_string(-5) == b"slot budget smaller than the step's selection"
    assert lib.spin_profile_enable(h, -1) == -1


def test_static_scratch_entry_point_refuses_shapes_beyond_its_array(lib):
    """spin_sparse_decode_static checks the scratch it needs against the fixed device array before any HIP call."""
    sp = binding.Spin(max_batch=64, num_q_heads=32, num_kv_heads=8, topk=128, max_context=32768, decode_splits=8)
    fake = 4096   # never dereferenced: the call returns before anything is launched
    big = lib.spin_sparse_decode_static(sp.h, 64, fake, fake, 1, fake, fake, fake, fake, None, None, None)
    assert big == -9 and lib.spin_status_string(big).startswith(b"shape needs more scratch")
    assert lib.spin_sparse_decode_static(sp.h, 65, fake, fake, 1, fake, fake, fake, fake, None, None, None) == -1
    assert lib.spin_sparse_decode_static(sp.h, 0, None, None, 1, None, None, None, None, None, None, None) == 0
    assert lib.spin_sparse_decode_static(sp.h, 1, None, fake, 1, fake, fake, fake, fake, None, None, None) == -1


def test_unsupported_combinations_are_refused_on_the_host(lib):
    """Refusals that need no GPU: partition tables on a context not sized for them, the calls that cannot follow
    tables, a key sketch with partitions other than one token, budget-mode shapes whose LDS need is too large."""
    fake = 4096   # never dereferenced: every call below returns before anything is launched
    base = dict(max_batch=2, num_q_heads=8, num_kv_heads=2, topk=8, max_context=4096, partition_tokens=64)
    uniform = binding.Spin(**base)
    assert lib.spin_set_partition_tables(uniform.h, fake, fake, fake, fake) == -2
    var = binding.Spin(variable_partitions=1, **base)
    assert lib.spin_set_partition_tables(var.h, fake, fake, fake, fake) == 0
    i64 = C.c_int64
    assert lib.spin_append_kv(var.h, 1, fake, fake, fake, fake, i64(8), fake, fake, i64(1), fake, None, fake, fake, None) == -2
    assert lib.spin_alloc_leaves(var.h, 1, fake, fake, fake, fake, fake, i64(4), fake, fake, None) == -2
    assert lib.spin_set_partition_tables(var.h, None, None, None, None) == 0
    with pytest.raises(binding.SpinError, match="UNSUPPORTED"):
        binding.Spin(max_batch=1, num_q_heads=8, num_kv_heads=2, topk=8, max_context=1024, score_kind=1,
                     partition_tokens=16)
    binding.Spin(max_batch=1, num_q_heads=8, num_kv_heads=2, topk=8, max_context=1024, score_kind=1, partition_tokens=1)

    def budget_call(sp):
        return lib.spin_resolve_slots(sp.h, 1, 0, fake, fake, fake, fake, fake, i64(4), fake, fake, fake, fake, fake,
                                      fake, fake, fake, fake, fake, None)
    big = dict(max_batch=1, num_q_heads=8, num_kv_heads=2, max_context=1 << 20, lru_timestamps=64)
    # bucketed LRU: 8 bytes per output entry + one byte per slot must fit in 60 KiB with slots >= entries
    assert binding.Spin(topk=7000, **big).page_stride == 7000
    assert budget_call(binding.Spin(topk=7000, **big)) == -2
    # set-associative: 16 bytes per output entry + 13/8 bytes per slot
    assert budget_call(binding.Spin(topk=3500, lru_policy=1, **big)) == -2


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(build, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load_library()


def test_header_is_plain_c(tmp_path):
    """include/spin.h must compile as C99 with no extensions: the boundary is a C ABI."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_spin.c"
    src.write_text('#include "spin.h"\n#include "spin_measure.h"\nint main(void) { spin_config c; (void)c; return spin_status_string(0) == 0; }\n')
    res = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                          "-c", str(src), "-o", str(tmp_path / "use_spin.o")], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only and says so (no collective is involved in this path)."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""

