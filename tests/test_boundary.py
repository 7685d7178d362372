"""The C-ABI library loads and exports every symbol that include/lgc.h declares; host-side
argument checks that need no GPU.  CPU only (no kernel is launched)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2103_08870_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lgc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lgc_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2103_08870_amd import binding
    names = declared_symbols()
    assert len(names) >= 16
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == names          # the binding covers the header, name for name


def test_status_strings(lib):
    assert lib.lgc_status_string(0) == b"ok"
    assert lib.lgc_status_string(1) == b"invalid argument"


def test_null_context_is_rejected_without_touching_a_device(lib):
    from paper_2103_08870_amd import binding
    assert lib.lgc_accumulate(None, None, None, None, 10, 1, 10, 0.9, None) == binding.LGC_EINVAL
    assert b"ctx" in lib.lgc_last_error(None)
    assert lib.lgc_topk(None, None, None, 10, 1, 10, 1, None, None, None) == binding.LGC_EINVAL
    assert lib.lgc_scatter(None, None, None, 1, 1, 1.0, None, 10, None) == binding.LGC_EINVAL
    assert lib.lgc_encode(None, None, None, 1, 1, None, None) == binding.LGC_EINVAL
    assert lib.lgc_set_option(None, 0, 0) == binding.LGC_EINVAL
    assert lib.lgc_latent_len(None, 100) == 0
    # the entry points of the per-layer, ring-allreduce and parameter-server forms
    assert lib.lgc_topk_segmented(None, None, None, None, 1, 10, None, None, None) == binding.LGC_EINVAL
    assert lib.lgc_accumulate_topk_segmented(None, None, None, None, None, 1, 10, 0.9, None, None, None) == binding.LGC_EINVAL
    assert lib.lgc_gather(None, None, None, 10, 1, 10, None, 1, None, None) == binding.LGC_EINVAL
    assert lib.lgc_accumulate_gather(None, None, None, None, 10, 1, 10, 0.9, None, 1, None, None) == binding.LGC_EINVAL
    assert lib.lgc_average(None, None, 10, 1, 0.5, None, None) == binding.LGC_EINVAL
    assert lib.lgc_innovation(None, None, None, 1, None, None) == binding.LGC_EINVAL
    assert lib.lgc_decode_innovation(None, None, None, None, 1, 1, None, None) == binding.LGC_EINVAL
    assert lib.lgc_segments_total_k(None) == 0
    assert lib.lgc_reserve(None, None, 0, 1, None) == binding.LGC_EINVAL
    h = C.c_void_p()
    assert lib.lgc_segments_create(C.byref(h), 0, 10, 1, None, None) == binding.LGC_EINVAL and not h.value


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_create_argument_checks(lib):
    from paper_2103_08870_amd import binding
    h = C.c_void_p()
    assert lib.lgc_create(None, 0, 10, 1, 1) == binding.LGC_EINVAL
    assert lib.lgc_create(C.byref(h), 0, 0, 0, 1) == binding.LGC_EINVAL
    assert lib.lgc_create(C.byref(h), 0, 1 << 31, 1, 1) == binding.LGC_EINVAL
    assert lib.lgc_create(C.byref(h), 0, 100, 101, 1) == binding.LGC_EINVAL
    assert lib.lgc_create(C.byref(h), 0, 100, 10, 0) == binding.LGC_EINVAL
    assert not h.value
    ah = C.c_void_p()
    assert lib.lgc_ae_create(C.byref(ah), 0, 0, None, 0, None, 0.0, None, None, None, None) == binding.LGC_EINVAL


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_2103_08870_amd import binding
    with pytest.raises(ValueError):
        binding._ptr(torch.zeros(4))
