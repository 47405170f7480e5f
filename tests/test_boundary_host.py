"""Host-side checks of the C boundary that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching a device."""
import os
import re

import numpy as np
import pytest

from paper_2512_00719_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "simple_sample.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(simple_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(binding._lib, name) is not None


def test_version_and_error_strings():
    assert binding.simple_version() >= 100
    for code in (0, -1, -2, -3, -4):
        assert binding.simple_strerror(code) != "unknown error code"
    assert binding.simple_strerror(-99) == "unknown error code"


def test_struct_layouts_match_the_header():
    header = open(os.path.join(ROOT, "include", "simple_sample.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} simple_row_params;", header, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(float|int32_t)\s+(\w+);", body)
    assert [n for _, n in fields] == list(synth.ROW_PARAMS_DTYPE.names)
    for (ctype, name) in fields:
        assert synth.ROW_PARAMS_DTYPE[name] == (np.float32 if ctype == "float" else np.int32)
    assert synth.ROW_PARAMS_DTYPE.itemsize == 32 and binding.ROW_DIAG_DTYPE.itemsize == 32


def test_null_context_and_bad_arguments_are_rejected_on_the_host():
    # NULL context: rejected before any device work
    assert binding.simple_sample(0, 0, 1, 8, 0, 8, 0, 0, 0, 0, 0, 1, 0, 0, 0, 0) == binding.SIMPLE_EINVAL
    assert binding.simple_set_hot_set(0, 0, 4, 8) == binding.SIMPLE_EINVAL
    assert binding.simple_set_stats(0, 0) == binding.SIMPLE_EINVAL
    assert binding.simple_sample_hot_first(0, 0, 1, 4096, 0, 4096, 0, 1024, 0, 1, 0, 0, 0, 0) == binding.SIMPLE_EINVAL   # no tail statistics
    assert binding.simple_sample_hot_first(0, 0, 1, 4096, 0, 4096, 0, 0, 1, 1, 0, 0, 0, 0) == binding.SIMPLE_EINVAL      # H <= 0
    # logit constraints: sizes and pointer pairs are checked before anything is enqueued
    assert binding.simple_apply_logit_constraints(0, 1, 0, 0, 8, 0, 0, 0, 0, 0, 0, 8) == binding.SIMPLE_EINVAL
    assert binding.simple_apply_logit_constraints(0, 1, 8, 0, 8, 1, 0, 0, 0, 0, 0, 8) == binding.SIMPLE_EINVAL   # offsets without ids
    assert binding.simple_apply_logit_constraints(0, 1, 8, 0, 8, 0, 0, 0, 0, 0, 0, 4) == binding.SIMPLE_EINVAL   # output stride below V
    assert binding.simple_apply_logit_constraints(0, 0, 8, 0, 8, 0, 0, 0, 0, 0, 0, 8) == binding.SIMPLE_OK       # empty batch
    assert binding.simple_apply_logit_constraints(0, 1, 1 << 22, 0, 1 << 22, 0, 0, 0, 1, 1, 0, 1 << 22) == binding.SIMPLE_EINVAL  # NULL logits
    # incremental penalty state: NULL handles and sizes are rejected on the host
    assert binding.simple_state_restart(0, 0, 1, 0, 0, 0) == binding.SIMPLE_EINVAL
    assert binding.simple_state_append(0, 0, 0, 1) == binding.SIMPLE_EINVAL
    assert binding.simple_sample_state(0, 0, 0, 0, 1, 8, 0, 8, 0, 0, 0, 1, 0, 0, 0, 0) == binding.SIMPLE_EINVAL
    binding.simple_state_destroy(None)  # accepted
    with pytest.raises(binding.SimpleError) as e:
        binding.simple_state_create(0, 4, 1024, 70000)  # counts are 16-bit
    assert e.value.code == binding.SIMPLE_ECAPACITY
    with pytest.raises(binding.SimpleError) as e:
        binding.simple_state_create(0, 0, 1024, 16)
    assert e.value.code == binding.SIMPLE_EINVAL
    assert binding.simple_lds_bytes(0) == binding.SIMPLE_EINVAL
    binding.simple_destroy(None)  # accepted
    with pytest.raises(binding.SimpleError) as e:
        binding.simple_create(0, 16, 0, 0)  # max_V <= 0
    assert e.value.code == binding.SIMPLE_EINVAL
    with pytest.raises(binding.SimpleError) as e:
        binding.simple_create(0, 0, 1024, 0)  # max_B <= 0
    assert e.value.code == binding.SIMPLE_EINVAL
    with pytest.raises(binding.SimpleError) as e:
        binding.simple_create(0, 16, 1024, 70000)  # counts are 16-bit
    assert e.value.code == binding.SIMPLE_ECAPACITY
    with pytest.raises(binding.SimpleError):
        binding.simple_create(-1, 16, 1024, 0)
    # the entry point without a context: sizes beyond its static workspace, and a hot set by reference
    assert binding.simple_static_limit(0) == 2 ** 18 - 1 and binding.simple_static_limit(3) == 8 << 20
    assert binding.simple_static_limit(9) == binding.SIMPLE_EINVAL
    V = binding.simple_static_limit(0) + 1
    assert binding.simple_sample_static(0, 1, V, 0, V, 0, 0, 0, 0, 0, 1, 0, 0, 0, 0) == binding.SIMPLE_ECAPACITY
    assert binding.simple_sample_static(0, 1, 8, 0, 8, 0, 0, 0, 0, -1, 1, 0, 0, 0, 0) == binding.SIMPLE_EINVAL


def test_synthetic_configs_have_the_stated_shapes():
    w = synth.make_config(1)
    assert (w.B, w.V, w.dtype) == (4, 1024, "f32") and w.hist_ids.size == 4 * 64
    w = synth.make_config(3, B=16, V=4096, nnz=64)
    assert w.logits.dtype == np.float32 and set(np.unique(w.params["top_k"])) <= {0, 20, 50, 1000}
    assert w.hist_ptr[-1] == w.hist_ids.size == 16 * 64
    w = synth.make_config(4, B=8, V=4096, H=256)
    assert w.logits.dtype == np.uint16 and w.hot_ids.size == 256 and np.unique(w.hot_ids).size == 256
    # bf16 round trip: upcast of the stored bits is exact and within half a bf16 ulp of the source
    x = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    b = synth.f32_to_bf16_bits(x)
    y = synth.bf16_bits_to_f32(b)
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)
    # reproducible from the seed
    w2 = synth.make_config(4, B=8, V=4096, H=256)
    assert np.array_equal(w.logits, w2.logits) and np.array_equal(w.hot_ids, w2.hot_ids)
