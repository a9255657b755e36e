"""The C boundary without a GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments on the host before anything touches a device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2605_06472_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in os.listdir(inc):
        if f.endswith(".h"):
            text = open(os.path.join(inc, f)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names.update(re.findall(r"\b(pbkv_[a-z_0-9]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    declared = _declared_symbols()
    assert {"pbkv_prefix_prefill", "pbkv_append_kv", "pbkv_swap_in_pages"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    assert binding.version().startswith("pbkv")


def _shape(**kw):
    base = dict(batch=1, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
                num_pages=64, max_pages_per_req=8, dtype="bf16")
    base.update(kw)
    return binding.make_shape(**base)


def test_page_bytes():
    assert binding.page_bytes(_shape()) == 65536
    assert binding.page_bytes(_shape(num_q_heads=2, num_kv_heads=1, head_dim=64, dtype="f32")) == 8192
    assert binding.page_bytes(_shape(page_size=32)) == 0


FAKE = 0x1000   # never dereferenced: the calls below fail on the host first


def _prefill(shape, pl, nl, q=FAKE):
    binding.prefix_prefill(shape, q, FAKE, FAKE, FAKE, FAKE, np.array(pl, np.int32),
                           np.array(nl, np.int32), FAKE, stream=0)


@pytest.mark.parametrize("kw,code", [
    (dict(page_size=32), -2), (dict(head_dim=96), -2), (dict(num_q_heads=30), -2),
    (dict(num_q_heads=24), -2), (dict(dtype=7), -3), (dict(num_pages=0), -2),
])
def test_prefill_rejects_bad_shapes(kw, code):
    with pytest.raises(binding.PbkvError) as e:
        _prefill(_shape(**kw), [16], [16])
    assert e.value.code == code
    assert str(e.value)


def test_prefill_rejects_null_and_ranges():
    with pytest.raises(binding.PbkvError) as e:
        _prefill(_shape(), [16], [16], q=None)
    assert e.value.code == -1
    with pytest.raises(binding.PbkvError) as e:
        _prefill(_shape(), [-1], [16])
    assert e.value.code == -4
    with pytest.raises(binding.PbkvError) as e:
        _prefill(_shape(), [100], [29])          # 129 tokens need 9 pages, table holds 8
    assert e.value.code == -4
    with pytest.raises(binding.PbkvError) as e:
        _prefill(_shape(), [16], [16], q=FAKE + 2)   # misaligned
    assert e.value.code == -2


def test_empty_batches_are_noops():
    _prefill(_shape(batch=0), [], [])
    _prefill(_shape(batch=2), [5, 0], [0, 0])
    binding.append_kv(_shape(batch=2), FAKE, FAKE, FAKE, FAKE, np.array([5, 0], np.int32),
                      np.array([0, 0], np.int32), stream=0)
    binding.swap_in_pages(_shape(), FAKE, np.zeros(0, np.int32), FAKE, stream=0)


def test_swap_in_rejects_bad_page_ids():
    with pytest.raises(binding.PbkvError) as e:
        binding.swap_in_pages(_shape(), FAKE, np.array([1, 64], np.int32), FAKE, stream=0)
    assert e.value.code == -4
    with pytest.raises(binding.PbkvError) as e:
        binding.swap_in_pages(_shape(), FAKE, np.array([3, 5, 3], np.int32), FAKE, stream=0)
    assert e.value.code == -5
    with pytest.raises(binding.PbkvError) as e:
        binding.swap_in_pages(_shape(), None, np.array([3], np.int32), FAKE, stream=0)
    assert e.value.code == -1


def test_pointer_kind_is_checked_before_any_launch():
    """A well-formed call with pointers that are not device memory fails with
    PBKV_ERR_DEVICE on the host (with or without a GPU present); nothing is launched."""
    with pytest.raises(binding.PbkvError) as e:
        _prefill(_shape(), [16], [16])
    assert e.value.code == -6
    buf = np.zeros(65536, np.uint8)            # pageable host memory is not acceptable
    addr = (buf.ctypes.data + 15) & ~15
    with pytest.raises(binding.PbkvError) as e:
        binding.swap_in_pages(_shape(), addr, np.array([3], np.int32), FAKE, stream=0)
    assert e.value.code == -6


# ---- predictor boundary (pbkv_predictor.h): host-side validation -------------------------------
def test_predictor_workspace_size_and_bad_shapes():
    from paper_2605_06472_amd import predictor as PR
    good = PR.make_shape(8, 64, 5120, 64, 3, 16)
    n = PR.predictor_workspace_bytes(good, 1024)
    # W_t twice in bf16 + the partial sums of 16 slices dominate
    assert n >= 2 * 64 * 5120 * 2 + 16 * 1024 * 64 * 4 and n % 256 == 0
    assert PR.predictor_workspace_bytes(good, 1) < n
    for bad in [PR.make_shape(0, 64, 5120, 64, 3, 16), PR.make_shape(65, 64, 5120, 64, 3, 16),
                PR.make_shape(8, 48, 5120, 64, 3, 16), PR.make_shape(8, 64, 5000, 64, 3, 16),
                PR.make_shape(8, 64, 32, 64, 3, 16), PR.make_shape(8, 64, 5120, 0, 3, 16),
                PR.make_shape(8, 64, 5120, 257, 3, 16), PR.make_shape(8, 64, 5120, 64, 9, 16),
                PR.make_shape(8, 64, 5120, 64, 3, 65)]:
        with pytest.raises(binding.PbkvError) as e:
            PR.predictor_workspace_bytes(bad, 16)
        assert e.value.code == -2 and str(e.value)
    with pytest.raises(binding.PbkvError) as e:
        PR.predictor_workspace_bytes(good, 0)
    assert e.value.code == -4


def test_predictor_calls_reject_bad_arguments_on_the_host():
    from paper_2605_06472_amd import predictor as PR
    good = PR.make_shape(8, 64, 5120, 64, 3, 16)
    n = PR.predictor_workspace_bytes(good, 64)
    w = {k: FAKE for k in PR.WEIGHT_NAMES}
    with pytest.raises(binding.PbkvError) as e:
        PR.predictor_prepare(good, w, FAKE, n - 1, 64, stream=0)            # workspace too small
    assert e.value.code == -4
    with pytest.raises(binding.PbkvError) as e:
        PR.predictor_prepare(good, w, None, n, 64, stream=0)
    assert e.value.code == -1
    with pytest.raises(binding.PbkvError) as e:
        PR.predictor_prepare(good, w, FAKE + 16, n, 64, stream=0)           # not 256-byte aligned
    assert e.value.code == -2
    with pytest.raises(binding.PbkvError) as e:
        PR.predictor_forward(good, FAKE, n, 64, FAKE, FAKE, FAKE, FAKE, 65, FAKE, stream=0)   # batch > max_batch
    assert e.value.code == -4
    with pytest.raises(binding.PbkvError) as e:
        PR.predictor_forward(good, FAKE, n, 64, FAKE, FAKE, FAKE, FAKE, -1, FAKE, stream=0)
    assert e.value.code == -4
    with pytest.raises(binding.PbkvError) as e:
        PR.predictor_forward(PR.make_shape(8, 64, 5120, 64, 3, 99), FAKE, n, 64, FAKE, FAKE, FAKE, FAKE, 1, FAKE, stream=0)
    assert e.value.code == -2


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; asking bench.py for more ends with a message and a non-zero status
    before anything touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_work_group_shape_follows_the_batch():
    """The bf16 attention kernel runs as four waves of 32 rows (32-token units) when the batch's 64-token
    blocks average fewer than 100 tile steps, else as four waves of 64 rows (64-token units); the size
    query of the gather diagnostic reports the unit the attention call will use, without touching a device."""
    binding.set_attn_waves(0)

    def units(batch, prefix, new, max_pages):
        shape = _shape(batch=batch, num_pages=4 * max_pages, max_pages_per_req=max_pages)
        return binding.gather_probe(shape, FAKE, FAKE, FAKE, FAKE, np.full(batch, prefix, np.int32),
                                    np.full(batch, new, np.int32), None, stream=0)

    n, tok = units(4, 2048, 512, 160)                 # the benchmark batch: 34-42 steps per block
    assert tok == 32 and n == 4 * 16 * 8
    n, tok = units(4, 32768, 2048, 2200)              # long histories: > 500 steps per block
    assert tok == 64 and n == 4 * 32 * 8
    n, tok = units(2, 6208, 64, 400)                  # 99 steps: just below the switch
    assert tok == 32
    n, tok = units(2, 6272, 64, 400)                  # 100 steps
    assert tok == 64
    try:
        binding.set_attn_waves(8)
        assert units(4, 2048, 512, 160)[1] == 64
        binding.set_attn_waves(4)
        assert units(4, 32768, 2048, 2200)[1] == 32
        binding.set_attn_waves(64)
        assert units(4, 2048, 512, 160)[1] == 64
        with pytest.raises(binding.PbkvError) as e:
            binding.set_attn_waves(6)
        assert e.value.code == -2
    finally:
        binding.set_attn_waves(0)
