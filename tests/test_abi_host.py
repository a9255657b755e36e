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
