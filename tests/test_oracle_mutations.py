"""The pins must notice a mistake: build copies of the oracle with one planted error
each (on the CPU, in a temp dir) and check that the pin suite rejects every one."""
import os
import subprocess

import numpy as np
import pytest

from paper_2605_06472_amd import workloads as W
from tests import bruteforce

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "pbkv_oracle.c")

MUTATIONS = {
    "dropped_scale": ("s[t] = dot * scale;", "s[t] = dot;"),
    "diagonal_masked": ("const int64_t L = p + i + 1;", "const int64_t L = p + i > 0 ? p + i : 1;"),
    "gqa_interleaved": ("const int g = h / G;", "const int g = h % Hkv;"),
    "values_from_keys": ("vidx = (((pg * 2 + 1) * Hkv + g) * P + t % P) * d;",
                         "vidx = (((pg * 2 + 0) * Hkv + g) * P + t % P) * d;"),
    "slot_reversed": ("kidx = (((pg * 2 + 0) * Hkv + g) * P + t % P) * d;",
                      "kidx = (((pg * 2 + 0) * Hkv + g) * P + (P - 1 - t % P)) * d;"),
    "head_and_slot_transposed": ("vidx = (((pg * 2 + 1) * Hkv + g) * P + t % P) * d;",
                                 "vidx = (((pg * 2 + 1) * P + t % P) * Hkv + g) * d;"),
    "suffix_offset_dropped": ("kidx = ((off[r] + (t - p)) * Hkv + g) * d;",
                              "kidx = (((t - p)) * Hkv + g) * d;"),
    "no_max_subtraction_sign": ("const double w = exp(s[t] - m);", "const double w = exp(m - s[t]);"),
    "append_wrong_slot": ("+ pos % P) * rowb;", "+ t % P) * rowb;"),
    "swap_in_wrong_source": ("(const char *)host_pages + (size_t)i * (size_t)page_bytes",
                             "(const char *)host_pages + (size_t)(n_pages - 1 - i) * (size_t)page_bytes"),
    "swap_out_wrong_page": ("(const char *)kv_pool + (size_t)page_ids[i] * (size_t)page_bytes",
                            "(const char *)kv_pool + (size_t)i * (size_t)page_bytes"),
}


def _pins_pass(oracle) -> bool:
    try:
        for b in (W.ragged_small(3, "bf16"), W.ragged_small(4, "f32", Hq=6, Hkv=3, d=64)):
            out = oracle.prefill(b.q, b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)
            ref, _ = bruteforce.attention(b)
            if not np.allclose(out, ref, rtol=0, atol=1e-12):
                return False
            got = oracle.append_kv(b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)
            want = b.kv_pool.copy()
            off = 0
            for r in range(b.B):
                pos = int(b.prefix_lens[r]) + np.arange(int(b.new_lens[r]))
                pg = b.block_table[r, pos // b.P]
                want[pg, 0, :, pos % b.P] = b.k_new[off:off + len(pos)]
                want[pg, 1, :, pos % b.P] = b.v_new[off:off + len(pos)]
                off += len(pos)
            if not np.array_equal(got, want):
                return False
        b = W.ragged_small(32, "bf16", Hq=4, Hkv=2, d=64, prefix_lens=(48, 100), new_lens=(3, 9),
                           nonresident=(2, 5))
        want = b.kv_pool.copy()
        want[b.swap_page_ids] = b.host_pages
        if not np.array_equal(oracle.swap_in(b.host_pages, b.swap_page_ids, b.kv_pool), want):
            return False
        ids = np.array([5, 0, 17, 5], np.int32)
        return bool(np.array_equal(oracle.swap_out(b.kv_pool, ids), b.kv_pool[ids]))
    except (ValueError, FloatingPointError):
        return False


def test_unmutated_oracle_passes(oracle):
    assert _pins_pass(oracle)


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(oracle, name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, "mutation anchor must be unique: %r" % old
    mutated = tmp_path / "mut.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "libmut.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", str(mutated),
                    "-o", str(lib), "-lm"], check=True)
    monkeypatch.setattr(oracle, "_LIB", oracle._bind(str(lib)))
    assert not _pins_pass(oracle)
