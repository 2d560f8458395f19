"""The method's communication / memory accounting against the values the paper prints
(tests/golden/accounting.txt cites each)."""
import os

import pytest

from oracle import accounting as acc

GOLDEN = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "accounting.txt")) as fh:
    for line in fh:
        line = line.strip()
        if line and not line.startswith("#"):
            key, val = line.split()
            GOLDEN[key] = float(val)


def test_vit_and_gpt2_bits_per_token_and_ratios():
    full = acc.full_precision_bits_per_token(12, 768, 32)
    assert full == GOLDEN["vit_base_full_bits"]
    for g in (1, 16, 32):
        bits = acc.bits_per_token(12, g, 1024)
        assert bits == GOLDEN[f"vit_base_bits_G{g}"]
        assert acc.compression_ratio(full, bits) == pytest.approx(GOLDEN[f"vit_base_ratio_G{g}"], abs=0.05)
        assert acc.bits_per_token(24, g, 1024) == GOLDEN[f"gpt2m_bits_G{g}"]
    assert acc.compression_ratio(32 * 768, acc.bits_per_token(1, 1, 1024)) == pytest.approx(GOLDEN["single_block_ratio"])


def test_llama_bits_per_token_and_ratios():
    full = acc.full_precision_bits_per_token(32, 1024, 16, tensors_per_layer=2)
    assert full == GOLDEN["llama_full_bits"]
    for g in (1, 16, 32):
        bits = acc.bits_per_token(32, g, 1024, codebooks_per_layer=2)
        assert bits == GOLDEN[f"llama_bits_G{g}"]
        assert acc.compression_ratio(full, bits) == pytest.approx(GOLDEN[f"llama_ratio_G{g}"], abs=0.05)


def test_codebook_size_sweep_ratios():
    full = acc.full_precision_bits_per_token(12, 768, 32)
    for k in (256, 512, 1024, 2048):
        assert acc.compression_ratio(full, acc.bits_per_token(12, 32, k)) == pytest.approx(GOLDEN[f"ksweep_ratio_{k}"], abs=0.05)


def test_memory_worked_examples():
    assert acc.codebook_bytes(32, 2, 1024, 1024, 2) == GOLDEN["codebook_bytes_llama"]
    assert acc.kv_cache_bytes_original(1024, 32, 1024, 2) == GOLDEN["kv_orig_bytes_llama"]
    assert acc.kv_cache_bytes_astra(1024, 32, 1024, 2, 4, 32, 1024) == GOLDEN["kv_astra_bytes_llama"]


def test_fpar_closed_forms():
    assert acc.fpar([256] * 4) == GOLDEN["fpar_even4"]
    n = [100, 300, 424, 200]
    big_n, k = sum(n), len(n)
    mu = big_n / k
    var = sum((v - mu) ** 2 for v in n) / k
    assert var == pytest.approx(big_n ** 2 / k * (acc.fpar(n) - 1 / k))     # variance identity of the appendix


def test_fpar_is_the_fraction_of_same_device_pairs():
    import numpy as np
    n = [3, 5, 2, 6]
    owner = np.repeat(np.arange(len(n)), n)
    same = owner[:, None] == owner[None, :]          # the training mask of Eq. 1: full precision iff same device
    assert same.mean() == pytest.approx(acc.fpar(n))
