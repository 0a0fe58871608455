"""The byte model behind the reported GB/s, pinned to what the paper prints
(Sec. 5.2 Analysis: bandwidth ratio 8.0x / 12.8x / -> 16x; App. Inference-Kernel
Details, Table kernel-flops: R(N+M)/8 + 2(N+R+M) weight bytes per row;
Eq. (lordba-bits): R(N+M) + 16 l (N+R+M) bits)."""
import os

import pytest

from paper_2605_24058_amd import inputs

GOLD = os.path.join(os.path.dirname(__file__), "golden", "adapter_bandwidth_ratio.txt")


def _printed():
    rows = []
    with open(GOLD) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                r0, ratio = line.split()
                rows.append((int(r0), ratio))
    return rows


@pytest.mark.parametrize("N,M", [(4096, 4096), (4096, 11008), (5120, 13824)])
def test_bandwidth_ratio_matches_printed_values(N, M):
    for r0, printed in _printed():
        sh = inputs.Shape("x", 1, N, M, r0)
        lora_fp16_bytes = 2 * r0 * (N + M)
        assert "%.1f" % (lora_fp16_bytes / sh.adapter_bytes()) == printed
    big = inputs.Shape("x", 1, N, M, 1 << 20)
    assert abs(2 * big.r * (N + M) / big.adapter_bytes() - 16.0) < 0.05   # the limit also needs N + M >> 16


def test_adapter_bytes_is_storage_formula():
    for sh in [inputs.C1, inputs.C2, inputs.C3_UP, inputs.C3_DOWN, inputs.C5_Q, inputs.C5_UP, inputs.C5_DOWN] + inputs.C4:
        bits = sh.r * (sh.d_in + sh.d_out) + 16 * 1 * (sh.d_in + sh.r + sh.d_out)   # Eq. (lordba-bits), l = 1
        assert 8 * sh.adapter_bytes() == bits


def test_algorithmic_bytes_of_headline_config():
    sh = inputs.C2
    x = y_base = y_out = 2048 * 4096 * 2
    packed = 16 * 4096 // 8
    scales = 2 * (4096 + 16 + 4096)
    assert sh.algorithmic_bytes() == x + y_base + y_out + 2 * packed + scales == 50364448
    assert sh.sign_macs() == 2048 * 16 * 8192


def test_c5_adapter_set_enumeration():
    items = list(inputs.c5_adapter_seeds(0))
    assert len(items) == 280 and len({s for *_, s in items}) == 280
    assert sum(sh.algorithmic_bytes() for _, _, sh, _ in items) == 99001230080
