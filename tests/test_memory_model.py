"""The paper's memory model (Appendix "Memory savings") against the terms it
is built from and against this library's own layout arithmetic."""
import os

GOLD = os.path.join(os.path.dirname(__file__), "golden", "memory_model.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def test_paper_constants_follow_from_the_listed_tensors():
    g = _gold()
    m = 1024
    per_d_fp32 = (4 * m + 4 * m) / 100 + 4 + 4          # I, V (k = d/100), xi, r_d
    per_d_bf16 = (4 * m + 2 * m) / 100 + 4 + 4
    assert abs(per_d_fp32 - g["sparse_fp32_bytes_per_d"]) < 1e-9
    assert abs(per_d_bf16 - g["sparse_bf16_bytes_per_d"]) < 1e-9
    assert g["dense_bytes_per_d"] == 4 * m
    assert abs(g["dense_bytes_per_d"] / 90 - g["saving_fp32"]) < 0.05     # the paper rounds 89.92 to 90
    assert abs(g["dense_bytes_per_d"] / 70 - g["saving_bf16"]) < 0.05


def test_ring_of_the_largest_workloads_needs_64_bit_offsets():
    from paper_2306_06098_amd import synth
    wl = synth.WORKLOADS["bert_large"]
    assert wl.m * wl.k > 2 ** 31                 # element offsets overflow int32
    assert wl.m * wl.k * 4 > 2 ** 32             # byte offsets overflow uint32
    wl = synth.WORKLOADS["bert_base"]
    assert abs(8 * wl.m * wl.k / 1e9 - 9.01) < 0.01      # "ring buffer ~9 GB"
