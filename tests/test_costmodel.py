"""The cost calculator against the numbers Appendix C prints."""
import os

from paper_1705_09786_amd import costmodel


def golden():
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "appendix_c.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def test_appendix_c_numbers():
    g = golden()
    r = costmodel.appendix_c(int(g["H"]), int(g["N"]), int(g["E"]), int(g["C"]), int(g["steps"]),
                             g["device_flops"], g["overhead"])
    nh2 = g["N"] * g["H"] ** 2
    assert r["ops_per_sample"] == g["ops_per_sample_in_NH2"] * nh2
    # the paper rounds to two significant digits
    assert abs(r["throughput"] - g["throughput_samples_per_s"]) / g["throughput_samples_per_s"] < 0.05
    assert abs(r["network_bits_per_s"] - g["network_bits_per_s"]) / g["network_bits_per_s"] < 0.05
    assert abs(r["device_memory_bytes"] / 1e6 - g["device_memory_MB"]) / g["device_memory_MB"] < 0.1
    assert r["min_devices"] == g["min_devices"]


def test_visit_cost_counts():
    c = costmodel.visit_cost(1000, rows=3)
    assert c["flops"] == 3 * (2 + 4) * 1000      # forward 2|W| per row, backward 4|W| per row
    assert c["weight_bytes"] == 8000             # W read once forward, once backward
