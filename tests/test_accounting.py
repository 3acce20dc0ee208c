"""The algorithmic byte/flop formulas reproduce the paper's kernel-metrics table."""
import os

from paper_2508_07101_amd import accounting as acc


def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "kernel_metrics_table.txt")
    out = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            name, value, _ = line.split()
            out[name] = float(value)
    return out


def test_closed_forms_match_the_printed_table():
    g = _golden()
    ours = {
        "sparse_flops": acc.attn_flops_per_q_head(2048, 128),
        "full_flops": acc.attn_flops_per_q_head(16384, 128),
        "sparse_g2s": acc.attn_bytes_per_kv_head(2048, 128),
        "full_g2s": acc.attn_bytes_per_kv_head(16384, 128),
    }
    for name, v in ours.items():
        assert abs(v - g[name]) / g[name] < 0.01, (name, v, g[name])
    assert ours["sparse_flops"] == 2048 * 128 * 4 and ours["full_g2s"] == 16384 * 128 * 2 * 2


def test_step_bytes_adds_up_per_layer_kind():
    sched = [0, 0, 1] + [2] * 29
    fused = acc.step_bytes(sched, [32768], G=8, budget=2048, window=512)
    assert fused["score"] == 0                                # the selection layer reads its K rows once
    b = acc.step_bytes(sched, [32768], G=8, budget=2048, window=512, fused_select=False)
    assert fused["total"] == b["total"] - b["score"]
    assert b["full"] == 3 * 2 * 8 * 32768 * 128 * 2
    assert b["score"] == 8 * (32768 - 512) * 128 * 2
    assert b["sparse"] == 29 * (2 * 8 * 2048 * 128 * 2 + 4 * 2048)
    assert b["total"] == b["full"] + b["score"] + b["sparse"]
    assert acc.score_bytes(8, 1000, 2048, 512) == 0          # budget covers the context: nothing scored
