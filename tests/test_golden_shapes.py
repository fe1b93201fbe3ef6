"""Shape bookkeeping against the numbers the paper prints (Table III, Sec. I)."""
import os

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table3_shapes.txt")


def _rows():
    models, active = {}, None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "mixtral_active_percent":
            active = float(f[1])
        else:
            models[f[0]] = dict(blocks=int(f[1]), experts=int(f[2]), k=int(f[3]), expert_b=float(f[4]),
                                total_b=float(f[5]), hidden=int(f[6]), ffn=int(f[7]))
    return models, active


def test_expert_parameter_counts_match_table3():
    models, _ = _rows()
    for name, m in models.items():
        params = m["blocks"] * m["experts"] * 3 * m["hidden"] * m["ffn"]
        assert abs(params / 1e9 - m["expert_b"]) < 0.05, (name, params)


def test_active_parameter_share():
    models, active = _rows()
    m = models["mixtral_8x7b"]
    share = (m["total_b"] - m["expert_b"] + m["expert_b"] * m["k"] / m["experts"]) / m["total_b"]
    assert abs(100 * share - active) < 0.1


def test_synth_layer_shapes_follow_table3():
    import torch
    from paper_2501_10375_amd import synth

    d = synth.moe_layer_inputs(2, 64, 128, 4, torch.float32)
    assert d["w1"].shape == (4, 128, 64) and d["w3"].shape == (4, 128, 64) and d["w2"].shape == (4, 64, 128)
    assert d["wg"].shape == (4, 64) and d["x"].shape == (2, 64)
