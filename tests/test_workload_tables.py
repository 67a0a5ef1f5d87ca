"""The paper-shaped workloads against the shape columns the paper prints (CPU only)."""
from paper_2512_06989_amd import inputs


def test_workloads_follow_the_paper_tables():
    """d_model, H, d_h and E x d_e of the paper_* workloads equal the shape columns printed
    in the paper's model table and efficiency-benchmark table (tests/golden/model_shapes.txt)."""
    import os
    rows = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "model_shapes.txt")):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            rows[f[0]] = [int(x) for x in f[1:6]]
    for wl, key in (("paper_128m", "flashmhf_128m"), ("paper_370m", "flashmhf_370m"),
                    ("paper_1p3b", "flashmhf_1p3b"), ("paper_bench", "bench_hopper")):
        w = inputs.WORKLOADS[wl]
        d_model, heads, d_h, inter, n_sub = rows[key]
        assert (w.d_model, w.n_heads, w.d_head, w.d_ff, w.n_sub) == (d_model, heads, d_h, inter, n_sub)
