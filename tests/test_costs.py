import os

from paper_2302_07475_amd import costs


def test_cost_table_matches_hand_evaluation():
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "cost_table.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = int(v)
    M, N, K = vals["M"], vals["N"], vals["K"]
    assert costs.vanilla_sgd(M, N) == vals["vanilla"]
    assert costs.topk_sgd(M, N, K) == vals["topk"]
    assert costs.signsgd_mv(M, N) == vals["signsgd"]
    assert costs.s3gd_mv(M, N, K) == vals["s3gd"]
    assert costs.s3gd_uplink(M, N, 0) == 0
