"""Writes tests/golden/fig_split_ratio.json: the range of v_gpu / v_com (flop per byte)
for which the oracle's Eq. 11 argmin reproduces the split points plotted in the paper's
appendix figure (tests/golden/fig_split_points.json).  Calls only oracle/.

    python tests/golden/fit_split_ratio.py
"""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import kvpr_plan_oracle as po  # noqa: E402


def main():
    fig = json.load(open(os.path.join(HERE, "fig_split_points.json")))
    h, p, b, s0 = fig["hidden"], fig["elem_bytes"], fig["batch"], fig["prompt"]
    want = fig["split_l"]
    v_com = 25.0e9
    good = []
    # scan ratios around 1e4 flop/B on a fine grid
    r = 9000.0
    while r < 11000.0:
        got = [po.plan_split(po.COST_EQ10, b, s0 + i, h, p, v_com, r * v_com)[0]
               for i in fig["tokens_generated"]]
        if got == want:
            good.append(r)
        r += 0.5
    if not good:
        raise SystemExit("no ratio reproduces the figure")
    out = {"_written_by": "tests/golden/fit_split_ratio.py (oracle only)",
           "v_com_bytes_per_s": v_com,
           "ratio_flop_per_byte_min": good[0], "ratio_flop_per_byte_max": good[-1],
           "ratio_flop_per_byte_mid": 0.5 * (good[0] + good[-1])}
    json.dump(out, open(os.path.join(HERE, "fig_split_ratio.json"), "w"), indent=1)
    print(out)


if __name__ == "__main__":
    main()
