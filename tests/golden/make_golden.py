"""Writes tests/golden/config1_oracle.json: the CPU oracle's outputs for benchmark configuration 1
(two tiny CNNs, fp32, batch 1, input U[0,1) from seed 7, He-normal weights from seeds 1000/1001,
zero bias).  Calls only the oracle and the seeded generators; run from the repository root:

    python tests/golden/make_golden.py
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from workloads import gen, zoo  # noqa: E402


def main():
    x = gen.make_input(7, 1, 3, 32, 32, "uniform", "f32")
    out = {"_citation": "oracle/fi_oracle.cpp on benchmark configuration 1; regenerate with tests/golden/make_golden.py",
           "members": []}
    for i in range(2):
        m = zoo.tiny_cnn("f32", softmax=True)
        blob = gen.make_blob(m, 1000 + i, bias_std=0.0)
        logits = oracle.run_model(m, blob, x, node=4)[0]
        probs = oracle.run_model(m, blob, x)[0]
        out["members"].append({"seed": 1000 + i, "logits": [float(v) for v in logits], "softmax": [float(v) for v in probs],
                               "top1": int(oracle.top1(logits[None])[0])})
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_oracle.json"), "w") as f:
        json.dump(out, f, indent=1)
    print("wrote config1_oracle.json")


if __name__ == "__main__":
    main()
