"""Writes the stored expected values under tests/golden/.  Calls only the
oracle (and the seeded input generators); never the HIP library.

    python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from oracle.replay import run_workload  # noqa: E402
from workloads import configs  # noqa: E402


def main():
    oracle.build()
    s = run_workload(configs.config1_tiny()).stream()
    out = {"what": "config 1 (tiny) expected host byte stream, completeness policy",
           "source": "oracle/ run over workloads.configs.config1_tiny(); record layout as "
                     "stated at the top of oracle/dmi_oracle.c",
           "bytes": int(s.size), "sha256": hashlib.sha256(s.tobytes()).hexdigest()}
    with open(os.path.join(HERE, "config1_stream.json"), "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(out)


if __name__ == "__main__":
    main()
