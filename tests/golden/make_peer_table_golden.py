"""Writes tests/golden/peer_table_N4_S8_R2_seed0_round0.txt from the CPU oracle.

The peer hash is this repository's own definition, so the values have no external
source; the file is a regression guard only.  Calls nothing but oracle/.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import ref  # noqa: E402

if __name__ == "__main__":
    T = ref.make_peer_table(4, 8, 2, 0, 0)
    with open(os.path.join(HERE, "peer_table_N4_S8_R2_seed0_round0.txt"), "w") as f:
        f.write("# peers[w][s][j] for N=4 S=8 R=2 seed=0 round=0; one line per worker w,\n"
                "# entries s-major then j.  Written by make_peer_table_golden.py (oracle only).\n")
        for w in range(4):
            f.write(" ".join(str(int(v)) for v in T[w].reshape(-1)) + "\n")
