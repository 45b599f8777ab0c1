"""Writes tests/golden/hash_kat.txt from the oracle alone (run from the repo
root: python tests/golden/make_golden.py).  The file freezes known-answer
vectors of the hash family so that a change to either side is noticed; a third,
independent numpy implementation in tests/test_oracle_hash.py checks the same
vectors."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(
    os.path.abspath(__file__)))))
from oracle import tagc_oracle as O  # noqa: E402

SEEDS = [0, 1, 0x0123456789ABCDEF, 2 ** 64 - 1]
INDICES = [0, 1, 2, 31, 32, 1000, 65535, 65536, 123456789, 2 ** 31,
           2 ** 32 - 2]
MSUBS = [1, 2, 7, 494, 8192, 65536, 10 ** 6 + 3]
SALTS = [0, 1, 7, 15]


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)),
                       "hash_kat.txt")
    with open(out, "w") as f:
        f.write("# seed index j m_sub salt slot sign   (written by make_golden.py "
                "from oracle/ only)\n")
        for s in SEEDS:
            for i in INDICES:
                for j in range(3):
                    for ms in MSUBS:
                        for salt in (SALTS if ms in (7, 8192) else [0]):
                            slot, sign = O.hash_slot(i, s, j, ms, salt)
                            f.write("%d %d %d %d %d %d %d\n" % (s, i, j, ms, salt,
                                                                slot, sign))


if __name__ == "__main__":
    main()
