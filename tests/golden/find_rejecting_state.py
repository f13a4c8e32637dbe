"""Finds a transcript state whose first challenge candidate is NOT canonical (>= p), so that the
rejection branch of the challenge derivation -- taken with probability 2^-32 -- can be exercised
in the library's host and device code, and writes it with the oracle's expected outcome to
tests/golden/rejecting_state.txt.

The search scans states  "IMM-TEST-REJECTING-STATE" (24 bytes) || u64le(i)  for i = 0, 1, 2, ... with
hashlib and the oracle's own acceptance predicate; the expected challenge value and next state come
from oracle.reference.Transcript alone.  About 2^32 candidates have to be hashed: tens of minutes on
a few cores.  Usage:  python tests/golden/find_rejecting_state.py [workers]
"""
import hashlib
import multiprocessing as mp
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import reference as ref  # noqa: E402

PREFIX = b"IMM-TEST-REJECTING-STATE"
assert len(PREFIX) == 24
BLOCK = 1 << 22


def scan(block: int):
    sha = hashlib.sha256
    tail = b"chal" + (0).to_bytes(4, "little")
    lo = block * BLOCK
    for i in range(lo, lo + BLOCK):
        h = sha(PREFIX + i.to_bytes(8, "little") + tail).digest()
        if h[7] == 255 and h[6] == 255 and not ref.Transcript.accepts(int.from_bytes(h[:8], "little")):
            return block, i
    return block, None


def main():
    workers = int(sys.argv[1]) if len(sys.argv) > 1 else max(1, (os.cpu_count() or 2) - 2)
    found = None
    with mp.Pool(workers) as pool:
        for block, i in pool.imap(scan, range(1 << 20)):     # in order: the smallest index wins
            if block % 64 == 0:
                print("scanned %d blocks of 2^22" % block, flush=True)
            if i is not None:
                found = i
                pool.terminate()
                break
    state = PREFIX + found.to_bytes(8, "little")
    tr = ref.Transcript(state)
    first = hashlib.sha256(state + b"chal" + (0).to_bytes(4, "little")).digest()
    v = tr.challenge()
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "rejecting_state.txt")
    with open(out, "w") as f:
        f.write("# A transcript state whose first challenge candidate is not canonical (challenge derivation with\n"
                "# rejection sampling: candidate = u64le(SHA256(s || \"chal\" || u32le(ctr))[0..8)), kept iff < p).\n"
                "# Written by tests/golden/find_rejecting_state.py from oracle/reference.py; index %d of its scan.\n" % found)
        f.write("state = %s\n" % state.hex())
        f.write("first_candidate = 0x%016X\n" % int.from_bytes(first[:8], "little"))
        f.write("challenge = 0x%016X\n" % v)
        f.write("state_after = %s\n" % tr.s.hex())
    print(open(out).read())


if __name__ == "__main__":
    main()
