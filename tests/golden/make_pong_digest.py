"""Writes tests/golden/pong_oracle_digest.txt from the CPU oracle alone (never from the HIP path).

The digest freezes the oracle's Pong arithmetic: SHA-256 of the raw obs / reward / done arrays of
config 0 (N = 64, T = 1000, seed 0) for max_score 21 and 2, plus a few literal rows for a reader.
Pong uses only IEEE float32 add / multiply / compare and integer Philox, so the bytes do not depend
on the host.  Run from the repository root:  python tests/golden/make_pong_digest.py
"""
import hashlib
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import oracle as orc  # noqa: E402


def digest(max_score):
    p = orc.Pong(64, 0, max_score=max_score)
    obs0 = p.reset()
    obs, rew, done = p.rollout(1000)
    h = hashlib.sha256()
    for a in (obs0, obs, rew, done):
        h.update(a.tobytes())
    return h.hexdigest(), obs, rew, done, p.stats()


def main():
    lines = ["# written by tests/golden/make_pong_digest.py from oracle/ only; config 0: N=64 T=1000 seed=0"]
    for ms in (21, 2):
        d, obs, rew, done, st = digest(ms)
        lines.append("max_score=%d sha256=%s episodes=%d return_sum=%d length_sum=%d" % (
            ms, d, st["episodes"], st["return_sum"], st["length_sum"]))
        lines.append("max_score=%d obs[999,0]=%s" % (ms, " ".join(float(x).hex() for x in obs[999, 0])))
        lines.append("max_score=%d reward_sum=%d done_sum=%d" % (ms, int(rew.sum()), int(done.sum())))
    path = os.path.join(ROOT, "tests", "golden", "pong_oracle_digest.txt")
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    print(path)


if __name__ == "__main__":
    main()
