"""Parser for the canonical bookkeeping image both libraries export (tests only)."""
import numpy as np


def parse(img):
    w = [int(x) for x in np.asarray(img, dtype=np.int32)]
    it = iter(w)
    nx = lambda: next(it)
    assert nx() == 0x53564B50 and nx() == 1
    st = {"n_frames": nx(), "page_tokens": nx()}
    n_free = nx()
    st["free"] = [nx() for _ in range(n_free)]
    st["owner"] = [nx() for _ in range(st["n_frames"])]
    st["models"] = {}
    for _ in range(nx()):
        mid = nx()
        m = dict(q_heads=nx(), kv_heads=nx(), head_dim=nx(), dtype=nx(), slots=nx())
        owned = nx()
        m["frames"] = [nx() for _ in range(owned)]
        nbits = nx()
        words = [nx() & 0xFFFFFFFF for _ in range((nbits + 31) // 32)]
        m["bits"] = [(words[j // 32] >> (j % 32)) & 1 for j in range(nbits)]
        m["max_seqs"] = nx()
        m["rows"] = {}
        for _ in range(nx()):
            s, n = nx(), nx()
            m["rows"][s] = [nx() for _ in range(n)]
        st["models"][mid] = m
    assert next(it, None) is None
    return st


def check_invariants(st):
    """Frames are conserved and never shared; slot bits and rows agree."""
    owned = [f for m in st["models"].values() for f in m["frames"]]
    everything = st["free"] + owned
    assert sorted(everything) == list(range(st["n_frames"])), "frames not conserved / not disjoint"
    for f in st["free"]:
        assert st["owner"][f] == -1
    for mid, m in st["models"].items():
        for f in m["frames"]:
            assert st["owner"][f] == mid
        blocks = [b for r in m["rows"].values() for b in r]
        assert len(blocks) == len(set(blocks)), "a block is in two rows"
        assert sum(m["bits"]) == len(blocks)
        pos = {f: i for i, f in enumerate(m["frames"])}
        for b in blocks:
            assert m["bits"][pos[b // m["slots"]] * m["slots"] + b % m["slots"]] == 1
