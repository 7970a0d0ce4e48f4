"""Independent list-and-set model of the pool bookkeeping, for tests only.

Written from the rules (paper Sec. 4.2 D1-D3 plus the stated tie-breaks) with
Python lists; it deliberately shares no structure with the C oracle: slots are a
set of (frame, slot) pairs rather than a byte array, and frame positions are
looked up through list.index.
"""


class PoolModel:
    def __init__(self, n_frames, order=None):
        self.n_frames = n_frames
        hand_out = list(order) if order is not None else list(range(n_frames))
        self.free = hand_out[::-1]            # pop() takes from the end
        self.owner = {}
        self.models = {}

    def register(self, mid, slots, page_tokens, max_blocks):
        self.models[mid] = dict(slots=slots, frames=[], used=set(), rows={}, T=page_tokens, max_blocks=max_blocks)

    def resize(self, mid, target):
        m = self.models[mid]
        owned = len(m["frames"])
        if target > owned:
            if target - owned > len(self.free):
                return -3
            for _ in range(target - owned):
                f = self.free.pop()
                self.owner[f] = mid
                m["frames"].append(f)
        elif target < owned:
            want = owned - target
            gone = []
            for f in reversed(m["frames"]):
                if len(gone) == want:
                    break
                if not any((f, s) in m["used"] for s in range(m["slots"])):
                    gone.append(f)
            for f in gone:
                self.free.append(f)
                del self.owner[f]
            m["frames"] = [f for f in m["frames"] if f not in gone]
        return len(m["frames"])

    def _free_slots(self, m):
        return [(f, s) for f in m["frames"] for s in range(m["slots"]) if (f, s) not in m["used"]]

    def reserve(self, mid, seq, ctx_len):
        m = self.models[mid]
        row = m["rows"].setdefault(seq, [])
        want = -(-ctx_len // m["T"])
        if want > m["max_blocks"]:
            return -6
        need = want - len(row)
        if need <= 0:
            return 0
        avail = self._free_slots(m)
        if need > len(avail):
            return -4
        for f, s in avail[:need]:
            m["used"].add((f, s))
            row.append(f * m["slots"] + s)
        return need

    def release(self, mid, seq):
        m = self.models[mid]
        row = m["rows"].get(seq, [])
        for b in row:
            m["used"].discard((b // m["slots"], b % m["slots"]))
        m["rows"][seq] = []
        return len(row)

    def bits(self, mid):
        m = self.models[mid]
        return [int((f, s) in m["used"]) for f in m["frames"] for s in range(m["slots"])]
