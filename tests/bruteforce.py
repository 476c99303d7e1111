"""Hash-free brute-force model of run-anchored matching, for tiny inputs only.

A request token at offset k of its run matches iff the k+1 tokens from the run
start equal the first k+1 tokens of some stored run; it is then served from the
slot of the earliest stored such token.  Everything is elementwise token
comparison over explicit lists (the O(n*m) substring check the paper's hashing
replaces, Sec. 4.2.2 first paragraph)."""


def runs(tok, mask, off):
    """Yield (request, start, end) for every maximal non-sensitive run."""
    for r in range(len(off) - 1):
        i, e = int(off[r]), int(off[r + 1])
        while i < e:
            if mask[i]:
                i += 1
                continue
            j = i
            while j < e and not mask[j]:
                j += 1
            yield r, i, j
            i = j


class BrutePool:
    def __init__(self, free_slots):
        self.free = [int(s) for s in free_slots]
        self.n_used = 0
        self.stored = []  # list of (list_of_tokens_prefix, slot): one entry per stored token
        self.slot_tok = {}
        self.slot_pos = {}

    def find(self, prefix):
        for p, s in self.stored:  # insertion order: the earliest wins
            if len(p) == len(prefix) and all(a == b for a, b in zip(p, prefix)):
                return s
        return None

    def insert(self, tok, mask, off):
        """Returns slot_out (None for sensitive or dropped tokens)."""
        out = [None] * len(tok)
        for r, a, b in runs(tok, mask, off):
            for i in range(a, b):
                prefix = [int(t) for t in tok[a : i + 1]]
                s = self.find(prefix)
                if s is None and self.n_used < len(self.free):
                    s = self.free[self.n_used]
                    self.n_used += 1
                    self.stored.append((prefix, s))
                    self.slot_tok[s] = int(tok[i])
                    self.slot_pos[s] = i - int(off[r])
                out[i] = s
        return out

    def probe(self, tok, mask, off):
        out = [None] * len(tok)
        for r, a, b in runs(tok, mask, off):
            for i in range(a, b):
                out[i] = self.find([int(t) for t in tok[a : i + 1]])
        return out
