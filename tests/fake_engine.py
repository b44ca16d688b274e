"""A stand-in engine for the serving-loop tests that run without a GPU."""
import time


class FakeEngine:
    """A stand-in engine for tests without a GPU: a fixed time per call and tokens that are a pure function
    of the sequence's history, so two runs over the same inputs produce the same tokens."""

    def __init__(self, per_token_s=0.002, prefill_s=0.004, vocab=1000):
        self.per_token_s, self.prefill_s, self.vocab = per_token_s, prefill_s, vocab
        self.hist, self.next_id, self.swapped = {}, 0, set()

    def _next(self, seq):
        h = 1469598103934665603
        for t in self.hist[seq][-16:]:
            h = ((h ^ (t + 1)) * 1099511628211) & ((1 << 64) - 1)
        tok = (h >> 20) % self.vocab
        self.hist[seq].append(tok)
        return tok

    def new_sequence(self):
        self.next_id += 1
        self.hist[self.next_id] = []
        return self.next_id

    def prefill(self, seq, tokens):
        assert seq not in self.swapped
        time.sleep(self.prefill_s)
        self.hist[seq].extend(tokens)
        return self._next(seq)

    def decode(self, seqs):
        time.sleep(self.per_token_s)
        return [self._next(s) for s in seqs]

    def free(self, seq):
        self.hist.pop(seq, None)

    def fork(self, parent, n_tokens):
        child = self.new_sequence()
        self.hist[child] = self.hist[parent][:n_tokens]
        return child

    def trim(self, seq):
        return 0

    def swap_out(self, seq):
        self.swapped.add(seq)

    def swap_in(self, seq):
        self.swapped.remove(seq)
