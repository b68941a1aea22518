"""The Actor loop's engine-side state machine (Alg. 2): a constant batch of H slots, refilled as
sequences finish, one token per slot per step, and a weight update that lands between two steps
and leaves every slot's K/V history untouched (Sec. 5.1: later tokens are sampled from the new
weights conditioned on the stale cache).

Life cycle of a slot holding a sequence with an n-token prompt: the step at position p consumes
prompt[p] while p < n, afterwards the token the previous step produced.  Steps at positions
p < n-1 emit nothing; the step at p = n-1 emits the first generated token; the sequence is
finished after max_new emitted tokens and holds n + max_new - 1 cached positions by then.
Every token of one step carries the same weight version.
"""
from dataclasses import dataclass, field
import numpy as np

from . import decoder
from .sampler import sample_row


@dataclass
class Record:
    slot: int
    seq_id: int
    token: int
    logprob: float
    weight_version: int
    position: int
    emitted: bool
    finished: bool


@dataclass
class _Seq:
    seq_id: int
    prompt: np.ndarray
    max_new: int
    temperature: float
    cache: decoder.Cache
    inputs: list = field(default_factory=list)   # tokens consumed so far (positions 0..pos-1)
    last_token: int = -1
    n_emitted: int = 0

    @property
    def pos(self):
        return len(self.inputs)


class OracleEngine:
    def __init__(self, cfg, weights, max_batch, seed, dtype=np.float64):
        self.cfg, self.W, self.H, self.seed = cfg, weights, max_batch, seed
        self.dtype = dtype
        self.slots = [None] * max_batch
        self.version = 0
        self.last_logits = {}

    # -- Alg. 2: "add H - len(S_prog) prompts" ------------------------------------------------
    def add_sequence(self, seq_id, prompt, max_new, temperature=1.0):
        if temperature <= 0 or max_new < 1 or len(prompt) < 1:
            raise ValueError("bad sequence parameters")
        for s, cur in enumerate(self.slots):
            if cur is None:
                self.slots[s] = _Seq(seq_id, np.asarray(prompt, dtype=np.int64), max_new,
                                     float(temperature), decoder.Cache(self.cfg, self.dtype))
                return s
        raise RuntimeError("batch full")

    # -- Alg. 2: "pop finished sequences" -----------------------------------------------------
    def retire_sequence(self, slot):
        if self.slots[slot] is None:
            raise RuntimeError("slot idle")
        self.slots[slot] = None

    def n_active(self):
        return sum(s is not None for s in self.slots)

    # -- Alg. 2: "mu <- receive_weight_update()" ----------------------------------------------
    def swap_weights(self, new_weights, recompute_kv=False):
        """Replace the weights for all later steps.  Caches are kept as they are, unless
        `recompute_kv` (the 'KV cache recomputed' variant of Sec. 5.1) rebuilds them by running
        every consumed token again under the new weights."""
        self.W = new_weights
        self.version += 1
        if recompute_kv:
            for seq in self.slots:
                if seq is None:
                    continue
                seq.cache = decoder.Cache(self.cfg, self.dtype)
                for p, tok in enumerate(seq.inputs):
                    decoder.step(self.cfg, self.W, tok, p, seq.cache, self.dtype)
        return self.version

    # -- Alg. 2: "generate next tokens with mu" -----------------------------------------------
    def decode_step(self, forced=None):
        """One token for every occupied slot.  forced[slot] >= 0 overrides the drawn token."""
        out = []
        self.last_logits = {}
        for s, seq in enumerate(self.slots):
            if seq is None:
                continue
            p = seq.pos
            n = len(seq.prompt)
            x = int(seq.prompt[p]) if p < n else seq.last_token
            logits = decoder.step(self.cfg, self.W, x, p, seq.cache, self.dtype)
            logits = logits.astype(np.float32)
            self.last_logits[s] = logits
            f = -1 if forced is None else int(forced[s])
            tok, lp = sample_row(logits, seq.temperature, self.seed, seq.seq_id, p, f)
            seq.inputs.append(x)
            emitted = p >= n - 1
            if emitted:
                seq.last_token = tok
                seq.n_emitted += 1
            out.append(Record(s, seq.seq_id, tok, lp, self.version, p, emitted,
                              emitted and seq.n_emitted >= seq.max_new))
        return out
