"""Seeded synthetic inputs for the Hanayo hot path.

Holds no arithmetic of the method: only random draws, the bf16 rounding of
generated values, and the table of workload configurations.  Both the HIP
binding's callers and the CPU oracle's callers take their arrays from here.

The paper names no dataset; its evaluation uses "GPT-style" and "BERT-style"
transformer stacks described by layer / head / hidden counts.  The workloads
below are the chunk shapes of that family that one rank of a (P, W, M) wave
pipeline holds.  Recipe: weights and biases N(0, 0.02^2), LayerNorm gamma = 1
and beta = 0, activations and upstream gradients N(0, 1), valid lengths
uniform integers on [lo, hi]; for bf16 workloads every generated value is
rounded to bf16 (round to nearest even) once, here, so both sides consume
identical numbers.

The model's ends (embedding, head, loss): vocabulary 50304 for the GPT-like
workloads (GPT-2's 50257 rounded up to a multiple of 128), 30592 for the
BERT-like one (BERT's 30522 likewise), 512 for the tiny one; token and position
tables N(0, 0.02^2), head tied to the token table, final LayerNorm (gamma 1,
beta 0) for pre-LN models only.  Token ids follow a Zipf law (probability
proportional to 1 / (id + 1)), so frequent tokens repeat inside a micro-batch as
they do in text.  GPT-like labels are the next token (none for the last
position); BERT-like labels are a random token on a seeded 15 % of the valid
positions and -1 (not counted) elsewhere.
"""

import numpy as np

SEED_BASE = 0x48414E41


class Workload:
    def __init__(self, name, index, dtype, norm, causal, hidden, heads, ffn, seq, mb,
                 n_blocks, P, W, M, valid_len_range=None, vocab=None):
        self.name, self.index, self.dtype = name, index, dtype
        self.norm, self.causal = norm, causal
        self.hidden, self.heads, self.ffn = hidden, heads, ffn
        self.seq, self.mb, self.n_blocks = seq, mb, n_blocks
        self.P, self.W, self.M = P, W, M
        self.valid_len_range = valid_len_range
        self.vocab = vocab if vocab is not None else (50304 if causal else 30592)
        self.seed = SEED_BASE + index

    @property
    def tokens(self):
        return self.seq * self.mb

    def scaled(self, **kw):
        """A copy with some fields replaced (reduced shapes for tests)."""
        w = Workload(self.name, self.index, self.dtype, self.norm, self.causal, self.hidden,
                     self.heads, self.ffn, self.seq, self.mb, self.n_blocks, self.P, self.W,
                     self.M, self.valid_len_range, self.vocab)
        for k, v in kw.items():
            setattr(w, k, v)
        return w


WORKLOADS = {
    "tiny_gpt_fp32": Workload("tiny_gpt_fp32", 0, "fp32", "pre", True, 256, 4, 1024, 128, 2, 1, 2, 1, 4, vocab=512),
    "gpt_1024_bf16": Workload("gpt_1024_bf16", 1, "bf16", "pre", True, 1024, 16, 4096, 1024, 4, 2, 4, 2, 8),
    "bert_1024_bf16": Workload("bert_1024_bf16", 2, "bf16", "post", False, 1024, 16, 4096, 512, 8, 3, 4, 1, 16,
                               valid_len_range=(256, 512)),
    "gpt_4096_bf16": Workload("gpt_4096_bf16", 3, "bf16", "pre", True, 4096, 32, 16384, 2048, 1, 2, 16, 2, 32),
    "gpt_2560_wave4_bf16": Workload("gpt_2560_wave4_bf16", 4, "bf16", "pre", True, 2560, 32, 10240, 1024, 2, 1,
                                    8, 4, 64),
}


def bf16_round(a):
    """float32 array -> nearest-even bf16 value, returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(a.shape)


def to_bf16_bits(a):
    """float32 array holding bf16-representable values -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def from_bf16_bits(u):
    u = np.ascontiguousarray(u, dtype=np.uint16)
    return (u.astype(np.uint32) << 16).view(np.float32).reshape(u.shape)


def rng_for(seed, *stream):
    """Independent Philox stream per (seed, stream ids)."""
    key = np.random.SeedSequence([int(seed)] + [int(s) for s in stream])
    return np.random.Generator(np.random.Philox(key))


def _finish(a, dtype):
    a = a.astype(np.float32)
    return bf16_round(a) if dtype == "bf16" else a


def block_params(rng, H, Fd, dtype, ln_random=False):
    """One block's parameters as float32 arrays (bf16-representable for bf16)."""
    n = lambda *shape: _finish(rng.normal(0.0, 0.02, size=shape), dtype)
    p = {}
    p["ln1_g"] = _finish(1.0 + 0.1 * rng.normal(size=H), dtype) if ln_random else np.ones(H, np.float32)
    p["ln1_b"] = _finish(0.1 * rng.normal(size=H), dtype) if ln_random else np.zeros(H, np.float32)
    p["wqkv"] = n(H, 3 * H)
    p["bqkv"] = n(3 * H)
    p["wo"] = n(H, H)
    p["bo"] = n(H)
    p["ln2_g"] = _finish(1.0 + 0.1 * rng.normal(size=H), dtype) if ln_random else np.ones(H, np.float32)
    p["ln2_b"] = _finish(0.1 * rng.normal(size=H), dtype) if ln_random else np.zeros(H, np.float32)
    p["w1"] = n(H, Fd)
    p["b1"] = n(Fd)
    p["w2"] = n(Fd, H)
    p["b2"] = n(H)
    return p


def chunk_params(wl, chunk, ln_random=False):
    """Parameters of local chunk `chunk` of the workload: list of n_blocks dicts."""
    rng = rng_for(wl.seed, 1, chunk)
    return [block_params(rng, wl.hidden, wl.ffn, wl.dtype, ln_random) for _ in range(wl.n_blocks)]


def stage_params(wl, stage, ln_random=False):
    """Parameters of global stage `stage` (whole-pipeline runs): list of n_blocks dicts."""
    rng = rng_for(wl.seed, 4, stage)
    return [block_params(rng, wl.hidden, wl.ffn, wl.dtype, ln_random) for _ in range(wl.n_blocks)]


def model_input(wl, mb):
    """Input of stage 0 for micro-batch `mb` (whole-pipeline runs)."""
    return activation(wl, 5, mb, 0)


def loss_grad(wl, mb):
    """Gradient of the loss w.r.t. the last stage's output for micro-batch `mb` (whole-pipeline runs)."""
    return activation(wl, 6, mb, 0)


def activation(wl, tag, mb, chunk):
    """N(0,1) tensor [mb_size, seq, hidden]; tag 2 = forward input, 3 = upstream gradient."""
    rng = rng_for(wl.seed, tag, mb, chunk)
    return _finish(rng.normal(size=(wl.mb, wl.seq, wl.hidden)), wl.dtype)


def forward_input(wl, mb, chunk):
    return activation(wl, 2, mb, chunk)


def upstream_grad(wl, mb, chunk):
    return activation(wl, 3, mb, chunk)


def valid_lengths(wl, mb):
    """int32 [mb_size] valid key counts of micro-batch `mb`, or None if unpadded."""
    if wl.valid_len_range is None:
        return None
    lo, hi = wl.valid_len_range
    rng = rng_for(wl.seed, 4, mb)
    return rng.integers(lo, hi + 1, size=wl.mb).astype(np.int32)


# ------------------------------------------------------------------ the model's ends

def ends_params(wl, ln_random=False):
    """dict(wte [V, H], wpe [seq, H], lnf (gamma, beta) or None); the head is tied to wte."""
    rng = rng_for(wl.seed, 7)
    H = wl.hidden
    p = {"wte": _finish(rng.normal(0.0, 0.02, size=(wl.vocab, H)), wl.dtype),
         "wpe": _finish(rng.normal(0.0, 0.02, size=(wl.seq, H)), wl.dtype), "lnf": None}
    if wl.norm == "pre":
        p["lnf"] = ((_finish(1.0 + 0.1 * rng.normal(size=H), wl.dtype), _finish(0.1 * rng.normal(size=H), wl.dtype))
                    if ln_random else (np.ones(H, np.float32), np.zeros(H, np.float32)))
    return p


def untied_head(wl):
    """A separate [V, H] head table, for the runs that do not tie it to the token table."""
    return _finish(rng_for(wl.seed, 10).normal(0.0, 0.02, size=(wl.vocab, wl.hidden)), wl.dtype)


def token_ids(wl, mb):
    """int32 [mb_size, seq], Zipf-distributed over the vocabulary."""
    rng = rng_for(wl.seed, 8, mb)
    w = 1.0 / np.arange(1, wl.vocab + 1)
    cdf = np.cumsum(w / w.sum())
    return np.minimum(np.searchsorted(cdf, rng.random(size=(wl.mb, wl.seq))), wl.vocab - 1).astype(np.int32)


def labels(wl, mb):
    """int32 [mb_size, seq]; -1 = position not counted."""
    tok = token_ids(wl, mb)
    if wl.causal:
        out = np.full_like(tok, -1)
        out[:, :-1] = tok[:, 1:]
        return out
    rng = rng_for(wl.seed, 9, mb)
    picked = rng.random(size=tok.shape) < 0.15
    vl = valid_lengths(wl, mb)
    if vl is not None:
        picked &= np.arange(wl.seq)[None, :] < vl[:, None]
    return np.where(picked, rng.integers(0, wl.vocab, size=tok.shape), -1).astype(np.int32)
