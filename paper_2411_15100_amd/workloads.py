"""Synthetic decode workloads driven through the library (used by the GPU
tests, the smoke check and the benchmark).  torch is used here for device
buffers and streams only; every mask comes from the HIP kernels."""

from __future__ import annotations

import numpy as np
import torch

import synth_inputs as si

from . import binding as xgm


def current_stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def make_xgm_vocab(vocab: si.Vocab) -> xgm.Vocab:
    return xgm.Vocab(vocab.data, vocab.offsets, vocab.stop_ids)


def unpack_rows(words: np.ndarray, V: int) -> np.ndarray:
    """int32 [B, W] -> bool [B, V] (bit i%32 of word i//32, LSB first)."""
    b = np.unpackbits(np.ascontiguousarray(words).view(np.uint8), axis=-1, bitorder="little")
    return b[..., :V].astype(bool)


class TokenInfo:
    """Per-vocabulary arrays the walk policy needs."""

    def __init__(self, vocab: si.Vocab):
        V = vocab.size
        lens = np.diff(vocab.offsets)
        first = np.full(V, -1, dtype=np.int16)
        nz = lens > 0
        first[nz] = vocab.data[vocab.offsets[:-1][nz]]
        self.first = first
        self.structural = np.isin(first, np.fromiter(si.STRUCTURAL_BYTES, dtype=np.int16))
        self.is_stop = np.zeros(V, dtype=bool)
        self.is_stop[vocab.stop_ids] = True
        opens = np.zeros(V, dtype=bool)
        data = vocab.data
        is_open = (data == ord("[")) | (data == ord("{")) | (data == ord("("))
        if data.size:
            csum = np.concatenate([[0], np.cumsum(is_open)])
            opens = (csum[vocab.offsets[1:]] - csum[vocab.offsets[:-1]]) > 0
        self.opens = opens  # token contains an opening bracket


class BatchWalker:
    """B requests walking at random through their grammars.

    Each step: fill the batch's bitmask on the GPU, copy it to the host, pick
    one allowed token per row with the seeded policy, accept it.  Rows that
    terminate are reset (re-seeded from the start state).  ``history[b]`` is
    the list of token ids accepted by row b since its last reset.
    """

    def __init__(self, caches, vocab: si.Vocab, seed: int, structural_bias: float = 0.35, max_depth: int = 32):
        self.vocab = vocab
        self.info = TokenInfo(vocab)
        self.V = vocab.size
        self.W = xgm.bitmask_words(self.V)
        self.matchers = [xgm.Matcher(cache=c) for c in caches]
        self.batch = xgm.MatcherBatch(self.matchers)
        self.B = len(self.matchers)
        self.rng = np.random.Generator(np.random.PCG64(seed))
        self.bias = structural_bias
        self.max_depth = max_depth
        self.d_mask = torch.zeros((self.B, self.W), dtype=torch.int32, device="cuda")
        self.history = [[] for _ in range(self.B)]
        self.frozen = np.zeros(self.B, dtype=bool)

    def fill(self) -> np.ndarray:
        """Run the fill kernel and return the packed masks int32 [B, W] (host)."""
        self.batch.fill_next_token_bitmask(self.d_mask.data_ptr(), current_stream())
        return self.d_mask.cpu().numpy()

    def depth(self, b: int) -> int:
        m = self.matchers[b]
        return max((len(m.stack(s)) for s in range(m.num_stacks())), default=0)

    def step(self, words: np.ndarray = None) -> np.ndarray:
        """One decode step for every non-frozen row; returns the chosen ids."""
        if words is None:
            words = self.fill()
        allowed = unpack_rows(words, self.V)
        for b in range(self.B):  # nesting guard: do not deepen very deep states
            if not self.frozen[b] and self.depth(b) > self.max_depth:
                allowed[b] &= ~self.info.opens
        picks = si.pick_tokens(self.rng, allowed, self.info.structural, self.info.is_stop, self.bias)
        for b in range(self.B):
            if self.frozen[b]:
                continue
            t = int(picks[b])
            if t < 0:
                raise RuntimeError(f"row {b}: no token is allowed (dead state)")
            self.matchers[b].accept_token(t)
            self.history[b].append(t)
            if self.matchers[b].is_terminated():
                self.matchers[b].reset()
                self.history[b] = []
        return picks


def uncertain_fraction(walker: BatchWalker, caches, plain: bool = False) -> np.ndarray:
    """Per row: mean over its stacks of |context-dependent tokens at the top node| / V.

    plain=True counts the context-dependent class of section 3.1 alone (what a
    cache without any context expansion would have to resolve at run time);
    plain=False what is left after the one-byte narrowing done at build time.
    """
    out = np.zeros(walker.B)
    for b, (m, c) in enumerate(zip(walker.matchers, caches)):
        n = m.num_stacks()
        if n:
            tops = [m.stack(s)[-1] for s in range(n)]
            out[b] = np.mean([c.num_uncertain(t) + (c.num_uncertain_plain(t) if plain else 0) for t in tops]) / walker.V
    return out


class ServingWorkload:
    """The serving decode step: B requests with distinct string-heavy schema
    grammars, each frozen in a state reached by a seeded random walk, a pool
    of `pool` such state sets, and rotating logits buffers.

    Recipe: vocabulary `bpe`(V, seed 0); grammar b = make_schema_grammar(b,
    string_heavy=True); state set k: rows walk with the structural-bias policy
    (seed 5000 + k) and freeze at the first step where their deepest stack has
    d_b + 1 frames, d_b ~ U{1..6}, or after 40 steps; then, while the mean
    fraction of context-dependent tokens (section 3.1's class, before any
    narrowing by context) at the stack tops is below `min_uncertain`, the
    quarter of rows with the lowest fraction keeps walking until it reaches a
    top with a fraction of at least one half.
    """

    def __init__(self, n_rows: int = 128, vocab_size: int = 151936, pool: int = 16, n_logit_buffers: int = 8,
                 min_uncertain: float = 0.20, log=None):
        log = log or (lambda *_: None)
        self.B, self.V = n_rows, vocab_size
        self.vocab = si.make_vocab("bpe", vocab_size, 0)
        self.xv = make_xgm_vocab(self.vocab)
        self.texts = [si.make_schema_grammar(b, string_heavy=True) for b in range(n_rows)]
        self.grammars = [xgm.Grammar(t, "root") for t in self.texts]
        log(f"compiled {n_rows} grammars, {sum(g.num_nodes for g in self.grammars)} nodes in total")
        self.caches = []
        self.build_kernel_seconds = 0.0
        self.build_pairs = 0
        for i, g in enumerate(self.grammars):
            c = xgm.Cache(g, self.xv, current_stream())
            self.caches.append(c)
            self.build_kernel_seconds += c.build_kernel_seconds
            self.build_pairs += g.num_nodes * vocab_size
            if i % 16 == 15:
                log(f"built {i + 1} mask caches ({self.build_pairs / max(self.build_kernel_seconds, 1e-9) / 1e9:.1f} G pairs/s in the kernel)")
        self.sets = []
        fractions, narrowed = [], []
        for k in range(pool):
            w = BatchWalker(self.caches, self.vocab, seed=5000 + k, structural_bias=0.35)
            rng = np.random.Generator(np.random.PCG64(7000 + k))
            target = rng.integers(1, 7, size=n_rows) + 1
            for step in range(40):
                for b in range(n_rows):
                    if not w.frozen[b] and step > 0 and w.depth(b) == target[b]:
                        w.frozen[b] = True
                if w.frozen.all():
                    break
                w.step()
            w.frozen[:] = True
            for _ in range(60):
                frac = uncertain_fraction(w, self.caches, plain=True)
                if frac.mean() >= min_uncertain:
                    break
                low = np.argsort(frac)[: max(1, n_rows // 4)]
                w.frozen[low] = False
                w.step()
                frac = uncertain_fraction(w, self.caches, plain=True)
                for b in low:
                    w.frozen[b] = frac[b] >= 0.5
                # rows still walking stay unfrozen for the next round
            w.frozen[:] = True
            fractions.append(uncertain_fraction(w, self.caches, plain=True))
            narrowed.append(uncertain_fraction(w, self.caches, plain=False))
            self.sets.append(w)
            log(f"state set {k}: mean context-dependent fraction {fractions[-1].mean():.3f} "
                f"(after the one-byte narrowing {narrowed[-1].mean():.3f})")
        self.uncertain_fraction = float(np.mean(fractions))
        self.uncertain_fraction_narrowed = float(np.mean(narrowed))
        if self.uncertain_fraction < min_uncertain:
            raise RuntimeError(f"state pool has only {self.uncertain_fraction:.3f} context-dependent tokens per row")
        self.W = xgm.bitmask_words(vocab_size)
        self.d_mask = torch.zeros((n_rows, self.W), dtype=torch.int32, device="cuda")
        gen = torch.Generator(device="cuda")
        gen.manual_seed(0)
        self.logits = [torch.randn((n_rows, vocab_size), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
                       for _ in range(n_logit_buffers)]

        # the same state sets resident on the device (no per-step packing or upload)
        self.device_sets = [xgm.DeviceBatch(w.matchers, history=0, stream=current_stream()) for w in self.sets]

    def fill(self, k: int, stream: int):
        self.sets[k % len(self.sets)].batch.fill_next_token_bitmask(self.d_mask.data_ptr(), stream)

    def fill_device(self, k: int, stream: int):
        """Fill from the device-resident copy of state set k."""
        self.device_sets[k % len(self.device_sets)].fill_next_token_bitmask(self.d_mask.data_ptr(), stream)

    def step_device(self, k: int, stream: int):
        self.fill_device(k, stream)
        self.apply(k, stream)

    def fused_step_device(self, k: int, stream: int):
        t = self.logits[k % len(self.logits)]
        self.device_sets[k % len(self.device_sets)].fill_and_apply(self.d_mask.data_ptr(), t.data_ptr(), xgm.DTYPE_BF16,
                                                                    self.V, t.stride(0), stream=stream)

    def apply(self, k: int, stream: int):
        t = self.logits[k % len(self.logits)]
        xgm.apply_token_bitmask_inplace(t.data_ptr(), xgm.DTYPE_BF16, self.B, self.V, t.stride(0),
                                        self.d_mask.data_ptr(), self.V, stream=stream)

    def step(self, k: int, stream: int):
        self.fill(k, stream)
        self.apply(k, stream)

    def fused_step(self, k: int, stream: int):
        """Fill and apply in one launch."""
        t = self.logits[k % len(self.logits)]
        xgm.fill_and_apply(self.sets[k % len(self.sets)].batch, self.d_mask.data_ptr(), t.data_ptr(), xgm.DTYPE_BF16,
                           self.V, t.stride(0), stream=stream)

    def refresh_logits(self):
        """Masked entries are -inf after a step; draw the buffers again."""
        gen = torch.Generator(device="cuda")
        gen.manual_seed(1)
        for t in self.logits:
            t.copy_(torch.randn(t.shape, generator=gen, device="cuda", dtype=torch.float32))

    def replay_tokens(self, k: int) -> np.ndarray:
        """The tokens that lead every row from its start state to its state in set k: int32 [steps, B],
        -1 where a row has arrived (its walk was shorter).  Accepting row after row of this array on a
        batch of fresh matchers replays the walk of state set k."""
        hist = self.sets[k].history
        steps = max(len(h) for h in hist)
        out = np.full((steps, self.B), -1, dtype=np.int32)
        for b, h in enumerate(hist):
            out[: len(h), b] = h
        return out


class WalkedWorkload:
    """A smaller decode workload: B rows over the given caches, a pool of state sets taken at equal
    distances along one seeded random valid-token walk (rows that terminate start again), each kept as host
    matchers and resident on the device; rotating logits buffers of the given dtype."""

    def __init__(self, caches, vocab: si.Vocab, seed: int, total_steps: int, pool: int = 8, dtype=torch.float32,
                 sigma: float = 1.0, n_logit_buffers: int = 4, structural_bias: float = 0.35):
        self.vocab, self.B, self.V = vocab, len(caches), vocab.size
        self.W = xgm.bitmask_words(self.V)
        self.caches = list(caches)
        walker = BatchWalker(self.caches, vocab, seed=seed, structural_bias=structural_bias)
        every = max(1, total_steps // pool)
        self.sets, self.device_sets, self.histories = [], [], []
        for step in range(1, total_steps + 1):
            walker.step()
            if step % every == 0 and len(self.sets) < pool:
                ms = []
                for b, c in enumerate(self.caches):
                    m = xgm.Matcher(cache=c)
                    for t in walker.history[b]:
                        m.accept_token(int(t))
                    ms.append(m)
                self.sets.append(xgm.MatcherBatch(ms))
                self.device_sets.append(xgm.DeviceBatch(ms, history=0, stream=current_stream()))
                self.histories.append([list(h) for h in walker.history])
        self.d_mask = torch.zeros((self.B, self.W), dtype=torch.int32, device="cuda")
        gen = torch.Generator(device="cuda")
        gen.manual_seed(0)
        self.dtype = dtype
        self.dtype_code = {torch.float32: xgm.DTYPE_F32, torch.bfloat16: xgm.DTYPE_BF16, torch.float16: xgm.DTYPE_F16}[dtype]
        self.logits = [(torch.randn((self.B, self.V), generator=gen, device="cuda", dtype=torch.float32) * sigma).to(dtype)
                       for _ in range(n_logit_buffers)]

    def refresh_logits(self):
        gen = torch.Generator(device="cuda")
        gen.manual_seed(1)
        for t in self.logits:
            t.copy_(torch.randn(t.shape, generator=gen, device="cuda", dtype=torch.float32))

    def fill_device(self, k: int, stream: int):
        self.device_sets[k % len(self.device_sets)].fill_next_token_bitmask(self.d_mask.data_ptr(), stream)

    def apply(self, k: int, stream: int):
        t = self.logits[k % len(self.logits)]
        xgm.apply_token_bitmask_inplace(t.data_ptr(), self.dtype_code, self.B, self.V, t.stride(0), self.d_mask.data_ptr(),
                                        self.V, stream=stream)

    def fused_step_device(self, k: int, stream: int):
        t = self.logits[k % len(self.logits)]
        self.device_sets[k % len(self.device_sets)].fill_and_apply(self.d_mask.data_ptr(), t.data_ptr(), self.dtype_code, self.V,
                                                                    t.stride(0), stream=stream)

    def fused_step(self, k: int, stream: int):
        t = self.logits[k % len(self.logits)]
        xgm.fill_and_apply(self.sets[k % len(self.sets)], self.d_mask.data_ptr(), t.data_ptr(), self.dtype_code, self.V,
                           t.stride(0), stream=stream)
