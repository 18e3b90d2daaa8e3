"""CPU oracle for the closed denoising loop around the cached step.  TEST INFRASTRUCTURE ONLY.

What it follows
---------------
Sec. 3.1 (inference process of a diffusion LLM): the response starts fully masked; at every
step the mask predictor gives a distribution over the clean sequence, the greedy estimate is
the per-position argmax (Eq. for y-hat^(0|k)), and a transition function S (Eq.
transition_step) produces the next state by updating some of the tokens.  The appendix on
experimental details fixes what S is in the paper's runs: low-confidence remasking, with a
number of steps, a block length and a generation length per task (semi-autoregressive blocks
when the block is shorter than the generation).

The paper gives S by reference to the LLaDA sampler only; the readings taken here:
  * confidence of a position = softmax probability of its greedy token (temperature 0);
  * the response is cut into blocks of `block_len` positions that are completed left to right,
    `steps / num_blocks` steps per block;
  * a step unmasks, inside the current block, the masked positions with the highest
    confidence; how many is fixed by the schedule: the block's positions are spread evenly
    over the block's steps, the first `block_len % steps_per_block` steps take one more;
  * exact confidence ties go to the lower position, exact logit ties to the lower token id;
  * unmasked positions never change again; every position left masked by a step stays masked
    (that is the "remasking": its prediction is discarded).
  * the predictor's head: final RMSNorm of the step's output rows, then the vocabulary
    projection (architecture of the workloads; the paper does not describe it).
In bf16 mode the normed rows are rounded once (a bf16 implementation materialises them); the
logits, the softmax and the confidence stay in the working precision.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this file; it
imports nothing from the product.

Pins (tests/test_oracle_generate.py): greedy token and confidence against scipy's softmax and
numpy's argmax, engineered ties; the unmask schedule's sum, monotonicity and closed form; the
transition against a brute-force sort by (-confidence, position), its invariants (unmasked
tokens frozen, nothing outside the block touched, exactly n new tokens, no mask left after the
last step, block_len = L_r equals global top-n); the loop's hidden states against the uncached
forward of the embedded tokens when rho = 1 and K_p = K_r = 1.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np

from oracle import dllm_cache_oracle as O


def greedy_with_confidence(logits: np.ndarray):
    """Per row of `logits` [rows, vocab]: greedy token (lowest id among exact ties) and its
    softmax probability (Sec. 3.1, greedy estimate; confidence of low-confidence remasking)."""
    logits = np.asarray(logits)
    x0 = np.argmax(logits, axis=-1)  # numpy returns the first maximum
    mx = np.max(logits, axis=-1, keepdims=True)
    conf = 1.0 / np.sum(np.exp(logits - mx), axis=-1)
    return x0.astype(np.int64), conf


def unmask_counts(block_len: int, steps_per_block: int) -> List[int]:
    """How many positions each step of a block unmasks: an even split of the block over its
    steps, the remainder going to the first steps."""
    if block_len < 1 or steps_per_block < 1:
        raise ValueError("need block_len >= 1 and steps_per_block >= 1")
    base, extra = divmod(block_len, steps_per_block)
    return [base + (1 if t < extra else 0) for t in range(steps_per_block)]


def block_of_step(i: int, L_r: int, block_len: int, steps: int):
    """(first position, one past the last position, number to unmask) of step i."""
    if L_r % block_len or steps % (L_r // block_len):
        raise ValueError("block_len must divide L_r and the block count must divide steps")
    spb = steps // (L_r // block_len)
    b, t = divmod(i, spb)
    return b * block_len, (b + 1) * block_len, unmask_counts(block_len, spb)[t]


def low_confidence_transition(tokens: np.ndarray, x0: np.ndarray, conf: np.ndarray, mask_id: int,
                              lo: int, hi: int, n_unmask: int):
    """Transition S (Eq. transition_step) for one sequence's response: among the masked
    positions of [lo, hi) the n_unmask with the highest confidence (ties: lower position) take
    their greedy token; everything else is unchanged.  Returns (new tokens, chosen ascending)."""
    tokens = np.asarray(tokens).copy()
    elig = np.flatnonzero(tokens[lo:hi] == mask_id) + lo
    if n_unmask > elig.size:
        raise ValueError("the schedule asks for more positions than are masked in the block")
    order = np.lexsort((elig, -np.asarray(conf, dtype=np.float64)[elig]))  # by -conf, then position
    chosen = np.sort(elig[order[:n_unmask]])
    tokens[chosen] = np.asarray(x0)[chosen]
    return tokens, chosen


def head_logits(hidden_rows: np.ndarray, final_norm_g: np.ndarray, lm_head: np.ndarray, eps: float,
                storage: str = "f64") -> np.ndarray:
    """Mask predictor head for the given rows: RMSNorm with the final gain, then the vocabulary
    projection; [rows, vocab]."""
    z = O.rmsnorm(np.asarray(hidden_rows, dtype=np.float64), np.asarray(final_norm_g, dtype=np.float64), eps)
    if storage == "bf16":
        z = O.round_bf16(z)
    return z @ np.asarray(lm_head, dtype=np.float64).T


@dataclass
class GenReport:
    lo: int
    hi: int
    n_unmask: int
    x0: np.ndarray        # [B, L_r] greedy tokens of every response position
    conf: np.ndarray      # [B, L_r] their confidences
    logit_gap: np.ndarray  # [B, L_r] best minus second-best logit
    chosen: List[np.ndarray]  # per sequence, ascending positions unmasked by this step
    logits: List[np.ndarray]  # per sequence [L_r, vocab] (kept for near-tie checks at test sizes)
    hidden_out: np.ndarray    # [B, n, d] output rows of the denoiser
    step_report: object


class Generator:
    """The denoising loop of Sec. 3.1 around a (cached or uncached) denoiser.

    tokens: [B, n] token ids, prompt first; the response part starts as mask_id everywhere.
    """

    def __init__(self, denoiser: O.CachedDenoiser, embed: np.ndarray, final_norm_g: np.ndarray,
                 lm_head: np.ndarray, mask_id: int, steps: int, block_len: Optional[int] = None):
        self.den = denoiser
        self.embed = np.asarray(embed, dtype=np.float64)
        self.final_norm_g, self.lm_head = final_norm_g, lm_head
        self.mask_id, self.steps = int(mask_id), int(steps)
        self.block_len = int(block_len) if block_len else denoiser.L_r
        block_of_step(0, denoiser.L_r, self.block_len, self.steps)  # validates the schedule

    def step(self, tokens: np.ndarray, i: int, forced_chosen=None, forced_x0=None, on_layer=None):
        """One step: embed, denoise, predict, transition.  forced_chosen[b] / forced_x0 [B, L_r]
        replace the oracle's own decisions (to continue along another valid choice among
        near-ties).  Returns (new tokens [B, n], GenReport)."""
        den = self.den
        L_p, L_r = den.L_p, den.L_r
        tokens = np.asarray(tokens)
        hidden_in = self.embed[tokens]                      # [B, n, d]
        hidden_out, rep = den.step(hidden_in, i, on_layer=on_layer)
        lo, hi, n_unmask = block_of_step(i, L_r, self.block_len, self.steps)
        B = tokens.shape[0]
        x0 = np.zeros((B, L_r), dtype=np.int64)
        conf = np.zeros((B, L_r))
        gap = np.zeros((B, L_r))
        new_tokens = tokens.copy()
        chosen, all_logits = [], []
        for b in range(B):
            logits = head_logits(hidden_out[b, L_p:], self.final_norm_g, self.lm_head,
                                 den.model.rms_eps, den.storage)
            x0[b], conf[b] = greedy_with_confidence(logits)
            all_logits.append(logits)
            top2 = np.partition(logits, -2, axis=-1)[:, -2:]
            gap[b] = top2[:, 1] - top2[:, 0]
            use_x0 = x0[b] if forced_x0 is None else np.asarray(forced_x0[b])
            if forced_chosen is not None:
                ch = np.sort(np.asarray(forced_chosen[b], dtype=np.int64))
                resp = tokens[b, L_p:].copy()
                resp[ch] = use_x0[ch]
            else:
                resp, ch = low_confidence_transition(tokens[b, L_p:], use_x0, conf[b], self.mask_id,
                                                     lo, hi, n_unmask)
            new_tokens[b, L_p:] = resp
            chosen.append(ch)
        return new_tokens, GenReport(lo=lo, hi=hi, n_unmask=n_unmask, x0=x0, conf=conf, logit_gap=gap,
                                     chosen=chosen, logits=all_logits, hidden_out=hidden_out,
                                     step_report=rep)
