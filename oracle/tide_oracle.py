"""CPU oracle for the TIDE MoE-step hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 statement of what the hot path computes, written from the
paper: per denoise step, every token of the block is routed to k of E experts;
experts that are in the GPU-resident set ("hits") contribute to the output and
the rest are listed as misses; a hit counter accumulates per-expert token hits
over the refresh interval; at a refresh step the resident set becomes the
current top-B experts by hits and only the newcomers are copied in.

The method is lossless (Sec. 3.3 "Lossless Inference"): placement decides where
a (token, expert) product is computed, never what it is.  The oracle is
therefore the plain definition of the routed MoE layer, evaluated in fp64 on
the bf16 / fp32 input values, one token and one expert at a time.  The only
library primitives used are numpy's matrix-vector / matrix-matrix products and
elementwise exp.

Nothing here is shared with, imported by, or derived from the HIP path.  Only
tests, the smoke check and the benchmark's cpu_baseline leg may import it.

Parity pins (tests/test_oracle_pins.py): every function below is pinned by at
least one of: brute-force full sort, scipy's expit / softmax, numpy bincount,
an independently written dense all-experts masked sum in torch fp64, the
lossless identity, hand-worked fixtures in tests/golden/, and brute-force
refresh rules; the policy driver is pinned to the Alg. 1 driver and to direct
statements of each counter rule.  No function is "parity unpinned".

Readings of points on which the paper is silent are marked R1..R12 and listed
in the design document.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

GATING_SOFTMAX = 0
GATING_SIGMOID = 1
BIAS_NONE = 0
BIAS_LOGIT = 1
BIAS_SELECT = 2

TIE_EPS = 1e-5


# --------------------------------------------------------------------------
# number formats
# --------------------------------------------------------------------------
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns (uint16) as fp64."""
    u32 = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u32.view(np.float32).astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bf16 value (ties to even) of fp64 numbers, returned as fp64.

    bf16 keeps 7 explicit mantissa bits; an fp64 has 52, so the low 45 bits are
    rounded away.  Inputs are assumed finite and inside bf16's normal range
    (true for every activation this path produces)."""
    u = np.ascontiguousarray(x, dtype=np.float64).view(np.uint64)
    low = np.uint64(45)
    r = u + ((np.uint64(1) << np.uint64(44)) - np.uint64(1)) + ((u >> low) & np.uint64(1))
    r = (r >> low) << low
    return r.view(np.float64)


# --------------------------------------------------------------------------
# routing: logits, gate, top-k   (Sec. 3.1: k of E experts per token)
# --------------------------------------------------------------------------
def router_logits(x_bits: np.ndarray, w_r: np.ndarray, bias: Optional[np.ndarray], bias_mode: int) -> np.ndarray:
    """z[n,e] = sum_j x[n,j] * W_r[e,j]  (+ b[e] when the bias is a logit offset)."""
    x = bf16_to_f64(x_bits)
    z = x @ np.asarray(w_r, dtype=np.float64).T
    if bias_mode == BIAS_LOGIT:
        z = z + np.asarray(bias, dtype=np.float64)[None, :]
    return z


def gate(z: np.ndarray, bias: Optional[np.ndarray], gating: int, bias_mode: int):
    """Return (sel, score, key).

    sel   : what the k largest are taken of
    score : what the routing weights are computed from (never includes a
            selection-only bias)
    key   : the quantity on which near-ties are measured -- the logit when the
            gate is a monotone function of it, else sel itself."""
    if gating == GATING_SOFTMAX:
        zs = z - z.max(axis=1, keepdims=True)
        p = np.exp(zs)
        p = p / p.sum(axis=1, keepdims=True)
        sel, score, key = p, p, z
    elif gating == GATING_SIGMOID:
        s = 1.0 / (1.0 + np.exp(-z))
        sel, score, key = s, s, z
    else:
        raise ValueError("gating")
    if bias_mode == BIAS_SELECT:
        sel = score + np.asarray(bias, dtype=np.float64)[None, :]
        key = sel
    return sel, score, key


def topk_route(sel: np.ndarray, score: np.ndarray, key: np.ndarray, k: int):
    """Pick the k largest sel per token.

    List order: descending sel, equal values by lower expert index (R3).
    w[n,i] = score_i / sum of the k selected scores (R1), so each token's
    weights sum to 1.  ``ambiguous[n]`` is set when any two neighbours among
    the k+1 largest keys are closer than TIE_EPS: fp32 arithmetic may order
    those differently, and such tokens are reported separately."""
    n_tok, n_exp = sel.shape
    idx = np.empty((n_tok, k), dtype=np.int32)
    w = np.empty((n_tok, k), dtype=np.float64)
    ambiguous = np.zeros(n_tok, dtype=bool)
    for n in range(n_tok):
        remaining = sel[n].copy()
        for i in range(k):
            e = int(np.argmax(remaining))        # first maximum = lowest index among equals
            idx[n, i] = e
            remaining[e] = -np.inf
        sc = score[n, idx[n]]
        w[n] = sc / sc.sum()
        top = np.sort(key[n])[::-1][: min(k + 1, n_exp)]
        ambiguous[n] = bool(np.any(top[:-1] - top[1:] < TIE_EPS))
    return idx, w, ambiguous


def route(x_bits, w_r, bias, gating: int, bias_mode: int, k: int):
    z = router_logits(x_bits, w_r, bias, bias_mode)
    sel, score, key = gate(z, bias, gating, bias_mode)
    idx, w, amb = topk_route(sel, score, key, k)
    return idx, w, amb, key


# --------------------------------------------------------------------------
# hit counter   (Fig. 1 caption: hits = number of tokens each expert processed)
# --------------------------------------------------------------------------
def step_histogram(idx: np.ndarray, n_experts: int) -> np.ndarray:
    hist = np.zeros(n_experts, dtype=np.int64)
    for e in idx.reshape(-1):
        hist[int(e)] += 1
    return hist


# --------------------------------------------------------------------------
# expert evaluation and the resident-partial output   (Alg. 1, token routing)
# --------------------------------------------------------------------------
def expert_ffn(x: np.ndarray, wg: np.ndarray, wu: np.ndarray, wd: np.ndarray, act_bf16: bool = True) -> np.ndarray:
    """e(x) = W_d ( silu(W_g x) * (W_u x) ),  silu(a) = a / (1 + exp(-a)).

    With act_bf16 the intermediate activation is stored in bf16 before the
    down projection (R10: bf16 storage, wide accumulation)."""
    g = wg @ x
    u = wu @ x
    a = (g / (1.0 + np.exp(-g))) * u
    if act_bf16:
        a = round_to_bf16(a)
    return wd @ a


WeightFn = Callable[[int], Tuple[np.ndarray, np.ndarray, np.ndarray]]   # expert id -> fp64 (Wg, Wu, Wd)


def moe_outputs(x_bits: np.ndarray, idx: np.ndarray, w: np.ndarray, slot_of: np.ndarray,
                weights: WeightFn, shared: Optional[Tuple[np.ndarray, np.ndarray, np.ndarray]],
                act_bf16: bool = True, tokens: Optional[Sequence[int]] = None,
                want_full: bool = True):
    """Resident-partial and full outputs plus the canonical miss list.

    y_res[n]  = shared(x_n) + sum over selected experts that are resident of w * e(x_n)
    y_full[n] = the same sum over all k selected experts
    miss      = every (n, expert, w) whose expert is not resident, ordered by
                token then by position in the token's top-k list.
    ``tokens`` restricts the (expensive) output evaluation to a sample of rows;
    the miss list always covers every token."""
    x = bf16_to_f64(x_bits)
    n_tok, k = idx.shape
    d = x.shape[1]
    rows = list(range(n_tok)) if tokens is None else [int(t) for t in tokens]
    y_res = np.zeros((len(rows), d))
    y_full = np.zeros((len(rows), d)) if want_full else None
    for r, n in enumerate(rows):
        if shared is not None:
            ys = expert_ffn(x[n], *shared, act_bf16=act_bf16)
            y_res[r] += ys
            if want_full:
                y_full[r] += ys
        for i in range(k):
            e = int(idx[n, i])
            hit = slot_of[e] >= 0
            if not hit and not want_full:
                continue
            contrib = w[n, i] * expert_ffn(x[n], *weights(e), act_bf16=act_bf16)
            if hit:
                y_res[r] += contrib
            if want_full:
                y_full[r] += contrib
    miss = [(n, int(idx[n, i]), float(w[n, i]))
            for n in range(n_tok) for i in range(k) if slot_of[int(idx[n, i])] < 0]
    return y_res, y_full, miss


# --------------------------------------------------------------------------
# refresh   (Alg. 1 refresh step; Sec. 3.3: the GPU set becomes the current top-B)
# --------------------------------------------------------------------------
def refresh(hits: np.ndarray, expert_in_slot: np.ndarray, capacity: int):
    """New placement from the interval's hit counts.

    Experts are ranked by (hits descending, currently resident first, lower
    index first); the first ``capacity`` are the new resident set, so a
    non-resident expert displaces a resident one only with strictly more hits
    (R7).  Leaving experts are ordered by (hits ascending, index), entering
    ones by (hits descending, index); the i-th entering expert takes the i-th
    freed slot, then empty slots in ascending order.  Returns
    (new expert_in_slot, plan) with plan = [(expert, slot), ...] -- one
    host-to-device copy per entering expert.  Eviction moves no bytes (R9)."""
    hits = np.asarray(hits)
    eis = np.asarray(expert_in_slot).copy()
    n_exp = len(hits)
    if capacity > len(eis) or capacity < 0 or capacity > n_exp:
        raise ValueError("capacity")
    resident = {int(e): s for s, e in enumerate(eis) if e >= 0}
    ranked = sorted(range(n_exp), key=lambda e: (-int(hits[e]), 0 if e in resident else 1, e))
    new = set(ranked[:capacity])
    leaving = sorted((e for e in resident if e not in new), key=lambda e: (int(hits[e]), e))
    entering = sorted((e for e in new if e not in resident), key=lambda e: (-int(hits[e]), e))
    free_slots = [resident[e] for e in leaving]
    for e in leaving:
        eis[resident[e]] = -1
    free_slots += [s for s in range(len(eis)) if expert_in_slot[s] < 0]
    plan = []
    for i, e in enumerate(entering):
        s = free_slots[i]
        eis[s] = e
        plan.append((e, s))
    return eis.astype(np.int32), plan


def slot_table(expert_in_slot: np.ndarray, n_experts: int) -> np.ndarray:
    slot_of = np.full(n_experts, -1, dtype=np.int32)
    for s, e in enumerate(expert_in_slot):
        if e >= 0:
            slot_of[int(e)] = s
    return slot_of


# --------------------------------------------------------------------------
# one block, in the driver's order (R4, R5, R6)
# --------------------------------------------------------------------------
def run_block(hidden_steps, w_r, bias, gating: int, bias_mode: int, k: int, n_experts: int,
              capacity: int, interval: int, initial_expert_in_slot: np.ndarray,
              weights: Optional[WeightFn] = None, shared=None, act_bf16: bool = True,
              output_steps: Optional[Sequence[int]] = None, output_tokens=None):
    """Run the denoise steps of one block for one layer.

    Per step t: if t > 0 and t % interval == 0, refresh from the hits of the
    interval just ended and clear the counter; then route step t, count its
    hits into the counter, split hits / misses against the placement now in
    force, and (for steps in ``output_steps``) evaluate the outputs.
    Returns a list of per-step dicts."""
    eis = np.asarray(initial_expert_in_slot, dtype=np.int32).copy()
    hits = np.zeros(n_experts, dtype=np.int64)
    log = []
    for t, x_bits in enumerate(hidden_steps):
        rec: Dict = {"t": t, "plan": None}
        if t > 0 and t % interval == 0:
            rec["hits_at_refresh"] = hits.copy()
            eis, plan = refresh(hits, eis, capacity)
            rec["plan"] = plan
            hits[:] = 0
        slot_of = slot_table(eis, n_experts)
        idx, w, amb, key = route(x_bits, w_r, bias, gating, bias_mode, k)
        hist = step_histogram(idx, n_experts)
        hits += hist
        rec.update(idx=idx, w=w, ambiguous=amb, key=key, hist=hist, hits=hits.copy(),
                   expert_in_slot=eis.copy(), slot_of=slot_of)
        rec["miss"] = [(n, int(idx[n, i]), float(w[n, i]))
                       for n in range(idx.shape[0]) for i in range(k) if slot_of[int(idx[n, i])] < 0]
        if weights is not None and (output_steps is None or t in output_steps):
            toks = None if output_tokens is None else output_tokens
            y_res, y_full, miss = moe_outputs(x_bits, idx, w, slot_of, weights, shared,
                                              act_bf16=act_bf16, tokens=toks)
            assert miss == rec["miss"]
            rec.update(y_res=y_res, y_full=y_full, tokens=toks)
        log.append(rec)
    return log


# --------------------------------------------------------------------------
# placement policies on the same layer (Sec. 4: the static and every-step baselines;
# Sec. 5 limitations: counters that outlive an interval or a block)
# --------------------------------------------------------------------------
def run_block_policy(hidden_steps, w_r, bias, gating: int, bias_mode: int, k: int, n_experts: int,
                     capacity: int, initial_expert_in_slot: np.ndarray, interval: Optional[int],
                     counter: str = "interval", decay: Tuple[int, int] = (1, 2), warm_start: bool = False,
                     initial_hits: Optional[np.ndarray] = None, deferred: int = 0):
    """Routing, counter, placement and miss lists of one block under a placement policy.

    interval = None: static placement, never refreshed (the Fiddler-like baseline); interval = 1:
    refresh before every step (the Mixtral-Offload-like baseline); otherwise Alg. 1.
    counter: what happens to H when a refresh has used it --
      "interval"    cleared (Alg. 1 as read in R4),
      "cumulative"  kept (hits since the start of the run),
      "decay"       H <- floor(H * num / den) with decay = (num, den): an exponentially fading memory.
    warm_start: step 0 is routed once on the initial placement only to count its hits, the placement is
    refreshed from them and the counter cleared (only with counter = "interval"), and step 0 is run again
    on the new placement, which counts it into the interval that starts there.
    initial_hits: H carried over from an earlier block (with initial_expert_in_slot its last placement).
    deferred = j > 0: the placement chosen by the refresh before step t (its copies overlap steps t..t+j-1)
    serves from step t+j on; until then the old placement does (R5's overlapped variant; True means j = 1).
    The counter is what it is without the delay; the choice is made against the placement in force, so with
    j <= interval the plans are those of the undelayed run too.  j must not exceed the interval.
    Returns (log, final expert_in_slot, final hits); log[t] has idx, w, hist, hits, expert_in_slot,
    slot_of, plan, miss like run_block's."""
    if warm_start and counter != "interval":
        raise ValueError("warm start is defined for the per-interval counter only")
    eis = np.asarray(initial_expert_in_slot, dtype=np.int32).copy()
    hits = np.zeros(n_experts, dtype=np.int64) if initial_hits is None else np.asarray(initial_hits, dtype=np.int64).copy()

    def after_refresh(h):
        if counter == "interval":
            h[:] = 0
        elif counter == "decay":
            h[:] = (h * decay[0]) // decay[1]
        elif counter != "cumulative":
            raise ValueError(counter)

    deferred = int(deferred)
    if deferred and warm_start:
        raise ValueError("a warm start is a blocking refresh")
    if deferred and (interval is None or deferred > interval):
        raise ValueError("the delay must not exceed the refresh interval")
    log = []
    pending, due = None, -1
    for t, x_bits in enumerate(hidden_steps):
        rec: Dict = {"t": t, "plan": None}
        if pending is not None and t == due:
            eis, pending = pending, None
        idx, w, amb, key = route(x_bits, w_r, bias, gating, bias_mode, k)
        hist = step_histogram(idx, n_experts)
        if t == 0 and warm_start:
            hits += hist
            eis, rec["plan"] = refresh(hits, eis, capacity)
            after_refresh(hits)
        elif interval is not None and t > 0 and t % interval == 0:
            new_eis, rec["plan"] = refresh(hits, eis, capacity)
            after_refresh(hits)
            if deferred:
                pending, due = new_eis, t + deferred
                rec["pending_expert_in_slot"] = new_eis.copy()
            else:
                eis = new_eis
        slot_of = slot_table(eis, n_experts)
        hits += hist
        rec.update(idx=idx, w=w, ambiguous=amb, key=key, hist=hist, hits=hits.copy(), expert_in_slot=eis.copy(),
                   slot_of=slot_of)
        rec["miss"] = [(n, int(idx[n, i]), float(w[n, i]))
                       for n in range(idx.shape[0]) for i in range(k) if slot_of[int(idx[n, i])] < 0]
        log.append(rec)
    return log, eis, hits


class ExpertStore:
    """Lazy fp64 view of a workload's bf16 expert weights (data handling only)."""

    def __init__(self, fetch_bits: Callable[[int], Tuple[np.ndarray, np.ndarray, np.ndarray]], max_cached: int = 512):
        self._fetch = fetch_bits
        self._cache: Dict[int, Tuple[np.ndarray, np.ndarray, np.ndarray]] = {}
        self._max = max_cached

    def __call__(self, e: int):
        got = self._cache.get(e)
        if got is None:
            if len(self._cache) >= self._max:
                self._cache.pop(next(iter(self._cache)))
            got = tuple(bf16_to_f64(m) for m in self._fetch(e))
            self._cache[e] = got
        return got
