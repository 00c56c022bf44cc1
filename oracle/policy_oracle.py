"""Oracle of the host-side policy: TEST INFRASTRUCTURE, not a product path.

Plain Python, exact rational arithmetic where a decision depends on a comparison, written from the
paper's equations.  Only ``tests/`` may import it.

* Section 3.1, Eq. 1: time a decoding request can give away to prefills of other requests.
* Section 3.1, Eq. 2 and Algorithm 1: how many queued prefills fit.
* Section 3.1, Eq. 3: prefill time model.
* Section 3.2.1, Eq. 4 (the second equation of the paper that carries the prefill label): offload
  time model; the smallest number x of layers to retain so that the offload hides behind the prefill.
* Section 3.2.1, Eq. 5: free-block forecast; the pressure rule (x/2 layers of the most recent
  requests first, then the rest).

Where the paper leaves something open, the function concerned states the reading it takes.
"""
from __future__ import annotations

from fractions import Fraction as F
from typing import List, Optional, Sequence, Tuple


def _f(x) -> F:
    return x if isinstance(x, F) else F(x)


# ----------------------------------------------------------------------------- Eq. 3, Eq. 4
def prefill_time(alpha, seqlen: int, n_param, n_hidden, device_flops) -> F:
    """Eq. 3: alpha * seqlen * (2 n_param + 2 seqlen n_hidden) / FLOPS."""
    s = _f(seqlen)
    return _f(alpha) * s * (2 * _f(n_param) + 2 * s * _f(n_hidden)) / _f(device_flops)


def offload_time(beta, seqlen: int, num_layers: int, x: int, head_dim: int, num_heads: int, bytes_per_elem,
                 link_bytes_per_s) -> F:
    """Eq. 4: beta * seqlen * 2 (L - x) d_heads n_heads f_precision / PCIe bandwidth.  n_heads are the heads
    whose K and V are stored (KV heads); the factor 2 is K and V; f_precision in bytes."""
    return (_f(beta) * _f(seqlen) * 2 * (num_layers - x) * head_dim * num_heads * _f(bytes_per_elem)
            / _f(link_bytes_per_s))


def min_retained_layers(alpha, n_param, n_hidden, device_flops, beta, num_layers: int, head_dim: int, num_heads: int,
                        bytes_per_elem, link_bytes_per_s, seqlen: int) -> int:
    """Smallest x in 0..L with T_offload(x) <= T_prefill (Section 3.2.1): tried in increasing order."""
    tp = prefill_time(alpha, seqlen, n_param, n_hidden, device_flops)
    for x in range(num_layers + 1):
        if offload_time(beta, seqlen, num_layers, x, head_dim, num_heads, bytes_per_elem, link_bytes_per_s) <= tp:
            return x
    raise AssertionError("x = L always satisfies the condition (nothing is offloaded)")


def retained_layers(num_layers: int, x: int) -> List[int]:
    """Even spread of Section 3.2.2 (8 layers, x = 4: layers 1, 3, 5, 7 stay)."""
    return [l for l in range(num_layers) if ((l + 1) * x) // num_layers > (l * x) // num_layers]


# ----------------------------------------------------------------------------- Eq. 1, Eq. 2, Algorithm 1
def n_future(n_past: int, predicted_lower_bound: int) -> int:
    """Tokens still to come: lower bound of the predicted length range minus what exists, at least 1."""
    return max(1, predicted_lower_bound - n_past)


def allow_prefill_time(t_tpot, n_past: int, t_past, predicted_lower_bound: int) -> F:
    """Eq. 1.  T_future = current TPOT * N_future, current TPOT = T_past / N_past (T_past includes waiting);
    a request that has produced nothing yet is taken to run at its target."""
    nf = n_future(n_past, predicted_lower_bound)
    tpot_now = _f(t_past) / n_past if n_past > 0 else _f(t_tpot)
    t_future = tpot_now * nf
    return _f(t_tpot) * (n_past + nf) - (_f(t_past) + t_future)


def max_prefills(allow: Sequence, t_prefill_queue: Sequence) -> int:
    """Algorithm 1: largest n with sum of the first n queued prefill times < min_i T_allow_i (strict);
    with no decoding request nothing constrains the queue."""
    if len(allow) == 0:
        return len(t_prefill_queue)
    budget = min(_f(a) for a in allow)
    total, n = F(0), 0
    for t in t_prefill_queue:
        total += _f(t)
        if not total < budget:
            break
        n += 1
    return n


# ----------------------------------------------------------------------------- Eq. 5 and the pressure rule
def forecast_avail(avail0: int, released: Sequence[int], allocated: Sequence[int]) -> List[int]:
    """Eq. 5 unrolled: Avail(t+1) = Avail(t) + Released(t) - Allocated(t); returns Avail(1..T)."""
    out, a = [], avail0
    for r, al in zip(released, allocated):
        a = a + r - al
        out.append(a)
    return out


def first_stage_below(avail0: int, released: Sequence[int], allocated: Sequence[int], threshold: int) -> int:
    """First stage t >= 1 whose forecast falls below the threshold, or -1."""
    for t, a in enumerate(forecast_avail(avail0, released, allocated), start=1):
        if a < threshold:
            return t
    return -1


def pressure_offload(deficit_blocks: int, retained: Sequence[int], blocks_per_layer: Sequence[int]) -> List[int]:
    """How many of its retained layers each request gives up.  Requests are listed MOST RECENT FIRST.  First pass:
    half of a request's retained layers (rounded up, so that a single retained layer can go), request after
    request, stopping as soon as the blocks freed cover the deficit; second pass, only if the first was not
    enough: the rest of each request's layers in the same order."""
    give = [0] * len(retained)
    freed = 0
    if deficit_blocks <= 0:
        return give
    for r, (x, b) in enumerate(zip(retained, blocks_per_layer)):
        if freed >= deficit_blocks:
            return give
        give[r] = (x + 1) // 2
        freed += give[r] * b
    for r, (x, b) in enumerate(zip(retained, blocks_per_layer)):
        if freed >= deficit_blocks:
            return give
        freed += (x - give[r]) * b
        give[r] = x
    return give


# ----------------------------------------------------------------------------- Section 3.2.3, link check per sub-unit
def gated_units(answers: Sequence[bool], units: int, max_checks: int) -> Tuple[int, int]:
    """Before each of `units` sub-units the link is asked whether it is busy; a busy answer delays and asks again,
    at most max_checks questions per unit, after which the unit goes anyway.  `answers` is the sequence of replies
    in the order asked (True = busy; exhausted = free).  Returns (questions asked, busy answers = delays)."""
    it = iter(answers)
    asked = busy = 0
    for _ in range(units):
        for _ in range(max_checks):
            asked += 1
            if not next(it, False):
                break
            busy += 1
    return asked, busy
