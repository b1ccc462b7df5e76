"""Oracle for the P/D allocation model, in plain Python floats (IEEE binary64).

TEST INFRASTRUCTURE ONLY; shares nothing with the C library.  Each step is the
paper's closed form written out:

  T_s          = TTFT - T_overhead                                   Eq. (12)
  TP_prefill   = TPhat_prefill - L_in / T_s                          Eq. (13)
  b*           = largest measured batch whose TPOT meets the target;
  TP_decode    = b* / TPOT(b*)            (section "Acquire decode throughput under TPOT constraints")
  N_prefill    = TP_total L_in  / ((L_in + L_out) TP_prefill)        Eq. (5)
  N_decode     = TP_total L_out / ((L_in + L_out) TP_decode)         Eq. (6)
  R_P/D        = L_in TP_decode / (L_out TP_prefill)                 Eq. (7)

Readings of points the paper leaves open:
  * integer counts: round half up, at least 1 (the only rule that reproduces the
    paper's "3P4D" from 3.07 and 3.77 in its Evaluation section); `rounding=1` = ceiling.
  * the decode point is the largest *measured* batch meeting the TPOT target over the
    whole curve (duplicates of a batch keep their smallest TPOT); no interpolation.
  * infeasible TTFT: T_s <= 0 or Eq. (13) <= 0; infeasible TPOT: no measured point meets it.

Pinned by tests/test_oracle_allocator.py against the numbers printed in the paper's
Evaluation section, the M/M/1 sojourn identity 1/(mu - lambda) = T_s, Eq. (4) balance,
Eq. (7) = Eq. (5)/Eq. (6), monotonicity and a discrete-event M/M/1 simulation.
"""
import math


class TTFTInfeasible(ValueError):
    pass


class TPOTInfeasible(ValueError):
    pass


def effective_prefill_throughput(tp_prefill_max, l_in, ttft, t_overhead=0.0):
    """Eq. (13); raises TTFTInfeasible when no positive arrival rate meets the TTFT."""
    t_s = ttft - t_overhead
    if not (t_s > 0.0):
        raise TTFTInfeasible("TTFT - T_overhead <= 0")
    tp = tp_prefill_max - l_in / t_s
    if not (tp > 0.0):
        raise TTFTInfeasible("Eq. (13) gives a non-positive prefill throughput")
    return tp


def decode_operating_point(batches, tpots, tpot_slo):
    """Largest measured batch whose TPOT <= target -> (batch, tpot, batch / tpot)."""
    best = {}
    for b, t in zip(batches, tpots):
        b = int(b)
        t = float(t)
        if b not in best or t < best[b]:
            best[b] = t
    feas = [b for b, t in best.items() if t <= tpot_slo]
    if not feas:
        raise TPOTInfeasible("no measured batch meets the TPOT target")
    b = max(feas)
    return b, best[b], b / best[b]


def round_count(n_real, rounding=0):
    if rounding == 0:
        n = math.floor(n_real + 0.5)
    else:
        n = math.ceil(n_real)
    return max(1, int(n))


def allocate(tp_total, l_in, l_out, ttft_slo, tpot_slo, prefill_max_tps, decode_batch, decode_tpot_s,
             t_overhead_s=0.0, rounding=0):
    vals = [tp_total, l_in, l_out, ttft_slo, tpot_slo, prefill_max_tps]
    if any((not math.isfinite(v)) or v <= 0.0 for v in vals):
        raise ValueError("non-positive or non-finite input")
    if (not math.isfinite(t_overhead_s)) or t_overhead_s < 0.0:
        raise ValueError("bad T_overhead")
    if len(decode_batch) == 0 or len(decode_batch) != len(decode_tpot_s):
        raise ValueError("bad curve")
    for b, t in zip(decode_batch, decode_tpot_s):
        if b <= 0 or (not math.isfinite(t)) or t <= 0.0:
            raise ValueError("bad curve point")
    tp_p = effective_prefill_throughput(prefill_max_tps, l_in, ttft_slo, t_overhead_s)
    b_star, tpot_star, tp_d = decode_operating_point(decode_batch, decode_tpot_s, tpot_slo)
    n_p = (tp_total * l_in) / ((l_in + l_out) * tp_p)
    n_d = (tp_total * l_out) / ((l_in + l_out) * tp_d)
    r = (l_in * tp_d) / (l_out * tp_p)
    return {
        "tp_prefill_eff": tp_p, "tp_decode_eff": tp_d, "decode_batch": b_star,
        "decode_tpot_s": tpot_star, "n_prefill_real": n_p, "n_decode_real": n_d, "ratio_pd": r,
        "n_prefill": round_count(n_p, rounding), "n_decode": round_count(n_d, rounding),
    }


# ---- M/M/1 pieces, Eqs. (9)-(12) ---------------------------------------------------------------

def service_rate(tp_prefill_max, l_in):
    return tp_prefill_max / l_in                     # Eq. (9)


def utilisation(lam, mu):
    return lam / mu                                  # Eq. (10)


def mm1_sojourn(mu, lam):
    if not lam < mu:
        raise ValueError("arrival rate must stay below the service rate")
    return 1.0 / (mu - lam)                          # Eq. (12)


def mg1_sojourn(lam, mean_s, mean_s2):
    """Pollaczek-Khinchine mean sojourn time (context for the queue check; not in the paper)."""
    rho = lam * mean_s
    return mean_s + lam * mean_s2 / (2.0 * (1.0 - rho))


def kv_transfer_overhead(l_in, n_layers, n_kv_heads, head_dim, bytes_per_elem, link_bytes_per_s, fixed_s=0.0):
    """The overhead term of Eq. (8) modelled from its named parts: a fixed part (user-side
    transmission) plus the prompt's keys and values of every layer over one link."""
    kv_bytes = l_in * (n_layers * 2.0 * n_kv_heads * head_dim * bytes_per_elem)
    return fixed_s + kv_bytes / link_bytes_per_s


def fifo_replay(arrivals, services):
    """Single FIFO server in virtual time: D_i = max(A_i, D_{i-1}) + S_i; returns D_i - A_i."""
    out = []
    done = -math.inf
    for a, s in zip(arrivals, services):
        start = a if a > done else done
        done = start + s
        out.append(done - a)
    return out


def fifo_replay_batched(arrivals, batch_service, max_batch):
    """One server that, whenever it becomes free, takes the first min(max_batch, waiting) requests
    of the FIFO queue and serves them together (the regime the paper's "Acquire prefill throughput
    under TTFT constraints" describes for a chunked prefill size much larger than the request
    length: several queued requests are batched into one chunk).  batch_service[b-1] is the service
    time of a batch of b equal-length requests; every request of a batch completes at the batch's
    end.  An idle server starts as soon as one request is present.  Returns each request's
    sojourn time (completion - arrival), in arrival order.  max_batch = 1 is fifo_replay with a
    constant service time."""
    n = len(arrivals)
    out = [0.0] * n
    free_at = -math.inf
    i = 0
    while i < n:
        start = arrivals[i] if arrivals[i] > free_at else free_at
        b = 1
        while b < max_batch and i + b < n and arrivals[i + b] <= start:
            b += 1
        done = start + batch_service[b - 1]
        for j in range(i, i + b):
            out[j] = done - arrivals[j]
        free_at = done
        i += b
    return out


def effective_prefill_throughput_dp(tp_prefill_max, l_in, ttft, t_overhead, groups):
    """Eq. (13) with prefill-side data parallelism: each of `groups` DP groups is its own M/M/1
    queue with 1/groups of the instance's maximum throughput and of its arrivals (the paper's
    remark under Eq. (8)), so per group TP = TP_max/groups - l_in/T_s and the instance achieves
    groups times that."""
    t_s = ttft - t_overhead
    if not (t_s > 0.0):
        raise TTFTInfeasible("TTFT - T_overhead <= 0")
    per_group = (tp_prefill_max / groups) - (l_in / t_s)
    if not (per_group > 0.0):
        raise TTFTInfeasible("Eq. (13) per DP group <= 0")
    return groups * per_group


def allocate_stages(tp_total, l_in, l_out, stage_work, stage_tps, rounding=0):
    """Eqs. (5), (6) for any number of independently deployed pipeline stages (the paper's
    conclusion names encode / prefill / decode disaggregation as the generalisation): requests
    arrive at tp_total / (l_in + l_out) per second (Eq. (1)); stage k does stage_work[k] units of
    work per request (tokens, images, ...) at stage_tps[k] units per second per instance, and
    every stage takes the same time (Eq. (4)), so N_k = (tp_total * work_k) / ((l_in + l_out) * tps_k).
    Returns (real counts, integer counts)."""
    vals = [tp_total, l_in, l_out] + list(stage_work) + list(stage_tps)
    if len(stage_work) == 0 or len(stage_work) != len(stage_tps):
        raise ValueError("bad stage lists")
    if any((not math.isfinite(v)) or v <= 0.0 for v in vals):
        raise ValueError("non-positive or non-finite input")
    real = [(tp_total * w) / ((l_in + l_out) * t) for w, t in zip(stage_work, stage_tps)]
    return real, [round_count(n, rounding) for n in real]
