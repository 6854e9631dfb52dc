"""TEST INFRASTRUCTURE -- placement closed forms written out with exact rationals.

Each function restates one definition or rule of the paper with Python
integers and ``fractions.Fraction`` so that no rounding enters.  Used by tests
to check the host-side evaluator of the GPU library; shares no code with it.
"""
from fractions import Fraction

MODES = ("R", "S", "S*", "M", "O")

# Table 2: (pi_Theta, pi_Omega, pi_G, pi_A) of the named strategies.
STRATEGIES = {
    "dp": ("R", "R", "R", "R"),
    "zero1": ("R", "S", "R", "R"),
    "zero2": ("R", "S", "S", "R"),
    "zero3": ("S*", "S", "S", "R"),
    "zero_offload": ("O", "O", "S", "R"),
    "tp": ("S", "S", "S", "S"),
    "pp": ("S", "S", "S", "R"),
}


def state_bytes(P):
    """Remark 1: |Theta| = 2P, |Omega| = 12P (master + m + v), |G| = 2P bytes."""
    return {"theta": 2 * P, "omega": 12 * P, "grad": 2 * P}


def mu(mode, s, N, s_unit=0):
    """Theorem 1, Eq. 7-11: per-device GPU bytes of a state of s bytes."""
    if mode == "R":
        return Fraction(s)
    if mode == "S":
        return Fraction(s, N)
    if mode == "S*":
        return Fraction(s, N) + s_unit
    if mode == "M":
        return Fraction(s_unit)
    if mode == "O":
        return Fraction(0)
    raise ValueError(mode)


def memory(spec, P, N, s_unit=0, act_bytes=0):
    """Theorem 1, Eq. 6: M(Pi) = sum of mu over the four states.  ``act_bytes``
    is the activation footprint |A| the caller accounts to one device."""
    sz = state_bytes(P)
    th, om, g, a = spec
    return (mu(th, sz["theta"], N, s_unit) + mu(om, sz["omega"], N, s_unit) +
            mu(g, sz["grad"], N, s_unit) + mu(a, act_bytes, N, s_unit))


def all_reduce(N, T):
    """Section 2.3: ring All-Reduce, bytes sent and received per device."""
    return Fraction(2 * (N - 1) * T, N)


def reduce_scatter(N, T):
    """Section 2.3: Reduce-Scatter, bytes per device."""
    return Fraction((N - 1) * T, N)


def all_gather(N, T):
    """Section 2.3: All-Gather, bytes per device."""
    return Fraction((N - 1) * T, N)


def communication(spec, P, N):
    """Theorem 2, Eq. 12-14: bytes per device per step.  Gradient sync is an
    All-Reduce under pi_G = R and a Reduce-Scatter under pi_G = S; pi_Theta =
    S* adds two All-Gathers of the parameters."""
    sz = state_bytes(P)
    th, _, g, _ = spec
    c = Fraction(0)
    if g == "R":
        c += all_reduce(N, sz["grad"])
    elif g == "S":
        c += reduce_scatter(N, sz["grad"])
    if th == "S*":
        c += 2 * all_gather(N, sz["theta"])
    return c


def shard_geometry(psi, N, i, align=1):
    """Definition 1, Eq. 2: device i holds X[i|X|/N : (i+1)|X|/N].  When N (times
    the alignment) does not divide psi the length is padded up to the next
    multiple and the pad falls at the end of the flat buffer.
    Returns (psi_padded, offset, length, valid_length)."""
    a = max(1, align)
    unit = N * a
    psi_pad = -(-psi // unit) * unit
    n = psi_pad // N
    off = i * n
    valid = min(max(psi - off, 0), n)
    return psi_pad, off, n, valid


def select_strategy(P, device_mem_bytes, N, layer_bytes=0, fast_interconnect=False):
    """Algorithm 1 (illustrative strategy selection), thresholds 0.7 and 0.3 as printed.
    Returns (spec, add_tp): data parallelism if 16P fits in 70 % of a device, else
    ZeRO-3 (whether or not 16P/N fits; that it does is the second test of the
    algorithm), with tensor parallelism added inside a node when a single layer
    exceeds 30 % of a device and the interconnect is fast.  add_tp is only
    considered on the path the algorithm reaches it: when ZeRO-3 alone does not fit."""
    m_model = 16 * P
    if Fraction(m_model) < Fraction(7, 10) * device_mem_bytes:
        return STRATEGIES["dp"], False
    if Fraction(m_model, N) < Fraction(7, 10) * device_mem_bytes:
        return STRATEGIES["zero3"], False
    add_tp = bool(Fraction(layer_bytes) > Fraction(3, 10) * device_mem_bytes and fast_interconnect)
    return STRATEGIES["zero3"], add_tp


def tp_dp_groups(T, D):
    """Theorem 6: on N = T*D devices TP group i is {iT, ..., (i+1)T-1}; data-parallel
    synchronisation runs across groups, between devices at the same position.
    Returns (tp_groups, dp_groups) as lists of device lists."""
    tp = [list(range(i * T, (i + 1) * T)) for i in range(D)]
    dp = [[i * T + j for i in range(D)] for j in range(T)]
    return tp, dp


def pp_dp_groups(K, D):
    """Theorem 7: on N = K*D devices stage k is replicated on {kD, ..., (k+1)D-1};
    gradient sync is among the replicas of one stage, activations move between
    corresponding replicas of adjacent stages.  Returns (stage_groups, pipelines)."""
    stages = [list(range(k * D, (k + 1) * D)) for k in range(K)]
    pipes = [[k * D + r for k in range(K)] for r in range(D)]
    return stages, pipes


def composed_cost(outer_spec, P, inner, D, s_unit=0):
    """Definition 5 with Theorems 6 and 7: an inner strategy of degree `inner` (TP degree,
    pipeline stages, or their product) leaves each device P/inner parameters; the outer
    data-parallel family specification acts on that share among the D devices holding the
    same share.  Returns (memory per device, bytes per device per step inside the outer
    group), Theorems 1 and 2 applied to the share.  The inner strategy's own activation
    traffic is not quantified by the paper and not included."""
    share = Fraction(P, inner)
    return memory(outer_spec, share, D, s_unit), communication(outer_spec, share, D)
