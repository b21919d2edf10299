"""Oracle adaptive draft-length controller (Sec. 3.3: the generation-length signal, the two
exponential moving averages and the one-line controller).  Test infrastructure only.

    L_gen = min(s - 1, k)                         s = 1-based index of the first EOS in the raw draft
    Lg~ = (1-rho) Lg~ + rho L_gen ;  La~ = (1-rho) La~ + rho L_acc
    k_next = clip( ceil( Lg~ + delta * [La~ >= Lg~] ), k_min, k_max )

Double precision; the indicator uses the already updated averages.
"""
from __future__ import annotations

import math


def first_eos_index(raw_draft, eos_id: int) -> int:
    """1-based index of the first EOS in the raw draft, 0 if there is none."""
    for i, t in enumerate(raw_draft):
        if int(t) == eos_id and eos_id >= 0:
            return i + 1
    return 0


class AdlState:
    def __init__(self, k_min: int, k_max: int, delta: float, rho: float):
        self.k_min, self.k_max, self.delta, self.rho = k_min, k_max, float(delta), float(rho)
        self.l_gen_ema = 0.0
        self.l_acc_ema = 0.0


def adl_update(st: AdlState, k_t: int, first_eos: int, l_acc: int) -> int:
    l_gen = min(first_eos - 1, k_t) if first_eos > 0 else k_t
    st.l_gen_ema = (1.0 - st.rho) * st.l_gen_ema + st.rho * l_gen
    st.l_acc_ema = (1.0 - st.rho) * st.l_acc_ema + st.rho * l_acc
    grow = st.delta if st.l_acc_ema >= st.l_gen_ema else 0.0
    z = math.ceil(st.l_gen_ema + grow)
    return int(min(max(z, st.k_min), st.k_max))
