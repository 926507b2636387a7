"""Per-round latency model of the device-edge loop (Sec. IV-A communication model, Sec. IV-B computation
model) and the FH / SH choice it implies (Sec. III-B, Sec. VII discussion of the two upload options).

Host-side arithmetic only: payload sizes in bits, serialisation times under the effective link rate
R (1 - PER), one interaction overhead tau_RTT per exchange, and the modelled per-round latencies
T^FH, T^SH.  The edge-side compute term T_T + T_J is meant to be a measurement of this library's
verify round (wisv_last_round_ms), the drafter term a measurement or a model of the device.
Nothing here touches the GPU path.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

PROTO_FH, PROTO_SH = 0, 1


@dataclass(frozen=True)
class Link:
    """Channel state of one round: achievable rates (bit/s), packet error rates, round-level overhead (s)."""
    rate_up: float
    rate_down: float
    per_up: float = 0.0
    per_down: float = 0.0
    tau_rtt: float = 0.0

    def t_up(self, bits: float) -> float:
        return bits / (self.rate_up * (1.0 - self.per_up))

    def t_down(self, bits: float) -> float:
        return bits / (self.rate_down * (1.0 - self.per_down))


@dataclass(frozen=True)
class Framing:
    """Message framing: vocabulary, drafter hidden width and element bits, header and position-index bits."""
    vocab: int
    d_hidden: int
    bits_hidden: int = 16
    hdr_up: int = 0
    hdr_down: int = 0
    bits_pos: int = 8

    @property
    def b_id(self) -> int:                      # bits of a token ID
        return math.ceil(math.log2(self.vocab))

    @property
    def b_hid(self) -> int:                     # bits of one uploaded hidden vector
        return self.d_hidden * self.bits_hidden

    @property
    def b_fb(self) -> int:                      # feedback: first rejected position + corrected token
        return self.hdr_down + self.bits_pos + self.b_id

    def b_up_fh(self, k: int) -> int:           # token IDs and all hidden states in one message
        return self.hdr_up + k * self.b_id + k * self.b_hid

    def b_up1_sh(self, k: int) -> int:          # token IDs only
        return self.hdr_up + k * self.b_id

    def b_req(self, m: int) -> int:             # the edge's request for m positions
        return self.hdr_down + m * self.bits_pos

    def b_up2_sh(self, m: int) -> int:          # the requested hidden states
        return self.hdr_up + m * self.b_hid


def t_comm_fh(fr: Framing, link: Link, k: int) -> float:
    """One uplink message, one feedback message, one interaction overhead."""
    return link.t_up(fr.b_up_fh(k)) + link.t_down(fr.b_fb) + link.tau_rtt


def t_comm_sh(fr: Framing, link: Link, k: int, m: int) -> float:
    """IDs up, request down, requested hidden states up, feedback down: two interaction overheads."""
    return (link.t_up(fr.b_up1_sh(k)) + link.t_down(fr.b_req(m)) + link.t_up(fr.b_up2_sh(m)) +
            link.t_down(fr.b_fb) + 2.0 * link.tau_rtt)


def t_round(proto: int, fr: Framing, link: Link, k: int, m: int, t_draft: float, t_edge: float) -> float:
    """T^FH or T^SH of one round: drafter time + communication + edge time (target forward and head)."""
    comm = t_comm_fh(fr, link, k) if proto == PROTO_FH else t_comm_sh(fr, link, k, m)
    return t_draft + comm + t_edge


def choose_protocol(fr: Framing, link: Link, k: int, m_expected: float) -> int:
    """The option with the smaller modelled communication latency for an expected number of requested
    positions (the compute terms are the same for both).  SH saves (k - m) hidden vectors of uplink and
    pays one more interaction overhead, one request message and one more uplink header."""
    sh = (link.t_up(fr.b_up1_sh(k)) + link.t_down(fr.hdr_down + m_expected * fr.bits_pos) +
          link.t_up(fr.hdr_up + m_expected * fr.b_hid) + link.t_down(fr.b_fb) + 2.0 * link.tau_rtt)
    return PROTO_FH if t_comm_fh(fr, link, k) <= sh else PROTO_SH


RTT_THRESHOLD_S = 10e-3   # Sec. VII "Hardware Implementation": the testbed's switch-over point


def select_protocol_by_rtt(rtt_s: float, threshold_s: float = RTT_THRESHOLD_S) -> int:
    """The testbed's per-request rule (Sec. VII "Hardware Implementation"): the device measures the round-trip time
    with a light handshake before each request; full-hidden upload when it exceeds the threshold (an extra exchange
    would cost more than the larger payload), selective-hidden upload otherwise."""
    if not (rtt_s >= 0.0):
        raise ValueError("round-trip time must be a non-negative number of seconds")
    return PROTO_FH if rtt_s > threshold_s else PROTO_SH


def end_to_end(rounds) -> float:
    """T_E2E: the sum of the per-round latencies."""
    return float(sum(rounds))


def average_accepted_length(accepted) -> float:
    """AAL over the rounds of a generation: mean of A_r."""
    accepted = list(accepted)
    return sum(accepted) / len(accepted) if accepted else 0.0
