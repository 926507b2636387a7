"""The latency model of Sec. IV-A / IV-B against numbers worked out by hand from its equations
(B_fb, B_u^FH, B_u1/B_req/B_u2^SH, T_comm^FH, T_comm^SH, T^FH, T^SH, T_E2E) and against what the
equations imply about the two upload options."""
from fractions import Fraction as Fr

import pytest

from paper_2604_17701_amd import link_model as lm

FRAME = lm.Framing(vocab=128256, d_hidden=2048, bits_hidden=16, hdr_up=256, hdr_down=128, bits_pos=8)
LINK = lm.Link(rate_up=20e6, rate_down=50e6, per_up=0.1, per_down=0.05, tau_rtt=5e-3)


def test_payload_sizes_follow_the_equations():
    assert FRAME.b_id == 17                       # ceil(log2 128256): 2^16 < 128256 <= 2^17
    assert lm.Framing(vocab=1024, d_hidden=1).b_id == 10 and lm.Framing(vocab=1025, d_hidden=1).b_id == 11
    assert FRAME.b_hid == 32768                   # 2048 elements of 16 bits
    assert FRAME.b_fb == 128 + 8 + 17
    assert FRAME.b_up_fh(4) == 256 + 4 * 17 + 4 * 32768
    assert FRAME.b_up1_sh(4) == 256 + 4 * 17
    assert FRAME.b_req(3) == 128 + 3 * 8
    assert FRAME.b_up2_sh(3) == 256 + 3 * 32768


def test_communication_latency_worked_example():
    up, down = Fr(18_000_000), Fr(47_500_000)     # R (1 - PER): 20e6 * 0.9, 50e6 * 0.95
    fh = Fr(131396) / up + Fr(153) / down + Fr(5, 1000)
    sh1 = Fr(324) / up + Fr(136) / down + Fr(33024) / up + Fr(153) / down + Fr(10, 1000)
    assert lm.t_comm_fh(FRAME, LINK, 4) == pytest.approx(float(fh), rel=1e-12)
    assert lm.t_comm_sh(FRAME, LINK, 4, 1) == pytest.approx(float(sh1), rel=1e-12)
    assert float(fh) == pytest.approx(0.0123029989, abs=1e-9) and float(sh1) == pytest.approx(0.0118587509, abs=1e-9)
    # per-round and end-to-end latencies add the compute terms
    t = lm.t_round(lm.PROTO_FH, FRAME, LINK, 4, 0, t_draft=0.020, t_edge=0.0037)
    assert t == pytest.approx(float(fh) + 0.0237, rel=1e-12)
    assert lm.t_round(lm.PROTO_SH, FRAME, LINK, 4, 1, 0.020, 0.0037) == pytest.approx(float(sh1) + 0.0237, rel=1e-12)
    assert lm.end_to_end([t, t, 0.5]) == pytest.approx(2 * t + 0.5)


def test_selective_upload_trades_payload_for_a_round_trip():
    k = 6
    for m in range(k + 1):
        diff = lm.t_comm_sh(FRAME, LINK, k, m) - lm.t_comm_fh(FRAME, LINK, k)
        # SH pays one more overhead, one more uplink header and the request; it saves (k - m) hidden vectors
        want = (LINK.tau_rtt + LINK.t_up(FRAME.hdr_up) + LINK.t_down(FRAME.b_req(m)) - LINK.t_up((k - m) * FRAME.b_hid))
        assert diff == pytest.approx(want, rel=1e-9, abs=1e-15)
    assert lm.t_comm_sh(FRAME, LINK, k, k) > lm.t_comm_fh(FRAME, LINK, k)     # nothing saved: SH can only lose
    # requesting fewer positions never costs more
    ts = [lm.t_comm_sh(FRAME, LINK, k, m) for m in range(k + 1)]
    assert all(a < b for a, b in zip(ts, ts[1:]))


def test_protocol_choice_follows_the_model():
    k = 4
    slow = lm.Link(rate_up=2e6, rate_down=10e6, tau_rtt=2e-3)      # payload dominates: upload only what is asked for
    far = lm.Link(rate_up=200e6, rate_down=200e6, tau_rtt=20e-3)   # the extra round trip dominates
    assert lm.choose_protocol(FRAME, slow, k, m_expected=1.0) == lm.PROTO_SH
    assert lm.choose_protocol(FRAME, far, k, m_expected=1.0) == lm.PROTO_FH
    assert lm.choose_protocol(FRAME, slow, k, m_expected=float(k)) == lm.PROTO_FH
    # the switch-over overhead: tau* = t_up((k - m) B_hid) - t_up(hdr) - t_down(B_req(m))
    m = 1
    tau_star = slow.t_up((k - m) * FRAME.b_hid) - slow.t_up(FRAME.hdr_up) - slow.t_down(FRAME.b_req(m))
    below = lm.Link(slow.rate_up, slow.rate_down, tau_rtt=tau_star * 0.99)
    above = lm.Link(slow.rate_up, slow.rate_down, tau_rtt=tau_star * 1.01)
    assert lm.choose_protocol(FRAME, below, k, m) == lm.PROTO_SH and lm.choose_protocol(FRAME, above, k, m) == lm.PROTO_FH


def test_average_accepted_length():
    assert lm.average_accepted_length([4, 0, 2, 2]) == 2.0 and lm.average_accepted_length([]) == 0.0
