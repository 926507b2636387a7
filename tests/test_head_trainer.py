"""The decision head's offline trainer (Sec. V-A eqs. mlp_form / bce; Sec. V-B instances) and the testbed's RTT rule
(Sec. VII "Hardware Implementation").  CPU only."""
import numpy as np
import pytest
import torch

from oracle import wisv_oracle as wo
from paper_2604_17701_amd import head_trainer as ht
from paper_2604_17701_amd import link_model as lm
from paper_2604_17701_amd import relabel
from wisv_inputs import configs, gen


def test_rtt_rule_of_the_testbed():
    assert lm.select_protocol_by_rtt(9.9e-3) == lm.PROTO_SH
    assert lm.select_protocol_by_rtt(10.1e-3) == lm.PROTO_FH
    assert lm.select_protocol_by_rtt(10e-3) == lm.PROTO_SH            # "exceeds 10 ms": the boundary itself stays selective
    assert lm.select_protocol_by_rtt(0.0) == lm.PROTO_SH and lm.select_protocol_by_rtt(50e-3) == lm.PROTO_FH
    assert lm.select_protocol_by_rtt(3e-3, threshold_s=2e-3) == lm.PROTO_FH
    with pytest.raises(ValueError):
        lm.select_protocol_by_rtt(float("nan"))
    # the rule agrees with the latency model where the model is unambiguous: a long round trip on a fast link
    # favours one exchange, a short one on a slow link favours the smaller payload
    fr = lm.Framing(vocab=128256, d_hidden=2048, bits_hidden=16, hdr_up=256, hdr_down=256, bits_pos=8)
    assert lm.choose_protocol(fr, lm.Link(500e6, 500e6, 0.0, 0.0, 50e-3), 8, 3.0) == lm.select_protocol_by_rtt(50e-3)
    assert lm.choose_protocol(fr, lm.Link(20e6, 20e6, 0.0, 0.0, 2e-3), 8, 3.0) == lm.select_protocol_by_rtt(2e-3)


@pytest.mark.parametrize("act", [ht.ACT_RELU, ht.ACT_SILU])
def test_gradient_matches_finite_differences(act):
    rng = np.random.default_rng(3)
    x, y = rng.normal(size=(17, 6)), (rng.random(17) < 0.4).astype(np.float64)
    p = ht.init_params(6, 5, seed=1)
    p.b1 += 0.3                                   # away from the ReLU kink at exactly zero pre-activations
    loss, g = ht.loss_and_grad(p, x, y, act, pos_weight=1.7, weight_decay=0.05)
    h = 1e-6
    for name, index in (("w1", (2, 3)), ("w1", (0, 0)), ("b1", (4,)), ("w2", (1,)), ("b2", None)):
        q = p.copy()
        if index is None:
            q.b2 += h
            got = g.b2
        else:
            getattr(q, name)[index] += h
            got = getattr(g, name)[index]
        up, _ = ht.loss_and_grad(q, x, y, act, pos_weight=1.7, weight_decay=0.05)
        assert abs((up - loss) / h - got) < 1e-4 * max(1.0, abs(got)), (name, index)


def test_loss_is_the_papers_bce_and_class_balancing_evens_the_classes():
    p = ht.HeadParams(np.zeros((2, 3)), np.zeros(2), np.zeros(2), 0.0)       # s = 0: p = 1/2 everywhere
    x, y = np.ones((5, 3)), np.array([1.0, 0, 0, 0, 0])
    loss, _ = ht.loss_and_grad(p, x, y, ht.ACT_RELU)
    assert abs(loss - np.log(2.0)) < 1e-12                                    # -E[y log p + (1 - y) log(1 - p)]
    assert abs(loss - relabel.bce_loss(np.full(5, 0.5), y)) < 1e-12
    pw = ht.balanced_pos_weight(y)
    assert pw == 4.0                                                          # one positive weighs like four negatives
    lw, _ = ht.loss_and_grad(p, x, y, ht.ACT_RELU, pos_weight=pw)
    assert abs(lw - relabel.bce_loss(np.full(5, 0.5), y, pos_weight=pw)) < 1e-12


def _episodes(n_ep: int, seed: int):
    """Synthetic episodes in the paper's format: per mismatch a feature vector [h^D ; h^T ; c] and a criticality
    flag b_t, here planted as a separable rule of the features that also depends on the channel (a position is
    critical when a fixed direction of the hidden states exceeds a bar that a good link lowers)."""
    rng = np.random.default_rng(seed)
    d_d, d_t, d_c, t_len = 6, 10, 4, 5
    w_true = np.random.default_rng(99).normal(size=d_d + d_t)     # the planted rule: the same for every seed
    xs, ys = [], []
    for e in range(n_ep):
        hid = rng.normal(size=(t_len, d_d + d_t))
        snr = rng.uniform(0.0, 30.0)
        c = np.array([snr, rng.choice([5.0, 10.0, 20.0]), 0.0, rng.uniform(5.0, 50.0)])
        c[2] = c[1] * np.log2(1.0 + 10.0 ** (snr / 10.0))
        b = (hid @ w_true / np.sqrt(d_d + d_t) > (snr - 15.0) / 30.0).astype(np.int64)
        # stage 2 of Sec. V-B: smoothed importance, one multiplier per sampled channel state, sampled repairs
        x, a = relabel.training_instances(np.hstack([hid, np.tile(c, (t_len, 1))]), b, alpha=0.5, lams=[0.5], rho=0.05,
                                          u=rng.random((1, t_len)))
        xs.append(x)
        ys.append(a)
    return np.concatenate(xs), np.concatenate(ys), (d_d, d_t, d_c)


def test_trainer_learns_a_planted_rule_and_its_loss_falls():
    x, y, _ = _episodes(400, seed=11)
    out = ht.train(x, y, d_hidden=16, act=ht.ACT_RELU, steps=600, lr=2e-2, weight_decay=1e-4, seed=5)
    losses = out["losses"]
    assert losses[-1] < 0.35 * losses[0] and min(losses[-50:]) <= min(losses[:50])
    xv, yv, _ = _episodes(150, seed=12)                     # fresh episodes of the same rule
    acc = np.mean((ht.forward(out["params"], xv, ht.ACT_RELU) >= 0.5) == (yv == 1))
    assert acc > 0.9, acc
    # class balancing: with few positives the balanced head still finds them
    keep = np.concatenate([np.nonzero(y == 0)[0], np.nonzero(y == 1)[0][:40]])
    bal = ht.train(x[keep], y[keep], d_hidden=16, steps=400, lr=2e-2, balance=True, seed=5)
    raw = ht.train(x[keep], y[keep], d_hidden=16, steps=400, lr=2e-2, balance=False, seed=5)
    assert bal["pos_weight"] > 3.0 and raw["pos_weight"] == 1.0
    recall = lambda r: np.mean(ht.forward(r["params"], xv[yv == 1], ht.ACT_RELU) >= 0.5)
    assert recall(bal) > 0.7 and recall(bal) > recall(raw) + 0.1, (recall(bal), recall(raw))


@pytest.mark.parametrize("act", [ht.ACT_RELU, ht.ACT_SILU])
def test_exported_head_is_the_head_the_round_evaluates(act):
    """A trained head, exported in the library's layout, gives through the oracle's head (the definition the HIP path
    is held to) the probabilities the trainer computes: same column order, same polarity (p is the rejection
    probability, the round reports 1 - p)."""
    x, y, (d_d, d_t, d_c) = _episodes(60, seed=21)
    out = ht.train(x, y, d_hidden=8, act=act, steps=60, seed=2)
    w = ht.export_weights(out["params"])
    shape = configs.ModelShape(n_layers=1, d_model=d_t, n_heads=1, n_kv_heads=1, head_dim=d_t, d_ff=8, vocab=16,
                               dtype="f32", d_draft=d_d, d_csi=d_c, d_head_hidden=8, head_act=act)
    wh = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in gen.make_weights(shape, 1, "cpu").items()}
    for k, v in w.items():
        wh[k] = torch.from_numpy(v).contiguous()
    orc = wo.Oracle(shape, wh)
    p_train = ht.forward(out["params"], x[:12], act)
    for i in range(12):
        s, p_rej, p_acc = orc.head(x[i, :d_d], x[i, d_d:d_d + d_t], x[i, d_d + d_t:])
        assert abs(p_rej - p_train[i]) < 2e-5 and abs(p_acc - (1.0 - p_train[i])) < 2e-5
