"""Pins of the oracle's individual equations against closed forms, special cases and
library routines.  None of these tests touches the HIP library."""
import math
from decimal import Decimal, getcontext

import numpy as np
import pytest
import torch

from oracle import oracle as orc

RNG = np.random.default_rng(20260321)


def paired_time_params(d_t):
    lad = 10.0 ** (-9.0 * np.arange(d_t // 2) / max(d_t // 2 - 1, 1))
    omega = np.repeat(lad, 2).astype(np.float32)
    phase = np.tile(np.array([0.0, -math.pi / 2]), d_t // 2).astype(np.float32)
    return omega, phase


# ---------------------------------------------------------------- time encoding (Sec. 2.2.1)

def test_phi_zero_is_one_zero_pattern():
    om, ph = paired_time_params(100)
    out = orc.time_encode(om, ph, 0.0)
    expect = np.tile([1.0, 0.0], 50) * math.sqrt(1 / 100)
    assert np.abs(out - expect).max() < 1e-8


@pytest.mark.parametrize("x", [0.3, 17.0, 12345.678, 9.87e6])
def test_phi_norm_is_half(x):
    om, ph = paired_time_params(64)
    out = orc.time_encode(om, ph, x)
    assert abs(np.dot(out, out) - 0.5) < 1e-6       # cos^2+sin^2 per pair, d_t/2 pairs, scale 1/d_t


def test_phi_pairs_are_cos_and_sin():
    om, ph = paired_time_params(8)
    x = 3.25
    out = orc.time_encode(om, ph, x) * math.sqrt(8)
    for j in range(4):
        w = float(om[2 * j])
        assert abs(out[2 * j] - math.cos(w * x)) < 1e-12
        assert abs(out[2 * j + 1] - math.sin(w * x)) < 1e-6    # fp32 phase -pi/2 is 4e-8 off


def test_phi_periodic():
    om = np.array([0.5, 0.25], dtype=np.float32)     # exact in fp32
    ph = np.array([0.3, -1.0], dtype=np.float32)
    a = orc.time_encode(om, ph, 11.0)
    b0 = orc.time_encode(om, ph, 11.0 + 2 * math.pi / 0.5)
    b1 = orc.time_encode(om, ph, 11.0 + 2 * math.pi / 0.25)
    assert abs(a[0] - b0[0]) < 1e-12 and abs(a[1] - b1[1]) < 1e-12


def test_phi_large_argument_against_high_precision_reduction():
    # x ~ 1e7: reduce omega*x + b modulo 2*pi with 60-digit decimals, then take the cosine
    getcontext().prec = 60
    pi = Decimal("3.14159265358979323846264338327950288419716939937510582097494")
    om = np.array([1.0, 0.8125, 0.001953125], dtype=np.float32)
    ph = np.array([0.0, 0.5, -1.25], dtype=np.float32)
    x = 9876543.21875
    out = orc.time_encode(om, ph, x) * math.sqrt(3)
    for i in range(3):
        arg = Decimal(float(om[i])) * Decimal(x) + Decimal(float(ph[i]))
        red = float(arg - (arg / (2 * pi)).to_integral_value() * 2 * pi)
        assert abs(out[i] - math.cos(red)) < 5e-9


# ---------------------------------------------------------------- message (Eq. msg_linear)

def _mk_oracle(d_mem=5, d_edge=3, d_time=4, d_msg=5, W_msg=None, b_msg=None):
    kin = 2 * d_mem + d_edge + d_time
    om, ph = paired_time_params(d_time)
    z = lambda *s: np.zeros(s, dtype=np.float32)
    w = dict(omega=om, phase=ph,
             W_msg=z(kin, d_msg) if W_msg is None else W_msg,
             b_msg=z(d_msg) if b_msg is None else b_msg,
             W_z=z(d_msg, d_mem), U_z=z(d_mem, d_mem), b_z=z(d_mem),
             W_r=z(d_msg, d_mem), U_r=z(d_mem, d_mem), b_r=z(d_mem),
             W_h=z(d_msg, d_mem), U_h=z(d_mem, d_mem), b_h=z(d_mem),
             W_Q=[z(d_mem + d_time, 4)], W_K=[z(d_mem + d_edge + d_time, 4)],
             W_V=[z(d_mem + d_edge + d_time, 4)], W_O=[z(4, 4)], b_O=[z(4)])
    return orc.Oracle(num_nodes=4, d_mem=d_mem, d_node=0, d_edge=d_edge, d_time=d_time, d_emb=4, d_msg=d_msg,
                      k=2, heads=2, layers=1, weights=w)


def test_message_selects_each_input_block():
    d_mem, d_edge, d_time = 5, 3, 4
    kin = 2 * d_mem + d_edge + d_time
    s_self = RNG.standard_normal(d_mem).astype(np.float32)
    s_other = RNG.standard_normal(d_mem).astype(np.float32)
    e = RNG.standard_normal(d_edge).astype(np.float32)
    dt = 2.75
    # block order must be [self | other | edge | phi(dt)]
    for off, width, expect in ((0, d_mem, s_self), (d_mem, d_mem, s_other), (2 * d_mem, d_edge, e)):
        W = np.zeros((kin, 5), dtype=np.float32)
        W[off:off + width, :width] = np.eye(width)
        o = _mk_oracle(W_msg=W, b_msg=np.arange(5, dtype=np.float32))
        m = o.message(s_self, s_other, e, dt)
        want = np.arange(5, dtype=np.float64)
        want[:width] += expect
        assert np.abs(m - want).max() < 1e-12
    W = np.zeros((kin, 5), dtype=np.float32)
    W[2 * d_mem + d_edge:, :d_time] = np.eye(d_time)
    o = _mk_oracle(W_msg=W)
    om, ph = paired_time_params(d_time)
    m = o.message(s_self, s_other, e, dt)
    assert np.abs(m[:d_time] - orc.time_encode(om, ph, dt)).max() < 1e-15


def test_message_matches_library_matmul():
    d_mem, d_edge, d_time = 5, 3, 4
    kin = 2 * d_mem + d_edge + d_time
    W = RNG.standard_normal((kin, 5)).astype(np.float32)
    b = RNG.standard_normal(5).astype(np.float32)
    o = _mk_oracle(W_msg=W, b_msg=b)
    s_self = RNG.standard_normal(d_mem).astype(np.float32)
    s_other = RNG.standard_normal(d_mem).astype(np.float32)
    e = RNG.standard_normal(d_edge).astype(np.float32)
    om, ph = paired_time_params(d_time)
    x = np.concatenate([s_self, s_other, e, orc.time_encode(om, ph, 7.5)]).astype(np.float64)
    want = x @ W.astype(np.float64) + b
    assert np.abs(o.message(s_self, s_other, e, 7.5) - want).max() < 1e-12


# ---------------------------------------------------------------- GRU (Eq. gru_detail)

def _zeros_gru(d_msg, d_mem):
    z = lambda *s: np.zeros(s, dtype=np.float32)
    return dict(W_z=z(d_msg, d_mem), U_z=z(d_mem, d_mem), b_z=z(d_mem),
                W_r=z(d_msg, d_mem), U_r=z(d_mem, d_mem), b_r=z(d_mem),
                W_h=z(d_msg, d_mem), U_h=z(d_mem, d_mem), b_h=z(d_mem))


def test_gru_all_zero_weights_halves_state():
    p = _zeros_gru(4, 4)
    s = RNG.standard_normal(4)
    out = orc.gru(**p, m=RNG.standard_normal(4), s=s)
    assert np.abs(out - 0.5 * s).max() < 1e-15      # z = 1/2, candidate = tanh(0) = 0


def test_gru_update_gate_saturated_keeps_state():
    p = _zeros_gru(4, 4)
    p["b_z"][:] = 40.0
    p["W_h"] = RNG.standard_normal((4, 4)).astype(np.float32)
    s = RNG.standard_normal(4)
    out = orc.gru(**p, m=RNG.standard_normal(4), s=s)
    assert np.abs(out - s).max() < 1e-15


def test_gru_update_gate_closed_gives_tanh_of_message():
    p = _zeros_gru(4, 4)
    p["b_z"][:] = -40.0
    p["W_h"] = np.eye(4, dtype=np.float32)
    m = RNG.standard_normal(4)
    out = orc.gru(**p, m=m, s=RNG.standard_normal(4))
    assert np.abs(out - np.tanh(m)).max() < 1e-15


def _torch_gru_cell(p, m, s):
    d_msg, d_mem = p["W_z"].shape
    cell = torch.nn.GRUCell(d_msg, d_mem, bias=True, dtype=torch.float64)
    with torch.no_grad():
        cell.weight_ih.copy_(torch.tensor(np.concatenate([p["W_r"].T, p["W_z"].T, p["W_h"].T]), dtype=torch.float64))
        cell.weight_hh.copy_(torch.tensor(np.concatenate([p["U_r"].T, p["U_z"].T, p["U_h"].T]), dtype=torch.float64))
        cell.bias_ih.copy_(torch.tensor(np.concatenate([p["b_r"], p["b_z"], p["b_h"]]), dtype=torch.float64))
        cell.bias_hh.zero_()
        return cell(torch.tensor(m)[None], torch.tensor(s)[None])[0].numpy()


def test_gru_matches_library_cell_when_Uh_is_diagonal():
    d_msg, d_mem = 6, 5
    p = {k: RNG.standard_normal(v.shape).astype(np.float32) * 0.5 for k, v in _zeros_gru(d_msg, d_mem).items()}
    p["U_h"] = np.diag(RNG.standard_normal(d_mem)).astype(np.float32)    # U_h(r.s) == r.(U_h s)
    m, s = RNG.standard_normal(d_msg), RNG.standard_normal(d_mem)
    assert np.abs(orc.gru(**p, m=m, s=s) - _torch_gru_cell(p, m, s)).max() < 1e-12


def test_gru_full_Uh_hand_case_differs_from_library_variant():
    # d = 2, numbers small enough to follow by hand.  Only U_h couples the two components.
    p = _zeros_gru(2, 2)
    p["b_r"][:] = [0.0, 40.0]              # r = (1/2, 1)
    p["U_h"] = np.array([[0.0, 1.0], [1.0, 0.0]], dtype=np.float32)   # swaps the components
    p["b_z"][:] = -40.0                    # z = 0: output is the candidate
    s = np.array([0.8, -0.6])
    out = orc.gru(**p, m=np.zeros(2), s=s)
    # candidate = tanh((r.s) U_h) = tanh([r2*s2, r1*s1]) = tanh([-0.6, 0.4])
    assert np.abs(out - np.tanh([-0.6, 0.4])).max() < 1e-15
    # the library cell applies r AFTER the recurrent product: tanh(r . (s U_h)) = tanh([0.5*-0.6, 1*0.8])
    lib_variant = _torch_gru_cell(p, np.zeros(2), s)
    assert np.abs(lib_variant - np.tanh([-0.3, 0.8])).max() < 1e-12
    assert np.abs(out - lib_variant).max() > 0.1


# ---------------------------------------------------------------- attention (Eq. attn_detail)

def test_attention_single_neighbour_ignores_query():
    d, H = 8, 2
    V = RNG.standard_normal((1, d))
    K = RNG.standard_normal((1, d))
    WO = RNG.standard_normal((d, d)).astype(np.float32)
    bO = RNG.standard_normal(d).astype(np.float32)
    want = V[0] @ WO.astype(np.float64) + bO
    for _ in range(3):
        out = orc.attention(RNG.standard_normal(d) * 5, K, V, WO, bO, H)
        assert np.abs(out - want).max() < 1e-12


def test_attention_zero_keys_is_uniform_mean():
    d, H, n = 8, 2, 5
    V = RNG.standard_normal((n, d))
    WO = RNG.standard_normal((d, d)).astype(np.float32)
    bO = RNG.standard_normal(d).astype(np.float32)
    out = orc.attention(RNG.standard_normal(d), np.zeros((n, d)), V, WO, bO, H)
    assert np.abs(out - (V.mean(0) @ WO.astype(np.float64) + bO)).max() < 1e-12


def test_attention_empty_neighbourhood_is_bias():
    d = 8
    WO = RNG.standard_normal((d, d)).astype(np.float32)
    bO = RNG.standard_normal(d).astype(np.float32)
    out = orc.attention(RNG.standard_normal(d), np.zeros((0, d)), np.zeros((0, d)), WO, bO, 2)
    assert np.array_equal(out, bO.astype(np.float64))


@pytest.mark.parametrize("heads", [1, 2, 4])
def test_attention_matches_library_sdpa(heads):
    d, n = 16, 7
    q, K, V = RNG.standard_normal(d), RNG.standard_normal((n, d)), RNG.standard_normal((n, d))
    WO = RNG.standard_normal((d, d)).astype(np.float32)
    bO = RNG.standard_normal(d).astype(np.float32)
    dk = d // heads
    tq = torch.tensor(q).reshape(1, heads, 1, dk)                      # [batch, head, 1, dk]
    tK = torch.tensor(K).reshape(n, heads, dk).permute(1, 0, 2)[None]  # [batch, head, n, dk]
    tV = torch.tensor(V).reshape(n, heads, dk).permute(1, 0, 2)[None]
    o = torch.nn.functional.scaled_dot_product_attention(tq, tK, tV)   # scale 1/sqrt(dk)
    o = o.reshape(d).numpy()                                           # heads concatenated
    want = o @ WO.astype(np.float64) + bO
    assert np.abs(orc.attention(q, K, V, WO, bO, heads) - want).max() < 1e-12


def test_attention_large_scores_do_not_overflow():
    d = 4
    q = np.array([300.0, 0, 0, 0])
    K = np.array([[10.0, 0, 0, 0], [9.0, 0, 0, 0]])
    V = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]])
    out = orc.attention(q, K, V, np.eye(d, dtype=np.float32), np.zeros(d, dtype=np.float32), 1)
    a = 1.0 / (1.0 + math.exp(-150.0))
    assert np.abs(out - np.array([a, 1 - a, 0, 0])).max() < 1e-12


# ---------------------------------------------------------------- printed arithmetic of the paper

def test_paper_bound_table():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "affected_bound_table.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    from paper_2603_21090_amd import binding          # imports without the built library
    for n, B, L, K, bound, speedup in rows:
        b = binding.paper_affected_bound(int(B), int(L), int(K))
        assert b == int(bound)                            # the printed bound column
        assert int(n) // b == int(speedup)                # the printed speed-up column, n / bound
