"""Pins of the learned scheduler's forward pass (oracle only, CPU): a hand-worked case, closed forms,
invariances, and a loop-by-loop evaluation in exact-ish arithmetic on a tiny case."""
import math

import numpy as np

import oracle
import pmpd_synth as synth


def test_hand_worked_case():
    """T = 2, D_k = 1: scores 0 and ln 3 -> p = (1/4, 3/4); V = 4 I -> O = (1, 3);
    W1 = [[1,-1],[-1,1]] -> hid = relu(-2, 2) = (0, 2); W2 = diag(1, ln2 / 2) -> z = (0, ln 2) -> (1/3, 2/3)."""
    O, probs, cls = oracle.learned_scheduler(
        q=[1.0], K=[[0.0], [math.log(3.0)]], V=[[4.0, 0.0], [0.0, 4.0]],
        W1=[[1.0, -1.0], [-1.0, 1.0]], b1=[0.0, 0.0], W2=[[1.0, 0.0], [0.0, math.log(2.0) / 2.0]], b2=[0.0, 0.0])
    assert np.allclose(O, [1.0, 3.0], rtol=1e-14)
    assert np.allclose(probs, [1.0 / 3.0, 2.0 / 3.0], rtol=1e-14)
    assert cls == 1


def test_score_scale_is_one_over_sqrt_dk():
    """D_k = 4 with q = K_1 = (1,1,1,1) * sqrt(ln 3): q.K_1 / sqrt(4) = 4 ln 3 / 2 = 2 ln 3, e^(2 ln 3) = 9
    -> p = (1/10, 9/10); a missing or squared scale gives 1/82 or 1/4."""
    r = math.sqrt(math.log(3.0))
    O, _, _ = oracle.learned_scheduler(q=[r] * 4, K=[[0.0] * 4, [r] * 4], V=[[10.0], [0.0]], W1=[[1.0]], b1=[0.0],
                                       W2=[[1.0], [0.0]], b2=[0.0, 0.0])
    assert np.allclose(O, [1.0], rtol=1e-13)


def test_zero_query_averages_the_values_and_bias_only_head():
    K, V, q, W1, b1, W2, b2 = synth.draw_learned_scheduler(3, 17, 16, 24, 8, 5)
    O, probs, cls = oracle.learned_scheduler(0 * q, K, V, 0 * W1, b1, 0 * W2, b2)
    assert np.allclose(O, V.astype(np.float64).mean(axis=0), rtol=1e-13, atol=1e-15)
    e = np.exp(b2.astype(np.float64))
    assert np.allclose(probs, e / e.sum(), rtol=1e-13)
    assert cls == int(np.argmax(b2))


def test_dominant_key_selects_its_value_row_and_shift_invariance():
    K, V, q, W1, b1, W2, b2 = synth.draw_learned_scheduler(4, 9, 8, 8, 4, 3)
    K = K.astype(np.float64)
    K[5] = 200.0 * q / np.dot(q, q) * math.sqrt(8.0)  # score 200 for row 5, O(1) for the others
    O, probs, _ = oracle.learned_scheduler(q, K, V, W1, b1, W2, b2)
    assert np.allclose(O, V[5].astype(np.float64), rtol=0, atol=1e-12)
    # adding the same vector c to every key shifts every score by q.c / sqrt(D_k): softmax does not move
    K2 = K + np.linspace(-1, 1, 8)[None, :]
    O2, probs2, _ = oracle.learned_scheduler(q, K2, V, W1, b1, W2, b2)
    assert np.allclose(O2, O, rtol=1e-9, atol=1e-12) and np.allclose(probs2, probs, rtol=1e-9)


def test_relu_and_transposition_are_where_they_belong():
    """hid = relu(W1 O + b1) with a non-square W1 and W2; negative pre-activations must vanish."""
    V = np.array([[1.0, 2.0, 3.0]])           # T = 1: O = V[0]
    W1 = np.array([[1.0, 0.0, 0.0], [0.0, -1.0, 0.0]])   # pre-activations 1 + 0.5, -2 + 0.5
    b1 = np.array([0.5, 0.5])
    W2 = np.array([[1.0, 5.0], [0.0, 5.0], [2.0, 5.0]])  # z = 1.5, 0, 3 (the second hidden unit is off)
    O, probs, cls = oracle.learned_scheduler([0.3], [[0.7]], V, W1, b1, W2, [0.0, 0.0, 0.0])
    e = np.exp([1.5, 0.0, 3.0])
    assert np.allclose(O, [1.0, 2.0, 3.0]) and np.allclose(probs, e / e.sum(), rtol=1e-14) and cls == 2


def test_against_plain_loops_in_python_floats():
    K, V, q, W1, b1, W2, b2 = synth.draw_learned_scheduler(8, 6, 8, 16, 5, 4, sharpness=2.0)
    T, Dk = K.shape
    s = [sum(float(q[i]) * float(K[t, i]) for i in range(Dk)) / math.sqrt(Dk) for t in range(T)]
    w = [math.exp(v) for v in s]
    O = [sum(w[t] * float(V[t, c]) for t in range(T)) / sum(w) for c in range(V.shape[1])]
    hid = [max(0.0, float(b1[j]) + sum(float(W1[j, c]) * O[c] for c in range(len(O)))) for j in range(len(b1))]
    z = [float(b2[k]) + sum(float(W2[k, j]) * hid[j] for j in range(len(hid))) for k in range(len(b2))]
    ez = [math.exp(v) for v in z]
    probs = [v / sum(ez) for v in ez]
    O_o, p_o, c_o = oracle.learned_scheduler(q, K, V, W1, b1, W2, b2)
    assert np.allclose(O_o, O, rtol=1e-12, atol=1e-14) and np.allclose(p_o, probs, rtol=1e-12)
    assert c_o == max(range(len(probs)), key=lambda k: (probs[k], -k))
    assert abs(sum(p_o) - 1.0) < 1e-14


def test_first_index_wins_a_tie():
    _, probs, cls = oracle.learned_scheduler([0.0], [[0.0]], [[1.0]], [[0.0]], [0.0], [[0.0], [0.0], [0.0]], [1.0, 2.0, 2.0])
    assert probs[1] == probs[2] and cls == 1
