"""Pins for the oracle's GPTQ on the E2M1 grid: the array encoder against the scalar C encoder on every boundary,
the identity-Hessian case against the plain packer (bit for bit), a two-channel case worked by hand, the
error-feedback invariant, and the layer-output error against round-to-nearest on correlated inputs."""
import numpy as np

import oracle
from paper_2307_09782_amd import inputs


def _bits(a):
    return inputs.f32_to_bf16_bits(np.asarray(a, np.float32))


def _hinv_u(H):
    """Upper Cholesky factor U of inv(H): inv(H) = U^T U."""
    return np.linalg.cholesky(np.linalg.inv(H)).T


def test_array_encoder_equals_the_scalar_encoder_on_values_midpoints_and_neighbours():
    grid = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    pts = set(grid) | {(a + b) / 2 for a, b in zip(grid, grid[1:])} | {6.5, 7.0, 100.0, 1e-9}
    ys = []
    for p in pts:
        for d in (0.0, 1e-7, -1e-7):
            ys += [p + d, -(p + d)]
    ys = np.array(ys + [0.0, -0.0])
    got = oracle.e2m1_encode_array(ys)
    want = np.array([oracle.e2m1_encode(float(y)) for y in ys], np.uint8)
    assert np.array_equal(got, want)


def test_identity_hessian_reduces_to_the_plain_packer():
    """With H = I nothing is fed back: every group is quantized from the original weights."""
    cfg = inputs.CONFIGS["tiny"]
    W = inputs.make_w(cfg)
    for G, mode in ((128, 1), (32, 1), (64, 2), (128, 2)):
        codes, exps, c, Q = oracle.gptq_fp4(W, np.eye(cfg.K), G, mode)
        codes_p, exps_p, c_p, _ = oracle.pack_weight(W, G, mode)
        assert np.array_equal(exps, exps_p) and np.array_equal(c, c_p)
        assert np.array_equal(codes, codes_p)  # both modes: M2 divides by c in binary32 on either side
        assert np.allclose(Q, oracle.dequant_weight(codes, exps, c, G), rtol=0, atol=0)


def test_identity_hessian_reduces_to_the_plain_packer_on_a_larger_matrix():
    """Half a million weights under M2, where a binary64 division in place of the packer's binary32 one would
    move a few hundred codes that sit next to a rounding boundary."""
    cfg = inputs.Config("g", 1024, 512, (1,), 128, 2, 0.0, 4, 20.0, 0, 7)
    W = inputs.make_w(cfg)
    for G, mode in ((128, 2), (256, 2), (128, 1)):
        codes, exps, c, _ = oracle.gptq_fp4(W, np.eye(cfg.K), G, mode)
        codes_p, exps_p, c_p, _ = oracle.pack_weight(W, G, mode)
        assert np.array_equal(codes, codes_p) and np.array_equal(exps, exps_p) and np.array_equal(c, c_p)


def test_two_channels_worked_by_hand():
    """K = 2 input channels (one group), one output channel: w = (2.6, 1.0), H = [[2, 1], [1, 2]].
    inv(H) = [[2,-1],[-1,2]]/3, U = [[sqrt(2/3), -1/sqrt(6)], [0, 1/sqrt(2)]].
    amax = 2.6 <= 6 * 2^-1 -> S = 0.5; w0/S = 5.2 -> code 6.0 -> q0 = 3.0; err = (2.6 - 3.0)/U00;
    w1' = 1.0 - U01 * err = 1.0 - (U01/U00) * (-0.4) = 1.0 - (-0.5)(-0.4) = 0.8 -> 0.8/S = 1.6 -> 1.5 -> q1 = 0.75."""
    K = 128  # the packer's shapes want K % 128 == 0: the other 126 channels are zero and uncoupled
    W = np.zeros((K, 1), np.float32)
    W[0, 0], W[1, 0] = 2.59375, 1.0  # 2.59375 is a bfloat16 value; the hand computation holds for it as well
    H = np.eye(K)
    H[:2, :2] = [[2.0, 1.0], [1.0, 2.0]]
    codes, exps, c, Q = oracle.gptq_fp4(_bits(W), _hinv_u(H), 128, 1)
    assert exps[0, 0] == 126 and c[0] == 1.0
    assert Q[0, 0] == 3.0
    w1 = 1.0 - (-0.5) * (2.59375 - 3.0)
    assert abs(w1 - 0.796875) < 1e-12 and Q[1, 0] == 0.75
    assert np.all(Q[2:] == 0)


def test_error_feedback_invariant_and_gain_over_round_to_nearest():
    """For every output channel the un-quantized tail absorbs the error so that, at the end,
    (W - Q) H (W - Q)^T is what the algorithm minimises greedily; on correlated inputs it must beat
    quantizing each channel on its own."""
    rng = np.random.default_rng(1)
    K, N, G = 256, 64, 128
    cfg = inputs.Config("g", K, N, (1,), G, 1, 0.0, 4, 20.0)
    W = inputs.make_w(cfg)
    A = rng.standard_normal((K, 4 * K)) + 2.0 * rng.standard_normal((1, 4 * K))  # strongly correlated channels
    H = A @ A.T / (4 * K) + 0.01 * np.eye(K)
    Wf = inputs.bf16_bits_to_f32(W).astype(np.float64)
    for mode in (1, 2):
        codes, exps, c, Q = oracle.gptq_fp4(W, _hinv_u(H), G, mode)
        assert np.array_equal(Q, oracle.dequant_weight(codes, exps, c, G))
        cp, ep, ccp, _ = oracle.pack_weight(W, G, mode)
        Qr = oracle.dequant_weight(cp, ep, ccp, G)
        obj = np.trace((Wf - Q).T @ H @ (Wf - Q))
        obj_rtn = np.trace((Wf - Qr).T @ H @ (Wf - Qr))
        assert obj < 0.8 * obj_rtn, (obj, obj_rtn)
        assert np.all((codes & 7) <= 7) and exps.min() >= 1
