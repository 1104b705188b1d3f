"""Pins for the low-rank query path oracle: torch fp64 matmul / rms_norm, closed forms, invariants."""
import numpy as np
import torch

from paper_2507_19427_amd import workloads as W


def _run(oracle, c, want_f64=True):
    b = oracle.bits_of
    return oracle.query_proj(b(c.x), b(c.w_qa), b(c.w_qb), c.eps,
                             gain=None if c.gain is None else c.gain.numpy(), want_f64=want_f64)


def _torch_ref(c):
    x, wa, wb = c.x.double(), c.w_qa.double(), c.w_qb.double()
    cc = x @ wa
    g = None if c.gain is None else c.gain.double()
    ch = torch.nn.functional.rms_norm(cc, (cc.shape[-1],), weight=g, eps=c.eps)
    return ch, ch @ wb


def test_against_torch_fp64(oracle):
    for with_gain in (False, True):
        c = W.make_query_proj_case("q", 31, B=5, d_model=96, r=40, n_out=72, w_std=0.1, with_gain=with_gain)
        q16, q64, ch = _run(oracle, c)
        ch_ref, q_ref = _torch_ref(c)
        assert np.abs(ch - ch_ref.numpy()).max() <= 1e-12
        assert np.abs(q64 - q_ref.numpy()).max() <= 1e-12
        # stored query = the fp64 query rounded once to bf16
        want = q_ref.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert (q16 != want).mean() <= 0.01      # torch rounds through fp32: rare double-rounding ties
        dec = np.array([[oracle.decode_bf16(v) for v in row] for row in q16])
        assert np.abs(dec - q64).max() <= np.abs(q64).max() * 2.0 ** -8


def test_normalised_activations_have_the_closed_form_norm(oracle):
    """|c_hat|^2 = r * ms / (ms + eps) with ms = mean(c^2), unit gain."""
    c = W.make_query_proj_case("q", 32, B=4, d_model=64, r=32, n_out=16, w_std=0.2)
    c.eps = 0.05                       # large eps so a misplaced eps (outside the root) would show
    _, _, ch = _run(oracle, c)
    cc = (c.x.double() @ c.w_qa.double()).numpy()
    ms = (cc ** 2).mean(1)
    assert np.allclose((ch ** 2).sum(1), 32 * ms / (ms + 0.05), rtol=1e-12)
    assert not np.allclose((ch ** 2).sum(1), 32 * ms / (np.sqrt(ms) + 0.05) ** 2, rtol=1e-3)


def test_selector_weights_reduce_to_a_normalised_prefix(oracle):
    """W_qa = [I;0] and W_qb = I: the query is RMSNorm of the first r inputs."""
    r, d_model = 16, 48
    c = W.make_query_proj_case("q", 33, B=3, d_model=d_model, r=r, n_out=r)
    wa = torch.zeros(d_model, r)
    wa[:r] = torch.eye(r)
    c.w_qa, c.w_qb = wa.bfloat16(), torch.eye(r).bfloat16()
    _, q64, _ = _run(oracle, c)
    x = c.x.double()[:, :r]
    ref = x / torch.sqrt((x ** 2).mean(1, keepdim=True) + c.eps)
    assert np.abs(q64 - ref.numpy()).max() <= 1e-13


def test_weight_layout_is_in_by_out(oracle):
    """y = x W with W [in, out]: a single nonzero weight W_qa[i0, j0] routes input i0 to rank channel j0."""
    d_model, r, n_out = 8, 4, 6
    c = W.make_query_proj_case("q", 34, B=1, d_model=d_model, r=r, n_out=n_out)
    c.x = torch.arange(1, d_model + 1, dtype=torch.float32).reshape(1, d_model).bfloat16()
    wa = torch.zeros(d_model, r)
    wa[5, 2] = 1.0
    wb = torch.zeros(r, n_out)
    wb[2, 4] = 2.0
    c.w_qa, c.w_qb = wa.bfloat16(), wb.bfloat16()
    c.eps = 0.0
    _, q64, ch = _run(oracle, c)
    # c = [0,0,6,0]; mean square = 9; c_hat = [0,0,2,0]; q = [0,0,0,0,4,0]
    assert np.allclose(ch[0], [0, 0, 2, 0]) and np.allclose(q64[0], [0, 0, 0, 0, 4, 0])


def test_input_scaling_leaves_query_unchanged_up_to_eps(oracle):
    c = W.make_query_proj_case("q", 35, B=3, d_model=64, r=32, n_out=24, w_std=0.2)
    _, q1, _ = _run(oracle, c)
    c.x = (c.x.float() * 4).bfloat16()         # exact in bf16
    _, q4, _ = _run(oracle, c)
    assert np.abs(q4 - q1).max() <= 1e-5 * np.abs(q1).max()
    assert np.abs(q4 - q1).max() > 0           # eps is really there


def test_gain_multiplies_channels(oracle):
    c = W.make_query_proj_case("q", 36, B=2, d_model=32, r=16, n_out=8, w_std=0.3, with_gain=True)
    _, _, ch_g = _run(oracle, c)
    gain = c.gain.double().numpy()
    c.gain = None
    _, _, ch_1 = _run(oracle, c)
    assert np.allclose(ch_g, ch_1 * gain, rtol=1e-14)
