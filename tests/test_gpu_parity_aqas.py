"""GPU parity of the AQAS scale search and the weight clipping (Sec. 3.2, Eq. 1; App. A.4) against the
CPU oracle: representatives and every member of the scale family bit-identical; the loss of every grid
point within 1e-4 relative of the oracle's float64 evaluation (the kernels sum fp16 outputs against an
fp32 matrix-core product); the chosen grid point / clipping indices valid minimizers of the oracle's own
losses (several may be, up to that tolerance), and the parameters of the chosen clipping bit-identical."""
import numpy as np
import pytest
import torch

import synthetic_inputs as syn
from gpu_util import dev, host

pytestmark = pytest.mark.gpu
LOSS_TOL = 1e-4


@pytest.fixture(scope="module")
def lib():
    import paper_2311_05161_amd as w
    w.load_library()
    assert torch.cuda.is_available()
    return w


def calib(seed, M, K, N, dtype="f16"):
    X, W, _ = syn.random_layer(seed, M, K, N, x_dtype=dtype, outlier_frac=0.02, outlier_gain=50.0)
    if K > 5:
        X[:, 5] = 0          # a dead input channel: s = 1 there
    return X, W


@pytest.mark.parametrize("shape", [(33, 384, "f16"), (300, 1024, "f16"), (7, 128, "f32"), (1000, 200, "f16")])
def test_channel_absmax_and_scale_family_bit_exact(lib, oracle, shape):
    R, K, dtype = shape
    aq = oracle.aqas_search
    X, W = calib(R, R, K, 48, dtype)
    ax, aw = lib.aqas_channel_absmax(dev(X)), lib.aqas_channel_absmax(dev(W))
    np.testing.assert_array_equal(host(ax), aq.channel_absmax(X))
    np.testing.assert_array_equal(host(aw), aq.channel_absmax(W))
    # a strided view and bf16
    buf = torch.zeros((R, K + 8), dtype=torch.bfloat16, device="cuda")
    buf[:, :K] = dev(X.astype(np.float32)).to(torch.bfloat16)
    np.testing.assert_array_equal(host(lib.aqas_channel_absmax(buf[:, :K])),
                                  aq.channel_absmax(host(buf[:, :K])))
    for j in range(17):
        np.testing.assert_array_equal(host(lib.aqas_scale(ax, aw, j)),
                                      aq.aqas_scale(aq.channel_absmax(X), aq.channel_absmax(W), j)), j


SEARCH_CASES = [
    # name, M (calibration tokens), K, N, G, dtype
    ("decode_sized", 16, 512, 256, 128, "f16"),
    ("per_channel", 96, 768, 272, 0, "f16"),
    ("grouped_256", 130, 1024, 128, 256, "f16"),
    ("f32_inputs", 40, 256, 64, 0, "f32"),
    ("ragged_tokens", 77, 384, 528, 128, "f16"),
]


@pytest.mark.parametrize("case", SEARCH_CASES, ids=[c[0] for c in SEARCH_CASES])
def test_scale_search_matches_oracle(lib, oracle, case):
    name, M, K, N, G, dtype = case
    aq = oracle.aqas_search
    X, W = calib(sum(name.encode()) % 983, M, K, N, dtype)
    ref = aq.aqas_search(X, W, G)
    s, best, losses = lib.aqas_search(dev(X), dev(W), G)
    losses, j = host(losses), int(host(best)[0])
    np.testing.assert_allclose(losses, ref["losses"], rtol=LOSS_TOL)
    assert ref["losses"][j] <= ref["losses"].min() * (1 + LOSS_TOL)      # a valid minimizer
    assert losses[j] == losses.min() and np.all(losses[:j] > losses[j])  # the first one of its own table
    np.testing.assert_array_equal(host(s), aq.aqas_scale(ref["ax"], ref["aw"], j))


@pytest.mark.parametrize("case", SEARCH_CASES[:3], ids=[c[0] for c in SEARCH_CASES[:3]])
def test_clip_search_matches_oracle(lib, oracle, case):
    name, M, K, N, G, dtype = case
    aq = oracle.aqas_search
    X, W = calib(sum(name.encode()) % 977, M, K, N, dtype)
    W = W.copy()
    W[3, 5] = 6.0            # an outlier weight on the dead input channel: clipping row 3 pays off
    s = aq.aqas_scale(aq.channel_absmax(X), aq.channel_absmax(W), 8)
    ref = aq.clip_search(X, W, s, G)
    idx, step, zero, table = lib.aqas_clip_search(dev(X), dev(W), dev(s), G, want_table=True)
    idx, table = host(idx), host(table)
    np.testing.assert_allclose(table, ref["err"], rtol=LOSS_TOL, atol=1e-30)
    for n in range(N):
        assert ref["err"][idx[n], n] <= ref["err"][:, n].min() * (1 + LOSS_TOL)
        assert table[idx[n], n] == table[:, n].min() and np.all(table[:idx[n], n] > table[idx[n], n])
    if G == 0:
        assert idx[3] >= 2   # (with groups the factor is shared by the row's other, ordinary groups)
    # parameters of the chosen factors: the oracle's for the same indices, bit for bit
    rho = np.array([aq.clip_factor(int(i)) for i in idx], np.float32)
    st, z = aq.clipped_params(W, s, G, rho)
    np.testing.assert_array_equal(host(step), st)
    np.testing.assert_array_equal(host(zero), z)
    # and the stand-alone entry point, uniform and per channel
    for i in (0, 4, 10):
        st_g, z_g = lib.dint4_clipped_params(dev(W), dev(s), G, uniform_index=i)
        st_o, z_o = aq.clipped_params(W, s, G, np.full(N, aq.clip_factor(i), np.float32))
        np.testing.assert_array_equal(host(st_g), st_o)
        np.testing.assert_array_equal(host(z_g), z_o)
    st_g, z_g = lib.dint4_clipped_params(dev(W), dev(s), G, index=dev(idx))
    np.testing.assert_array_equal(host(st_g), st)
    # codes quantized with the clipped parameters saturate instead of stretching the range
    codes, _, _ = lib.quantize_weight_dint4(dev(W), dev(s), G, step=st_g, zero=z_g)
    oc, _, _ = oracle.quantize_weight_dint4(W, s, G, step=st, zero=z)
    np.testing.assert_array_equal(host(codes), oc)


def test_full_size_c2_layer_scale_search(lib, oracle):
    """The search on the LLaMA-7B attention-projection layer of the decode workload (K = N = 4096,
    group-128) with 64 calibration tokens drawn like its activations."""
    aq = oracle.aqas_search
    X, W, _, G = syn.make_layer("C2", M=64)
    ref = aq.aqas_search(X, W, G)
    s, best, losses = lib.aqas_search(dev(X), dev(W), G)
    losses, j = host(losses), int(host(best)[0])
    np.testing.assert_allclose(losses, ref["losses"], rtol=LOSS_TOL)
    assert ref["losses"][j] <= ref["losses"].min() * (1 + LOSS_TOL)
    np.testing.assert_array_equal(host(s), aq.aqas_scale(ref["ax"], ref["aw"], j))
    # with 0.5 % outlier channels x50 the best exponent lies strictly inside the grid
    assert 0 < j < 16 and ref["losses"][j] < 0.9 * min(ref["losses"][0], ref["losses"][16])
