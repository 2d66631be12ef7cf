"""GPU parity of gla_srem_dwconv (3x3 depth-wise convolution of the SREM, Algorithm 1) against the CPU fp64 oracle.
fp32 in / fp32 out: 1e-5 of the RMS (nine fp32 multiply-adds per output); bf16 out adds its rounding, 2^-8 of the
largest magnitude at most."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2405_18428_amd as gla
from paper_2405_18428_amd import inputs as gi

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    gla.load_library()


def make(B, gh, gw, D, dtype, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((B, gh * gw, D), dtype=np.float32)
    w = (rng.standard_normal((D, 3, 3), dtype=np.float32) * np.float32(0.3)).astype(np.float32)
    w[:, 1, 1] += np.float32(1)          # around the identity initialisation
    b = (rng.standard_normal((D,), dtype=np.float32) * np.float32(0.1)).astype(np.float32)
    bits = gi.round_to_bf16_bits(x) if dtype == "bf16" else None
    if bits is not None:
        x = gi.bf16_bits_to_f32(bits)
    return x, bits, w, b


def run(x, bits, w, b, gh, gw, orient, out_dtype, with_bias=True):
    dev = torch.device("cuda:0")
    xt = (torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16) if bits is not None
          else torch.from_numpy(x).to(dev))
    y = gla.gla_srem_dwconv(xt, torch.from_numpy(w).to(dev), torch.from_numpy(b).to(dev) if with_bias else None,
                            gh, gw, orient, out_dtype=out_dtype)
    torch.cuda.synchronize()
    return y.float().cpu().numpy()


SHAPES = [
    # B, gh, gw, D, dtype
    (1, 1, 1, 8, "bf16"),
    (2, 5, 13, 72, "bf16"),
    (1, 16, 16, 384, "bf16"),       # DiG-S token matrix at 256 px
    (1, 9, 17, 1152, "bf16"),       # DiG-XL channel count, strips with a ragged end
    (2, 7, 3, 10, "bf16"),          # channel count not a multiple of 8: one channel per thread
    (1, 12, 11, 24, "f32"),
    (1, 1, 9, 5, "f32"),            # single row
    (1, 9, 1, 16, "f32"),           # single column
]


@pytest.mark.parametrize("shape", SHAPES)
def test_shapes_all_orientations(shape):
    from oracle import srem_oracle as so
    B, gh, gw, D, dtype = shape
    x, bits, w, b = make(B, gh, gw, D, dtype, seed=51)
    for orient in range(4):
        ref = so.srem_dwconv(x, w, b, gh, gw, orient)
        rms = np.sqrt(np.mean(ref ** 2))
        got = run(x, bits, w, b, gh, gw, orient, torch.float32)
        err = np.abs(got - ref).max() / rms
        print("  orient=%d fp32 out err=%.3e" % (orient, err), flush=True)
        assert err <= 1e-5, err
        got = run(x, bits, w, b, gh, gw, orient, torch.bfloat16)
        err = np.abs(got - ref).max() / rms
        assert err <= 1e-5 + 2.0 ** -8 * np.abs(ref).max() / rms, err
    ref = so.srem_dwconv(x, w, None, gh, gw, 0)
    got = run(x, bits, w, b, gh, gw, 0, torch.float32, with_bias=False)
    assert np.abs(got - ref).max() / np.sqrt(np.mean(ref ** 2)) <= 1e-5


def test_identity_initialisation_copies_the_tokens():
    x, bits, _, _ = make(1, 32, 32, 1152, "bf16", seed=52)
    w = np.zeros((1152, 3, 3), dtype=np.float32)
    w[:, 1, 1] = 1
    for orient in (0, 3):
        got = run(x, bits, w, np.zeros(1152, dtype=np.float32), 32, 32, orient, torch.bfloat16)
        np.testing.assert_array_equal(got, x)     # bit-exact: a copy


def test_headline_token_matrix():
    from oracle import srem_oracle as so
    x, bits, w, b = make(1, 128, 128, 1152, "bf16", seed=53)
    ref = so.srem_dwconv(x, w, b, 128, 128, 2)
    got = run(x, bits, w, b, 128, 128, 2, torch.float32)
    assert np.abs(got - ref).max() / np.sqrt(np.mean(ref ** 2)) <= 1e-5


def test_argument_checks():
    dev = torch.device("cuda:0")
    x = torch.zeros((1, 16, 8), dtype=torch.bfloat16, device=dev)
    w = torch.zeros((8, 3, 3), dtype=torch.float32, device=dev)
    with pytest.raises(gla.GlaError):
        gla.gla_srem_dwconv(x, w, None, 4, 4, orient=4)
    with pytest.raises(gla.GlaError):
        gla.gla_srem_dwconv(x, w, None, 4, 4, out=x)      # in place
