"""GPU parity of the NVFP4-faithful encoder variant (paper Appendix "Implementation Details",
Quantization Details) against the oracle, through the C ABI: bit-exact scale bytes and codes."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import nvfp4 as onv, bf16 as obf

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def R():
    import paper_2604_19503_amd as R
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return R


def _say(msg):
    print(f"[nvfp4] {msg}", flush=True)


def _case(name):
    rng = np.random.default_rng({"weights": 21, "activations": 22, "mixed_magnitudes": 23, "heavy_tail": 24}[name])
    if name == "weights":
        x = rng.standard_normal((700, 2048)).astype(np.float32) * 0.02
    elif name == "activations":
        x = rng.standard_normal((333, 1408 + 16)).astype(np.float32)
    elif name == "mixed_magnitudes":       # rows of very different size: subnormal E4M3 scales, zero groups, scales that round to 0
        x = rng.standard_normal((512, 256)).astype(np.float32) * (10.0 ** rng.uniform(-7, 2, size=(512, 1))).astype(np.float32)
        x[5, :32] = 0.0
        x[6, 16:48] = -0.0
        x[7] = 0.0
    else:                                  # heavy tail: a few large outliers set the global scale
        x = rng.standard_normal((256, 512)).astype(np.float32)
        x[rng.integers(256, size=20), rng.integers(512, size=20)] *= 50.0
    return W.f32_to_bf16_bits(x)


@pytest.mark.parametrize("name", ["weights", "activations", "mixed_magnitudes", "heavy_tail"])
def test_nvfp4_encoder_is_bit_exact(R, name):
    bits = _case(name)
    _say(f"case {name} shape {bits.shape}")
    x = R.bf16_from_bits(bits)
    amax = float(R.amax_bf16(x).cpu()[0])
    assert amax == float(np.abs(obf.bits_to_f64(bits)).max())
    g = onv.global_scale(bits)
    assert g == np.float32(np.float32(amax) / np.float32(6.0 * 448.0))
    q, s = R.quantize_rows_nvfp4(x, float(g))
    torch.cuda.synchronize()
    codes, sc = onv.quantize(bits, g)
    assert np.array_equal(s.cpu().numpy(), sc)
    assert np.array_equal(q.cpu().numpy(), onv.pack(codes))


def test_nvfp4_every_bf16_pattern_against_a_few_scales(R):
    """All finite BF16 magnitudes as the group maximum and as ordinary members, for several global scales."""
    pats = np.arange(0x7F80, dtype=np.uint16)
    pats = np.concatenate([pats, pats | np.uint16(0x8000)])
    n = pats.size                                              # 65280
    rows = np.zeros((n, 16), dtype=np.uint16)
    rows[:, 0] = pats
    rows[:, 1] = (pats & np.uint16(0x7FFF)) // np.uint16(2)    # some smaller members
    rows[:, 2] = np.uint16(0x3F80)                             # 1.0
    x = R.bf16_from_bits(rows)
    for g in (np.float32(1.0), np.float32(2.0 ** -9), np.float32(0.0137), np.float32(3.3e-7), np.float32(517.0)):
        _say(f"all patterns, g={g}")
        q, s = R.quantize_rows_nvfp4(x, float(g))
        torch.cuda.synchronize()
        codes, sc = onv.quantize(rows, g)
        assert np.array_equal(s.cpu().numpy(), sc)
        assert np.array_equal(q.cpu().numpy(), onv.pack(codes))


def test_nvfp4_argument_errors(R):
    from paper_2604_19503_amd.binding import RealbError
    x = torch.zeros((4, 24), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(RealbError):
        R.quantize_rows_nvfp4(x, 1.0)                         # K not a multiple of 16
    x = torch.zeros((4, 32), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(RealbError):
        R.quantize_rows_nvfp4(x, 0.0)                         # global scale must be positive
    q, s = R.quantize_rows_nvfp4(x[:0], 1.0)                  # empty input is fine
    assert q.shape[0] == 0
