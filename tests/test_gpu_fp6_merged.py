"""The FP6 (E3M2) merged kernel for asymmetric power-of-two scales (the default for that format; per-call option pot_kernel = "merged_fp6"): groups
whose two scale exponents lie within 5 of each other become one FP6 operand, exactly; group positions where some row's
scales lie further apart are written twice along K, split by sign. Against the oracle on identical operands, bit for bit
where the sums are exact."""
import numpy as np
import pytest

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL = 1e-3


def fp6():
    return binding.gemm_options(pot_kernel="merged_fp6", few_rows=-1)


@pytest.mark.parametrize("scale", [ref.E8M0_FLOOR, ref.E8M0_ROUND])
@pytest.mark.parametrize("M,N,K", [(1, 1, 32), (33, 65, 96), (100, 200, 160), (257, 255, 544), (300, 520, 1024),
                                   (31, 257, 384), (260, 300, 768), (64, 1024, 1024), (513, 129, 4096)])
def test_ragged_shapes(M, N, K, scale):
    """Partial tiles in M and N; K from one group (padded to twelve K steps of zero blocks) to many ring turns, with
    and without a K tail. The activations carry an outlier channel, so some group positions of A are split."""
    a = synth.activations(M, K, seed=M + K, n_outlier=1, outlier_gain=60.0)
    b = synth.weights(N, K, seed=N)
    ac, as_ = ref.quantize(a, 32, scale, 1)
    bc, bs = ref.quantize(b, 32, scale, 1)
    C = G.gpu_gemm(ac, as_, bc, bs, scale, 1, options=fp6())
    Cr = ref.gemm(ac, as_, bc, bs, 32, scale, 1)
    assert C.shape == (M, N)
    assert G.rel_fro(C, Cr) <= TOL


def test_integer_exact_bit_for_bit_and_batched():
    """Scales 1 and integer codes: every partial sum is an integer below 2^24, so the result must equal the oracle bit
    for bit. Batch of 3, several tiles."""
    rng = np.random.default_rng(3)
    batch, M, N, K = 3, 300, 270, 256
    mags = np.array([0, 2, 4, 5, 6, 7])

    def operand(rows):
        mag = rng.choice(mags, size=(batch, rows, K))
        sgn = rng.integers(0, 2, size=(batch, rows, K))
        nib = (mag | (sgn << 3)).astype(np.uint8)
        return nib[..., 0::2] | (nib[..., 1::2] << 4), np.full((batch, rows, K // 32, 2), 127, np.uint8)

    ac, as_ = operand(M)
    bc, bs = operand(N)
    C = G.gpu_gemm(ac, as_, bc, bs, ref.E8M0_FLOOR, 1, options=fp6())
    Cr = ref.gemm(ac, as_, bc, bs, 32, ref.E8M0_FLOOR, 1)
    assert C.shape == (batch, M, N)
    assert np.array_equal(C, Cr)


def hand_made(rows, K, rng, gaps):
    """Codes with every magnitude and both signs; scale pairs whose exponents differ by the given gaps, one gap per
    group position (the same for every row) except that row 0 keeps gap 0 everywhere: a position is split as soon as
    ONE row needs it."""
    nib = rng.integers(0, 16, size=(rows, K)).astype(np.uint8)
    codes = nib[:, 0::2] | (nib[:, 1::2] << 4)
    Gn = K // 32
    scales = np.empty((rows, Gn, 2), np.uint8)
    base = rng.integers(120, 134, size=(rows, Gn))
    for g in range(Gn):
        gap = gaps[g % len(gaps)]
        pos_high = rng.integers(0, 2, size=rows).astype(bool)
        scales[:, g, 0] = np.where(pos_high, base[:, g] + gap, base[:, g])
        scales[:, g, 1] = np.where(pos_high, base[:, g], base[:, g] + gap)
    scales[0, :, 1] = scales[0, :, 0]
    return codes, scales


@pytest.mark.parametrize("gaps_a,gaps_b", [((0, 1, 2, 3, 4, 5), (5, 4, 3, 2, 1, 0)),      # every in-window shift
                                           ((0, 6, 3, 9, 5, 20), (0, 0, 1, 2, 3, 4)),      # A split at some positions
                                           ((1, 2, 3), (0, 7, 5, 30, 2)),                  # B split
                                           ((6, 0, 7, 2, 40, 5), (8, 0, 1, 6, 9, 5))])     # both, together and apart
def test_every_shift_and_the_split_positions_exactly(gaps_a, gaps_b):
    """All products are multiples of a common power of two and the sums stay far below 2^24 of it... only where the
    gaps are small; in general the FP32 accumulation rounds. The merged operands themselves are exact, so the result
    must agree with the oracle to FP32 accumulation accuracy (1e-6), for every in-window shift (gaps 0..5, either class
    the larger), for positions split in A, in B, and in both."""
    rng = np.random.default_rng(11)
    M, N, K = 70, 90, 32 * 12
    ac, as_ = hand_made(M, K, rng, gaps_a)
    bc, bs = hand_made(N, K, rng, gaps_b)
    Cr = ref.gemm(ac, as_, bc, bs, 32, ref.E8M0_FLOOR, 1)
    C = G.gpu_gemm(ac, as_, bc, bs, ref.E8M0_FLOOR, 1, options=fp6())
    assert G.rel_fro(C, Cr) <= 2e-6
    assert max(G.rel_fro(C[i], Cr[i]) for i in range(M)) <= 1e-5
    # the sign-split FP4 kernel on the same operands: the two exact kernels agree to the same accuracy
    Cs = G.gpu_gemm(ac, as_, bc, bs, ref.E8M0_FLOOR, 1, options=binding.gemm_options(pot_kernel="split", few_rows=-1))
    assert G.rel_fro(C, Cs) <= 2e-6


def test_one_sided_groups_and_zero_groups():
    """What the cast writes for a class without elements is scale byte 0: such a class is dropped (not split). All-
    positive operands (attention probabilities), all-negative ones and all-zero groups."""
    rng = np.random.default_rng(5)
    M, N, K = 64, 96, 256
    a = np.abs(rng.standard_normal((M, K))).astype(np.float32)
    a[:, 64:96] = 0.0                                  # a zero group in every row
    a[3] *= -1.0                                       # one all-negative row
    b = rng.standard_normal((N, K)).astype(np.float32) * 0.05
    ac, as_ = ref.quantize(synth.f32_to_bf16_bits(a), 32, ref.E8M0_FLOOR, 1)
    bc, bs = ref.quantize(synth.f32_to_bf16_bits(b), 32, ref.E8M0_FLOOR, 1)
    assert np.all(as_[0, :, 1] == 0) and np.all(as_[3, :, 0] == 0)
    C = G.gpu_gemm(ac, as_, bc, bs, ref.E8M0_FLOOR, 1, options=fp6())
    Cr = ref.gemm(ac, as_, bc, bs, 32, ref.E8M0_FLOOR, 1)
    assert G.rel_fro(C, Cr) <= 2e-6


@pytest.mark.parametrize("name,M,N", [("c2_llama7b_qkvo_2048x4096x4096", 512, 768),
                                      ("c3_70b_up_4096x8192x28672", 300, 512),
                                      ("c3_70b_down_4096x28672x8192", 256, 256)])
def test_llm_shapes_cut_down(name, M, N):
    """Full K of the LLaMA-7B / 70B shaped linears (outlier channels x60 / x100: split positions in A)."""
    x, w = synth.linear_operands(name, seed=0, M=M, N=N)
    ac, as_ = ref.quantize(x, 32, ref.E8M0_FLOOR, 1)
    bc, bs = ref.quantize(w, 32, ref.E8M0_FLOOR, 1)
    C = G.gpu_gemm(ac, as_, bc, bs, ref.E8M0_FLOOR, 1, options=fp6())
    assert G.rel_fro(C, ref.gemm(ac, as_, bc, bs, 32, ref.E8M0_FLOOR, 1)) <= 1e-5
