"""Fused attention on the GPU against the CPU oracle, through the C ABI.

Both gates of the other floating-point operators apply (|err| <= 1e-2 (|ref| + 1) elementwise,
relative Frobenius error <= 5e-3), plus a bound derived from each kernel's arithmetic:
  general kernel   fp32 throughout: summation-order noise only, ~1e-6
  mfma kernel      the probabilities are rounded to bf16 (relative error <= 2^-9, rms 2^-9/sqrt(3)
                   = 1.1e-3) before they multiply V, everything else is fp32: the relative
                   Frobenius error of a row of independent terms is that rms value; bound 2.5e-3
"""
import numpy as np
import pytest

from paper_2505_02146_amd import inputs
from tests.helpers import GATE_ELEM, GATE_FRO, dev

pytestmark = pytest.mark.gpu

TIGHT = {0: 2e-5, 1: 2.5e-3, 2: 2.5e-3, 3: 2.5e-3, 4: 2.5e-3, 5: 2.5e-3, 6: 2.5e-3}     # variant 0 is the general kernel, the rest are mfma kernels
MFMA = [1, 2, 5]                                        # head size 64 (5: eight waves, 128 queries per workgroup)
MFMA128 = [3, 4, 6]                                     # head size 128 (6: eight waves)
DEFAULT = 2                                             # what the library picks for head size 64 when it can (small problems)
DEFAULT128 = 4                                          # ... and for head size 128
BIG128 = 6                                              # with at least 256 workgroups of 128 queries (512 at head size 64): the eight-wave kernels
NVARIANTS = 7


@pytest.fixture(scope="module")
def xp():
    import torch
    assert torch.cuda.is_available()
    from paper_2505_02146_amd import xp as m
    yield m
    for t in ("f32", "bf16"):
        m.xp_force_config(m.XP_OP_ATTENTION, t, -1)


def _pack(m, ld, stride, fill):
    """batch x rows x cols array -> flat buffer with row pitch ld and batch stride `stride`."""
    b, rows, cols = m.shape
    buf = np.full(max(b - 1, 0) * stride + rows * ld + 16, fill, dtype=m.dtype)
    for x in range(b):
        view = buf[x * stride: x * stride + rows * ld].reshape(rows, ld)
        view[:, :cols] = m[x]
    return buf


def _gate(got, ref, what, tight):
    got = np.asarray(got, np.float64)
    assert np.isfinite(got).all(), what
    worst = np.max(np.abs(got - ref) / (np.abs(ref) + 1.0))
    fro = np.linalg.norm((got - ref).ravel()) / np.linalg.norm(ref.ravel())
    assert worst <= GATE_ELEM, (what, worst)
    assert fro <= GATE_FRO, (what, fro)
    assert fro <= tight, f"{what}: relative Frobenius error {fro:.3e} above the bound {tight} of this kernel's arithmetic"
    return fro


def _run(xp, oracle, *, batch, Lq, Lk, d, dv, scale, kind="bf16", variant=None, pad=(0, 0, 0, 0), gap=0,
         share_kv=False, seed=3, sigma=1.0, stream=None):
    import torch
    rnd = lambda shape, tid: inputs.normal(shape, seed, tid, sigma).astype(np.float32)
    conv = inputs.to_bf16_bits if kind == "bf16" else (lambda a: a)
    kb = 1 if share_kv else batch
    Q, K, V = conv(rnd((batch, Lq, d), 1)), conv(rnd((kb, Lk, d), 2)), conv(rnd((kb, Lk, dv), 3))
    ldq, ldk, ldv, ldo = d + pad[0], d + pad[1], dv + pad[2], dv + pad[3]
    sq, sk, sv, so = Lq * ldq + gap, Lk * ldk + gap, Lk * ldv + gap, Lq * ldo + gap
    nan = 0x7FC0 if kind == "bf16" else np.nan
    Qb, Kb, Vb = _pack(Q, ldq, sq, nan), _pack(K, ldk, sk, nan), _pack(V, ldv, sv, nan)
    SENT = -12345.0
    O = torch.full(((batch - 1) * so + Lq * ldo + 16,), SENT, dtype=torch.float32, device="cuda")
    xp.xp_force_config(xp.XP_OP_ATTENTION, kind, -1 if variant is None else variant)
    args = (batch, Lq, Lk, d, dv, scale, dev(Qb), ldq, sq, dev(Kb), ldk, 0 if share_kv else sk,
            dev(Vb), ldv, 0 if share_kv else sv, O, ldo, so)
    if stream is None:
        xp.xp_attention(*args, q_type=kind, k_type=kind, v_type=kind)
    else:
        with torch.cuda.stream(stream):
            xp.xp_attention(*args, q_type=kind, k_type=kind, v_type=kind)
        stream.synchronize()
    torch.cuda.synchronize()
    used = xp.xp_last_config(xp.XP_OP_ATTENTION, kind)
    out = O.cpu().numpy()
    got = np.stack([out[x * so: x * so + Lq * ldo].reshape(Lq, ldo)[:, :dv] for x in range(batch)])
    # nothing outside the output rows was written
    mask = np.ones(out.shape, bool)
    for x in range(batch):
        m = mask[x * so: x * so + Lq * ldo].reshape(Lq, ldo)
        m[:, :dv] = False
    assert (out[mask] == SENT).all(), "wrote outside the output"
    ref = oracle.attention(Qb, Kb, Vb, batch=batch, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=scale, ldq=ldq, ldk=ldk, ldv=ldv,
                           strideQ=sq, strideK=0 if share_kv else sk, strideV=0 if share_kv else sv)
    return got, ref, used, (Q, K, V)


MFMA_SHAPES = [  # batch, Lq, Lk: whole tiles, ragged query and key tails, single elements, several key tiles
    (3, 64, 64), (2, 128, 192), (2, 100, 130), (1, 1, 1), (2, 17, 257), (1, 200, 63), (2, 65, 65), (8, 70, 300),
]


@pytest.mark.parametrize("variant", [0] + MFMA)
@pytest.mark.parametrize("shape", MFMA_SHAPES)
def test_head64_bf16_both_kernels(xp, oracle, shape, variant):
    batch, Lq, Lk = shape
    got, ref, used, _ = _run(xp, oracle, batch=batch, Lq=Lq, Lk=Lk, d=64, dv=64, scale=0.125, variant=variant)
    assert used == variant
    _gate(got, ref, f"{shape} variant {variant}", TIGHT[variant])


@pytest.mark.parametrize("variant", [0] + MFMA128)
@pytest.mark.parametrize("shape", MFMA_SHAPES)
def test_head128_bf16_both_kernels(xp, oracle, shape, variant):
    batch, Lq, Lk = shape
    got, ref, used, _ = _run(xp, oracle, batch=batch, Lq=Lq, Lk=Lk, d=128, dv=128, scale=0.0884, variant=variant)
    assert used == variant
    _gate(got, ref, f"head 128 {shape} variant {variant}", TIGHT[variant])


@pytest.mark.parametrize("variant", MFMA128)
def test_head128_padded_shared_peaked_and_single_key(xp, oracle, variant):
    got, ref, used, _ = _run(xp, oracle, batch=3, Lq=90, Lk=150, d=128, dv=128, scale=0.0884, variant=variant,
                             pad=(8, 16, 24, 4), gap=64)
    assert used == variant
    _gate(got, ref, "head 128 padded", TIGHT[variant])
    got, ref, used, _ = _run(xp, oracle, batch=4, Lq=80, Lk=100, d=128, dv=128, scale=0.0884, variant=variant, share_kv=True)
    _gate(got, ref, "head 128 shared K/V", TIGHT[variant])
    got, ref, _, _ = _run(xp, oracle, batch=2, Lq=66, Lk=200, d=128, dv=128, scale=20.0, variant=variant)
    _gate(got, ref, "head 128 peaked", 4e-3)
    got, ref, _, (Q, K, V) = _run(xp, oracle, batch=2, Lq=70, Lk=1, d=128, dv=128, scale=0.7, variant=variant)
    expect = inputs.bf16_bits_to_f32(V).astype(np.float64)
    assert np.array_equal(got, np.broadcast_to(expect, got.shape))


def test_head128_is_selected_and_head64_variants_decline_it(xp, oracle):
    got, ref, used, _ = _run(xp, oracle, batch=2, Lq=130, Lk=260, d=128, dv=128, scale=0.0884)
    assert used == DEFAULT128
    _gate(got, ref, "selected head 128", TIGHT[DEFAULT128])
    with pytest.raises(xp.XpError) as e:
        _run(xp, oracle, batch=2, Lq=33, Lk=47, d=128, dv=128, scale=0.2, variant=1)
    assert e.value.status == 6
    with pytest.raises(xp.XpError) as e:
        _run(xp, oracle, batch=2, Lq=33, Lk=47, d=64, dv=64, scale=0.2, variant=3)
    assert e.value.status == 6
    got, ref, used, _ = _run(xp, oracle, batch=2, Lq=33, Lk=47, d=128, dv=64, scale=0.2)     # mixed sizes: the general kernel
    assert used == 0
    _gate(got, ref, "d 128 dv 64", TIGHT[0])


@pytest.mark.parametrize("variant", [0] + MFMA)
def test_padded_pitches_and_batch_gaps(xp, oracle, variant):
    got, ref, used, _ = _run(xp, oracle, batch=3, Lq=90, Lk=150, d=64, dv=64, scale=0.125, variant=variant,
                             pad=(8, 16, 24, 4), gap=64)
    assert used == variant
    _gate(got, ref, "padded", TIGHT[variant])


def test_selection_takes_the_mfma_kernel_when_it_can_and_the_general_one_otherwise(xp, oracle):
    got, ref, used, _ = _run(xp, oracle, batch=2, Lq=70, Lk=90, d=64, dv=64, scale=0.125)
    assert used == DEFAULT and xp.xp_num_configs(xp.XP_OP_ATTENTION, "bf16") == NVARIANTS
    _gate(got, ref, "selected mfma", TIGHT[DEFAULT])
    # row pitch not a multiple of 16 bytes: the matrix-core kernel declines
    got, ref, used, _ = _run(xp, oracle, batch=2, Lq=70, Lk=90, d=64, dv=64, scale=0.125, pad=(3, 0, 0, 0))
    assert used == 0
    _gate(got, ref, "selected general (pitch)", TIGHT[0])
    got, ref, used, _ = _run(xp, oracle, batch=2, Lq=33, Lk=47, d=32, dv=64, scale=0.2)
    assert used == 0
    _gate(got, ref, "selected general (head size)", TIGHT[0])
    with pytest.raises(xp.XpError) as e:
        _run(xp, oracle, batch=2, Lq=33, Lk=47, d=32, dv=64, scale=0.2, variant=1)
    assert e.value.status == 6


@pytest.mark.parametrize("case", [
    dict(batch=2, Lq=9, Lk=21, d=40, dv=72, kind="bf16"),        # odd head sizes, two column blocks
    dict(batch=1, Lq=5, Lk=1100, d=16, dv=8, kind="f32"),        # more keys than one score chunk
    dict(batch=2, Lq=7, Lk=13, d=1, dv=130, kind="f32"),         # three column blocks
    dict(batch=3, Lq=4, Lk=6, d=0, dv=5, kind="f32"),            # no head dimension: plain average of V
    dict(batch=1, Lq=64, Lk=64, d=64, dv=64, kind="f32"),
])
def test_general_kernel_shapes(xp, oracle, case):
    got, ref, used, _ = _run(xp, oracle, scale=0.3, **case)
    assert used == 0
    _gate(got, ref, str(case), TIGHT[0])


@pytest.mark.parametrize("variant", [0] + MFMA)
def test_single_key_returns_the_value_row_exactly(xp, oracle, variant):
    got, ref, _, (Q, K, V) = _run(xp, oracle, batch=2, Lq=70, Lk=1, d=64, dv=64, scale=0.7, variant=variant)
    expect = inputs.bf16_bits_to_f32(V).astype(np.float64)
    assert np.array_equal(got, np.broadcast_to(expect, got.shape))
    assert np.array_equal(ref, np.broadcast_to(expect, ref.shape))


@pytest.mark.parametrize("variant", [0] + MFMA)
def test_shared_keys_and_values_across_the_batch(xp, oracle, variant):
    got, ref, used, _ = _run(xp, oracle, batch=4, Lq=80, Lk=100, d=64, dv=64, scale=0.125, variant=variant, share_kv=True)
    assert used == variant
    _gate(got, ref, "shared K/V", TIGHT[variant])


@pytest.mark.parametrize("variant", [0] + MFMA)
def test_peaked_softmax_stays_finite(xp, oracle, variant):
    # scores with a spread of several hundred: nearly one-hot rows, exp() of large negatives
    got, ref, _, _ = _run(xp, oracle, batch=2, Lq=66, Lk=200, d=64, dv=64, scale=30.0, variant=variant)
    _gate(got, ref, "peaked", 4e-3 if variant else 2e-4)


def test_runs_on_the_callers_stream(xp, oracle):
    import torch
    s = torch.cuda.Stream()
    got, ref, used, _ = _run(xp, oracle, batch=2, Lq=64, Lk=128, d=64, dv=64, scale=0.125, stream=s)
    _gate(got, ref, "side stream", TIGHT[DEFAULT])


def test_attention_workload_full_size(xp, oracle):
    """The benchmark's attention workload in the configuration the benchmark times."""
    import torch
    w = inputs.workload("attention_bf16_512")
    b, L, d = w["batch"], w["Lq"], w["d"]
    xp.xp_force_config(xp.XP_OP_ATTENTION, "bf16", -1)
    O = torch.full((b, L, d), float("nan"), device="cuda")
    xp.xp_attention(b, L, L, d, d, w["scale"], dev(w["Q"].reshape(-1)), d, L * d, dev(w["K"].reshape(-1)), d, L * d,
                    dev(w["V"].reshape(-1)), d, L * d, O, d, L * d, q_type="bf16", k_type="bf16", v_type="bf16")
    torch.cuda.synchronize()
    assert xp.xp_last_config(xp.XP_OP_ATTENTION, "bf16") == DEFAULT
    ref = oracle.attention(w["Q"].reshape(-1), w["K"].reshape(-1), w["V"].reshape(-1), batch=b, Lq=L, Lk=L, d=d, dv=d,
                           scale=w["scale"])
    _gate(O.cpu().numpy(), ref, "attention_bf16_512", TIGHT[DEFAULT])


def test_attention_head128_workload_sampled(xp, oracle):
    """The decoder-block workload (32 x 2048 x 2048 x 128) as the benchmark runs it; three batch indices
    are checked in full against the oracle."""
    import torch
    w = inputs.workload("attention_bf16_2048_d128")
    b, L, d = w["batch"], w["Lq"], w["d"]
    xp.xp_force_config(xp.XP_OP_ATTENTION, "bf16", -1)
    O = torch.full((b, L, d), float("nan"), device="cuda")
    xp.xp_attention(b, L, L, d, d, w["scale"], dev(w["Q"].reshape(-1)), d, L * d, dev(w["K"].reshape(-1)), d, L * d,
                    dev(w["V"].reshape(-1)), d, L * d, O, d, L * d, q_type="bf16", k_type="bf16", v_type="bf16")
    torch.cuda.synchronize()
    assert xp.xp_last_config(xp.XP_OP_ATTENTION, "bf16") == BIG128       # 32 x 16 workgroups of 128 queries
    got = O.cpu().numpy()
    assert np.isfinite(got).all()
    for x in (0, 13, 31):
        ref = oracle.attention(w["Q"][x].reshape(-1), w["K"][x].reshape(-1), w["V"][x].reshape(-1), batch=1, Lq=L, Lk=L, d=d, dv=d,
                               scale=w["scale"])
        _gate(got[x:x + 1], ref, f"attention_bf16_2048_d128 batch index {x}", TIGHT[BIG128])
