"""Per-kernel parity: each operator of the step, called through the C ABI, against
the matching piece of the CPU oracle on the same seeded inputs."""
import math

import numpy as np
import pytest

from oracle import dit, sampler
from paper_2501_04012_amd import synth
from util import dev, host, max_abs, record, rel_l2

pytestmark = pytest.mark.gpu
BF = synth.round_to_bf16


def _torch():
    import torch
    return torch


# --------------------------------------------------------------------------- linear layers

LIN_SHAPES = [
    (1, 32, 64), (300, 200, 128), (513, 384, 256), (64, 1152, 1152), (127, 96, 64),   # few tiles: split-K kernel
    (2100, 1024, 128),       # the 128x128 configuration, ragged M
    (2500, 48, 192),         # narrow N, many rows (the output head's shape class), ragged both ways
    (8209, 2048, 128),       # enough tiles for the 256x256 configuration, ragged M
    (8200, 1152, 128),       # N a multiple of 192 that 256 would pad: the 256x192 configuration, ragged M
    (8209, 2048, 192),       # an odd number of K tiles: the general form of the tile kernel, 256x256
    (8200, 1152, 320),       # the same, 256x192
    (8209, 2304, 384),       # six K tiles, 256x256, ragged M
    (250, 160, 72),          # K not a multiple of 64: plain kernel
]


@pytest.mark.parametrize("M,N,K", LIN_SHAPES)
@pytest.mark.parametrize("epilogue", [0, 1])
def test_linear_bf16(fc, M, N, K, epilogue):
    torch = _torch()
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    A = BF(rng.standard_normal((M, K), dtype=np.float32))
    W = BF(rng.standard_normal((K, N), dtype=np.float32) * np.float32(1 / math.sqrt(K)))
    b = rng.standard_normal(N, dtype=np.float32)
    want = A.astype(np.float64) @ W.astype(np.float64) + b
    if epilogue:
        want = dit.gelu_tanh(want)
    out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda:0")
    fc.fc_op_linear(fc.FC_BF16, dev(A, True), dev(W.T.copy(), True), dev(b), None, out, M, N, K, epilogue)
    torch.cuda.synchronize()
    got = host(out)
    assert rel_l2(got, want) < 4e-3, (rel_l2(got, want), max_abs(got, want))
    assert max_abs(got, want) < 3e-2


@pytest.mark.parametrize("M,N,K,epilogue", [
    (27 * 256 - 37, 29 * 256, 2048, 1),   # 783 tiles of 256 x 256: 15 left over, 4 ranges of K; ragged M; GELU
    (44 * 256 - 50, 1152, 2112, 2),       # 44 x 6 = 264 tiles of 256 x 192: 8 left over; gated epilogue
    (20 * 256, 39 * 256, 3072, 0),        # 780 tiles: 12 left over, 4 ranges of 12 K tiles
    (5 * 256, 155 * 256, 2240, 0),        # 775 tiles, K = 35 tiles: ranges of unequal length
    (70 * 256 - 144, 3072, 3072, 2),      # the full-3D configuration's output projection: 840 tiles, 72 left over, 3 ranges
    (226, 3072, 4096, 0),                 # its text projection: 48 tiles of 128 x 128, all of them split in 4
    (1000, 1152, 3072, 1),                # 72 tiles of 128 x 128, ragged M, 3 ranges
    (17550, 64, 3072, 0),                 # the full-3D configuration's output head: 138 tiles of 128 x 128 (half of N empty), 3 ranges
    (150 * 128 - 7, 128, 2048, 1),        # 150 tiles of 128 x 128: 3 ranges, 450 units on 512 slots
])
def test_linear_bf16_split_k_remainder(fc, M, N, K, epilogue):
    """Products whose tile count leaves a nearly empty last round: with scratch memory that
    round is split along K and finished by the fix-up launch.  Against the float64 product, and
    against the unsplit launch (the sums along K are merely associated differently)."""
    torch = _torch()
    rng = np.random.default_rng(M + N + K)
    A = BF(rng.standard_normal((M, K), dtype=np.float32))
    W = BF(rng.standard_normal((K, N), dtype=np.float32) * np.float32(1 / math.sqrt(K)))
    b = rng.standard_normal(N, dtype=np.float32)
    g = rng.standard_normal(N, dtype=np.float32) if epilogue == 2 else None
    want = A.astype(np.float64) @ W.astype(np.float64) + b
    want = dit.gelu_tanh(want) if epilogue == 1 else want * g if epilogue == 2 else want
    dA, dW, db, dg = dev(A, True), dev(W.T.copy(), True), dev(b), dev(g) if g is not None else None
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    scratch = torch.empty(128 << 20, dtype=torch.uint8, device="cuda:0")
    fc.fc_op_linear_scratch(fc.FC_BF16, dA, dW, db, dg, out, M, N, K, epilogue, scratch)
    ref = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    fc.fc_op_linear(fc.FC_BF16, dA, dW, db, dg, ref, M, N, K, epilogue)
    again = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    fc.fc_op_linear_scratch(fc.FC_BF16, dA, dW, db, dg, again, M, N, K, epilogue, scratch)
    torch.cuda.synchronize()
    got = host(out)
    assert np.isfinite(got).all()
    assert rel_l2(got, want) < 4e-3, rel_l2(got, want)
    # element by element: the rounding of the bf16 output (half an ulp: 2^-9 relative) plus the fp32 sums
    assert (np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 2e-2).all()
    assert rel_l2(got, host(ref)) < 2e-3
    assert torch.equal(out, again)                         # fixed order of the partial sums
    # the split really happened where it should: the unsplit result differs in a few roundings
    # (no assertion on that: equality would be legal, just improbable)
    # too little scratch: runs unsplit, bit-identical to fc_op_linear
    small = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    out2 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    fc.fc_op_linear_scratch(fc.FC_BF16, dA, dW, db, dg, out2, M, N, K, epilogue, small)
    torch.cuda.synchronize()
    assert torch.equal(out2, ref)


def test_linear_bf16_operand_beyond_32_bit_offsets(fc):
    """An activation matrix of more than 4 GB: the tile kernel's buffer-addressed form covers
    32-bit ranges only, so the dispatcher must hand this product to the general form.  The
    operand is drawn on the device (it is 4.3 GB) with a seeded generator; the float64 product
    is checked on sampled rows copied back to the host, the rest for finiteness."""
    torch = _torch()
    M, N, K = 65600 + 37, 256, 32768
    assert M * K * 2 >= 2 ** 32
    g = torch.Generator(device="cuda:0").manual_seed(4321)
    A = torch.randn((M, K), device="cuda:0", generator=g, dtype=torch.float32).to(torch.bfloat16)
    rng = np.random.default_rng(99)
    W = BF(rng.standard_normal((K, N), dtype=np.float32) * np.float32(1 / math.sqrt(K)))
    b = rng.standard_normal(N, dtype=np.float32)
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    fc.fc_op_linear(fc.FC_BF16, A, dev(W.T.copy(), True), dev(b), None, out, M, N, K, 0)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out.float()).all())
    rows = np.unique(np.concatenate([np.arange(0, 4), np.arange(M - 4, M), rng.integers(0, M, 56),
                                     [32767, 32768, 65535, 65536]]))      # around 2^31 and 2^32 bytes of row offset
    idx = torch.from_numpy(rows).to("cuda:0")
    a_rows = A.index_select(0, idx).float().cpu().numpy().astype(np.float64)
    want = a_rows @ W.astype(np.float64) + b
    got = out.index_select(0, idx).float().cpu().numpy()
    record(rel_l2=rel_l2(got, want), max_abs=max_abs(got, want))
    assert rel_l2(got, want) < 4e-3
    assert (np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 2e-2).all()


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (70, 65, 33), (256, 64, 64)])
def test_linear_fp32(fc, M, N, K):
    torch = _torch()
    rng = np.random.default_rng(M + N + K)
    A = rng.standard_normal((M, K), dtype=np.float32)
    W = rng.standard_normal((K, N), dtype=np.float32)
    b = rng.standard_normal(N, dtype=np.float32)
    out = torch.empty((M, N), dtype=torch.float32, device="cuda:0")
    fc.fc_op_linear(fc.FC_F32, dev(A), dev(W.T.copy()), dev(b), None, out, M, N, K, 1)
    torch.cuda.synchronize()
    want = dit.gelu_tanh(A.astype(np.float64) @ W.astype(np.float64) + b)
    assert rel_l2(host(out), want) < 1e-5


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("gated", [True, False])
def test_linear_gated_branch_then_residual_layernorm(fc, dtype, gated):
    """The gated branch output (epilogue 2) and the LayerNorm that folds it into the
    residual stream, against x + gate * (A W + b) and LayerNorm of that."""
    torch = _torch()
    M, N, K = 333, 192, 128
    rng = np.random.default_rng(5)
    bf = dtype == "bf16"
    A = rng.standard_normal((M, K), dtype=np.float32)
    W = rng.standard_normal((K, N), dtype=np.float32) * np.float32(0.1)
    if bf:
        A, W = BF(A), BF(W)
    b = rng.standard_normal(N, dtype=np.float32)
    g = rng.standard_normal(N, dtype=np.float32) if gated else None
    x = rng.standard_normal((M, N), dtype=np.float32)
    sh, sc = rng.standard_normal(N, dtype=np.float32), rng.standard_normal(N, dtype=np.float32)
    branch = (g if gated else 1.0) * (A.astype(np.float64) @ W.astype(np.float64) + b)
    want_x = x + branch
    want_u = dit.modulate(dit.layernorm(want_x, 1e-6), sh, sc)
    code = fc.FC_BF16 if bf else fc.FC_F32
    tdt = torch.bfloat16 if bf else torch.float32
    y = torch.empty((M, N), dtype=tdt, device="cuda:0")
    fc.fc_op_linear(code, dev(A, bf), dev(W.T.copy(), bf), dev(b), dev(g) if gated else None, y, M, N, K, 2)
    dx, u = dev(x), torch.empty((M, N), dtype=tdt, device="cuda:0")
    fc.fc_op_layernorm_modulate(code, dx, y, dev(sh), dev(sc), u, M, N, 1e-6)
    torch.cuda.synchronize()
    assert rel_l2(host(y), branch) < (4e-3 if bf else 1e-5)
    assert rel_l2(host(dx), want_x) < (3e-3 if bf else 1e-5)      # bf16: the branch is rounded before the add
    assert rel_l2(host(u), want_u) < (6e-3 if bf else 1e-5)


# --------------------------------------------------------------------------- attention

def _attn_inputs(G, nq, nk, d, gain, bf):
    qs, ks, vs = [], [], []
    for g in range(G):
        q, k, v = synth.sharp_qkv(1000 + 17 * g + nq + nk + d, nq, nk, d, gain=gain)
        qs.append(q); ks.append(k); vs.append(v)
    q, k, v = np.stack(qs), np.stack(ks), np.stack(vs)
    return (BF(q), BF(k), BF(v)) if bf else (q, k, v)


def _attn_case(fc, G, nq, nk, d, gain, bf, impl):
    """(got, want) for the entry point on raw q, k, v: want is the oracle on exactly those."""
    torch = _torch()
    q, k, v = _attn_inputs(G, nq, nk, d, gain, bf)
    want = dit.attention(np.asarray(q, dtype=np.float64), k.astype(np.float64), v.astype(np.float64))
    out = torch.full((G, nq, d), float("nan"), dtype=torch.bfloat16 if bf else torch.float32, device="cuda:0")
    fc.fc_op_attention(fc.FC_BF16 if bf else fc.FC_F32, dev(q, bf), dev(k, bf), dev(v, bf), out, G, nq, nk, d, impl)
    torch.cuda.synchronize()
    return host(out), want


def _check_flash_both_forms(fc, G, nq, nk, d, gain):
    """The MFMA attention kernels in the two forms the entry point offers.
    (1) As a step runs them: the query tensor holds q' = bf16(q log2(e)/sqrt(d)) (inside a
    step the QKV epilogue writes that).  The oracle gets the same q', turned back into the
    query of the plain definition (q' sqrt(d)/log2(e) in float64), so both sides see the
    inputs the ABI receives.  Bar: the step's (rel-L2 <= 1e-2, max-abs <= 5e-2); the
    kernels do better, which the second pair of bounds records.
    (2) On a raw bf16 q, which the kernel has to scale and round a second time.  That second
    rounding moves a score s by up to |s| 2^-9 before the kernel's arithmetic starts; its
    effect on the output is measured between two oracle evaluations and widens the max-abs
    bound (it alone exceeds 5e-2 for peaked rows), rel-L2 stays at 1e-2."""
    torch = _torch()
    q, k, v = _attn_inputs(G, nq, nk, d, gain, True)
    k64, v64 = k.astype(np.float64), v.astype(np.float64)
    c = np.float32(1.4426950408889634 / math.sqrt(d))
    q_pre = BF(q.astype(np.float32) * c)                               # the input of form (1)
    want_pre = dit.attention(q_pre.astype(np.float64) / np.float64(c), k64, v64)
    out = torch.full((G, nq, d), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    fc.fc_op_attention(fc.FC_BF16, dev(q_pre, True), dev(k, True), dev(v, True), out, G, nq, nk, d, 2)
    torch.cuda.synchronize()
    got_pre = host(out)
    assert np.all(np.isfinite(got_pre))
    assert rel_l2(got_pre, want_pre) <= 1e-2 and max_abs(got_pre, want_pre) <= 5e-2
    assert rel_l2(got_pre, want_pre) < 4e-3, (rel_l2(got_pre, want_pre), max_abs(got_pre, want_pre))
    assert max_abs(got_pre, want_pre) < 2.5e-2

    want_raw = dit.attention(q.astype(np.float64), k64, v64)
    out.fill_(float("nan"))
    fc.fc_op_attention(fc.FC_BF16, dev(q, True), dev(k, True), dev(v, True), out, G, nq, nk, d, 0)
    torch.cuda.synchronize()
    got_raw = host(out)
    rounding_effect = max_abs(want_pre, want_raw)
    record(gain=gain, rel_l2=rel_l2(got_pre, want_pre), max_abs=max_abs(got_pre, want_pre),
           raw_q_rel_l2=rel_l2(got_raw, want_raw), raw_q_max_abs=max_abs(got_raw, want_raw),
           second_rounding_effect=rounding_effect)
    assert np.array_equal(got_raw, got_pre)            # same kernel, same operand after the second rounding
    assert rel_l2(got_raw, want_raw) <= 1e-2, (rel_l2(got_raw, want_raw), max_abs(got_raw, want_raw))
    assert max_abs(got_raw, want_raw) <= 2.5e-2 + rounding_effect


@pytest.mark.parametrize("G,nq,nk,d", [(3, 300, 333, 64), (2, 64, 64, 64), (1, 1, 1, 64), (2, 257, 120, 72),
                                       (1, 700, 1000, 64), (4, 256, 256, 72), (1, 33, 7, 72), (2, 600, 333, 64),
                                       (1, 1100, 1000, 64), (2, 513, 129, 64),
                                       (1, 4200, 650, 64)])      # long enough for the 8-wave workgroup, ragged both ways
@pytest.mark.parametrize("gain", [1.0, 2.5, 4.0])
def test_attention_flash_bf16(fc, G, nq, nk, d, gain):
    _check_flash_both_forms(fc, G, nq, nk, d, gain)


@pytest.mark.parametrize("G,nq,nk,d", [(3, 1000, 120, 72), (2, 4096, 26, 64), (1, 515, 128, 72), (2, 700, 1, 64),
                                       (1, 2048, 97, 64), (5, 512, 33, 72), (1, 9000, 120, 72)])
@pytest.mark.parametrize("gain", [1.0, 2.5, 4.0])
def test_attention_few_keys_many_queries_bf16(fc, G, nq, nk, d, gain):
    """At most 128 keys shared by at least 512 queries (the text cross-attention shape): keys
    and values stay in LDS, every key-group count 1..4, ragged query ranges and chunks."""
    _check_flash_both_forms(fc, G, nq, nk, d, gain)


@pytest.mark.parametrize("G,nq,nk,d", [(2, 4200, 2100, 64),      # 8-wave workgroups, ragged both ways
                                       (3, 600, 2300, 64),       # 4-wave workgroups
                                       (2, 700, 2048, 72),       # head dim 72, whole tiles
                                       (1, 300, 333, 64)])       # too short to use the bound: plain path
@pytest.mark.parametrize("gain", [0.5, 1.0, 2.5, 4.0])
def test_attention_with_the_key_norm_bound(fc, G, nq, nk, d, gain):
    """Long key sequences in the form a step runs them: scores bounded by |q| max|k|.  Small
    gains keep every query column inside the slack (no running maximum after the first tile),
    large gains do not (the lazy-maximum loop); gain 1 mixes both among the waves of a launch.
    The result must meet the step's bar against the oracle on the same inputs either way, and
    agree with the unbounded kernel to rounding."""
    torch = _torch()
    q, k, v = _attn_inputs(G, nq, nk, d, gain, True)
    c = np.float32(1.4426950408889634 / math.sqrt(d))
    q_pre = BF(q.astype(np.float32) * c)
    want = dit.attention(q_pre.astype(np.float64) / np.float64(c), k.astype(np.float64), v.astype(np.float64))
    out = torch.full((G, nq, d), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    scratch = torch.full((32 * G,), float("nan"), device="cuda:0")
    fc.fc_op_attention_bounded(dev(q_pre, True), dev(k, True), dev(v, True), out, G, nq, nk, d, scratch)
    torch.cuda.synchronize()
    got = host(out)
    assert np.all(np.isfinite(got))
    record(gain=gain, rel_l2=rel_l2(got, want), max_abs=max_abs(got, want))
    assert rel_l2(got, want) < 4e-3 and max_abs(got, want) < 2.5e-2, (rel_l2(got, want), max_abs(got, want))
    # the scratch holds the largest key norm of each problem (maximum over its 32 partial maxima)
    norms = host(scratch).reshape(G, 32).max(axis=1)
    np.testing.assert_allclose(norms, np.linalg.norm(k.astype(np.float64), axis=2).max(axis=1), rtol=1e-5)
    ref = torch.full((G, nq, d), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    fc.fc_op_attention(fc.FC_BF16, dev(q_pre, True), dev(k, True), dev(v, True), ref, G, nq, nk, d, 2)
    torch.cuda.synchronize()
    assert rel_l2(got, host(ref)) < 4e-3


@pytest.mark.parametrize("G,nq,nk,d,bf", [(2, 50, 70, 16, False), (3, 16, 16, 72, True), (1, 100, 130, 64, True),
                                          (2, 9, 5, 8, False), (1, 20, 40, 128, False)])
def test_attention_plain(fc, G, nq, nk, d, bf):
    got, want = _attn_case(fc, G, nq, nk, d, 2.0, bf, 1)
    assert rel_l2(got, want) < (5e-3 if bf else 2e-5)


def test_attention_rows_are_convex_combinations(fc):
    """Property that holds at any size: with all-ones V every output is exactly 1
    (softmax rows sum to 1), also across a ragged last key tile."""
    torch = _torch()
    G, nq, nk, d = 2, 130, 1000, 64
    q, k, _ = synth.sharp_qkv(3, nq, nk, d, gain=2.0)
    q, k = np.stack([BF(q)] * G), np.stack([BF(k)] * G)
    v = np.ones((G, nk, d), dtype=np.float32)
    out = torch.empty((G, nq, d), dtype=torch.bfloat16, device="cuda:0")
    fc.fc_op_attention(fc.FC_BF16, dev(q, True), dev(k, True), dev(v, True), out, G, nq, nk, d, 0)
    torch.cuda.synchronize()
    np.testing.assert_allclose(host(out), 1.0, atol=8e-3)


# --------------------------------------------------------------------------- LayerNorm + modulate

@pytest.mark.parametrize("M,D", [(1, 64), (37, 1152), (130, 3072), (5, 4), (9, 4096), (3, 260)])
@pytest.mark.parametrize("bf", [False, True])
@pytest.mark.parametrize("mod", [True, False])
def test_layernorm_modulate(fc, M, D, bf, mod):
    torch = _torch()
    rng = np.random.default_rng(M + D)
    x = rng.standard_normal((M, D), dtype=np.float32) * 3 + 1
    sh = rng.standard_normal(D, dtype=np.float32) if mod else None
    sc = rng.standard_normal(D, dtype=np.float32) if mod else None
    want = dit.layernorm(x.astype(np.float64), 1e-6)
    if mod:
        want = dit.modulate(want, sh, sc)
    out = torch.empty((M, D), dtype=torch.bfloat16 if bf else torch.float32, device="cuda:0")
    dx = dev(x)
    fc.fc_op_layernorm_modulate(fc.FC_BF16 if bf else fc.FC_F32, dx, None, dev(sh) if mod else None,
                                dev(sc) if mod else None, out, M, D, 1e-6)
    torch.cuda.synchronize()
    assert rel_l2(host(out), want) < (4e-3 if bf else 2e-6)
    assert np.array_equal(host(dx), x)                        # no pending branch: x untouched


@pytest.mark.parametrize("M,D", [(37, 1152), (130, 3072), (9, 4096), (3, 260), (5, 4)])
@pytest.mark.parametrize("bf", [False, True])
@pytest.mark.parametrize("gated", [False, True])
def test_layernorm_with_deferred_residual_additions(fc, M, D, bf, gated):
    """The residual additions of a pre-LN block, two per write of x: the first call adds one
    pending branch output and must leave x untouched, the second adds both and writes the sum.
    Expected values: x + g1 y1 (+ g2 y2) in float64 on the values the kernel is given (branch
    outputs rounded to the activation type first), then the oracle's LayerNorm and modulation."""
    torch = _torch()
    rng = np.random.default_rng(7 * M + D)
    x = rng.standard_normal((M, D), dtype=np.float32) * 3 + 1
    y1 = rng.standard_normal((M, D), dtype=np.float32)
    y2 = rng.standard_normal((M, D), dtype=np.float32) * 2
    if bf:
        y1, y2 = BF(y1), BF(y2)
    g1 = rng.standard_normal(D, dtype=np.float32) if gated else None
    g2 = rng.standard_normal(D, dtype=np.float32) if gated else None
    sh, sc = rng.standard_normal(D, dtype=np.float32), rng.standard_normal(D, dtype=np.float32)
    code = fc.FC_BF16 if bf else fc.FC_F32
    tdt = torch.bfloat16 if bf else torch.float32
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    v1 = f64(x) + (f64(g1) if gated else 1.0) * f64(y1)
    v2 = v1 + (f64(g2) if gated else 1.0) * f64(y2)
    dx, dy1, dy2 = dev(x), dev(y1, bf), dev(y2, bf)
    dg1, dg2 = (dev(g1), dev(g2)) if gated else (None, None)
    out = torch.empty((M, D), dtype=tdt, device="cuda:0")
    # one pending, not written back
    fc.fc_op_layernorm_residual2(code, dx, dy1, dg1, None, None, dev(sh), dev(sc), out, M, D, 1e-6, 0)
    torch.cuda.synchronize()
    assert rel_l2(host(out), dit.modulate(dit.layernorm(v1, 1e-6), sh, sc)) < (4e-3 if bf else 2e-6)
    assert np.array_equal(host(dx), x)
    # both, written back
    fc.fc_op_layernorm_residual2(code, dx, dy1, dg1, dy2, dg2, None, None, out, M, D, 1e-6, 1)
    torch.cuda.synchronize()
    assert rel_l2(host(out), dit.layernorm(v2, 1e-6)) < (4e-3 if bf else 2e-6)
    assert np.abs(host(dx) - v2).max() <= 2e-6 * np.abs(v2).max() + 1e-6
    # the same sum as adding each branch when it arrives (two writes of x): bit for bit
    dx2 = dev(x)
    fc.fc_op_layernorm_residual2(code, dx2, dy1, dg1, None, None, None, None, out, M, D, 1e-6, 1)
    fc.fc_op_layernorm_residual2(code, dx2, dy2, dg2, None, None, None, None, out, M, D, 1e-6, 1)
    torch.cuda.synchronize()
    assert np.array_equal(host(dx2), host(dx))


@pytest.mark.parametrize("impl", [1, 2])
@pytest.mark.parametrize("shape", [
    # T, H, W, C, D, R, B, row_off
    (3, 12, 20, 16, 256, 2, 4, 5),        # ragged spatial tile (60 positions), guidance rows reuse latents, text rows ahead
    (2, 16, 16, 16, 512, 1, 1, 0),
])
def test_patch_embed_kernels(fc, shape, impl):
    """Both patch-embedding kernels against patchify + matmul + position add in float64.
    The matrix-core kernel multiplies bf16 high/low splits of both fp32 operands
    (hi*hi + hi*lo + lo*hi): the bound is relative 2^-15 of sum |patch| |w| per output."""
    import torch
    T, H, W, C, D, R, B, row_off = shape
    p = 2
    rng = np.random.default_rng(1234)
    S = (H // p) * (W // p)
    lat = rng.standard_normal((R, T, H, W, C)).astype(np.float32)
    Wp = (rng.standard_normal((p * p * C, D)) * 0.05).astype(np.float32)
    bp = rng.standard_normal(D).astype(np.float32)
    pos_sp = rng.standard_normal((S, D)).astype(np.float32)
    pos_t = rng.standard_normal((T, D)).astype(np.float32)
    rows_per_b = row_off + T * S + 3
    x = torch.full((B, rows_per_b, D), -7.0, device="cuda:0")
    fc.fc_op_patch_embed(dev(lat), R, B, dev(Wp), dev(bp), dev(pos_sp), dev(pos_t), x, T, H, W, C, p, D, rows_per_b,
                         row_off, impl)
    torch.cuda.synchronize()
    got = host(x)
    for b in range(B):
        patches = dit.patchify(lat[b % R].astype(np.float64), p)
        want = patches @ Wp.astype(np.float64) + bp + (pos_t[:, None, :] + pos_sp[None, :, :]).reshape(T * S, D)
        bound = 2.0 ** -15 * (np.abs(patches) @ np.abs(Wp).astype(np.float64)) + 1e-5
        assert (np.abs(got[b, row_off:row_off + T * S] - want) <= bound).all()
        # rows outside the video tokens are not touched
        assert (got[b, :row_off] == -7.0).all() and (got[b, row_off + T * S:] == -7.0).all()



# --------------------------------------------------------------------------- guidance + DDIM

@pytest.mark.parametrize("n", [1, 7, 4096, 65536 + 3])
@pytest.mark.parametrize("guided", [True, False])
def test_cfg_ddim(fc, n, guided):
    torch = _torch()
    rng = np.random.default_rng(n)
    x, ec, eu = (rng.standard_normal(n, dtype=np.float32) for _ in range(3))
    sched = synth.Schedule()
    coef, _ = fc.fc_schedule_coefficients(sched, 25)
    _, a_t, a_p = sampler.step_coefficients(sched, 25)
    e = sampler.guide(ec.astype(np.float64), eu.astype(np.float64), 7.5) if guided else ec.astype(np.float64)
    want = sampler.ddim_update(x.astype(np.float64), e, a_t, a_p)
    dx, de = dev(x), torch.empty(n, dtype=torch.float32, device="cuda:0")
    fc.fc_op_cfg_ddim(dx, dev(ec), dev(eu) if guided else None, de, n, 7.5, coef)
    torch.cuda.synchronize()
    assert rel_l2(host(dx), want) < 1e-6
    assert rel_l2(host(de), e) < 1e-6


def test_cfg_ddim_misaligned_pointers(fc):
    torch = _torch()
    n = 1001
    rng = np.random.default_rng(1)
    x, ec = rng.standard_normal(n + 1, dtype=np.float32), rng.standard_normal(n + 1, dtype=np.float32)
    coef, _ = fc.fc_schedule_coefficients(synth.Schedule(), 50)
    _, a_t, a_p = sampler.step_coefficients(synth.Schedule(), 50)
    dx, de = dev(x), dev(ec)
    fc.fc_op_cfg_ddim(dx[1:], de[1:], None, None, n, 1.0, coef)     # 4-byte aligned only
    torch.cuda.synchronize()
    got = host(dx)
    assert got[0] == x[0]
    assert rel_l2(got[1:], sampler.ddim_update(x[1:].astype(np.float64), ec[1:].astype(np.float64), a_t, a_p)) < 1e-6
