"""GPU parity of every head dimension with every switch of Section 4.4: the squared-distance
estimator, 1-bit and 3-bit codes, with and without the transform, query groups up to 8.

One routine drives every stage through the C ABI and compares with the oracle at the same head
dimension: bulk key encode and query encode (code bytes), the fused step (indices, attention,
appended K / V / code rows), and the stand-alone distance + top-k call (every distance).
"""

import numpy as np
import pytest
import torch

import synth_inputs as synth

pytestmark = pytest.mark.gpu

THR = {1: (0.0,), 2: synth.DEFAULT_THRESHOLDS, 3: (-1.5, -1.0, -0.5, 0.0, 0.5, 1.0, 1.5)}


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    assert torch.cuda.is_available()
    return gpu_harness


def run_all_stages(H, oracle, hd, bits, variant, seed, B, Hq, Hkv, lens, k, append):
    import paper_2510_18413_amd as A
    G = Hq // Hkv
    thr = THR[bits]
    hadamard = not (variant & A.VARIANT_NO_HADAMARD)
    squared = bool(variant & A.VARIANT_L2)
    print("head_dim", hd, "bits", bits, "variant", variant, "B/Hq/Hkv", B, Hq, Hkv, "lens", lens,
          "k", k, "append", append, flush=True)
    case = synth.make_case("hd", seed, B, Hq, Hkv, lens, [0],
                           lambda b, L, h, rng: rng.choice(L, (G, min(1, L // G)), replace=False),
                           append=append, head_dim=hd)
    d = H.DeviceCase(case, k, variant=variant, code_bits=0 if bits == 2 else bits, thresholds=thr)
    row_bytes = hd // 8 * bits
    assert d.codes.shape[-1] == row_bytes
    with oracle.head_dim(hd):
        _, rows0 = oracle.encode_bits(case.K, thr, bits, hadamard=hadamard)
        _, qrows = oracle.encode_bits(case.q, thr, bits, hadamard=hadamard)
        K, V, rows = case.K.copy(), case.V.copy(), rows0.copy()
        scale = 1.0 / np.sqrt(float(hd))
        if bits == 2:
            ref_out, ref_idx, ref_dist = oracle.decode_step(
                case.q, K, V, rows, case.seq_start, case.seq_len, k, thr, thr, scale,
                k_new=case.k_new, v_new=case.v_new, want_dist=True, hadamard=hadamard,
                squared=squared)
        else:
            ref_out, ref_idx, ref_dist = oracle.decode_step_bits(
                case.q, K, V, rows, case.seq_start, case.seq_len, k, thr, thr, bits, scale,
                k_new=case.k_new, v_new=case.v_new, want_dist=True, hadamard=hadamard)
    assert np.array_equal(d.codes.cpu().numpy(), rows0), "bulk key encode"
    qcodes = torch.zeros(B, Hq, row_bytes, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    torch.cuda.synchronize()
    assert np.array_equal(qcodes.cpu().numpy(), qrows), "query encode"
    out, idx = d.decode_step()
    assert np.array_equal(idx, ref_idx), "fused step: indices"
    assert H.attn_rel_err(out, ref_out) <= H.ATTN_TOL
    if append:
        assert np.array_equal(d.codes.cpu().numpy(), rows), "appended code rows"
        assert np.array_equal(H.host_u16(d.K), K) and np.array_equal(H.host_u16(d.V), V)
    dist = torch.full((B, Hq, d.max_len), 0xFFFF, dtype=torch.uint16, device="cuda")
    idx2 = torch.full((B, Hq, k), -7, dtype=torch.int32, device="cuda")
    A.adamas_select_topk(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, k, idx2, d.max_len,
                         d.workspace, dist_out=dist)
    torch.cuda.synchronize()
    got = H.host_dist(dist)
    for b in range(B):
        L = int(case.seq_len[b])
        assert np.array_equal(got[b, :, :L], ref_dist[b, :, :L]), "distances"
    assert np.array_equal(idx2.cpu().numpy(), ref_idx), "stand-alone top-k"


SHAPES = [
    # B, Hq, Hkv, lens, k, append
    (2, 8, 2, [4097, 333], 128, True),
    (1, 8, 1, [9000], 300, False),          # a query group of 8
    (3, 3, 3, [0, 2500, 1], 64, True),
]


@pytest.mark.parametrize("hd", [64, 256, 96, 160, 192])
@pytest.mark.parametrize("bits,variant", [(2, 2), (2, 3), (1, 0), (3, 0), (3, 1)])
def test_head_dim_with_every_switch(H, oracle, hd, bits, variant):
    for i, (B, Hq, Hkv, lens, k, append) in enumerate(SHAPES):
        run_all_stages(H, oracle, hd, bits, variant, 3000 + 10 * hd + 3 * bits + variant + i,
                       B, Hq, Hkv, lens, k, append)


@pytest.mark.parametrize("hd", [96, 160, 192])
def test_head_dims_two_to_the_n_times_12_and_20(H, oracle, hd):
    """The method itself (Hadamard transform H_{2^n} (x) H_m with Paley's H_12 / H_20, 2-bit
    codes, Eq. 6) at d = 96, 160, 192: every stage against the oracle, several shapes."""
    for i, (B, Hq, Hkv, lens, k, append) in enumerate(SHAPES + [(1, 4, 4, [20000], 256, True),
                                                                 (2, 6, 2, [1, 700], 16, False)]):
        run_all_stages(H, oracle, hd, 2, 0, 5000 + 10 * hd + i, B, Hq, Hkv, lens, k, append)
    run_all_stages(H, oracle, hd, 2, 1, 5900 + hd, 2, 4, 2, [3000, 129], 64, True)   # without the transform


@pytest.mark.parametrize("hd", [96, 160, 192])
def test_head_dims_two_to_the_n_times_m_values_on_thresholds(H, oracle, hd):
    """Coefficients that fall exactly on a threshold (strict comparison, Eq. 5), and zero vectors."""
    import paper_2510_18413_amd as A
    rng = np.random.default_rng(hd)
    n = 512
    x = np.zeros((1, n, hd), dtype=np.float32)
    # one element -> every coefficient is +-that element; sqrt(d) scales the thresholds, so choose
    # thresholds t = v / sqrt(d) with v a bf16 value: coefficients equal to +-v sit on +-t * sqrt(d)
    vals = rng.choice([0.5, 1.0, 2.0, 3.0], n).astype(np.float32)
    pos = rng.integers(0, hd, n)
    x[0, np.arange(n), pos] = vals * rng.choice([-1.0, 1.0], n).astype(np.float32)
    x[0, :8] = 0.0
    xb = synth.f32_to_bf16_bits(x)
    for v in (0.5, 1.0, 2.0):
        t = float(np.float32(v / np.sqrt(np.float64(hd))))
        thr = (-t, 0.0, t)
        cfg = A.Config.make(1, 1, n, thr_k=thr, head_dim=hd)
        K = H.dev_bf16(xb)
        codes = torch.zeros(1, n, hd // 4, dtype=torch.uint8, device="cuda")
        A.adamas_encode_keys(cfg, K, codes, 0, n)
        torch.cuda.synchronize()
        with oracle.head_dim(hd):
            _, rows = oracle.encode(xb, thr)
        assert np.array_equal(codes.cpu().numpy(), rows), v


def test_group_of_eight_at_head_dim_256(H, oracle):
    run_all_stages(H, oracle, 256, 2, 0, 3900, 1, 16, 2, [6000], 200, True)


@pytest.mark.parametrize("hd", [64, 256, 96, 160, 192])
@pytest.mark.parametrize("bits,squared", [(1, False), (3, False), (2, True), (2, False)])
def test_head_dim_largest_distance(H, oracle, hd, bits, squared):
    """Lowest against highest code in every coefficient: the largest distance of the metric."""
    import paper_2510_18413_amd as A
    case = synth.make_case("far", 3950, 1, 1, 1, [2000], [0],
                           lambda b, L, h, rng: np.zeros((1, 0), dtype=np.int64), head_dim=hd)
    case.K[:] = 0
    case.K[0, :, 0] = int(synth.f32_to_bf16_bits(np.float32([64.0]))[0])    # every coefficient +64
    case.q[:] = 0
    case.q[0, 0, 0] = int(synth.f32_to_bf16_bits(np.float32([-64.0]))[0])   # every coefficient -64
    d = H.DeviceCase(case, 16, variant=A.VARIANT_L2 if squared else 0,
                     code_bits=0 if bits == 2 else bits, thresholds=THR[bits])
    qcodes = torch.zeros(1, 1, hd // 8 * bits, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    dist = torch.zeros(1, 1, 2000, dtype=torch.uint16, device="cuda")
    A.adamas_manhattan_distance(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, dist)
    torch.cuda.synchronize()
    top = (1 << bits) - 1
    assert np.all(H.host_dist(dist) == (top * top if squared else top) * hd)
    out, idx = d.decode_step()
    assert idx[0, 0].tolist() == list(range(16))
