"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.

Codes, distances and indices must match bit for bit; attention outputs within ATTN_TOL.
Sizes here are small enough for the oracle to finish in seconds but span several scan tiles,
select segments and ragged tails.  Full-size configurations live in test_gpu_configs.py.
"""

import numpy as np
import pytest
import torch

import synth_inputs as synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    assert torch.cuda.is_available()
    return gpu_harness


def small_case(seed, B, Hq, Hkv, lens, append=False, needles=1, head_dim=128):
    G = Hq // Hkv
    return synth.make_case("small", seed, B, Hq, Hkv, lens, [0],
                           lambda b, L, h, rng: rng.choice(L, (G, min(needles, L // G)), replace=False),
                           append=append, head_dim=head_dim)


# ----------------------------------------------------------------------------- encode

def test_encode_keys_and_query_bit_exact(H, oracle):
    import paper_2510_18413_amd as A
    case = small_case(101, 2, 8, 4, [777, 1300])
    d = H.DeviceCase(case, 16)
    torch.cuda.synchronize()
    _, rows = oracle.encode(case.K, case.thresholds)
    assert np.array_equal(d.codes.cpu().numpy(), rows)
    qcodes = torch.zeros(case.B, case.Hq, 32, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    torch.cuda.synchronize()
    assert np.array_equal(qcodes.cpu().numpy(), oracle.encode(case.q, case.thresholds)[1])


def test_encode_keys_row_ranges_and_thresholds(H, oracle):
    import paper_2510_18413_amd as A
    case = small_case(102, 1, 2, 2, [500])
    thr = (-0.4, 0.25, 1.7)
    cfg = A.Config.make(2, 2, case.pool_tokens, thr_k=thr)
    K = H.dev_bf16(case.K)
    codes = torch.full((2, case.pool_tokens, 32), 0xEE, dtype=torch.uint8, device="cuda")
    A.adamas_encode_keys(cfg, K, codes, 37, 101)
    torch.cuda.synchronize()
    got = codes.cpu().numpy()
    _, rows = oracle.encode(case.K, thr)
    assert np.array_equal(got[:, 37:138], rows[:, 37:138])
    assert np.all(got[:, :37] == 0xEE) and np.all(got[:, 138:] == 0xEE)   # untouched outside


def test_encode_values_on_thresholds_and_zeros(H, oracle):
    import paper_2510_18413_amd as A
    # vectors whose transform hits thresholds exactly: +-e_i combinations give coefficients in
    # {0, +-2, ...}; with thresholds at 2/sqrt(128) multiples the strict '>' decides.
    x = np.zeros((6, 128), dtype=np.float32)
    x[1, 0] = 1.0
    x[2, 0], x[2, 1] = 1.0, -1.0
    x[3, 5], x[3, 77] = 0.5, 0.5
    x[4, :] = 0.125
    x[5, 3] = -0.0
    bits = synth.f32_to_bf16_bits(x)
    root = np.float32(np.sqrt(128.0))
    for thr in ((-1.0, 0.0, 1.0), (0.0, float(np.float32(1.0) / root), float(np.float32(2.0) / root))):
        cfg = A.Config.make(1, 1, 6, thr_k=thr)
        K = H.dev_bf16(bits.reshape(1, 6, 128))
        codes = torch.zeros(1, 6, 32, dtype=torch.uint8, device="cuda")
        A.adamas_encode_keys(cfg, K, codes, 0, 6)
        torch.cuda.synchronize()
        assert np.array_equal(codes.cpu().numpy()[0], oracle.encode(bits, thr)[1])


def test_encode_coefficients_within_rounding_of_a_threshold(H, oracle):
    """The bulk encode first tries single precision and keeps a vector's result only when every
    coefficient is provably on the right side of every threshold.  near_threshold_cases feeds it
    vectors for which that cannot be certified and on which plain single precision is wrong (a
    CPU test shows that).  Bulk and query encode must equal the oracle bit for bit."""
    import paper_2510_18413_amd as A
    import near_threshold_cases as ntc
    n, above = ntc.N_VECTORS, 0
    for trial, (bits, thr, picks) in enumerate(ntc.trials(oracle)):
        tau = np.array(thr, dtype=np.float64) * np.sqrt(128.0)
        above += int(np.sum(np.array(picks) > tau))        # exact sums just above their threshold
        cfg = A.Config.make(1, 1, n, thr_k=thr)
        codes = torch.zeros(1, n, 32, dtype=torch.uint8, device="cuda")
        A.adamas_encode_keys(cfg, H.dev_bf16(bits.reshape(1, n, 128)), codes, 0, n)
        qcodes = torch.zeros(n, 1, 32, dtype=torch.uint8, device="cuda")
        A.adamas_encode_query(A.Config.make(1, 1, n, thr_k=thr, thr_q=thr),
                              H.dev_bf16(bits.reshape(n, 1, 128)), qcodes)
        torch.cuda.synchronize()
        ref = oracle.encode(bits, thr)[1]
        assert np.array_equal(codes.cpu().numpy()[0], ref), trial
        assert np.array_equal(qcodes.cpu().numpy()[:, 0], ref), trial
    assert above > 5       # both sides of the thresholds occurred


@pytest.mark.parametrize("hd", [64, 128, 256, 96, 160, 192])
def test_encode_symmetric_thresholds_within_rounding_of_a_coefficient(H, oracle, hd):
    """Thresholds (-t, 0, t) take a route of their own through the bulk encode (|y| against t and
    the sign of y).  Here t is the magnitude of one of a vector's exact coefficients rounded to
    float, the vectors have the wide exponent spread on which single precision rounds, and some
    have coefficients that are exactly zero (equal elements, zeros of either sign)."""
    import paper_2510_18413_amd as A
    rng = np.random.default_rng(4100 + hd)
    n = 512
    above = below = 0
    for trial in range(12):
        x = rng.standard_normal((n, hd), dtype=np.float32)
        x[:, 1::2] *= np.float32(2.0 ** -10)
        x[0::7, :] = x[0::7, :1]                  # constant vectors: every coefficient but one is 0
        x[1::7, hd // 2:] = x[1::7, :hd // 2]     # repeated halves: half of the coefficients are 0
        x[2::7, :] = 0.0
        x[2::7, 3::5] = -0.0
        bits = synth.f32_to_bf16_bits(x)
        xs = synth.bf16_bits_to_f32(bits).astype(np.float64)
        with oracle.head_dim(hd):
            y = oracle.hadamard_transform(xs[3 + 7 * int(rng.integers(40))])
        pick = float(np.abs(y[rng.integers(hd)]))
        t = float(np.float32(pick / np.sqrt(float(hd))))
        if not t > 0.0:
            continue
        tau = t * np.sqrt(float(hd))
        above += pick > tau
        below += pick < tau
        thr = (-t, 0.0, t)
        cfg = A.Config.make(1, 1, n, thr_k=thr, head_dim=hd)
        codes = torch.zeros(1, n, hd // 4, dtype=torch.uint8, device="cuda")
        A.adamas_encode_keys(cfg, H.dev_bf16(bits.reshape(1, n, hd)), codes, 0, n)
        torch.cuda.synchronize()
        with oracle.head_dim(hd):
            ref = oracle.encode(bits, thr)[1]
        assert np.array_equal(codes.cpu().numpy()[0], ref), trial
    assert above > 0 and below > 0


@pytest.mark.parametrize("hd,bits", [(128, 2), (64, 2), (256, 2), (128, 1), (128, 3),
                                     (96, 2), (160, 2), (192, 2), (96, 3), (160, 1), (192, 3)])
def test_encode_wide_exponent_spread(H, oracle, hd, bits):
    """60 000 vectors whose elements span about 28 binary orders of magnitude (so that single
    precision sums round all the time) against odd thresholds: every code byte as the oracle's."""
    import paper_2510_18413_amd as A
    rng = np.random.default_rng(900 + hd + bits)
    n = 60000
    x = rng.standard_normal((n, hd), dtype=np.float32)
    x *= np.exp2(rng.integers(-20, 9, size=(n, hd))).astype(np.float32)
    x[rng.random((n, hd)) < 0.05] = 0.0
    xb = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))          # synth flushes |x| < 2^-24
    bf = (xb.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    thr = {1: (0.13,), 2: (-0.7, 0.13, 0.9), 3: (-2.1, -0.7, -0.2, 0.13, 0.5, 0.9, 3.3)}[bits]
    cfg = A.Config.make(1, 1, n, thr_k=thr, head_dim=hd, code_bits=0 if bits == 2 else bits)
    codes = torch.zeros(1, n, cfg.code_row_bytes, dtype=torch.uint8, device="cuda")
    A.adamas_encode_keys(cfg, H.dev_bf16(bf.reshape(1, n, hd)), codes, 0, n)
    torch.cuda.synchronize()
    with oracle.head_dim(hd):
        ref = oracle.encode_bits(bf, thr, bits)[1] if bits != 2 else oracle.encode(bf, thr)[1]
    assert np.array_equal(codes.cpu().numpy()[0], ref)


def test_encode_extreme_magnitudes(H, oracle):
    """Vectors scaled by 2^100 and 2^-100 (thresholds scaled alike): the single-precision
    attempt must step aside where its sums could overflow, and stay exact where they are tiny."""
    import paper_2510_18413_amd as A
    rng = np.random.default_rng(78)
    x = rng.standard_normal((512, 128), dtype=np.float32)
    for scale in (2.0 ** 100, 2.0 ** -100):
        xb = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x)) * np.float32(scale)   # exact: a power of two
        bits = (xb.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
        assert np.array_equal(synth.bf16_bits_to_f32(bits), xb)
        thr = tuple(float(np.float32(t * scale)) for t in (-1.0, 0.0, 1.0))
        cfg = A.Config.make(1, 1, 512, thr_k=thr)
        codes = torch.zeros(1, 512, 32, dtype=torch.uint8, device="cuda")
        A.adamas_encode_keys(cfg, H.dev_bf16(bits.reshape(1, 512, 128)), codes, 0, 512)
        torch.cuda.synchronize()
        ref_codes, ref = oracle.encode(bits, thr)
        assert np.array_equal(codes.cpu().numpy()[0], ref), scale
        assert len(np.unique(ref_codes)) == 4


# -------------------------------------------------------------------- distance + top-k

@pytest.mark.parametrize("B,Hq,Hkv,lens,k", [
    (1, 1, 1, [1024], 64),
    (1, 4, 4, [5000], 128),          # two 4096-token segments with a ragged tail
    (2, 8, 2, [4097, 333], 256),     # GQA group 4, k close to one sequence's length
    (3, 6, 2, [1, 64, 65], 8),       # group 3, tiny sequences
    (1, 8, 1, [9000], 100),          # group 8
    (1, 2, 2, [70000], 1024),        # 18 segments -> longer segments, several passes
])
def test_distance_and_topk_bit_exact(H, oracle, B, Hq, Hkv, lens, k):
    import paper_2510_18413_amd as A
    case = small_case(200 + Hq + B, B, Hq, Hkv, lens)
    d = H.DeviceCase(case, k)
    qcodes = torch.zeros(B, Hq, 32, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    dist = torch.full((B, Hq, d.max_len), 0xFFFF, dtype=torch.uint16, device="cuda")
    A.adamas_manhattan_distance(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, dist)
    dist2 = torch.full((B, Hq, d.max_len), 0xFFFF, dtype=torch.uint16, device="cuda")
    A.adamas_select_topk(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, k, d.idx, d.max_len,
                         d.workspace, dist_out=dist2)
    torch.cuda.synchronize()
    ref = H.oracle_step(case, k)
    got, got2 = H.host_dist(dist), H.host_dist(dist2)
    for b in range(B):
        L = int(case.seq_len[b])
        assert np.array_equal(got[b, :, :L], ref["dist"][b, :, :L])
        assert np.array_equal(got2[b, :, :L], ref["dist"][b, :, :L])
        assert np.all(got[b, :, L:] == 0xFFFF)                 # untouched past the sequence
    assert np.array_equal(d.idx.cpu().numpy(), ref["idx"])


def test_topk_ties_everywhere(H, oracle):
    """All keys identical: every distance equal, so the rule 'lowest position first' decides
    everything; then two distance levels with the boundary inside the second."""
    import paper_2510_18413_amd as A
    case = small_case(301, 1, 2, 1, [6000])
    case.K[0, :] = case.K[0, 0]
    case.K[0, 4500:4600] = synth.f32_to_bf16_bits(
        synth.bf16_bits_to_f32(case.q[0, 0]))                  # 100 near-exact matches of head 0
    for k in (1, 37, 100, 101, 4096):
        d = H.DeviceCase(case, k)
        qcodes = torch.zeros(1, 2, 32, dtype=torch.uint8, device="cuda")
        A.adamas_encode_query(d.cfg, d.q, qcodes)
        A.adamas_select_topk(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, k, d.idx, d.max_len,
                             d.workspace)
        torch.cuda.synchronize()
        ref = H.oracle_step(case, k, want_dist=False)
        assert np.array_equal(d.idx.cpu().numpy(), ref["idx"]), k


def test_topk_k_at_least_length_and_empty(H, oracle):
    import paper_2510_18413_amd as A
    case = small_case(302, 3, 2, 2, [0, 5, 300], needles=0)
    k = 300
    d = H.DeviceCase(case, k)
    qcodes = torch.zeros(3, 2, 32, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    A.adamas_select_topk(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, k, d.idx, d.max_len,
                         d.workspace)
    torch.cuda.synchronize()
    got = d.idx.cpu().numpy()
    assert np.all(got[0] == -1)
    assert np.all(got[1, :, :5] == np.arange(5)) and np.all(got[1, :, 5:] == -1)
    assert np.all(got[2] == np.arange(300))
    assert np.array_equal(got, H.oracle_step(case, k, want_dist=False)["idx"])


# ------------------------------------------------------------------- sparse attention

def test_sparse_attn_matches_oracle(H, oracle):
    import paper_2510_18413_amd as A
    case = small_case(401, 2, 4, 2, [900, 2000])
    for k in (1, 17, 64, 700):
        d = H.DeviceCase(case, k, encode=False)
        rng = np.random.default_rng(k)
        idx = np.full((2, 4, k), -1, dtype=np.int32)
        for b in range(2):
            for h in range(4):
                n = int(rng.integers(0, k + 1)) if (b, h) != (0, 0) else k
                if (b, h) == (1, 3):
                    n = 0                                         # nothing selected -> zeros
                sel = np.sort(rng.choice(int(case.seq_len[b]), n, replace=False))
                slots = np.sort(rng.choice(k, n, replace=False))  # -1 holes anywhere
                idx[b, h, slots] = sel
        A.adamas_sparse_attn(d.cfg, d.q, d.K, d.V, d.seq_start, torch.from_numpy(idx).cuda(), d.out,
                             d.max_len, d.workspace)
        torch.cuda.synchronize()
        got = d.out.cpu().numpy()
        ref = np.zeros_like(got)
        for b in range(2):
            s, L = int(case.seq_start[b]), int(case.seq_len[b])
            for h in range(4):
                ref[b, h] = oracle.sparse_attention(case.q[b, h], case.K[h // 2, s:s + L],
                                                    case.V[h // 2, s:s + L], idx[b, h], H.SM_SCALE)
        assert np.all(got[1, 3] == 0)
        assert H.attn_rel_err(got, ref) <= H.ATTN_TOL


def test_sparse_attn_equals_full_attention_when_all_rows_listed(H, oracle):
    import paper_2510_18413_amd as A
    case = small_case(402, 1, 2, 1, [513])
    d = H.DeviceCase(case, 513, encode=False)
    idx = torch.arange(513, dtype=torch.int32, device="cuda").repeat(1, 2, 1)
    A.adamas_sparse_attn(d.cfg, d.q, d.K, d.V, d.seq_start, idx, d.out, d.max_len, d.workspace)
    torch.cuda.synchronize()
    ref = np.stack([oracle.full_attention(case.q[0, h], case.K[0, :513], case.V[0, :513], H.SM_SCALE)
                    for h in range(2)])[None]
    assert H.attn_rel_err(d.out.cpu().numpy(), ref) <= H.ATTN_TOL


def test_sparse_attn_large_scores_do_not_overflow(H, oracle):
    import paper_2510_18413_amd as A
    case = small_case(403, 1, 1, 1, [64])
    case.q[:] = synth.f32_to_bf16_bits(np.full(128, 30.0, np.float32))
    case.K[0, :32] = synth.f32_to_bf16_bits(np.full(128, 30.0, np.float32))
    d = H.DeviceCase(case, 64, encode=False)
    idx = torch.arange(64, dtype=torch.int32, device="cuda").view(1, 1, 64)
    A.adamas_sparse_attn(d.cfg, d.q, d.K, d.V, d.seq_start, idx, d.out, d.max_len, d.workspace)
    torch.cuda.synchronize()
    ref = oracle.full_attention(case.q[0, 0], case.K[0, :64], case.V[0, :64], H.SM_SCALE)[None, None]
    got = d.out.cpu().numpy()
    assert np.all(np.isfinite(got)) and H.attn_rel_err(got, ref) <= H.ATTN_TOL


@pytest.mark.parametrize("B,Hq,Hkv,lens", [
    (1, 1, 1, [1024]),
    (1, 4, 4, [5000]),
    (3, 8, 2, [4097, 0, 333]),
    (2, 8, 1, [300, 9000]),
    (1, 6, 2, [20001]),
])
def test_full_attention_matches_oracle(H, oracle, B, Hq, Hkv, lens):
    """The dense comparison kernel (Eq. 1 over every cached row) against the oracle's full
    attention, per (sequence, query head); an empty sequence gives zeros."""
    import paper_2510_18413_amd as A
    case = small_case(700 + Hq, B, Hq, Hkv, lens)
    d = H.DeviceCase(case, 16, encode=False)
    ws = torch.full((A.adamas_full_attn_workspace_bytes(d.cfg, B, d.max_len),), 0xA5,
                    dtype=torch.uint8, device="cuda")
    A.adamas_full_attn(d.cfg, d.q, d.K, d.V, d.seq_start, d.seq_len, d.out, d.max_len, ws)
    torch.cuda.synchronize()
    got = d.out.cpu().numpy()
    G = Hq // Hkv
    ref = np.zeros_like(got, dtype=np.float64)
    for b in range(B):
        s, L = int(case.seq_start[b]), int(case.seq_len[b])
        for h in range(Hq):
            if L > 0:
                ref[b, h] = oracle.full_attention(case.q[b, h], case.K[h // G, s:s + L],
                                                  case.V[h // G, s:s + L], H.SM_SCALE)
            else:
                assert np.all(got[b, h] == 0)
    assert np.all(np.isfinite(got)) and H.attn_rel_err(got, ref) <= H.ATTN_TOL


def test_stream_read_probe_touches_nothing(H, oracle):
    """The bandwidth probe only reads: source and sink stay as they were, for full and ragged
    launch sizes."""
    import paper_2510_18413_amd as A
    for n in (32, 32 * 513, 1 << 20):
        src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
        keep = src.clone()
        sink = torch.full((4,), 7, dtype=torch.int32, device="cuda")
        A.adamas_stream_read(src, sink)
        torch.cuda.synchronize()
        assert torch.equal(src, keep) and sink.tolist() == [7, 7, 7, 7]


# ----------------------------------------------------------------------- fused decode step

@pytest.mark.parametrize("B,Hq,Hkv,lens,k,append", [
    (1, 1, 1, [1024], 64, False),
    (1, 4, 4, [5000], 128, False),
    (2, 8, 2, [4097, 333], 256, True),
    (4, 8, 2, [0, 1, 4096, 8193], 64, True),
    (3, 6, 2, [100, 64, 65], 128, False),      # k above every length: full attention
    (1, 8, 1, [20000], 4096, True),
    (1, 2, 2, [70000], 1024, False),
])
def test_decode_step_matches_oracle(H, oracle, B, Hq, Hkv, lens, k, append):
    case = small_case(500 + B + Hq, B, Hq, Hkv, lens, append=append)
    d = H.DeviceCase(case, k)
    out, idx = d.decode_step()
    ref = H.oracle_step(case, k, want_dist=False)
    assert np.array_equal(idx, ref["idx"])
    assert H.attn_rel_err(out, ref["out"]) <= H.ATTN_TOL
    for b in range(B):
        if case.seq_len[b] == 0:
            assert np.all(out[b] == 0) and np.all(idx[b] == -1)
    if append:   # Algorithm 1, cache update: cache rows and code rows of the new token, bit for bit
        assert np.array_equal(H.host_u16(d.K), ref["K"])
        assert np.array_equal(H.host_u16(d.V), ref["V"])
        assert np.array_equal(d.codes.cpu().numpy(), ref["rows"])
    # same call without the index output, on a fresh poisoned workspace: same attention result
    d2 = H.DeviceCase(case, k)
    out2, _ = d2.decode_step(with_idx=False)
    assert np.array_equal(out, out2)


def test_decode_step_prologue_on_vectors_within_rounding_of_a_threshold(H, oracle):
    """The decode step encodes its queries and the appended keys in its own prologue, one vector
    per wave (exact sums in double precision).  Queries and new keys here are the vectors of near_threshold_cases, some of whose coefficients lie within a
    rounding of a threshold (plain single precision misjudges them).  The appended code rows must
    equal the oracle's bit for bit, and so must the selection: a query code off by one moves every
    distance and with it the ties."""
    import near_threshold_cases as ntc
    B, Hq, Hkv = 8, 4, 2
    for trial, (bits, thr, picks) in enumerate(ntc.trials(oracle, n_trials=8)):
        case = small_case(1300 + trial, B, Hq, Hkv, [300 + 170 * b for b in range(B)], append=True)
        special = [17, 117, 217]                    # the vectors the thresholds were taken from
        others = [i for i in range(ntc.N_VECTORS) if i not in special]
        kn = (special + others[:B * Hkv - 3])
        qs = (others[40:40 + B * Hq - 3] + special)
        case.k_new = np.ascontiguousarray(bits[kn].reshape(B, Hkv, 128))
        case.q = np.ascontiguousarray(bits[qs].reshape(B, Hq, 128))
        case.thresholds = thr
        d = H.DeviceCase(case, 48)
        out, idx = d.decode_step()
        ref = H.oracle_step(case, 48, want_dist=False)
        assert np.array_equal(d.codes.cpu().numpy(), ref["rows"]), trial
        assert np.array_equal(idx, ref["idx"]), trial
        assert H.attn_rel_err(out, ref["out"]) <= H.ATTN_TOL


def test_decode_step_repeatable_and_workspace_reusable(H, oracle):
    case = small_case(601, 2, 8, 2, [3000, 9000])
    d = H.DeviceCase(case, 128)
    first = d.decode_step()
    for _ in range(3):
        again = d.decode_step()
        assert np.array_equal(first[0], again[0]) and np.array_equal(first[1], again[1])


def test_decode_step_back_to_back_on_one_workspace(H, oracle):
    """Different inputs alternate on ONE workspace with no host synchronisation between the
    calls.  The one-call step combines the segments' attention partials inside the select
    kernel (last segment to finish, device-scope atomics only); the staged call uses the
    separate merge kernel.  Both must give the same bits every time, and the oracle's answer."""
    import paper_2510_18413_amd as A
    cases = [small_case(610 + i, 2, 16, 4, [30000, 9000 + 4000 * i]) for i in range(2)]
    devs = [H.DeviceCase(c, 256) for c in cases]
    shared = devs[0].workspace
    assert devs[1].workspace.numel() == shared.numel()
    want = []
    for d in devs:        # scan, then select + merge kernel, as two calls
        for stages in (A.STAGE_SCAN, A.STAGE_SELECT_ATTN):
            A.adamas_decode_step_stages(d.cfg, d.q, d.K, d.V, d.codes, d.seq_start, d.seq_len, d.k,
                                        d.out, d.max_len, shared, idx_out=d.idx, stages=stages)
        torch.cuda.synchronize()
        want.append(d.out.clone())
        ref = H.oracle_step(d.case, d.k, want_dist=False)
        assert np.array_equal(d.idx.cpu().numpy(), ref["idx"])
        assert H.attn_rel_err(d.out.cpu().numpy(), ref["out"]) <= H.ATTN_TOL
    got = []
    for it in range(48):
        d = devs[it % 2]
        d.out.fill_(float("nan"))
        A.adamas_decode_step(d.cfg, d.q, d.K, d.V, d.codes, d.seq_start, d.seq_len, d.k, d.out,
                             d.max_len, shared)
        got.append(d.out.clone())
    torch.cuda.synchronize()
    for it, g in enumerate(got):
        assert torch.equal(g, want[it % 2]), f"call {it}"


def test_decode_step_in_a_replayed_graph(H, oracle):
    """The fused step captured in a HIP graph (two layers with different inputs on one
    workspace) and replayed several times, with eager calls and synchronisations between the
    replays: every replay must give the eager result, which must be the oracle's."""
    import paper_2510_18413_amd as A
    cases = [small_case(620 + i, 2, 8, 2, [20000, 5000 + 3000 * i], append=(i == 1)) for i in range(2)]
    devs = [H.DeviceCase(c, 128) for c in cases]
    shared = devs[0].workspace
    eager = []
    for d in devs:
        A.adamas_decode_step(d.cfg, d.q, d.K, d.V, d.codes, d.seq_start, d.seq_len, d.k, d.out,
                             d.max_len, shared, k_new=d.k_new, v_new=d.v_new, idx_out=d.idx)
        torch.cuda.synchronize()
        ref = H.oracle_step(d.case, d.k, want_dist=False)
        assert np.array_equal(d.idx.cpu().numpy(), ref["idx"])
        assert H.attn_rel_err(d.out.cpu().numpy(), ref["out"]) <= H.ATTN_TOL
        eager.append((d.out.clone(), d.idx.clone()))
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for d in devs:      # warm-up on the capture stream
            A.adamas_decode_step(d.cfg, d.q, d.K, d.V, d.codes, d.seq_start, d.seq_len, d.k,
                                 d.out, d.max_len, shared, k_new=d.k_new, v_new=d.v_new,
                                 idx_out=d.idx)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            for d in devs:
                A.adamas_decode_step(d.cfg, d.q, d.K, d.V, d.codes, d.seq_start, d.seq_len, d.k,
                                     d.out, d.max_len, shared, k_new=d.k_new, v_new=d.v_new,
                                     idx_out=d.idx)
    torch.cuda.synchronize()
    for rep in range(5):
        for d in devs:
            d.out.fill_(float("nan"))
            d.idx.fill_(-9)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for d, (o, i) in zip(devs, eager):
            assert torch.equal(d.out, o) and torch.equal(d.idx, i), f"replay {rep}"
        # eager work of the program itself between replays, on the same workspace
        d = devs[rep % 2]
        A.adamas_decode_step(d.cfg, d.q, d.K, d.V, d.codes, d.seq_start, d.seq_len, d.k, d.out,
                             d.max_len, shared, k_new=d.k_new, v_new=d.v_new)
        torch.cuda.synchronize()


def test_plain_c_client_of_the_abi(H, oracle):
    """tests/c_abi_client.c: hipMalloc'ed buffers and adamas.h only, no Python in the process.
    It runs the fused step (ragged batch, GQA, append) and checks it against the oracle itself."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = os.path.join(root, "tests", "c_abi_client")
    if not os.path.exists(exe):
        sys.path.insert(0, root)
        import __graft_entry__
        __graft_entry__.build_c_client()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "C ABI client: OK" in r.stdout


def test_appended_token_is_a_candidate(H, oracle):
    case = small_case(602, 1, 2, 2, [4097], append=True)     # new token alone in the 2nd segment
    case.q[0, 0] = case.k_new[0, 0]
    d = H.DeviceCase(case, 8)
    out, idx = d.decode_step()
    assert 4096 in idx[0, 0].tolist()
    ref = H.oracle_step(case, 8, want_dist=False)
    assert np.array_equal(idx, ref["idx"]) and H.attn_rel_err(out, ref["out"]) <= H.ATTN_TOL


def test_invalid_device_lengths_are_treated_as_empty(H, oracle):
    case = small_case(603, 2, 2, 2, [500, 600], needles=0)
    d = H.DeviceCase(case, 16)
    d.seq_len = torch.tensor([500, 10 ** 6], dtype=torch.int32, device="cuda")   # beyond max/pool
    out, idx = d.decode_step()
    assert np.all(idx[1] == -1) and np.all(out[1] == 0)
    case.seq_len[1] = 0
    ref = H.oracle_step(case, 16, want_dist=False)
    assert np.array_equal(idx[0], ref["idx"][0])


# ------------------------------------------------------- ablation variants (Section 4.4)

@pytest.mark.parametrize("variant", [1, 2, 3])      # NO_HADAMARD, L2, both
@pytest.mark.parametrize("B,Hq,Hkv,lens,k,append", [
    (1, 1, 1, [1024], 64, False),
    (2, 8, 2, [4097, 333], 128, True),
    (3, 4, 4, [0, 5000, 9000], 256, False),
    (1, 8, 1, [20000], 1024, True),
])
def test_variant_decode_step_matches_oracle(H, oracle, variant, B, Hq, Hkv, lens, k, append):
    """Every stage of the step under the ablation switches: code bytes, distances (through
    adamas_select_topk's optional output), indices bit for bit; attention within tolerance."""
    import paper_2510_18413_amd as A
    case = small_case(800 + variant + Hq, B, Hq, Hkv, lens, append=append)
    d = H.DeviceCase(case, k, variant=variant)
    hadamard = not (variant & A.VARIANT_NO_HADAMARD)
    _, rows0 = oracle.encode(case.K, case.thresholds, hadamard=hadamard)
    assert np.array_equal(d.codes.cpu().numpy(), rows0)                   # bulk key encode
    qcodes = torch.zeros(B, Hq, 32, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    torch.cuda.synchronize()
    _, qrows = oracle.encode(case.q, case.thresholds, hadamard=hadamard)
    assert np.array_equal(qcodes.cpu().numpy(), qrows)
    out, idx = d.decode_step()
    ref = H.oracle_step(case, k, want_dist=True, variant=variant)
    assert np.array_equal(idx, ref["idx"])
    assert H.attn_rel_err(out, ref["out"]) <= H.ATTN_TOL
    if append:
        assert np.array_equal(d.codes.cpu().numpy(), ref["rows"])
        assert np.array_equal(H.host_u16(d.K), ref["K"])
    # stand-alone select on the updated cache: distances and indices once more
    dist = torch.full((B, Hq, d.max_len), 0xFFFF, dtype=torch.uint16, device="cuda")
    idx2 = torch.full((B, Hq, k), -7, dtype=torch.int32, device="cuda")
    A.adamas_select_topk(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, k, idx2, d.max_len,
                         d.workspace, dist_out=dist)
    torch.cuda.synchronize()
    got = H.host_dist(dist)
    for b in range(B):
        L = int(case.seq_len[b])
        assert np.array_equal(got[b, :, :L], ref["dist"][b, :, :L])
    assert np.array_equal(idx2.cpu().numpy(), ref["idx"])


def test_variant_l2_extreme_distances(H, oracle):
    """All-0 against all-3 codes: 1152, the largest squared distance, and ties everywhere."""
    import paper_2510_18413_amd as A
    case = small_case(850, 1, 1, 1, [3000], needles=0)
    case.K[:] = synth.f32_to_bf16_bits(np.full(case.K.shape, 0.0, np.float32))
    case.K[0, :, 0] = int(synth.f32_to_bf16_bits(np.float32([64.0]))[0])    # every coefficient = +64
    case.q[:] = 0
    case.q[0, 0, 0] = int(synth.f32_to_bf16_bits(np.float32([-64.0]))[0])   # every coefficient = -64
    d = H.DeviceCase(case, 32, variant=A.VARIANT_L2)
    out, idx = d.decode_step()
    ref = H.oracle_step(case, 32, want_dist=True, variant=A.VARIANT_L2)
    assert int(ref["dist"].max()) == 1152
    assert np.array_equal(idx, ref["idx"]) and idx[0, 0].tolist() == list(range(32))
    assert H.attn_rel_err(out, ref["out"]) <= H.ATTN_TOL


def test_variant_without_hadamard_loses_the_true_top_k(H, oracle):
    """Direction of the paper's ablation (Section 4.4, Table 7) on the synthetic outlier data:
    without the transform the selected set overlaps the exact attention top-k far less."""
    import paper_2510_18413_amd as A
    case = small_case(860, 1, 4, 4, [8192], needles=8)
    k = 256
    overlap = {}
    for variant in (0, A.VARIANT_NO_HADAMARD):
        d = H.DeviceCase(case, k, variant=variant)
        _, idx = d.decode_step()
        q = synth.bf16_bits_to_f32(case.q[0]).astype(np.float64)
        K = synth.bf16_bits_to_f32(case.K[:, :8192]).astype(np.float64)
        ov = []
        for h in range(4):
            true_top = np.argsort(-(K[h] @ q[h]), kind="stable")[:k]
            ov.append(len(set(true_top.tolist()) & set(idx[0, h].tolist())) / k)
        overlap[variant] = float(np.mean(ov))
    assert overlap[0] > 0.3 and overlap[0] > 2.0 * overlap[A.VARIANT_NO_HADAMARD], overlap


# ----------------------------------- bucketization ablation: 1-bit and 3-bit codes

BITS_THR = {1: (0.0,), 3: (-1.5, -1.0, -0.5, 0.0, 0.5, 1.0, 1.5)}


@pytest.mark.parametrize("bits", [1, 3])
@pytest.mark.parametrize("B,Hq,Hkv,lens,k,append,variant", [
    (1, 1, 1, [1024], 64, False, 0),
    (2, 8, 2, [4097, 333], 128, True, 0),
    (3, 4, 4, [0, 5000, 9000], 256, False, 1),
    (1, 8, 1, [20000], 1024, True, 0),
    (1, 6, 2, [2500], 32, True, 1),
])
def test_code_bits_decode_step_matches_oracle(H, oracle, bits, B, Hq, Hkv, lens, k, append, variant):
    """1-bit and 3-bit codes through every stage: code bytes of keys and queries, distances,
    indices bit for bit; attention within tolerance; appended rows in the cache."""
    import paper_2510_18413_amd as A
    thr = BITS_THR[bits]
    hadamard = not (variant & A.VARIANT_NO_HADAMARD)
    case = small_case(1000 + 10 * bits + Hq, B, Hq, Hkv, lens, append=append)
    d = H.DeviceCase(case, k, variant=variant, code_bits=bits, thresholds=thr)
    assert d.codes.shape[-1] == 16 * bits
    _, rows0 = oracle.encode_bits(case.K, thr, bits, hadamard=hadamard)
    assert np.array_equal(d.codes.cpu().numpy(), rows0)
    qcodes = torch.zeros(B, Hq, 16 * bits, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    torch.cuda.synchronize()
    _, qrows = oracle.encode_bits(case.q, thr, bits, hadamard=hadamard)
    assert np.array_equal(qcodes.cpu().numpy(), qrows)
    out, idx = d.decode_step()
    K, V = case.K.copy(), case.V.copy()
    rows = rows0.copy()
    ref_out, ref_idx, ref_dist = oracle.decode_step_bits(
        case.q, K, V, rows, case.seq_start, case.seq_len, k, thr, thr, bits, H.SM_SCALE,
        k_new=case.k_new, v_new=case.v_new, want_dist=True, hadamard=hadamard)
    assert np.array_equal(idx, ref_idx)
    assert H.attn_rel_err(out, ref_out) <= H.ATTN_TOL
    if append:
        assert np.array_equal(d.codes.cpu().numpy(), rows)
        assert np.array_equal(H.host_u16(d.K), K) and np.array_equal(H.host_u16(d.V), V)
    dist = torch.full((B, Hq, d.max_len), 0xFFFF, dtype=torch.uint16, device="cuda")
    idx2 = torch.full((B, Hq, k), -7, dtype=torch.int32, device="cuda")
    A.adamas_select_topk(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, k, idx2, d.max_len,
                         d.workspace, dist_out=dist)
    torch.cuda.synchronize()
    got = H.host_dist(dist)
    for b in range(B):
        L = int(case.seq_len[b])
        assert np.array_equal(got[b, :, :L], ref_dist[b, :, :L])
    assert np.array_equal(idx2.cpu().numpy(), ref_idx)


@pytest.mark.parametrize("bits", [1, 3])
def test_code_bits_extreme_distances(H, oracle, bits):
    """Lowest against highest code everywhere: the largest distance, (2^bits - 1) * 128."""
    import paper_2510_18413_amd as A
    case = small_case(1050, 1, 1, 1, [2000], needles=0)
    case.K[:] = 0
    case.K[0, :, 0] = int(synth.f32_to_bf16_bits(np.float32([64.0]))[0])
    case.q[:] = 0
    case.q[0, 0, 0] = int(synth.f32_to_bf16_bits(np.float32([-64.0]))[0])
    d = H.DeviceCase(case, 16, code_bits=bits, thresholds=BITS_THR[bits])
    qcodes = torch.zeros(1, 1, 16 * bits, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    dist = torch.zeros(1, 1, 2000, dtype=torch.uint16, device="cuda")
    A.adamas_manhattan_distance(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, dist)
    torch.cuda.synchronize()
    assert np.all(H.host_dist(dist) == ((1 << bits) - 1) * 128)
    out, idx = d.decode_step()
    assert idx[0, 0].tolist() == list(range(16))


def test_code_bits_with_paged_cache(H, oracle):
    """3-bit codes on a paged cache: the two switches compose."""
    import paper_2510_18413_amd as A
    thr = BITS_THR[3]
    case = small_case(1060, 2, 4, 2, [3000, 700], append=True)
    pc = synth.paginate(case, 128, seed=13)
    cfg = A.Config.make(4, 2, pc.pool_tokens, thr_k=thr, code_bits=3)
    Kd, Vd, qd = H.dev_bf16(pc.K), H.dev_bf16(pc.V), H.dev_bf16(case.q)
    codes = torch.zeros(2, pc.pool_tokens, 48, dtype=torch.uint8, device="cuda")
    A.adamas_encode_keys(cfg, Kd, codes, 0, pc.pool_tokens)
    ws = torch.empty(A.adamas_workspace_bytes(cfg, 2, 3000, 64), dtype=torch.uint8, device="cuda")
    out = torch.zeros(2, 4, 128, device="cuda")
    idx = torch.zeros(2, 4, 64, dtype=torch.int32, device="cuda")
    A.adamas_decode_step_paged(cfg, qd, Kd, Vd, codes, torch.from_numpy(pc.page_table).cuda(), 128,
                               torch.from_numpy(case.seq_len).cuda(), 64, out, 3000, ws,
                               k_new=H.dev_bf16(case.k_new), v_new=H.dev_bf16(case.v_new),
                               idx_out=idx)
    torch.cuda.synchronize()
    # reference: the contiguous 3-bit step of the oracle on the unscattered case
    K, V = case.K.copy(), case.V.copy()
    _, rows = oracle.encode_bits(K, thr, 3)
    ref_out, ref_idx, _ = oracle.decode_step_bits(case.q, K, V, rows, case.seq_start, case.seq_len,
                                                  64, thr, thr, 3, H.SM_SCALE, k_new=case.k_new,
                                                  v_new=case.v_new)
    assert np.array_equal(idx.cpu().numpy(), ref_idx)
    assert H.attn_rel_err(out.cpu().numpy(), ref_out) <= H.ATTN_TOL


# --------------------------------------------------------------------- paged cache layout

@pytest.mark.parametrize("variant", [0, 3])
@pytest.mark.parametrize("B,Hq,Hkv,lens,k,page,append", [
    (1, 1, 1, [1024], 64, 64, False),
    (2, 8, 2, [4097, 333], 128, 256, True),       # 4097 = 16 * 256 + 1: the new token opens a page
    (3, 4, 4, [0, 5000, 9000], 256, 64, True),
    (1, 8, 1, [20000], 1024, 1024, True),
    (2, 6, 2, [70000, 129], 512, 128, False),
])
def test_paged_decode_step_matches_oracle(H, oracle, variant, B, Hq, Hkv, lens, k, page, append):
    """The step on a cache scattered over randomly placed pages: indices (token positions) bit
    for bit, attention within tolerance, and the appended row in the right physical page while
    every other pool row stays as it was."""
    import paper_2510_18413_amd as A
    case = small_case(900 + Hq + variant, B, Hq, Hkv, lens, append=append)
    pc = synth.paginate(case, page, seed=11)
    hadamard = not (variant & A.VARIANT_NO_HADAMARD)
    cfg = A.Config.make(Hq, Hkv, pc.pool_tokens, thr_k=case.thresholds, variant=variant)
    Kd, Vd, qd = H.dev_bf16(pc.K), H.dev_bf16(pc.V), H.dev_bf16(case.q)
    knd = None if case.k_new is None else H.dev_bf16(case.k_new)
    vnd = None if case.v_new is None else H.dev_bf16(case.v_new)
    codes = torch.zeros(Hkv, pc.pool_tokens, 32, dtype=torch.uint8, device="cuda")
    A.adamas_encode_keys(cfg, Kd, codes, 0, pc.pool_tokens)
    table = torch.from_numpy(pc.page_table).cuda()
    seq_len = torch.from_numpy(case.seq_len).cuda()
    max_len = max(case.max_seq_len, 1)
    ws = torch.full((A.adamas_workspace_bytes(cfg, B, max_len, k),), 0xA5, dtype=torch.uint8,
                    device="cuda")
    out = torch.full((B, Hq, 128), float("nan"), device="cuda")
    idx = torch.full((B, Hq, k), -7, dtype=torch.int32, device="cuda")
    A.adamas_decode_step_paged(cfg, qd, Kd, Vd, codes, table, page, seq_len, k, out, max_len, ws,
                               k_new=knd, v_new=vnd, idx_out=idx)
    torch.cuda.synchronize()
    Kr, Vr = pc.K.copy(), pc.V.copy()
    _, rows = oracle.encode(Kr, case.thresholds, hadamard=hadamard)
    ref_out, ref_idx = oracle.decode_step_paged(
        case.q, Kr, Vr, rows, pc.page_table, page, case.seq_len, k, case.thresholds,
        case.thresholds, H.SM_SCALE, k_new=case.k_new, v_new=case.v_new, hadamard=hadamard,
        squared=bool(variant & A.VARIANT_L2))
    assert np.array_equal(idx.cpu().numpy(), ref_idx)
    assert H.attn_rel_err(out.cpu().numpy(), ref_out) <= H.ATTN_TOL
    assert np.array_equal(H.host_u16(Kd), Kr) and np.array_equal(H.host_u16(Vd), Vr)
    assert np.array_equal(codes.cpu().numpy(), rows)


def test_paged_step_clamps_page_numbers_outside_the_pool(H, oracle):
    """A page table with entries beyond the pool must not fault: rows come from clamped pages."""
    import paper_2510_18413_amd as A
    case = small_case(950, 1, 2, 2, [1000], needles=0)
    pc = synth.paginate(case, 64, seed=12)
    cfg = A.Config.make(2, 2, pc.pool_tokens, thr_k=case.thresholds)
    Kd, Vd, qd = H.dev_bf16(pc.K), H.dev_bf16(pc.V), H.dev_bf16(case.q)
    codes = torch.zeros(2, pc.pool_tokens, 32, dtype=torch.uint8, device="cuda")
    A.adamas_encode_keys(cfg, Kd, codes, 0, pc.pool_tokens)
    bad = pc.page_table.copy()
    bad[0, 3], bad[0, 7] = 10 ** 6, -5
    ws = torch.empty(A.adamas_workspace_bytes(cfg, 1, 1000, 32), dtype=torch.uint8, device="cuda")
    out = torch.zeros(1, 2, 128, device="cuda")
    idx = torch.zeros(1, 2, 32, dtype=torch.int32, device="cuda")
    A.adamas_decode_step_paged(cfg, qd, Kd, Vd, codes, torch.from_numpy(bad).cuda(), 64,
                               torch.from_numpy(case.seq_len).cuda(), 32, out, 1000, ws, idx_out=idx)
    torch.cuda.synchronize()
    got = idx.cpu().numpy()
    assert np.all((got >= 0) & (got < 1000)) and np.all(np.isfinite(out.cpu().numpy()))


def test_decode_step_random_shapes(H, oracle):
    """Seeded sweep over batch, group size, lengths, budgets, thresholds, scale and append:
    every case against the oracle."""
    import paper_2510_18413_amd as A
    rng = np.random.default_rng(20251018)
    for case_no in range(24):
        Hkv = int(rng.choice([1, 2, 3]))
        G = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8]))
        B = int(rng.integers(1, 4))
        lens = [int(x) for x in rng.choice([0, 1, 2, 63, 64, 65, 255, 1000, 4095, 4096, 4097, 9001,
                                            12345], size=B)]
        k = int(rng.choice([1, 2, 31, 64, 100, 256, 1000, 4096]))
        append = bool(rng.integers(0, 2))
        case = small_case(7000 + case_no, B, Hkv * G, Hkv, lens, append=append)
        if case_no % 3 == 0:       # coarse keys: few distinct code rows, ties everywhere
            for h in range(Hkv):
                rows = case.K[h, :8].copy()
                pick = rng.integers(0, 8, size=case.K.shape[1])
                case.K[h] = rows[pick]
        thr = [(-1.0, 0.0, 1.0), (-0.3, 0.4, 2.5), (-2.0, -1.0, -0.5)][case_no % 3]
        case.thresholds = thr
        scale = [0.0, 0.05, 0.2][case_no % 3]
        d = H.DeviceCase(case, k)
        d.cfg = A.Config.make(case.Hq, case.Hkv, case.pool_tokens, thr_k=thr, sm_scale=scale)
        A.adamas_encode_keys(d.cfg, d.K, d.codes, 0, case.pool_tokens)
        out, idx = d.decode_step()
        K, V = case.K.copy(), case.V.copy()
        _, rows = oracle.encode(K, thr)
        ref_out, ref_idx, _ = oracle.decode_step(case.q, K, V, rows, case.seq_start, case.seq_len, k,
                                                 thr, thr, scale if scale > 0 else H.SM_SCALE,
                                                 k_new=case.k_new, v_new=case.v_new)
        tag = "case %d: B=%d Hkv=%d G=%d lens=%s k=%d append=%s" % (case_no, B, Hkv, G, lens, k, append)
        assert np.array_equal(idx, ref_idx), tag
        assert H.attn_rel_err(out, ref_out) <= H.ATTN_TOL, tag
        if append:
            assert np.array_equal(d.codes.cpu().numpy(), rows), tag
            assert np.array_equal(H.host_u16(d.K), K), tag


# ------------------------------------------------------------- head dimensions 64 and 256

@pytest.mark.parametrize("hd", [64, 256])
def test_head_dim_encode_bit_exact(H, oracle, hd):
    """Bulk key and query encode at d = 64 / 256: rows of d/4 bytes, bit for bit, including a
    row range that leaves the rest of the plane untouched."""
    import paper_2510_18413_amd as A
    case = small_case(900 + hd, 2, 8, 4, [777, 1300], head_dim=hd)
    d = H.DeviceCase(case, 16)
    assert d.cfg.code_row_bytes == hd // 4
    torch.cuda.synchronize()
    with oracle.head_dim(hd):
        _, rows = oracle.encode(case.K, case.thresholds)
        _, qrows = oracle.encode(case.q, case.thresholds)
    assert rows.shape[-1] == hd // 4
    assert np.array_equal(d.codes.cpu().numpy(), rows)
    qcodes = torch.zeros(case.B, case.Hq, hd // 4, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    part = torch.full_like(d.codes, 0xEE)
    A.adamas_encode_keys(d.cfg, d.K, part, 41, 333)
    torch.cuda.synchronize()
    assert np.array_equal(qcodes.cpu().numpy(), qrows)
    got = part.cpu().numpy()
    assert np.array_equal(got[:, 41:374], rows[:, 41:374])
    assert np.all(got[:, :41] == 0xEE) and np.all(got[:, 374:] == 0xEE)


@pytest.mark.parametrize("hd", [64, 256])
def test_head_dim_values_on_thresholds(H, oracle, hd):
    """Vectors whose transform lands exactly on a threshold (strict comparison of Eq. 5) and
    all-zero vectors, at d = 64 / 256."""
    import paper_2510_18413_amd as A
    root = int(np.sqrt(hd))                       # 8 or 16: x = c * e_0 gives y_j = c / sqrt(d)
    vals = np.array([-1.0, 0.0, 1.0, 2.0, -2.0, 0.5], dtype=np.float32) * root
    K = np.zeros((1, len(vals) * 2, hd), dtype=np.float32)
    K[0, :len(vals), 0] = vals                    # every coefficient equals vals / sqrt(d)
    K[0, len(vals):, 3] = vals                    # signs follow column 3 of the Hadamard matrix
    Kb = synth.f32_to_bf16_bits(K)
    cfg = A.Config.make(1, 1, Kb.shape[1], head_dim=hd)
    codes = torch.zeros(1, Kb.shape[1], hd // 4, dtype=torch.uint8, device="cuda")
    A.adamas_encode_keys(cfg, H.dev_bf16(Kb), codes, 0, Kb.shape[1])
    torch.cuda.synchronize()
    with oracle.head_dim(hd):
        vals_ref, rows = oracle.encode(Kb, synth.DEFAULT_THRESHOLDS)
    assert np.array_equal(codes.cpu().numpy(), rows)
    assert set(np.unique(vals_ref[0, :3])) == {0, 1, 2}     # -1 -> 0, 0 -> 1, 1 -> 2 (strict >)


@pytest.mark.parametrize("hd,B,Hq,Hkv,lens,k", [
    (64, 1, 1, 1, [1024], 64),
    (64, 2, 8, 2, [4097, 333], 256),       # group 4
    (64, 1, 8, 1, [9000], 100),            # group 8
    (64, 3, 6, 2, [1, 64, 65], 8),         # group 3, tiny sequences
    (256, 1, 1, 1, [1024], 64),
    (256, 2, 8, 2, [4097, 333], 256),      # group 4 (the largest built at d = 256)
    (256, 1, 6, 2, [9000], 100),           # group 3
    (256, 1, 2, 2, [70000], 1024),
])
def test_head_dim_distance_and_topk_bit_exact(H, oracle, hd, B, Hq, Hkv, lens, k):
    import paper_2510_18413_amd as A
    case = small_case(920 + hd + Hq + B, B, Hq, Hkv, lens, head_dim=hd)
    d = H.DeviceCase(case, k)
    qcodes = torch.zeros(B, Hq, hd // 4, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    dist = torch.full((B, Hq, d.max_len), 0xFFFF, dtype=torch.uint16, device="cuda")
    A.adamas_manhattan_distance(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, dist)
    dist2 = torch.full((B, Hq, d.max_len), 0xFFFF, dtype=torch.uint16, device="cuda")
    A.adamas_select_topk(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, k, d.idx, d.max_len,
                         d.workspace, dist_out=dist2)
    torch.cuda.synchronize()
    ref = H.oracle_step(case, k)
    got, got2 = H.host_dist(dist), H.host_dist(dist2)
    for b in range(B):
        L = int(case.seq_len[b])
        assert np.array_equal(got[b, :, :L], ref["dist"][b, :, :L])
        assert np.array_equal(got2[b, :, :L], ref["dist"][b, :, :L])
        assert np.all(got[b, :, L:] == 0xFFFF)
    assert np.array_equal(d.idx.cpu().numpy(), ref["idx"])


@pytest.mark.parametrize("hd", [64, 256])
def test_head_dim_extreme_distances(H, oracle, hd):
    """All codes 3 against all codes 0: the largest distance 3d must survive the 16-bit
    distance, the histogram bins and the threshold search."""
    import paper_2510_18413_amd as A
    case = small_case(940 + hd, 1, 1, 1, [3000], head_dim=hd)
    big = synth.f32_to_bf16_bits(np.full(hd, 64.0, np.float32))
    # x = 64 * (1, ..., 1) transforms to (64 sqrt(d), 0, ..., 0): not all codes 3.  Use a vector
    # whose transform is constant instead: 64 * sqrt(d) * e_0 -> every coefficient 64.
    e0 = np.zeros(hd, np.float32)
    e0[0] = 64.0 * np.sqrt(hd)
    case.q[0, 0] = synth.f32_to_bf16_bits(e0)               # codes all 3
    case.K[0, 1000:1200] = synth.f32_to_bf16_bits(-e0)      # codes all 0: distance 3d
    case.K[0, 2000:2100] = synth.f32_to_bf16_bits(e0)       # distance 0
    del big
    k = 2950                                                # reaches into the 3d bin
    d = H.DeviceCase(case, k)
    qcodes = torch.zeros(1, 1, hd // 4, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    dist = torch.zeros((1, 1, d.max_len), dtype=torch.uint16, device="cuda")
    A.adamas_select_topk(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, k, d.idx, d.max_len,
                         d.workspace, dist_out=dist)
    torch.cuda.synchronize()
    ref = H.oracle_step(case, k)
    got = H.host_dist(dist)
    assert got[0, 0, 1000:1200].min() == 3 * hd and got[0, 0, 2000:2100].max() == 0
    assert np.array_equal(got[0, :, :3000], ref["dist"][0, :, :3000])
    assert np.array_equal(d.idx.cpu().numpy(), ref["idx"])


@pytest.mark.parametrize("hd,B,Hq,Hkv,lens,k,append", [
    (64, 1, 1, 1, [1024], 64, False),
    (64, 2, 8, 2, [4097, 333], 256, True),
    (64, 4, 8, 1, [0, 1, 4096, 8193], 64, True),      # group 8, an empty sequence
    (64, 3, 6, 2, [100, 64, 65], 128, False),          # k above every length
    (64, 1, 2, 2, [70000], 1024, True),
    (256, 1, 1, 1, [1024], 64, False),
    (256, 2, 8, 2, [4097, 333], 256, True),
    (256, 4, 4, 1, [0, 1, 4096, 8193], 64, True),
    (256, 3, 6, 2, [100, 64, 65], 128, False),
    (256, 1, 2, 2, [40000], 4096, True),
])
def test_head_dim_decode_step_matches_oracle(H, oracle, hd, B, Hq, Hkv, lens, k, append):
    case = small_case(960 + hd + B + Hq, B, Hq, Hkv, lens, append=append, head_dim=hd)
    d = H.DeviceCase(case, k)
    out, idx = d.decode_step()
    ref = H.oracle_step(case, k, want_dist=False)
    assert out.shape[-1] == hd
    assert np.array_equal(idx, ref["idx"])
    assert H.attn_rel_err(out, ref["out"]) <= H.ATTN_TOL
    for b in range(B):
        if case.seq_len[b] == 0:
            assert np.all(out[b] == 0) and np.all(idx[b] == -1)
    if append:
        assert np.array_equal(H.host_u16(d.K), ref["K"])
        assert np.array_equal(H.host_u16(d.V), ref["V"])
        assert np.array_equal(d.codes.cpu().numpy(), ref["rows"])


@pytest.mark.parametrize("hd", [64, 256])
def test_head_dim_staged_entry_points_and_full_attention(H, oracle, hd):
    """select_topk -> sparse_attn (the stand-alone kernels) reproduce the fused step, and the
    dense comparison kernel matches the oracle's full attention, at d = 64 / 256."""
    import paper_2510_18413_amd as A
    B, Hq, Hkv, lens, k = 2, 4, 2, [5000, 700], 96
    case = small_case(980 + hd, B, Hq, Hkv, lens, head_dim=hd)
    d = H.DeviceCase(case, k)
    out, idx = d.decode_step()
    qcodes = torch.zeros(B, Hq, hd // 4, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    idx2 = torch.full_like(d.idx, -9)
    A.adamas_select_topk(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, k, idx2, d.max_len,
                         d.workspace)
    out2 = torch.full_like(d.out, float("nan"))
    A.adamas_sparse_attn(d.cfg, d.q, d.K, d.V, d.seq_start, idx2, out2, d.max_len, d.workspace)
    torch.cuda.synchronize()
    ref = H.oracle_step(case, k, want_dist=False)
    assert np.array_equal(idx2.cpu().numpy(), ref["idx"]) and np.array_equal(idx, ref["idx"])
    assert H.attn_rel_err(out2.cpu().numpy(), ref["out"]) <= H.ATTN_TOL
    ws = torch.full((A.adamas_full_attn_workspace_bytes(d.cfg, B, d.max_len),), 0xA5,
                    dtype=torch.uint8, device="cuda")
    A.adamas_full_attn(d.cfg, d.q, d.K, d.V, d.seq_start, d.seq_len, d.out, d.max_len, ws)
    torch.cuda.synchronize()
    got = d.out.cpu().numpy()
    full = np.zeros_like(got, dtype=np.float64)
    with oracle.head_dim(hd):
        for b in range(B):
            s, L = int(case.seq_start[b]), int(case.seq_len[b])
            for h in range(Hq):
                full[b, h] = oracle.full_attention(case.q[b, h], case.K[h // 2, s:s + L],
                                                   case.V[h // 2, s:s + L], 1.0 / np.sqrt(hd))
    assert H.attn_rel_err(got, full) <= H.ATTN_TOL


@pytest.mark.parametrize("hd,B,Hq,Hkv,lens,k,page,append", [
    (64, 2, 8, 2, [4097, 333], 128, 256, True),        # the new token opens a page
    (64, 3, 8, 1, [0, 5000, 9000], 256, 64, True),     # group 8, an empty sequence
    (256, 2, 8, 2, [4097, 333], 128, 256, True),
    (256, 1, 3, 1, [20000], 1024, 1024, False),        # group 3
])
def test_head_dim_paged_decode_step_matches_oracle(H, oracle, hd, B, Hq, Hkv, lens, k, page, append):
    """The paged step at d = 64 / 256 against the oracle's paged step."""
    import paper_2510_18413_amd as A
    case = small_case(990 + hd + Hq, B, Hq, Hkv, lens, append=append, head_dim=hd)
    pc = synth.paginate(case, page, seed=13)
    cfg = A.Config.make(Hq, Hkv, pc.pool_tokens, thr_k=case.thresholds, head_dim=hd)
    Kd, Vd, qd = H.dev_bf16(pc.K), H.dev_bf16(pc.V), H.dev_bf16(case.q)
    knd = None if case.k_new is None else H.dev_bf16(case.k_new)
    vnd = None if case.v_new is None else H.dev_bf16(case.v_new)
    codes = torch.zeros(Hkv, pc.pool_tokens, hd // 4, dtype=torch.uint8, device="cuda")
    A.adamas_encode_keys(cfg, Kd, codes, 0, pc.pool_tokens)
    table = torch.from_numpy(pc.page_table).cuda()
    seq_len = torch.from_numpy(case.seq_len).cuda()
    max_len = max(case.max_seq_len, 1)
    ws = torch.full((A.adamas_workspace_bytes(cfg, B, max_len, k),), 0xA5, dtype=torch.uint8,
                    device="cuda")
    out = torch.full((B, Hq, hd), float("nan"), device="cuda")
    idx = torch.full((B, Hq, k), -7, dtype=torch.int32, device="cuda")
    A.adamas_decode_step_paged(cfg, qd, Kd, Vd, codes, table, page, seq_len, k, out, max_len, ws,
                               k_new=knd, v_new=vnd, idx_out=idx)
    torch.cuda.synchronize()
    Kr, Vr = pc.K.copy(), pc.V.copy()
    with oracle.head_dim(hd):
        _, rows = oracle.encode(Kr, case.thresholds)
        ref_out, ref_idx = oracle.decode_step_paged(
            case.q, Kr, Vr, rows, pc.page_table, page, case.seq_len, k, case.thresholds,
            case.thresholds, 1.0 / np.sqrt(hd), k_new=case.k_new, v_new=case.v_new)
    assert np.array_equal(idx.cpu().numpy(), ref_idx)
    assert H.attn_rel_err(out.cpu().numpy(), ref_out) <= H.ATTN_TOL
    assert np.array_equal(H.host_u16(Kd), Kr) and np.array_equal(H.host_u16(Vd), Vr)
    assert np.array_equal(codes.cpu().numpy(), rows)


@pytest.mark.parametrize("hd", [64, 256])
def test_head_dim_without_hadamard(H, oracle, hd):
    """The no-transform ablation is a run-time switch of the same kernels: also at d = 64 / 256."""
    import paper_2510_18413_amd as A
    case = small_case(995 + hd, 2, 4, 2, [3000, 4100], append=True, head_dim=hd)
    d = H.DeviceCase(case, 96, variant=A.VARIANT_NO_HADAMARD)
    out, idx = d.decode_step()
    ref = H.oracle_step(case, 96, want_dist=False, variant=A.VARIANT_NO_HADAMARD)
    assert np.array_equal(idx, ref["idx"])
    assert H.attn_rel_err(out, ref["out"]) <= H.ATTN_TOL
    assert np.array_equal(d.codes.cpu().numpy(), ref["rows"])


def test_head_dims_that_are_not_built_are_refused(H, oracle):
    import paper_2510_18413_amd as A
    for hd in (32, 100, 512):
        assert A.adamas_workspace_bytes(A.Config.make(1, 1, 1024, head_dim=hd), 1, 1024, 16) == 0, hd
    assert A.adamas_workspace_bytes(A.Config.make(8, 1, 1024, head_dim=64), 1, 1024, 16) > 0
    assert A.adamas_workspace_bytes(A.Config.make(8, 1, 1024, head_dim=256), 1, 1024, 16) > 0


def test_generation_loop_of_appending_steps(H, oracle):
    """Six consecutive decode steps on a growing cache (one sequence crosses a scan-tile
    boundary on the way), device lengths bumped in place, one workspace, no host round trip
    between the library calls of a step: every step's selection and output against the oracle,
    which keeps its own copy of the cache, and the final caches bit for bit."""
    B, Hq, Hkv, k, steps = 2, 8, 4, 48, 6
    start_len = [700, 2046]
    case = small_case(1200, B, Hq, Hkv, [n + steps for n in start_len])   # pools sized for the end
    rng = np.random.default_rng(1201)
    d = H.DeviceCase(case, k)          # encodes the whole pool: rows beyond the lengths are ignored
    K_ref, V_ref = case.K.copy(), case.V.copy()
    with oracle.head_dim(128):
        _, rows_ref = oracle.encode(K_ref, case.thresholds)
    lens = np.array(start_len, dtype=np.int32)
    d.seq_len.copy_(torch.from_numpy(lens))
    import paper_2510_18413_amd as A
    for step in range(steps):
        lens = lens + 1
        d.seq_len.add_(1)
        q = synth.f32_to_bf16_bits(rng.standard_normal((B, Hq, 128), dtype=np.float32))
        kn = synth.f32_to_bf16_bits(rng.standard_normal((B, Hkv, 128), dtype=np.float32) * 1.5)
        vn = synth.f32_to_bf16_bits(rng.standard_normal((B, Hkv, 128), dtype=np.float32))
        A.adamas_decode_step(d.cfg, H.dev_bf16(q), d.K, d.V, d.codes, d.seq_start, d.seq_len, k,
                             d.out, d.max_len, d.workspace, k_new=H.dev_bf16(kn),
                             v_new=H.dev_bf16(vn), idx_out=d.idx)
        torch.cuda.synchronize()
        out, idx, _ = oracle.decode_step(q, K_ref, V_ref, rows_ref, case.seq_start, lens, k,
                                         case.thresholds, case.thresholds, H.SM_SCALE,
                                         k_new=kn, v_new=vn)
        assert np.array_equal(d.idx.cpu().numpy(), idx), step
        assert H.attn_rel_err(d.out.cpu().numpy(), out) <= H.ATTN_TOL, step
    assert np.array_equal(H.host_u16(d.K), K_ref) and np.array_equal(H.host_u16(d.V), V_ref)
    assert np.array_equal(d.codes.cpu().numpy(), rows_ref)


@pytest.mark.parametrize("hd", [128, 64, 256])
@pytest.mark.parametrize("far_share,k", [(0.02, 200), (0.5, 64), (0.9, 1500), (0.9, 4000), (1.0, 100)])
def test_distances_above_255_in_some_tiles(H, oracle, hd, far_share, k):
    """Byte-sized distances carry a ninth bit only in tiles that need one.  Rows far from the
    query (every code 3 against every code 0: distance 3 * d) are sprinkled over some tiles or
    fill most of the cache, so that the threshold distance lies below 256 in one case and above
    it (with ties broken by position among the far rows) in the others; two sequences, the
    second without any far row; several scan tiles and select segments."""
    rng = np.random.default_rng(1234 + hd + k)
    L0, L1 = 9000, 2500
    case = synth.make_case("far", 4242 + hd, 2, 4, 2, [L0, L1], [0],
                           lambda b, L, h, rng: rng.choice(L, (2, 1), replace=False), head_dim=hd)
    big = int(synth.f32_to_bf16_bits(np.float32([64.0]))[0])
    neg = int(synth.f32_to_bf16_bits(np.float32([-64.0]))[0])
    case.q[0] = 0
    case.q[0, :, 0] = neg                      # sequence 0: every query coefficient -64 -> code 0
    far = rng.random(L0) < far_share
    if far_share < 0.1:                        # only in a few tiles
        far &= (np.arange(L0) // 1024) % 3 == 1
    rows = np.flatnonzero(far)
    case.K[:, rows] = 0
    case.K[:, rows, 0] = big                   # every coefficient +64 -> code 3
    d = H.DeviceCase(case, k)
    out, idx = d.decode_step()
    ref = H.oracle_step(case, k, want_dist=True)
    if hd >= 128:
        assert int(ref["dist"][0].max()) == 3 * hd and int(ref["dist"][1].max()) < 3 * hd
    assert np.array_equal(idx, ref["idx"])
    assert H.attn_rel_err(out, ref["out"]) <= H.ATTN_TOL
    # the stand-alone entry point on the same cache, with the user-visible distances
    import paper_2510_18413_amd as A
    qcodes = torch.zeros(2, 4, d.cfg.code_row_bytes, dtype=torch.uint8, device="cuda")
    A.adamas_encode_query(d.cfg, d.q, qcodes)
    dist = torch.full((2, 4, d.max_len), 0xFFFF, dtype=torch.uint16, device="cuda")
    idx2 = torch.full((2, 4, k), -7, dtype=torch.int32, device="cuda")
    A.adamas_select_topk(d.cfg, qcodes, d.codes, d.seq_start, d.seq_len, k, idx2, d.max_len,
                         d.workspace, dist_out=dist)
    torch.cuda.synchronize()
    got = H.host_dist(dist)
    for b, L in enumerate((L0, L1)):
        assert np.array_equal(got[b, :, :L], ref["dist"][b, :, :L])
    assert np.array_equal(idx2.cpu().numpy(), ref["idx"])


@pytest.mark.parametrize("k", [1, 64, 300])
def test_ragged_batch_of_every_length_up_to_257(H, oracle, k):
    """257 sequences of lengths 1, 2, ..., 257 in one call (one token of each appended in the
    same step), a query group of three: indices bit for bit, attention within tolerance, the
    appended K / V / code rows in place."""
    lens = list(range(1, 258))
    case = synth.make_case("ragged257", 7100 + k, 257, 6, 2, lens, [0],
                           lambda b, L, h, rng: rng.choice(L, (3, min(1, L // 3)), replace=False),
                           append=True)
    d = H.DeviceCase(case, k)
    out, idx = d.decode_step()
    ref = H.oracle_step(case, k, want_dist=False)
    assert np.array_equal(idx, ref["idx"])
    assert H.attn_rel_err(out, ref["out"]) <= H.ATTN_TOL
    assert np.array_equal(d.codes.cpu().numpy(), ref["rows"])
    assert np.array_equal(H.host_u16(d.K), ref["K"]) and np.array_equal(H.host_u16(d.V), ref["V"])


def test_merge_inside_the_select_kernel_equals_the_merge_kernel_on_a_ragged_batch(H, oracle):
    """Sixteen segments per head for the longest sequence, fewer for the others (down to one and
    to an empty sequence), four query heads per sequence: the one-call step (segments merged by the
    last workgroup to arrive, device-scope atomics) and the staged call (separate merge kernel)
    must agree bit for bit, call after call on one workspace, and match the oracle."""
    import paper_2510_18413_amd as A
    lens = [65536, 40000, 4097, 4096, 300, 0, 20481, 61441]
    case = synth.make_case("ragged_merge", 7200, len(lens), 4, 2, lens, [0],
                           lambda b, L, h, rng: rng.choice(L, (2, min(1, L // 2)), replace=False))
    k = 192
    d = H.DeviceCase(case, k)
    for stages in (A.STAGE_SCAN, A.STAGE_SELECT_ATTN):
        A.adamas_decode_step_stages(d.cfg, d.q, d.K, d.V, d.codes, d.seq_start, d.seq_len, k, d.out,
                                    d.max_len, d.workspace, idx_out=d.idx, stages=stages)
    torch.cuda.synchronize()
    staged_out, staged_idx = d.out.clone(), d.idx.clone()
    ref = H.oracle_step(case, k, want_dist=False)
    assert np.array_equal(staged_idx.cpu().numpy(), ref["idx"])
    assert H.attn_rel_err(staged_out.cpu().numpy(), ref["out"]) <= H.ATTN_TOL
    outs = []
    for it in range(12):
        o = torch.full_like(d.out, float("nan"))
        A.adamas_decode_step(d.cfg, d.q, d.K, d.V, d.codes, d.seq_start, d.seq_len, k, o, d.max_len,
                             d.workspace, idx_out=d.idx)
        outs.append(o)
    torch.cuda.synchronize()
    for it, o in enumerate(outs):
        assert torch.equal(o, staged_out), f"call {it}"
    assert torch.equal(d.idx, staged_idx)
