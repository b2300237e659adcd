"""The five benchmark configurations at FULL size, in the launch configuration bench.py times,
against the oracle: every head's code plane and index set bit for bit, attention within
tolerance, and the planted needles inside the top-k (the synthetic stand-in for the paper's
passkey retrieval test, Table 1)."""

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


def check_case(H, oracle, case, budgets, check_cache=False):
    _, rows = oracle.encode(case.K, case.thresholds)          # cache before the step
    first = True
    for k in budgets:
        d = H.DeviceCase(case, k)
        if first:
            torch.cuda.synchronize()
            assert np.array_equal(d.codes.cpu().numpy(), rows), "code plane"
            first = False
        out, idx = d.decode_step()
        Kc, Vc, rc = case.K.copy(), case.V.copy(), rows.copy()
        ref_out, ref_idx, _ = oracle.decode_step(case.q, Kc, Vc, rc, case.seq_start, case.seq_len, k,
                                                 case.thresholds, case.thresholds, H.SM_SCALE,
                                                 k_new=case.k_new, v_new=case.v_new)
        assert np.array_equal(idx, ref_idx), "indices, k=%d" % k
        err = H.attn_rel_err(out, ref_out)
        assert err <= H.ATTN_TOL, "attention rel err %g, k=%d" % (err, k)
        # with fp64 scores the step is far inside the bound (measured <= 3.5e-5 on these
        # configurations); a regression to fp32-score accuracy (1e-4 .. 2e-3) would show here
        assert err <= H.ATTN_TOL / 10, "attention rel err %g, k=%d" % (err, k)
        for b in range(case.B):
            for h in range(case.Hq):
                sel = set(idx[b, h].tolist())
                missing = [p for p in case.needles[b][h] if p not in sel]
                assert not missing, "needles %s of (b=%d, h=%d) not selected at k=%d" % (missing, b, h, k)
        if check_cache and case.k_new is not None:
            assert np.array_equal(H.host_u16(d.K), Kc)
            assert np.array_equal(H.host_u16(d.V), Vc)
            assert np.array_equal(d.codes.cpu().numpy(), rc)
        del d
        torch.cuda.empty_cache()


def test_config0_tiny_single_head(H, oracle):
    case = synth.tiny_single_head()
    check_case(H, oracle, case, case.budgets)


def test_config1_mha_32k(H, oracle):
    case = synth.mha_32k()
    check_case(H, oracle, case, case.budgets)


def test_config2_gqa_32k(H, oracle):
    case = synth.gqa_32k()
    check_case(H, oracle, case, case.budgets)


def test_config3_long_128k_with_append(H, oracle):
    case = synth.long_128k_append()
    check_case(H, oracle, case, case.budgets, check_cache=True)


def test_config4_batched_ragged(H, oracle):
    case = synth.batched_ragged()
    assert case.seq_len.min() >= 8192 and case.seq_len.max() <= 32768
    check_case(H, oracle, case, case.budgets)


def test_maximum_sequence_length_and_budget(H, oracle):
    """The documented limits at once: one sequence of ADAMAS_MAX_SEQ_LEN = 2^20 tokens (with an
    append as its last token), the largest budget k = 4096, a group of two query heads."""
    L = 1 << 20
    case = synth.make_case("max", 4242, 1, 2, 1, [L], [4096],
                           lambda b, Lc, h, rng: rng.choice(Lc, (2, 3), replace=False), append=True)
    check_case(H, oracle, case, [4096], check_cache=True)
