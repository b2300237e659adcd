"""adamas_decode_step_static (the entry point that allocates nothing: its scratch is a static
device array inside the library) against adamas_decode_step on a caller-owned workspace.

Both run the same kernels, so indices must be bit-equal and the attention output equal to the
bit; the oracle is consulted as well, to the usual tolerance.  Two calls in a row share the
one static array, the second on a smaller input, so stale contents of the first call's scratch
would show.  Runs last in the suite and must also pass alone in a fresh process.
"""

import ctypes

import numpy as np
import pytest
import torch

import paper_2510_18413_amd as A
import synth_inputs as synth

FAKE = ctypes.c_void_p(0x1000)


def test_oversize_request_is_refused_without_a_gpu():
    """Sizes whose scratch would not fit the static array are rejected on the host."""
    lib = A.library()
    c = A.Config.make(32, 8, 16 * 32768)
    assert A.adamas_workspace_bytes(c, 16, 32768, 128) > A.STATIC_SCRATCH_BYTES
    args = [ctypes.byref(c), FAKE, None, None, FAKE, FAKE, FAKE, FAKE, FAKE, 16, 128, FAKE, None,
            32768, None]
    assert lib.adamas_decode_step_static(*args) == -3
    a = list(args)
    a[9] = 0
    assert lib.adamas_decode_step_static(*a) == -1          # batch
    a = list(args)
    a[0] = ctypes.byref(A.Config.make(32, 3, 1024))
    assert lib.adamas_decode_step_static(*a) == -1          # heads not divisible
    small = [ctypes.byref(A.Config.make(4, 2, 4096)), FAKE, None, None, FAKE, FAKE, FAKE, FAKE, FAKE,
             1, 16, FAKE, None, 4096, None]
    for pos in (1, 4, 5, 6, 7, 8, 11):
        a = list(small)
        a[pos] = None
        assert lib.adamas_decode_step_static(*a) == -1      # null pointers, before any HIP call


def _case(seed, B, Hq, Hkv, lens, append):
    G = Hq // Hkv
    return synth.make_case("static_%d" % seed, seed, B, Hq, Hkv, lens, [0],
                           lambda b, Lc, h, rng: rng.choice(Lc, size=(G, 1), replace=False),
                           append=append)


@pytest.mark.gpu
def test_static_scratch_step_equals_workspace_step_twice_in_a_row(oracle):
    from gpu_harness import DeviceCase, attn_rel_err, oracle_step, ATTN_TOL
    # first a large input (9 scan tiles per head, 3 select segments), then a smaller one
    for seed, B, Hq, Hkv, lens, k, append in [(501, 2, 8, 2, [9000, 4097], 96, True),
                                              (502, 1, 4, 4, [700], 33, False)]:
        print("static-scratch step: seed", seed, "lens", lens, "k", k, flush=True)
        case = _case(seed, B, Hq, Hkv, lens, append)
        ref = DeviceCase(case, k)
        want_out, want_idx = ref.decode_step()
        dev = DeviceCase(case, k)           # its own pools: an append writes them
        assert A.adamas_workspace_bytes(dev.cfg, B, dev.max_len, k) <= A.STATIC_SCRATCH_BYTES
        A.adamas_decode_step_static(dev.cfg, dev.q, dev.K, dev.V, dev.codes, dev.seq_start,
                                    dev.seq_len, k, dev.out, dev.max_len, k_new=dev.k_new,
                                    v_new=dev.v_new, idx_out=dev.idx)
        torch.cuda.synchronize()
        got_out, got_idx = dev.out.cpu().numpy(), dev.idx.cpu().numpy()
        assert np.array_equal(got_idx, want_idx)
        assert np.array_equal(got_out.view(np.uint32), want_out.view(np.uint32))
        for name in ("K", "V", "codes"):    # the appended rows went to the same places
            assert torch.equal(getattr(dev, name), getattr(ref, name)), name
        o = oracle_step(case, k, want_dist=False)
        assert np.array_equal(got_idx, o["idx"])
        assert attn_rel_err(got_out, o["out"]) <= ATTN_TOL
