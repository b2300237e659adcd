"""CPU-side checks of the C ABI: the library loads, exports what the header declares, and
rejects bad arguments before touching the GPU (none of these calls launches anything)."""

import ctypes
import os
import re

import pytest

import paper_2510_18413_amd as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)      # non-null, 256-byte aligned; never dereferenced on these paths
ODD = ctypes.c_void_p(0x1008)


def header_functions():
    text = open(os.path.join(ROOT, "include", "adamas.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adamas_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = A.library()
    declared = header_functions()
    assert len(declared) >= 9
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(A.EXPORTED_SYMBOLS) == declared


def test_status_strings():
    assert A.adamas_status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert A.adamas_status_string(code)


def cfg(**kw):
    base = dict(num_q_heads=32, num_kv_heads=8, pool_tokens=32768)
    base.update(kw)
    return A.Config.make(**base)


def test_workspace_bytes():
    c = cfg()
    w = A.adamas_workspace_bytes(c, 1, 32768, 128)
    assert w > 32 * 32768 and w % 256 == 0
    assert A.adamas_workspace_bytes(c, 2, 32768, 128) > w
    assert A.adamas_workspace_bytes(c, 1, 65536, 128) > w
    assert A.adamas_workspace_bytes(c, 0, 32768, 128) == 0
    assert A.adamas_workspace_bytes(c, 1, 0, 128) == 0
    assert A.adamas_workspace_bytes(c, 1, 32768, 0) == 0
    assert A.adamas_workspace_bytes(c, 1, 32768, 4097) == 0
    assert A.adamas_workspace_bytes(c, 1, (1 << 20) + 1, 128) == 0
    assert A.adamas_workspace_bytes(cfg(head_dim=80), 1, 32768, 128) == 0
    assert A.adamas_workspace_bytes(cfg(head_dim=96), 1, 32768, 128) > 0
    # head dimensions 64 and 256: distances are 2 bytes either way, partials scale with d
    w64 = A.adamas_workspace_bytes(cfg(head_dim=64), 1, 32768, 128)
    w256 = A.adamas_workspace_bytes(cfg(head_dim=256, num_q_heads=32, num_kv_heads=8), 1, 32768, 128)
    assert 0 < w64 < w < w256


@pytest.mark.parametrize("bad, status", [
    (dict(head_dim=80), -2),
    (dict(head_dim=512), -2),
    (dict(head_dim=100), -2),
    (dict(num_q_heads=32, num_kv_heads=3), -1),
    (dict(num_q_heads=0), -1),
    (dict(pool_tokens=0), -1),
    (dict(thr_k=(0.0, 0.0, 1.0)), -1),
    (dict(thr_q=(1.0, 0.0, -1.0)), -1),
    (dict(thr_k=(float("nan"), 0.0, 1.0)), -1),
    (dict(sm_scale=-1.0), -1),
    (dict(sm_scale=float("inf")), -1),
    (dict(num_q_heads=32, num_kv_heads=2), -2),        # group of 16 > ADAMAS_MAX_GROUP
    (dict(variant=4), -2),                             # unknown variant bit
    (dict(code_bits=3, thr_k=(0.0,) * 7), -1),          # seven thresholds must increase
    (dict(code_bits=1, thr_k=(0.0,), variant=2), -2),   # L2 needs 2-bit codes
])
def test_bad_config_rejected_everywhere(bad, status):
    lib, c = A.library(), cfg(**bad)
    p = ctypes.byref(c)
    assert lib.adamas_encode_keys(p, FAKE, FAKE, 0, 16, None) == status
    assert lib.adamas_encode_query(p, FAKE, FAKE, 1, None) == status
    assert lib.adamas_manhattan_distance(p, FAKE, FAKE, FAKE, FAKE, 1, FAKE, 1024, None) == status
    assert lib.adamas_select_topk(p, FAKE, FAKE, FAKE, FAKE, 1, 64, FAKE, None, 1024, FAKE,
                                  1 << 30, None) == status
    assert lib.adamas_sparse_attn(p, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 64, FAKE, 1024, FAKE,
                                  1 << 30, None) == status
    assert lib.adamas_decode_step(p, FAKE, None, None, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 64, FAKE,
                                  None, 1024, FAKE, 1 << 30, None) == status


def test_null_and_misaligned_pointers_rejected():
    lib, c = A.library(), cfg()
    p = ctypes.byref(c)
    assert lib.adamas_encode_keys(None, FAKE, FAKE, 0, 16, None) == -1
    assert lib.adamas_encode_keys(p, None, FAKE, 0, 16, None) == -1
    assert lib.adamas_encode_keys(p, FAKE, None, 0, 16, None) == -1
    assert lib.adamas_encode_keys(p, ODD, FAKE, 0, 16, None) == -1
    assert lib.adamas_encode_keys(p, FAKE, FAKE, -1, 16, None) == -1
    assert lib.adamas_encode_keys(p, FAKE, FAKE, 32760, 16, None) == -1      # past the pool
    assert lib.adamas_encode_keys(p, FAKE, FAKE, 0, 0, None) == 0            # empty: no-op
    assert lib.adamas_encode_query(p, FAKE, FAKE, 0, None) == -1
    assert lib.adamas_manhattan_distance(p, FAKE, FAKE, None, FAKE, 1, FAKE, 1024, None) == -1
    assert lib.adamas_manhattan_distance(p, FAKE, FAKE, FAKE, FAKE, 1, None, 1024, None) == -1
    args = [p, FAKE, FAKE, FAKE, FAKE, 1, 64, FAKE, None, 1024, FAKE, 1 << 30, None]
    for pos in (1, 2, 3, 4, 7, 10):
        a = list(args)
        a[pos] = None
        assert lib.adamas_select_topk(*a) == -1
    a = list(args)
    a[10] = ODD
    assert lib.adamas_select_topk(*a) == -1                                   # workspace alignment
    pargs = [p, FAKE, None, None, FAKE, FAKE, FAKE, FAKE, 16, 256, FAKE, 1, 64, FAKE, None, 1024,
             FAKE, 1 << 30, None, 3]
    assert lib.adamas_decode_step_paged(*(pargs[:-1] + [2])) == -1           # select stage alone
    for pos in (1, 4, 5, 6, 7, 10, 13, 16):
        a = list(pargs)
        a[pos] = None
        assert lib.adamas_decode_step_paged(*a) == -1
    for bad_page in (48, 32, 8192):
        a = list(pargs)
        a[9] = bad_page
        assert lib.adamas_decode_step_paged(*a) == -2                         # page size
    a = list(pargs)
    a[8] = 2
    assert lib.adamas_decode_step_paged(*a) == -1                             # table too short for max_seq_len
    fargs = [p, FAKE, FAKE, FAKE, FAKE, FAKE, 1, FAKE, 1024, FAKE, 1 << 30, None]
    for pos in (1, 2, 3, 4, 5, 7, 9):
        a = list(fargs)
        a[pos] = None
        assert lib.adamas_full_attn(*a) == -1
    a = list(fargs)
    a[10] = 16
    assert lib.adamas_full_attn(*a) == -3                                     # workspace too small
    assert A.adamas_full_attn_workspace_bytes(c, 1, 32768) > 0
    assert A.adamas_full_attn_workspace_bytes(c, 0, 32768) == 0
    assert lib.adamas_stream_read(None, 64, FAKE, None) == -1
    assert lib.adamas_stream_read(FAKE, 64, None, None) == -1
    assert lib.adamas_stream_read(ODD, 64, FAKE, None) == -1
    assert lib.adamas_stream_read(FAKE, 48, FAKE, None) == -1                 # not whole rows
    assert lib.adamas_stream_read(FAKE, 0, FAKE, None) == 0                   # empty: no-op
    dargs = [p, FAKE, None, None, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 64, FAKE, None, 1024, FAKE,
             1 << 30, None]
    for pos in (1, 4, 5, 6, 7, 8, 11, 14):
        a = list(dargs)
        a[pos] = None
        assert lib.adamas_decode_step(*a) == -1
    a = list(dargs)
    a[2] = FAKE                                                               # k_new without v_new
    assert lib.adamas_decode_step(*a) == -1


def test_size_limits_and_workspace_check():
    lib, c = A.library(), cfg()
    p = ctypes.byref(c)
    need = A.adamas_workspace_bytes(c, 1, 1024, 64)
    base = [p, FAKE, FAKE, FAKE, FAKE, 1, 64, FAKE, None, 1024, FAKE, need - 1, None]
    assert lib.adamas_select_topk(*base) == -3
    for k, st in ((0, -1), (-5, -1), (4097, -2)):
        a = list(base)
        a[6] = k
        assert lib.adamas_select_topk(*a) == st
    a = list(base)
    a[9] = (1 << 20) + 1
    assert lib.adamas_select_topk(*a) == -2
    a = list(base)
    a[5] = 0
    assert lib.adamas_select_topk(*a) == -1
    d = [p, FAKE, None, None, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 64, FAKE, None, 1024, FAKE, need - 1,
         None]
    assert lib.adamas_decode_step(*d) == -3
    s = [p, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 64, FAKE, 1024, FAKE, need - 1, None]
    assert lib.adamas_sparse_attn(*s) == -3


def test_binding_rejects_cpu_tensors():
    import torch
    c = cfg(num_q_heads=1, num_kv_heads=1, pool_tokens=8)
    K = torch.zeros(1, 8, 128, dtype=torch.bfloat16)
    codes = torch.zeros(1, 8, 32, dtype=torch.uint8)
    with pytest.raises(ValueError):
        A.adamas_encode_keys(c, K, codes, 0, 8, stream=0)


def test_product_code_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2510_18413_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)
    assert "oracle" not in open(os.path.join(ROOT, "include", "adamas.h")).read().lower()


def test_merge_uses_device_scope_accesses(tmp_path):
    """The attention merge inside the select kernel exchanges partials between workgroups that may
    run on different XCDs without a cache write-back or invalidate: it relies on every access to
    a partial being a device-scope access (the `sc1` bit on gfx950), which goes to the memory
    side instead of the XCD's own L2, and on the arrival counter being a hardware atomic.  A compiler that lowered the
    relaxed agent-scope atomics of the source differently would break the merge silently, so the
    kernel's assembly (of our own source, compiled here) must show the three kinds of access."""
    import subprocess
    from paper_2510_18413_amd import build as B
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    out = tmp_path / "select.s"
    flags = [f for f in B.HIPCC_FLAGS if f != "-fPIC"]
    subprocess.run([hipcc] + flags + ["-w", "-DADAMAS_INST_D=128", "-DADAMAS_INST_METRIC=0",
                                      "-I", os.path.join(ROOT, "include"), "-I", str(B.CSRC),
                                      "-S", "--cuda-device-only", "-o", str(out),
                                      str(B.CSRC / "kernels_inst.hip")], check=True)
    text = out.read_text()
    # the decode step's select kernels (a pass at a time / eight passes per barrier): 256 threads,
    # with attention, Eq. 6, contiguous cache, d = 128
    starts = list(re.finditer(r"^_ZN6adamas13select_kernelILi256ELb1ELi0ELb0ELi128ELi\d+EEE\w*:", text, re.M))
    assert len(starts) == 2, "select kernels not found in the assembly"
    body = ""
    for start in starts:
        one = text[start.end():text.index(".Lfunc_end", start.end())]
        sc1 = [l.split() for l in one.splitlines() if re.search(r"\bsc1\b", l)]
        kinds = {w[0] for w in sc1}
        assert any(k.startswith("global_store_dword") for k in kinds), kinds      # partials out
        assert any(k.startswith("global_load_dword") for k in kinds), kinds       # partials read back
        # the arrival counter: a returning atomic add (device-wide atomicity is the hardware's; the
        # compiler marks only system scope with sc1 on read-modify-write instructions)
        assert re.search(r"^\s*global_atomic_add\w* v\d+, .*\bsc0\b", one, re.M)
        body += one
    # and no whole-cache write-back / invalidate crept in (the fence that cost 23 us per step)
    assert "buffer_wbl2" not in body and "buffer_inv" not in body
