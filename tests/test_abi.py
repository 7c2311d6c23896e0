"""The C-ABI library loads, exports every symbol declared in include/rkv.h, and its host-side
validation returns the documented status codes without touching a GPU.  CPU only."""
import ctypes
import os
import re

import pytest

from paper_2505_24133_amd import rkv


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(rkv.LIB_PATH):
        from paper_2505_24133_amd.build import build
        build()
    return rkv.load_library()


def declared_symbols(repo_root):
    text = open(os.path.join(repo_root, "include", "rkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rkv_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib, repo_root):
    names = declared_symbols(repo_root)
    assert names == ["rkv_cache_append", "rkv_compact", "rkv_compact_inplace", "rkv_compress", "rkv_compress_events", "rkv_compress_inplace", "rkv_compress_static", "rkv_probe_mfma", "rkv_score_importance", "rkv_score_redundancy",
                     "rkv_select_topk", "rkv_should_compress", "rkv_status_string", "rkv_workspace_size"]
    for n in names:
        assert hasattr(lib, n), n
    assert set(rkv.__dict__) >= set(names) - {"rkv_status_string", "rkv_compress_events"}


def test_params_struct_layout_matches_header(repo_root, tmp_path):
    """The ctypes mirror against the header itself: a C program compiled from include/rkv.h prints
    the size of rkv_params and the offset of every field."""
    import subprocess
    names = [f[0] for f in rkv.RkvParams._fields_]
    c_names = ["lambda" if n == "lam" else n for n in names]
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "rkv.h"\nint main(void) {\n'
                   '  printf("%zu\\n", sizeof(rkv_params));\n'
                   + "".join(f'  printf("%zu\\n", offsetof(rkv_params, {n}));\n' for n in c_names)
                   + "  return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(repo_root, "include"), "-o", str(exe), str(src)], check=True)
    out = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert out[0] == ctypes.sizeof(rkv.RkvParams)
    assert out[1:] == [getattr(rkv.RkvParams, n).offset for n in names]
    assert rkv.RkvParams.k_stride_problem.offset == 56 and rkv.RkvParams.page_size.offset == 56 + 12 * 8


def shape(**kw):
    base = dict(num_problems=2, kv_heads=8, q_heads=32, n_tokens=1152, budget=1024)
    base.update(kw)
    return rkv.Shape(**base)


def ws_status(lib, s):
    n = ctypes.c_size_t(0)
    p = s.params()
    return lib.rkv_workspace_size(ctypes.byref(p), ctypes.byref(n)), n.value


def test_workspace_size_and_validation(lib):
    st, nbytes = ws_status(lib, shape())
    assert st == rkv.RKV_OK and nbytes > 0 and nbytes % 256 == 0
    st2, nbytes2 = ws_status(lib, shape(num_problems=4))
    assert st2 == rkv.RKV_OK and nbytes2 > nbytes
    assert ws_status(lib, shape(num_problems=0)) == (rkv.RKV_OK, 0)
    assert ws_status(lib, shape(num_problems=-1))[0] == rkv.RKV_ERR_SHAPE
    assert ws_status(lib, shape(pool_w=1025, alpha=8))[0] == rkv.RKV_ERR_UNSUPPORTED
    assert ws_status(lib, shape(q_heads=30))[0] == rkv.RKV_ERR_SHAPE
    assert ws_status(lib, shape(budget=8))[0] == rkv.RKV_ERR_SHAPE
    assert ws_status(lib, shape(n_tokens=8))[0] == rkv.RKV_ERR_SHAPE
    assert ws_status(lib, shape(head_dim=64))[0] == rkv.RKV_ERR_UNSUPPORTED
    assert ws_status(lib, shape(flags=128))[0] == rkv.RKV_ERR_UNSUPPORTED          # unknown flag bit
    # the triangular schedule of the similarity pass: beta = 1 only, not with the other direction of the rule or the shortcut
    assert ws_status(lib, shape(flags=64))[0] == rkv.RKV_OK
    assert ws_status(lib, shape(flags=64, num_problems=64))[1] > ws_status(lib, shape(num_problems=64))[1]     # 16 more bytes per candidate
    assert ws_status(lib, shape(flags=64, beta=2))[0] == rkv.RKV_ERR_PARAM
    assert ws_status(lib, shape(flags=64 | 32))[0] == rkv.RKV_ERR_PARAM
    assert ws_status(lib, shape(flags=64 | 1))[0] == rkv.RKV_ERR_PARAM
    assert ws_status(lib, shape(flags=15))[0] == rkv.RKV_OK
    assert ws_status(lib, shape(flags=8 | 16))[0] == rkv.RKV_ERR_PARAM             # two ways of merging the group at once
    # merging after the softmax keeps G * alpha logit rows per head: a larger workspace
    assert ws_status(lib, shape(flags=8))[1] > ws_status(lib, shape())[1]
    assert ws_status(lib, shape(flags=32, beta=2))[1] > ws_status(lib, shape(beta=2))[1]     # 8 more bytes per candidate
    # pooling stage holds alpha rows, one more when the mean is taken before the pooling
    assert ws_status(lib, shape(alpha=63, q_heads=8, pool_w=130))[0] == rkv.RKV_OK            # 63 * 260 <= 16384
    assert ws_status(lib, shape(alpha=63, q_heads=8, pool_w=130, flags=2))[0] == rkv.RKV_ERR_UNSUPPORTED
    assert ws_status(lib, shape(q_heads=8 * 9))[0] == rkv.RKV_ERR_UNSUPPORTED     # G * alpha = 72 > 64
    assert ws_status(lib, shape(n_tokens=40000, budget=30000))[0] == rkv.RKV_ERR_UNSUPPORTED
    assert ws_status(lib, shape(lam=1.5))[0] == rkv.RKV_ERR_PARAM
    assert ws_status(lib, shape(lam=float("nan")))[0] == rkv.RKV_ERR_PARAM
    assert ws_status(lib, shape(sim_threshold=-0.1))[0] == rkv.RKV_ERR_PARAM
    assert ws_status(lib, shape(beta=-1))[0] == rkv.RKV_ERR_PARAM
    assert ws_status(lib, shape(pool_w=-1))[0] == rkv.RKV_ERR_PARAM
    assert ws_status(lib, shape(eps=-1.0))[0] == rkv.RKV_ERR_PARAM
    assert ws_status(lib, shape(eps=0.0))[0] == rkv.RKV_ERR_PARAM                  # Eq. 5's eps is what keeps a zero key finite
    assert ws_status(lib, shape(eps=float("inf")))[0] == rkv.RKV_ERR_PARAM
    # observation queries: dense by default, or strided rows (16-byte aligned)
    def qs(sp, sh, st):
        p = shape().params()
        p.q_stride_problem, p.q_stride_head, p.q_stride_token = sp, sh, st
        n = ctypes.c_size_t(0)
        return lib.rkv_workspace_size(ctypes.byref(p), ctypes.byref(n))
    assert qs(8 * 32 * 128, 128, 32 * 128) == rkv.RKV_OK                           # [P, alpha, q_heads, d]
    assert qs(8 * 32 * 128, 128, 100) == rkv.RKV_ERR_SHAPE
    assert qs(8 * 32 * 128, 0, 32 * 128) == rkv.RKV_ERR_SHAPE
    assert qs(0, 128, 32 * 128) == rkv.RKV_ERR_SHAPE
    assert qs(8 * 32 * 128, 132, 32 * 128) == rkv.RKV_ERR_SHAPE
    assert lib.rkv_workspace_size(None, ctypes.byref(ctypes.c_size_t(0))) == rkv.RKV_ERR_NULL


def test_paged_cache_validation(lib):
    """Paged layouts are checked on the host: page size, table, strides; the workspace grows by the
    dense copy of the candidate keys."""
    def paged(**kw):
        p = shape().params()
        p.page_size, p.table_stride, p.block_table = 16, 72, 0x1000       # 72 * 16 = 1152 tokens
        p.k_stride_page = p.v_stride_page = 8 * 16 * 128
        p.k_stride_head = p.v_stride_head = 16 * 128
        p.k_stride_token = p.v_stride_token = 128
        for k_, v_ in kw.items():
            setattr(p, k_, v_)
        n = ctypes.c_size_t(0)
        return lib.rkv_workspace_size(ctypes.byref(p), ctypes.byref(n)), n.value
    ok, nbytes = paged()
    assert ok == rkv.RKV_OK and nbytes >= ws_status(lib, shape())[1] + 2 * 8 * 1144 * 256   # + bf16 [heads][n][128]
    assert paged(page_size=24)[0] == rkv.RKV_ERR_UNSUPPORTED
    assert paged(page_size=256)[0] == rkv.RKV_ERR_UNSUPPORTED
    assert paged(block_table=None)[0] == rkv.RKV_ERR_NULL
    assert paged(table_stride=71)[0] == rkv.RKV_ERR_SHAPE                  # 71 pages hold 1136 < 1152 tokens
    assert paged(k_stride_page=0)[0] == rkv.RKV_ERR_SHAPE
    assert paged(v_stride_token=64)[0] == rkv.RKV_ERR_SHAPE
    assert paged(k_stride_head=0)[0] == rkv.RKV_ERR_SHAPE                  # several heads need a head stride
    assert paged(k_stride_token=132)[0] == rkv.RKV_ERR_SHAPE               # rows must stay 16-byte aligned
    for ps in (16, 32, 64, 128):
        assert paged(page_size=ps, table_stride=(1152 + ps - 1) // ps)[0] == rkv.RKV_OK


def test_null_and_workspace_errors_return_before_any_launch(lib):
    p = shape().params()
    assert lib.rkv_compress(ctypes.byref(p), None, None, None, None, None, None, None, None, 0, None) == rkv.RKV_ERR_NULL
    fake = ctypes.c_void_p(0x1000)        # never dereferenced: validation fails first
    assert lib.rkv_compress(ctypes.byref(p), fake, fake, fake, fake, fake, None, None, None, 0, None) == rkv.RKV_ERR_WORKSPACE
    assert lib.rkv_compress(ctypes.byref(p), fake, fake, fake, fake, fake, None, None, ctypes.c_void_p(0x1001), 1 << 40, None) == rkv.RKV_ERR_WORKSPACE
    assert lib.rkv_compress(ctypes.byref(p), fake, fake, fake, fake, fake, None, None, fake, 16, None) == rkv.RKV_ERR_WORKSPACE
    # cache does not exceed the budget: nothing to do (Alg. 1 early return)
    p2 = shape(n_tokens=1024, budget=1024).params()
    assert lib.rkv_compress(ctypes.byref(p2), fake, fake, fake, fake, fake, None, None, fake, 1 << 40, None) == rkv.RKV_NOT_TRIGGERED
    assert lib.rkv_compress_inplace(ctypes.byref(p), fake, None, fake, None, None, fake, 1 << 40, None) == rkv.RKV_ERR_NULL
    assert lib.rkv_compress_inplace(ctypes.byref(p), fake, fake, fake, None, None, None, 0, None) == rkv.RKV_ERR_WORKSPACE
    assert lib.rkv_compress_inplace(ctypes.byref(p2), fake, fake, fake, None, None, fake, 1 << 40, None) == rkv.RKV_NOT_TRIGGERED
    assert lib.rkv_compact_inplace(ctypes.byref(p), fake, fake, None, None) == rkv.RKV_ERR_NULL
    bad = shape().params()
    bad.k_stride_token = 100
    bad.k_stride_head = 8
    bad.k_stride_problem = 8
    assert lib.rkv_compress(ctypes.byref(bad), fake, fake, fake, fake, fake, None, None, fake, 1 << 40, None) == rkv.RKV_ERR_SHAPE


def test_static_scratch_entry_point_validates_on_the_host(lib):
    """rkv_compress_static refuses what does not fit its fixed scratch, and what rkv_compress refuses,
    before it looks anything up on a device."""
    fake = ctypes.c_void_p(0x1000)
    big = shape(num_problems=32, n_tokens=4224, budget=4096)
    assert ws_status(lib, big)[1] > rkv.RKV_STATIC_SCRATCH_BYTES
    p = big.params()
    assert lib.rkv_compress_static(ctypes.byref(p), fake, fake, fake, fake, fake, None, None, None) == rkv.RKV_ERR_WORKSPACE
    fits = shape(num_problems=32)
    assert 0 < ws_status(lib, fits)[1] <= rkv.RKV_STATIC_SCRATCH_BYTES          # one sequence of the 8B model, budget 1024
    p = fits.params()
    assert lib.rkv_compress_static(ctypes.byref(p), None, fake, fake, fake, fake, None, None, None) in (rkv.RKV_ERR_NULL, rkv.RKV_ERR_HIP)
    p = shape(n_tokens=1024, budget=1024).params()
    assert lib.rkv_compress_static(ctypes.byref(p), fake, fake, fake, fake, fake, None, None, None) == rkv.RKV_NOT_TRIGGERED
    p = shape(eps=0.0).params()
    assert lib.rkv_compress_static(ctypes.byref(p), fake, fake, fake, fake, fake, None, None, None) == rkv.RKV_ERR_PARAM
    assert lib.rkv_compress_static(None, fake, fake, fake, fake, fake, None, None, None) == rkv.RKV_ERR_NULL
    p = shape(num_problems=0).params()
    assert lib.rkv_compress_static(ctypes.byref(p), None, None, None, None, None, None, None, None) == rkv.RKV_OK
    header = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "rkv.h")).read()
    assert "#define RKV_STATIC_SCRATCH_BYTES (32u << 20)" in header and rkv.RKV_STATIC_SCRATCH_BYTES == 32 << 20


def test_mfma_probe_validates_on_the_host(lib, repo_root):
    fake = ctypes.c_void_p(0x1000)
    assert lib.rkv_probe_mfma(None, fake, 1, None, None) == rkv.RKV_ERR_NULL
    assert lib.rkv_probe_mfma(fake, None, 1, None, None) == rkv.RKV_ERR_NULL
    assert lib.rkv_probe_mfma(fake, fake, 0, None, None) == rkv.RKV_ERR_PARAM
    assert lib.rkv_probe_mfma(fake, fake, (1 << 20) + 1, None, None) == rkv.RKV_ERR_PARAM
    assert lib.rkv_probe_mfma(ctypes.c_void_p(0x1008), fake, 1, None, None) == rkv.RKV_ERR_SHAPE
    assert lib.rkv_probe_mfma(fake, ctypes.c_void_p(0x1002), 1, None, None) == rkv.RKV_ERR_SHAPE
    header = open(os.path.join(repo_root, "include", "rkv.h")).read()
    assert "#define RKV_PROBE_OPERAND_BYTES (64u << 10)" in header and rkv.RKV_PROBE_OPERAND_BYTES == 64 << 10
    assert "#define RKV_PROBE_SINK_BYTES (1u << 20)" in header and rkv.RKV_PROBE_SINK_BYTES == 1 << 20


def test_status_strings(lib):
    seen = {rkv.status_string(s) for s in range(-6, 2)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert rkv.status_string(99) == "unknown status"


def test_binding_refuses_cpu_tensors():
    import torch
    s = shape(num_problems=1, kv_heads=1, q_heads=4, n_tokens=256, budget=128)
    k = torch.zeros((1, 1, 256, 128), dtype=torch.bfloat16)
    q = torch.zeros((1, 4, 8, 128), dtype=torch.bfloat16)
    with pytest.raises(RuntimeError, match="no CPU path"):
        rkv.rkv_compress(s, q, k, k)


def test_trigger_rule(lib):
    """Alg. 1: nothing happens until the rows held beyond the budget fill the buffer."""
    p = shape(n_tokens=1152, budget=1024).params()
    for held, want in [(0, rkv.RKV_NOT_TRIGGERED), (1024, rkv.RKV_NOT_TRIGGERED), (1151, rkv.RKV_NOT_TRIGGERED),
                       (1152, rkv.RKV_OK)]:
        assert lib.rkv_should_compress(ctypes.byref(p), held) == want
    p2 = shape(n_tokens=1024, budget=1024).params()
    assert lib.rkv_should_compress(ctypes.byref(p2), 1024) == rkv.RKV_NOT_TRIGGERED
    fake = ctypes.c_void_p(0x1000)
    assert lib.rkv_cache_append(ctypes.byref(p), fake, fake, fake, fake, fake, fake, 1152, 0, None) == rkv.RKV_ERR_SHAPE
    assert lib.rkv_cache_append(ctypes.byref(p), fake, fake, fake, fake, fake, fake, 0, 8, None) == rkv.RKV_ERR_SHAPE
    assert lib.rkv_cache_append(ctypes.byref(p), None, fake, fake, fake, fake, fake, 0, 0, None) == rkv.RKV_ERR_NULL
