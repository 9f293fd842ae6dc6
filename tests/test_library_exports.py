"""The C-ABI library loads and exports every symbol the header declares (no GPU needed, no compute calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "turboboa.h")
LIB = os.path.join(ROOT, "paper_2602_04929_amd", "libturboboa.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tboa_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("libturboboa.so is not built: run __graft_entry__.build()")
    return ctypes.CDLL(LIB)


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for must in ("tboa_create", "tboa_destroy", "tboa_last_error", "tboa_build_hessians", "tboa_build_hessian_out_proj", "tboa_fp_cache_bytes",
                 "tboa_quantize_layer", "tboa_act_fakequant", "tboa_hadamard_rotate", "tboa_build_hessian_linear", "tboa_swiglu_forward", "tboa_pack_codes", "tboa_dequant_gemv", "tboa_packed_words_per_row", "tboa_chol_inv_upper", "tboa_gemm_f64", "tboa_gemm_bf16_nt"):
        assert must in names


def test_every_declared_symbol_is_exported(lib):
    missing = [n for n in declared_functions() if not hasattr(lib, n)]
    assert not missing, missing


def test_binding_signatures_cover_the_header():
    import paper_2602_04929_amd as tb
    src = open(os.path.join(ROOT, "paper_2602_04929_amd", "binding.py")).read()
    assert tb.LIB_PATH == LIB
    for n in declared_functions():
        assert '"%s"' % n in src, "binding.py has no signature for " + n


def test_null_context_is_rejected_without_touching_a_device(lib):
    lib.tboa_last_error.restype = ctypes.c_char_p
    assert lib.tboa_last_error(None) == b"null context"
    assert lib.tboa_workspace_bytes(None) == 0
    lib.tboa_counter.restype = ctypes.c_int64
    assert lib.tboa_counter(None, 0) == -1
    assert lib.tboa_profile_enable(None, 1) == -1
    assert lib.tboa_create(None, 0, None) == -1


def test_descriptor_structs_match_the_header():
    """Field order of the ctypes mirrors equals the order in the header's typedefs."""
    import paper_2602_04929_amd as tb
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    for cname, cls in (("tboa_attn_desc", tb.AttnDesc), ("tboa_layer_desc", tb.LayerDesc)):
        body = re.search(r"typedef struct \{([^}]*)\} %s;" % cname, text).group(1)
        fields = []
        for decl in body.split(";"):
            decl = decl.strip()
            if decl:
                ctype, names = decl.split(None, 1)
                fields += [(n.strip(), ctype) for n in names.split(",")]
        got = [(n, {"c_int": "int", "c_double": "double", "c_float": "float"}[t.__name__]) for n, t in cls._fields_]
        assert got == fields


def test_workspace_queries_are_host_arithmetic():
    """tboa_hessian_workspace_bytes / tboa_quantize_workspace_bytes run the library's own planning code on the host: no device
    is touched, sizes grow with the problem, an invalid descriptor gives 0."""
    import paper_2602_04929_amd as tb
    import torch
    C = tb.Context
    small = C.hessian_workspace_bytes(256, 4, 4, 64, 8, 128, torch.float32)
    big = C.hessian_workspace_bytes(4096, 32, 32, 128, 128, 2048, torch.bfloat16)
    gqa = C.hessian_workspace_bytes(8192, 64, 8, 128, 128, 2048, torch.bfloat16)
    assert 0 < small < big < gqa < 288 * 2 ** 30
    assert C.hessian_workspace_bytes(256, 4, 3, 64, 8, 128, torch.float32) == 0        # heads not divisible
    d = tb.LayerDesc(4096, 4096, 32, 0, 2, 32, 0, tb.BF16, 1, 1, 100, 0.8, 0.01, 0.0)
    per_head = tb.LayerDesc(4096, 4096, 32, 1, 2, 32, 0, tb.BF16, 1, 1, 100, 0.8, 0.01, 0.0)
    a, b = C.quantize_workspace_bytes(d), C.quantize_workspace_bytes(per_head)
    assert 0 < a < b < 288 * 2 ** 30
    assert C.quantize_workspace_bytes(tb.LayerDesc(4096, 4096, 32, 0, 5, 32, 0, tb.BF16, 1, 1, 100, 0.8, 0.01, 0.0)) == 0
    # every layer of every named configuration fits one GPU: W_O goes without H_out (its rows are independent), which is what
    # keeps the group-wise refinement of the 13B-shaped layer small (one Gram entry per row instead of a block per head)
    from paper_2602_04929_amd import synth
    for name in ("llama2-7b", "llama2-13b", "llama2-70b", "llama2-7b-w4a4"):
        cfg = synth.CONFIGS[name]
        desc = lambda d_out, d_in, nh, per, block: tb.LayerDesc(d_out, d_in, nh, per, cfg.bits, block, cfg.group, tb.BF16, 1, 1, 100, 0.8, 0.01, 0.0)
        o = C.quantize_workspace_bytes(desc(cfg.d_model, cfg.d_q, 1, 0, cfg.d_model), with_H_out=False)
        v = C.quantize_workspace_bytes(desc(cfg.d_kv, cfg.d_model, cfg.n_kv_heads, 1, cfg.block))
        qk = C.quantize_workspace_bytes(desc(cfg.d_q + cfg.d_kv, cfg.d_model, cfg.n_q_heads + cfg.n_kv_heads, 0, cfg.block))
        assert 0 < o < 64 * 2 ** 30 and 0 < v < 64 * 2 ** 30 and 0 < qk < 64 * 2 ** 30, (name, o, v, qk)
    print("workspace: 7B Hessians %.1f GiB, 70B Hessians %.1f GiB, 7B W_Q %.1f GiB, 7B W_V %.1f GiB" % (big / 2 ** 30, gqa / 2 ** 30, a / 2 ** 30, b / 2 ** 30))
