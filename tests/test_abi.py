"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and its
host-side argument checks behave as the header says.  No compute call is made."""
import ctypes
import dataclasses
import os
import re

import pytest

import paper_2603_03592_amd as sv
import stage_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "stageverify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sv_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"sv_create", "sv_destroy", "sv_verify_forward", "sv_verify_backward", "sv_score_and_flag",
            "sv_ema_update", "sv_check_desc", "sv_workspace_bytes", "sv_last_error", "sv_gemm_bf16"} <= set(names)
    lib = ctypes.CDLL(sv.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None, n


def test_result_struct_is_32_bytes():
    assert sv.RESULT_DTYPE.itemsize == 32
    assert sv.RESULT_DTYPE.fields["flag"][1] == 16 and sv.RESULT_DTYPE.fields["argmax_token"][1] == 28


@pytest.mark.parametrize("wl", [si.TINY, si.SMALL, si.MEDIUM, si.LARGE, si.sweep_point(4096, 16), si.MOE_TOP1, si.MOE_TOP6],
                         ids=lambda w: w.name)
def test_benchmark_stages_are_supported(wl):
    st, msg = sv.sv_check_desc(wl.desc, 1 if wl.backward else 0)
    assert st == 0, msg
    fwd = sv.sv_workspace_bytes(wl.desc, wl.batch * wl.seq, wl.seq, 0)
    bwd = sv.sv_workspace_bytes(wl.desc, wl.batch * wl.seq, wl.seq, 1)
    assert 0 < fwd < bwd < 64 * 2 ** 30
    assert sv.sv_workspace_bytes(wl.desc, 2 * wl.batch * wl.seq, wl.seq, 0) > fwd


def test_malformed_and_unsupported_descriptors_are_rejected():
    d = si.SMALL.desc
    bad = [
        (dataclasses.replace(d, n_heads=24), 1, "multiple of n_heads"),        # 1024 % 24
        (dataclasses.replace(d, n_kv_heads=5), 1, "multiple of n_kv_heads"),
        (dataclasses.replace(d, n_blocks=0), 1, "positive"),
        (dataclasses.replace(d, d_model=1008, n_heads=14, n_kv_heads=14), 2, "head_dim"),     # hd = 72
        (dataclasses.replace(d, ffn_hidden=2812), 2, "multiples of 8"),
        (dataclasses.replace(d, rope_theta=0.0), 1, "rope_theta"),
    ]
    for desc, status, frag in bad:
        st, msg = sv.sv_check_desc(desc)
        assert st == status and frag in msg, (desc, st, msg)
        assert sv.sv_workspace_bytes(desc, 128, 64) == -1
    st, msg = sv.sv_check_desc(d, flags=64)
    assert st == 1 and "flag" in msg


def test_fused_norm_flag_sizes_the_gain_folded_weight_copies():
    """SV_FLAG_FUSE_NORM: the context holds a copy of wq, wk, wv and of the dense MLP's first weights per block plus the
    per-row scalars; stages the flag does not apply to (fp32, LayerNorm, plain kernels) are sized as without it, and
    the rule that says where it paid when measured covers exactly the dense bf16 RMSNorm stages of width <= 2048."""
    wl = si.LARGE
    d, T = wl.desc, wl.batch * wl.seq
    plain = sv.sv_workspace_bytes(d, T, wl.seq, 0)
    fused = sv.sv_workspace_bytes(d, T, wl.seq, 8)
    hd = d.d_model // d.n_heads
    folded = d.n_blocks * 2 * d.d_model * ((d.n_heads + 2 * d.n_kv_heads) * hd + 2 * d.ffn_hidden)      # bf16 bytes
    scalars = 4 * T * (1 + d.d_model // 128)
    assert folded + scalars <= fused - plain <= folded + scalars + 64 * 1024
    assert sv.sv_check_desc(d, flags=8)[0] == 0 and sv.sv_check_desc(d, flags=9)[0] == 0
    for other in (si.TINY.desc, dataclasses.replace(d, dtype="f32"), dataclasses.replace(d, norm="ln")):
        assert sv.sv_workspace_bytes(other, 128, 64, 8) == sv.sv_workspace_bytes(other, 128, 64, 0)
    assert sv.sv_workspace_bytes(d, T, wl.seq, 8 | 2) == sv.sv_workspace_bytes(d, T, wl.seq, 2)
    m = si.MOE_TOP6.desc                                   # a mixture keeps its second norm: only wq, wk, wv are copied
    extra = sv.sv_workspace_bytes(m, 8192, 1024, 8) - sv.sv_workspace_bytes(m, 8192, 1024, 0)
    qkv = m.n_blocks * 2 * m.d_model * 3 * m.d_model
    assert qkv <= extra <= qkv + 4 * 8192 * (1 + m.d_model // 128) + 64 * 1024
    assert [sv.fuse_norm_pays(w.desc) for w in (si.TINY, si.SMALL, si.MEDIUM, si.LARGE, si.MOE_TOP1, si.sweep_point(512, 1))] == \
        [False, True, True, False, False, False]


def test_mixture_of_experts_descriptors():
    d = si.MOE_TOP6.desc
    assert sv.sv_check_desc(d)[0] == 0
    bad = [
        (dataclasses.replace(d, top_k=9), 1, "top_k"),                       # more than n_experts
        (dataclasses.replace(d, top_k=0), 1, "top_k"),
        (dataclasses.replace(d, n_experts=17, top_k=2), 2, "16 experts"),
        (dataclasses.replace(d, n_experts=16, top_k=9), 2, "top_k <= 8"),
        (dataclasses.replace(d, mlp="gelu"), 2, "SwiGLU"),
        (dataclasses.replace(d, n_experts=0), 1, "dense MLP"),               # routing fields without experts
    ]
    for desc, status, frag in bad:
        st, msg = sv.sv_check_desc(desc)
        assert st == status and frag in msg, (desc, st, msg)
    # the expert-sorted buffers are part of the workspace: more experts per token, more rows
    one = sv.sv_workspace_bytes(dataclasses.replace(d, top_k=1), 8192, 1024, 0)
    six = sv.sv_workspace_bytes(d, 8192, 1024, 0)
    assert 0 < one < six
