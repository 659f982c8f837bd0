"""CPU-side checks of the C ABI: the library loads, exports every declared
symbol, and validates arguments on the host (no kernel is launched)."""
import ctypes as C
import os
import re

import pytest

from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import synth_inputs as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for hdr in ("lemix_stage.h", "lemix_kernels.h", "lemix_sched.h", "lemix_serve.h", "lemix_profile.h"):
        txt = open(os.path.join(ROOT, "include", hdr)).read()
        txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
        names |= set(re.findall(r"\b((?:ls|lsk|stage)_[a-z0-9_]+)\s*\(", txt))
    return names


def test_library_exports_every_declared_symbol():
    lib = Bd.lib()
    decl = declared_symbols()
    assert len(decl) >= 25
    for name in decl:
        assert hasattr(lib, name), f"{name} is declared in include/ but not exported"
    assert decl == set(Bd.SIGNATURES), decl ^ set(Bd.SIGNATURES)


def test_config_struct_matches_header_field_order():
    txt = open(os.path.join(ROOT, "include", "lemix_stage.h")).read()
    body = re.search(r"typedef struct \{([^}]*)\} ls_config;", txt, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = [f.strip() for decl in body.split(";") for f in re.sub(r"^\s*\w+\s+", "", decl.strip()).split(",") if f.strip()]
    assert fields == [n for n, _ in Bd.ls_config._fields_]


def _create(cfg_over=None, **kw):
    cfg = dict(S.CONFIGS["tiny_gpt_f32"])
    cfg.update(cfg_over or {})
    c = Bd.make_config(cfg, **kw)
    h = C.c_void_p()
    st = Bd.lib().ls_create(C.byref(c), C.byref(h))
    return st, h


@pytest.mark.parametrize("over,frag", [
    (dict(d_model=130), "d_model"),
    (dict(head_dim=48, d_model=192), "head_dim"),
    (dict(d_ff=509), "d_ff"),
    (dict(page_size=12), "page_size"),
    (dict(act="swiglu"), "GELU"),
    (dict(n_layers=0), "non-positive"),
])
def test_create_rejects_bad_configs_on_the_host(over, frag):
    st, _ = _create(over)
    assert st == Bd.LS_EINVAL
    assert frag in Bd.lib().ls_last_error().decode()


def test_create_rejects_mixed_precision_mismatch():
    st, _ = _create(None, mma_dtype="bf16")
    assert st == Bd.LS_EINVAL
    cfg = dict(S.CONFIGS["gpt2s_bf16"])
    c = Bd.make_config(cfg, mma_dtype="f32")
    h = C.c_void_p()
    assert Bd.lib().ls_create(C.byref(c), C.byref(h)) == Bd.LS_EINVAL


def test_null_arguments_are_errors_not_crashes():
    lib = Bd.lib()
    assert lib.ls_create(None, None) == Bd.LS_EINVAL
    assert lib.ls_param_count(None) == 0
    assert lib.ls_workspace_bytes(None, 10) == 0
    assert lib.stage_decode(None, None, 1, None, None, None, None) == Bd.LS_EINVAL
    assert lib.stage_train_fwd(None, None, 1, 1, None, None, None, None) == Bd.LS_EINVAL
    assert lib.lsk_gemm(Bd.LS_BF16, 0, 8, 8, None, 8, 1, None, 8, 1, None, 8, Bd.LS_BF16, None, 0, None, 0,
                        0, None) == Bd.LS_EINVAL
    assert b"non-positive" in lib.ls_last_error()
    lib.ls_destroy(None)
    # the decode-batch entry points and the serving loop validate on the host too
    splits = C.c_int(0)
    assert lib.lsk_gemm_partials(Bd.LS_F16, 64, 128, 64, None, 64, None, 64, None, 0, C.byref(splits), None) == Bd.LS_EINVAL
    assert lib.lsk_finish_resid_norm(None, 1, 4, 64, None, None, None, 1, None, None, 0, 1e-5, None, 0, None) == Bd.LS_EINVAL
    assert lib.lsk_finish_act(None, 1, 4, 64, Bd.LS_ACT_SWIGLU, None, 0, None, 0, None) == Bd.LS_EINVAL
    assert lib.lsk_finish_qkv(None, 1, 4, 2, 64, None, 0, None, None, None, None, Bd.LS_F16, None, None, None, 4, 16,
                              None) == Bd.LS_EINVAL
    srv = C.c_void_p()
    assert lib.ls_server_create(None, None, None, None, C.byref(srv)) == Bd.LS_EINVAL
    assert lib.ls_server_submit(None, 0, None, None, 1, 1) == Bd.LS_EINVAL
    assert lib.ls_server_pass(None, 0.0, None, None, None, None, None) == Bd.LS_EINVAL
    assert lib.ls_server_in_flight(None) == 0
    lib.ls_server_destroy(None)
    assert lib.ls_get_config(None, None) == Bd.LS_EINVAL
    assert lib.ls_node_plan(None, None, 0, None, None, None, None) == Bd.LS_EINVAL
    assert lib.ls_node_queue_len(None, 0) == 0 and lib.ls_node_prune(None) == 0
    assert lib.ls_batcher_form(None, 0.0, None, None, None, None) == Bd.LS_EINVAL
    assert lib.ls_batcher_queued(None) == 0 and lib.ls_batcher_batch_size(None) == 0
    lib.ls_node_destroy(None)
    lib.ls_batcher_destroy(None)


def test_probe_validates_its_arguments_before_any_launch():
    """The interference probe's own checks (two different streams, two different workspaces, a positive
    repetition count, somewhere to write the times) need no GPU: an fp32 stage allocates nothing."""
    st, h = _create()
    assert st == Bd.LS_OK
    lib = Bd.lib()
    out = (C.c_float * 6)()
    kv = Bd.ls_kv(0x1000, 0x1000, 0x1000, 0x1000, None, 4, 2)
    P = 0x1000            # never dereferenced: every case below fails validation on the host

    def call(ws_a=P, ws_b=2 * P, sa=P, sb=2 * P, iters=1, out_ms=out, dec_B=1, trn_B=1, dec_X=P):
        return lib.stage_probe_interference(h, dec_X, dec_B, C.byref(kv), P, ws_a, P, trn_B, 8, P, P, P, P, P, ws_b,
                                            sa, sb, iters, out_ms)

    assert call() == Bd.LS_ESTATE                      # no parameters bound yet
    assert lib.ls_bind_params(h, P, None) == Bd.LS_OK
    assert call(sb=P) == Bd.LS_EINVAL and b"streams" in lib.ls_last_error()
    assert call(ws_b=P) == Bd.LS_EINVAL and b"workspaces" in lib.ls_last_error()
    assert call(ws_a=None) == Bd.LS_EINVAL
    assert call(iters=0) == Bd.LS_EINVAL and call(iters=-3) == Bd.LS_EINVAL
    assert call(out_ms=None) == Bd.LS_EINVAL
    assert call(dec_B=0) == Bd.LS_EINVAL and call(trn_B=0) == Bd.LS_EINVAL
    assert call(dec_X=None) == Bd.LS_EINVAL and b"decode" in lib.ls_last_error()
    lib.ls_destroy(h)


def test_no_instruction_touches_a_register_with_an_assembly_issued_lds_read_in_flight(tmp_path):
    """Compiles the sources that issue LDS reads or MFMAs from assembly to ISA and lints them."""
    import shutil
    import subprocess
    import isa_lint
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not available")
    csrc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2507_21276_amd", "csrc")
    # a planted hazard is found (the checker itself works)
    planted = "_Zk:\n\tds_read_b64_tr_b16 v[4:5], v9\n\tv_mov_b32_e32 v4, 0\n\ts_waitcnt lgkmcnt(0)\n\ts_endpgm\n"
    assert isa_lint.scan(planted) == {"_Zk": [(2, "v_mov_b32_e32 v4, 0")]}
    # a counted wait retires the older read only
    counted = ("_Zk:\n\tds_read_b128 v[4:7], v9\n\tds_read_b128 v[10:13], v9\n\ts_waitcnt lgkmcnt(1)\n"
               "\tv_mov_b32_e32 v0, v4\n\tv_mov_b32_e32 v1, v10\n\ts_waitcnt lgkmcnt(0)\n\ts_endpgm\n")
    assert isa_lint.scan(counted) == {"_Zk": [(5, "v_mov_b32_e32 v1, v10")]}
    # a read issued late in a loop body and used at the top of the next iteration before any wait
    looped = ("_Zk:\n.LBB0_1:\n\tv_mov_b32_e32 v0, v4\n\ts_waitcnt lgkmcnt(0)\n\tds_read_b128 v[4:7], v9\n"
              "\ts_cbranch_scc0 .LBB0_1\n\ts_waitcnt lgkmcnt(0)\n\ts_endpgm\n")
    assert isa_lint.scan(looped) == {"_Zk": [(2, "v_mov_b32_e32 v0, v4")]}
    # a scalar load in flight does not stop a counted wait from retiring the older LDS reads, and is never retired by one
    mixed = ("_Zk:\n\tds_read_b128 v[4:7], v9\n\ts_load_dwordx2 s[0:1], s[2:3], 0x0\n\tds_read_b128 v[10:13], v9\n"
             "\ts_waitcnt lgkmcnt(1)\n\tv_mov_b32_e32 v0, v4\n\tv_mov_b32_e32 v1, v10\n\ts_waitcnt lgkmcnt(0)\n\ts_endpgm\n")
    assert isa_lint.scan(mixed) == {"_Zk": [(6, "v_mov_b32_e32 v1, v10")]}
    # an MFMA result named by another kind of instruction before the MFMA's passes + 3 wait states are over
    early = ("_Zk:\n\tv_mfma_f32_32x32x16_f16 a[0:15], v[0:3], v[4:7], a[0:15]\n\tv_add_u32_e32 v9, 1, v9\n"
             "\tv_accvgpr_read_b32 v8, a3\n\ts_endpgm\n")
    assert isa_lint.scan(early) == {"_Zk": [(3, "v_accvgpr_read_b32 v8, a3")]}
    settled = ("_Zk:\n\tv_mfma_f32_32x32x16_f16 a[0:15], v[0:3], v[4:7], a[0:15]\n\tv_mfma_f32_32x32x16_f16 a[0:15], v[0:3], v[4:7], a[0:15]\n"
               "\ts_nop 10\n\tv_accvgpr_read_b32 v8, a3\n\ts_endpgm\n")
    assert isa_lint.scan(settled) == {}
    # an MFMA reading a register that a vector instruction wrote less than two wait states before
    close = "_Zk:\n\tv_cvt_pk_f16_f32 v4, v8, v9\n\ts_nop 0\n\tv_mfma_f32_32x32x16_f16 a[0:15], v[0:3], v[4:7], a[0:15]\n\ts_endpgm\n"
    assert isa_lint.scan(close) == {"_Zk": [(3, "v_mfma_f32_32x32x16_f16 a[0:15], v[0:3], v[4:7], a[0:15]")]}
    apart = "_Zk:\n\tv_cvt_pk_f16_f32 v4, v8, v9\n\ts_nop 1\n\tv_mfma_f32_32x32x16_f16 a[0:15], v[0:3], v[4:7], a[0:15]\n\ts_endpgm\n"
    assert isa_lint.scan(apart) == {}
    # both sides of a branch are walked: the read is in flight on the path that skips the wait
    forked = ("_Zk:\n\tds_read_b128 v[4:7], v9\n\ts_cbranch_scc1 .LBB0_2\n\ts_waitcnt lgkmcnt(0)\n.LBB0_2:\n"
              "\tv_mov_b32_e32 v0, v4\n\ts_waitcnt lgkmcnt(0)\n\ts_endpgm\n")
    assert isa_lint.scan(forked) == {"_Zk": [(5, "v_mov_b32_e32 v0, v4")]}
    for src in ("gemm_dma.hip", "gemm_dma16.hip", "attention_mfma.hip"):
        out = tmp_path / (src + ".s")
        subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                        "-packed-fp32-ops", "-S", "--cuda-device-only", os.path.join(csrc, src), "-o", str(out)],
                       check=True, capture_output=True)
        text = out.read_text()
        assert "ds_read_b64_tr_b16" in text
        assert isa_lint.scan(text) == {}, src
