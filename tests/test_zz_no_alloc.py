"""The entry point that allocates nothing (lsk_attn_paged_noalloc) against the entry point it is a variant of
(lsk_attn_paged, impl 1, caller-provided scratch): two calls in a row on one GPU, the second with a smaller
input, each bit-identical to the existing entry point's result and within the bar of the float64 oracle."""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import synth_inputs as S
from parity_util import assert_close, host, out_rounding_bound

pytestmark = pytest.mark.gpu


def decode_case(seed, ctx, h, dh, P, dt):
    ctx = np.asarray(ctx, np.int64)
    T, d = len(ctx), h * dh
    table, n_pages = S.page_tables(ctx, np.ones_like(ctx), P, seed=seed)
    kp = S.normal_torch(seed, "K", (n_pages, h, P, dh), 1.0, "cuda", dt)
    vp = S.normal_torch(seed, "V", (n_pages, h, P, dh), 1.0, "cuda", dt)
    qkv = S.normal_torch(seed, "qkv", (T, 3 * d), 1.0, "cuda", dt)
    pos = torch.as_tensor(ctx, dtype=torch.int32, device="cuda")
    req = torch.arange(T, dtype=torch.int32, device="cuda")
    bt = torch.as_tensor(table, dtype=torch.int32, device="cuda")
    Bd.lsk_kv_write(qkv, h, dh, pos, req, kp, vp, bt, P)
    return dict(ctx=ctx, T=T, h=h, dh=dh, P=P, table=table, kp=kp, vp=vp, qkv=qkv, pos=pos, req=req, bt=bt,
                max_ctx=int(ctx.max()) + 1)


def oracle_rows(c):
    d, h, dh, P = c["h"] * c["dh"], c["h"], c["dh"], c["P"]
    kp, vp, q = host(c["kp"]), host(c["vp"]), host(c["qkv"])
    ref = np.empty((c["T"], d))
    for b, n in enumerate(c["ctx"]):
        j = np.arange(int(n) + 1)
        K, V = kp[c["table"][b, j // P], :, j % P, :], vp[c["table"][b, j // P], :, j % P, :]
        ob, _ = O.attention(q[b:b + 1, :d].reshape(1, h, dh), K, V, int(n))
        ref[b] = ob.reshape(d)
    return ref


def test_attention_over_pages_without_any_allocation_two_calls_the_second_smaller():
    dt = torch.float16
    # few (row, head) pairs and long contexts: both launches split the context and go through the scratch
    big = decode_case(31, [2044, 1500, 900, 777, 130, 2047, 64, 1], 4, 128, 16, dt)
    small = decode_case(32, [300, 1200, 15], 2, 128, 16, dt)
    for c in (big, small):
        assert Bd.lib().lsk_attn_paged_scratch_floats(c["T"], c["h"], c["dh"], c["max_ctx"], c["P"]) > 0
    got = []
    for c in (big, small):                       # back to back on the current stream, no synchronisation between
        o = torch.full((c["T"], c["h"] * c["dh"]), 7.0, dtype=dt, device="cuda")
        Bd.lsk_attn_paged_noalloc(c["qkv"], c["h"], c["dh"], c["pos"], c["req"], c["kp"], c["vp"], c["bt"], c["P"],
                                  c["max_ctx"], o)
        got.append(o)
    torch.cuda.synchronize()
    for c, o in zip((big, small), got):
        ref_o = torch.empty_like(o)
        Bd.lsk_attn_paged(1, c["qkv"], c["h"], c["dh"], c["pos"], c["req"], c["kp"], c["vp"], c["bt"], c["P"],
                          c["max_ctx"], ref_o)
        torch.cuda.synchronize()
        assert torch.equal(o, ref_o), "differs from lsk_attn_paged with a caller-provided scratch"
        r = oracle_rows(c)
        assert_close(host(o), r, 2e-2 + out_rounding_bound(r, "f16"), "against the float64 definition")


def test_no_alloc_entry_point_rejects_what_it_cannot_hold():
    c = decode_case(33, [40, 7], 2, 128, 16, torch.float16)
    o = torch.empty(c["T"], 2 * 128, dtype=torch.float16, device="cuda")
    lib = Bd.lib()
    args = lambda dh, T: (c["qkv"].data_ptr(), Bd.LS_F16, T, 2, dh, c["pos"].data_ptr(), c["req"].data_ptr(),
                          c["kp"].data_ptr(), c["vp"].data_ptr(), c["bt"].data_ptr(), c["bt"].shape[1], 16, 64,
                          o.data_ptr(), None)
    assert lib.lsk_attn_paged_noalloc(*args(32, 2)) == Bd.LS_EINVAL          # head size outside the kernel's
    assert lib.lsk_attn_paged_noalloc(*args(128, 0)) == Bd.LS_EINVAL         # no rows
    # 128 rows x 40 heads with contexts up to 4096 tokens split into eight 512-token chunks: 21 MB of partials
    big = list(args(128, 128))
    big[3], big[12] = 40, 4096
    assert lib.lsk_attn_paged_scratch_floats(128, 40, 128, 4096, 16) > (2 << 20)
    assert lib.lsk_attn_paged_noalloc(*big) == Bd.LS_EINVAL and b"static scratch" in lib.ls_last_error()
    assert lib.lsk_attn_paged_noalloc(*args(128, 2)) == Bd.LS_OK
    torch.cuda.synchronize()
