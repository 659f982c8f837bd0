"""GPU parity of the KV offload / reload path (through the C ABI): byte work, so bit-exact."""
import numpy as np
import pytest
import torch

from oracle import kv_offload_oracle as KO
from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import synth_inputs as S
from test_gpu_stage import SMALL_GPT, SMALL_LLAMA, make_stage

pytestmark = pytest.mark.gpu


def bits(t):
    """Pool tensor -> numpy array of its raw 16-bit (or 32-bit) patterns."""
    return t.view(torch.int16 if t.element_size() == 2 else torch.int32).cpu().numpy()


def setup(cfg, mma, ctx, spare=1.0):
    st, _, _ = make_stage(cfg, mma=mma, io="f32" if cfg["dtype"] == "bf16" else None)
    table, n_pages = S.page_tables(ctx, np.ones_like(ctx), cfg["page_size"], seed=4, spare=spare)
    kv = Bd.KV(st, n_pages, table, ctx)
    kv.k_pool.copy_(S.normal_torch(4, "K", kv.k_pool.shape, 1.0, "cuda", kv.k_pool.dtype))
    kv.v_pool.copy_(S.normal_torch(4, "V", kv.v_pool.shape, 1.0, "cuda", kv.v_pool.dtype))
    return st, kv, table, n_pages


@pytest.mark.parametrize("which,mma", [("llama", "f16"), ("gpt", "bf16"), ("tiny", None)])
def test_offloaded_bytes_are_the_packed_pages_of_the_request(which, mma):
    cfg = {"llama": SMALL_LLAMA, "gpt": SMALL_GPT, "tiny": S.CONFIGS["tiny_gpt_f32"]}[which]
    ctx = np.array([37, 5, 130, 64])
    st, kv, table, _ = setup(cfg, mma, ctx)
    for b in (2, 1):
        n = int(ctx[b])
        nbytes = Bd.lsk_kv_packed_bytes(st, n)
        ref = KO.pack(bits(kv.k_pool), bits(kv.v_pool), table[b], n)
        assert nbytes == ref.nbytes
        staging = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        hbuf = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
        Bd.lsk_kv_offload(st, kv, b, n, staging, hbuf)
        torch.cuda.synchronize()
        assert np.array_equal(hbuf.numpy().view(ref.dtype).reshape(ref.shape), ref)
    assert Bd.lsk_kv_packed_bytes(st, 0) == 0
    st.close()


def test_decode_after_offload_and_reload_into_other_pages_is_bit_identical():
    cfg = SMALL_LLAMA
    ctx = np.array([37, 5, 130, 64, 16])
    st, kv, table, n_pages = setup(cfg, "f16", ctx)
    B, d, P = len(ctx), cfg["d_model"], cfg["page_size"]
    X = S.normal_torch(4, "X", (B, d), 1.0, "cuda", st.io_torch)
    ws = st.new_workspace(B)
    k_before, v_before = kv.k_pool.clone(), kv.v_pool.clone()
    Y0 = torch.empty_like(X)
    st.stage_decode(X, B, kv, Y0, ws)
    torch.cuda.synchronize()
    kv.k_pool.copy_(k_before); kv.v_pool.copy_(v_before)       # undo the rows the decode step wrote
    b = 2
    n = int(ctx[b])
    nbytes = Bd.lsk_kv_packed_bytes(st, n)
    staging = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    hbuf = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    Bd.lsk_kv_offload(st, kv, b, n, staging, hbuf)
    # the request's pages are handed to someone else ...
    old = table[b][table[b] >= 0].copy()
    kv.k_pool[:, torch.as_tensor(old, device="cuda")] = 777.0
    kv.v_pool[:, torch.as_tensor(old, device="cuda")] = -777.0
    # ... and it comes back into pages nobody uses (the spare half of the pool)
    free = sorted(set(range(n_pages)) - set(int(p) for p in table[table >= 0]))
    assert len(free) >= len(old)
    new_table = table.copy()
    new_table[b, :len(old)] = free[:len(old)][::-1]
    kv.block_table.copy_(torch.as_tensor(new_table, dtype=torch.int32))
    staging.zero_()
    Bd.lsk_kv_reload(st, kv, b, n, hbuf, staging)
    Y1 = torch.empty_like(X)
    st.stage_decode(X, B, kv, Y1, ws)
    torch.cuda.synchronize()
    assert torch.equal(Y0, Y1)
    # the pool after the round trip, by the oracle's index map
    kr, vr = bits(k_before).copy(), bits(v_before).copy()
    packed = KO.pack(kr, vr, table[b], n)
    KO.unpack(packed, kr, vr, new_table[b])
    got_k = bits(kv.k_pool)
    npg = KO.n_pages_of(n, P)
    sel = new_table[b, :npg]
    # whole reloaded pages except the slot the second decode step wrote (position n)
    for j, pg in enumerate(sel):
        for slot in range(P):
            if j * P + slot == n:
                continue
            assert np.array_equal(got_k[:, pg, :, slot], kr[:, pg, :, slot])
    st.close()


def test_offload_argument_checks_and_memory_test():
    cfg = SMALL_LLAMA
    st, kv, table, _ = setup(cfg, "f16", np.array([20, 3]))
    staging = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    hbuf = torch.empty(1 << 20, dtype=torch.uint8, pin_memory=True)
    with pytest.raises(Bd.LsError):
        Bd.lsk_kv_offload(st, kv, 0, 10 ** 6, staging, hbuf)        # more pages than a table row holds
    with pytest.raises(Bd.LsError):
        Bd.lsk_kv_offload(st, kv, -1, 4, staging, hbuf)
    ok, used = Bd.lsk_memory_available(0, 1 << 62)
    assert ok and used > 0
    ok2, _ = Bd.lsk_memory_available(1 << 40, used)     # a terabyte more than what is in use now
    assert not ok2
    st.close()
