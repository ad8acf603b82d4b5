"""The entry point that allocates nothing (lychee_decode_attn_static: scratch in the library's own
device array) against lychee_decode_attn on a caller-owned workspace, through the C ABI: two calls
in a row, the second on a smaller input, so that whatever the first call left in the shared array
is there when the second one runs."""
import numpy as np
import pytest
import torch

from paper_2602_04541_amd import workloads as wl
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def _both_ways(ctx, w, l_cap, seed_layer):
    lb = H.binding()
    inp = wl.make_layer(w, layer=seed_layer, l_cap=l_cap)
    idx_in = H.previous_layer_sets(inp, w.k)
    dl = H.DeviceLayer(inp, w.k, idx_in)
    out_ws, idx_ws = H.run_hybrid(ctx, dl, inp.mask)                    # the existing entry point
    out_st = torch.full_like(dl.out, float("nan"))
    idx_st = torch.full_like(dl.idx_out, -7)
    assert lb.workspace_bytes(dl.shape) <= lb.STATIC_SCRATCH_BYTES
    ctx.decode_attn_static(dl.shape, dl.q, dl.k_cache, dl.v_cache, inp.mask, dl.idx_in, out_st, idx_st, dl.lengths)
    torch.cuda.synchronize()
    out_st, idx_st = H.bf16_tensor_to_f64(out_st), idx_st.cpu().numpy()
    # same kernels, same launch shapes: index sets bit for bit, outputs to the bar of the parity tests
    assert (idx_st == idx_ws).all(), "index sets differ between the two entry points"
    H.assert_outputs_close(out_st, out_ws, "static scratch vs workspace")
    # and against the oracle, like every other layer call
    out_ref, idx_ref, sel_ref = H.oracle_layer(inp, inp.mask, w.k, idx_in)
    H.assert_outputs_close(out_st, out_ref, "static scratch vs oracle")
    H.assert_sets_match(idx_st, idx_ref, sel_ref, inp.mask, inp, w.k, idx_in, "static scratch vs oracle")


def test_static_scratch_entry_point_two_calls_the_second_smaller():
    lb = H.binding()
    ctx = lb.Context(0)
    try:
        print("static scratch: call 1, B2 8q/2kv L=9000 (lengths 9000, 5100) k=700", flush=True)
        big = wl.scaled(wl.WORKLOADS["c1"], batch=2, max_len=9000, k=700, planted=16)
        inp_lens = np.asarray([9000, 5100], np.int32)
        inp = wl.make_layer(big, lens=inp_lens, l_cap=9000)
        idx_in = H.previous_layer_sets(inp, big.k)
        dl = H.DeviceLayer(inp, big.k, idx_in)
        out_ws, idx_ws = H.run_hybrid(ctx, dl, inp.mask)
        out_st = torch.full_like(dl.out, float("nan"))
        idx_st = torch.full_like(dl.idx_out, -7)
        ctx.decode_attn_static(dl.shape, dl.q, dl.k_cache, dl.v_cache, inp.mask, dl.idx_in, out_st, idx_st,
                               dl.lengths)
        torch.cuda.synchronize()
        assert (idx_st.cpu().numpy() == idx_ws).all()
        H.assert_outputs_close(H.bf16_tensor_to_f64(out_st), out_ws, "static scratch vs workspace, call 1")
        out_ref, idx_ref, sel_ref = H.oracle_layer(inp, inp.mask, big.k, idx_in)
        H.assert_outputs_close(H.bf16_tensor_to_f64(out_st), out_ref, "static scratch vs oracle, call 1")
        H.assert_sets_match(idx_st.cpu().numpy(), idx_ref, sel_ref, inp.mask, inp, big.k, idx_in, "call 1")

        print("static scratch: call 2, B1 8q/2kv L=1300 k=64", flush=True)
        small = wl.scaled(wl.WORKLOADS["c1"], max_len=1300, k=64, planted=8)
        _both_ways(ctx, small, 1300, 1)
    finally:
        ctx.close()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    lb = H.binding()
    ctx = lb.Context(0)
    try:
        # batch 8 of the 128K layer shape needs far more scratch than the static array holds
        shape = lb.make_shape(8, 32, 8, 131072, 4096)
        assert lb.workspace_bytes(shape) > lb.STATIC_SCRATCH_BYTES
        t = torch.zeros(64, dtype=torch.int32, device="cuda")
        with pytest.raises(lb.LycheeError) as e:
            ctx.decode_attn_static(shape, t, t, t, np.ones(32, np.uint8), None, t, t, t)
        assert e.value.code == lb.EWORKSPACE
        ctx.timing_enable(True)
        small = lb.make_shape(1, 8, 2, 1024, 64)
        with pytest.raises(lb.LycheeError) as e:
            ctx.decode_attn_static(small, t, t, t, np.ones(8, np.uint8), None, t, t, t)
        assert e.value.code == lb.EUNSUPPORTED
        ctx.timing_enable(False)
    finally:
        ctx.close()
