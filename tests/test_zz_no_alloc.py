"""qkv_card_attend_static - the attention entry point for callers that cannot allocate - against
qkv_card_attend with a caller's workspace: the same kernels over the library's fixed scratch array, so
out and lse must be bit-identical.  Two calls in a row, the second on a smaller card (the array then
still holds the first call's partials), through the C ABI with raw ctypes; then the refusal of a shape
beyond the fixed array."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_03884_amd as qkv
import qkv_synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_case(L, H, rep, T, G, budget, seed):
    D = 128
    K, V = qkv_synth.make_kv(L, H, T, D, seed, "llama", device=DEV)
    scores = qkv_synth.make_scores(T, seed + 1, DEV)
    desc = qkv.Desc.make(L, H, T, D, G)
    counts = qkv.budget_counts(T, budget)
    card = torch.empty(qkv.card_bytes(desc, counts), dtype=torch.uint8, device=DEV)
    qkv.assign_quantize_pack(desc, K, V, scores, budget, card)
    q = qkv_synth.normal(seed + 2, 9, 0, L * H * rep * D, DEV).view(L, H * rep, D).to(torch.float16)
    return desc, card, q


def with_workspace(desc, card, q, scale):
    out = torch.full((desc.layers, q.shape[1], 128), float("nan"), dtype=torch.float32, device=DEV)
    lse = torch.full((desc.layers, q.shape[1]), float("nan"), dtype=torch.float32, device=DEV)
    qkv.card_attend(card, desc, q, scale, out, lse=lse)
    torch.cuda.synchronize()
    return out, lse


def static_call(desc, card, q, scale, out, lse, status):
    """Straight through the C ABI: no binding helper, no allocation between the arguments and the library."""
    L = qkv.lib()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return L.qkv_card_attend_static(ctypes.c_void_p(card.data_ptr()), ctypes.c_uint64(card.numel()), ctypes.byref(desc),
                                    ctypes.c_void_p(q.data_ptr()), ctypes.c_int32(q.shape[1]), ctypes.c_float(scale),
                                    ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(lse.data_ptr()),
                                    ctypes.c_void_p(status.data_ptr()), st)


def test_static_scratch_matches_workspace_on_two_calls_in_a_row():
    scale = 128 ** -0.5
    big = make_case(4, 8, 4, 3000, 32, 4.0, 9100)          # 4 layers x 8 kv heads, 32 query heads, mixed widths
    small = make_case(2, 2, 2, 333, 32, 6.0, 9200)         # fewer planes, fewer tasks, other widths
    wants = [with_workspace(d, c, q, scale) for d, c, q in (big, small)]
    # results first, then both static calls back to back so that nothing else touches the scratch in between
    outs = []
    for desc, card, q in (big, small):
        out = torch.full((desc.layers, q.shape[1], 128), float("nan"), dtype=torch.float32, device=DEV)
        lse = torch.full((desc.layers, q.shape[1]), float("nan"), dtype=torch.float32, device=DEV)
        status = torch.full((1,), 0x7777, dtype=torch.int32, device=DEV)
        outs.append((out, lse, status))
    for (desc, card, q), (out, lse, status) in zip((big, small), outs):
        print("[case] static attend T=%d L=%d" % (desc.tokens, desc.layers), flush=True)
        assert static_call(desc, card, q, scale, out, lse, status) == 0
    torch.cuda.synchronize()
    for (out, lse, status), (want_out, want_lse) in zip(outs, wants):
        assert int(status.item()) == 0
        assert torch.isfinite(out).all() and torch.isfinite(lse).all()
        assert torch.equal(out.view(torch.int32), want_out.view(torch.int32))
        assert torch.equal(lse.view(torch.int32), want_lse.view(torch.int32))
    # and the big one once more after the small one
    desc, card, q = big
    out, lse, status = outs[0]
    out.fill_(float("nan")); lse.fill_(float("nan"))
    assert static_call(desc, card, q, scale, out, lse, status) == 0
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), wants[0][0].view(torch.int32))
    assert torch.equal(lse.view(torch.int32), wants[0][1].view(torch.int32))


def test_static_scratch_refuses_what_does_not_fit_and_bad_arguments():
    L = qkv.lib()
    desc = qkv.Desc.make(32, 8, 32768, 128, 32)
    need = qkv.card_attend_workspace(desc, 32)
    assert need > (16 << 20)
    dummy = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    f32 = torch.zeros(32 * 32 * 128, dtype=torch.float32, device=DEV)
    args = (ctypes.c_void_p(dummy.data_ptr()), ctypes.c_uint64(dummy.numel()), ctypes.byref(desc), ctypes.c_void_p(dummy.data_ptr()),
            ctypes.c_int32(32), ctypes.c_float(0.1), ctypes.c_void_p(f32.data_ptr()), None, None, None)
    assert L.qkv_card_attend_static(*args) == -5                       # QKV_ERR_CAPACITY: nothing launched
    ok = qkv.Desc.make(2, 2, 100, 128, 32)
    assert L.qkv_card_attend_static(None, 4096, ctypes.byref(ok), ctypes.c_void_p(dummy.data_ptr()), 4, ctypes.c_float(0.1),
                                    ctypes.c_void_p(f32.data_ptr()), None, None, None) == -1
    assert L.qkv_card_attend_static(ctypes.c_void_p(dummy.data_ptr()), 4096, ctypes.byref(ok), ctypes.c_void_p(dummy.data_ptr()), 3,
                                    ctypes.c_float(0.1), ctypes.c_void_p(f32.data_ptr()), None, None, None) == -2
    # a buffer that is no card: refused on the device, outputs untouched
    out = torch.full((2, 4, 128), 7.0, dtype=torch.float32, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    q = torch.zeros((2, 4, 128), dtype=torch.float16, device=DEV)
    assert L.qkv_card_attend_static(ctypes.c_void_p(dummy.data_ptr()), 4096, ctypes.byref(ok), ctypes.c_void_p(q.data_ptr()), 4,
                                    ctypes.c_float(0.1), ctypes.c_void_p(out.data_ptr()), None, ctypes.c_void_p(status.data_ptr()),
                                    None) == 0
    torch.cuda.synchronize()
    assert int(status.item()) == qkv.STATUS_BAD_HEADER and bool((out == 7.0).all())
