"""The boundary used without Python: a plain HIP host program (paper_2605_03884_amd/csrc/handoff_client.cpp, built beside the
library) takes seeded inputs from a file, runs one handoff through the C ABI with buffers from hipMalloc, and writes
what it got; widths, card and dequantized cache are compared with the oracle byte for byte."""
import os
import struct
import subprocess

import numpy as np
import pytest

import paper_2605_03884_amd as qkv
import qkv_synth
from oracle import ref

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("L,H,T,D,G,budget", [(2, 2, 333, 128, 32, 4.0), (1, 3, 1000, 64, 64, 3.0), (3, 1, 77, 256, 128, 7.5)])
def test_handoff_from_a_plain_hip_program(tmp_path, L, H, T, D, G, budget):
    client = os.path.join(os.path.dirname(qkv.lib_path()), "handoff_client")
    if not os.path.exists(client):                        # built with the library; compiled here only if it is not there
        qkv.lib()
        from paper_2605_03884_amd import build as lib_build
        lib_build.build_client()
    print("[case] C client L%d H%d T%d D%d G%d budget %.1f" % (L, H, T, D, G, budget), flush=True)
    K, V = qkv_synth.make_kv(L, H, T, D, 900 + T, "llama")
    scores = qkv_synth.make_scores(T, 901 + T).numpy()
    k16, v16 = K.numpy().view(np.uint16), V.numpy().view(np.uint16)
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        f.write(struct.pack("<4iqd", L, H, D, G, T, budget))
        f.write(scores.astype(np.float32).tobytes())
        f.write(k16.tobytes())
        f.write(v16.tobytes())
    run = subprocess.run([client, str(src), str(dst)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stderr
    raw = np.fromfile(dst, dtype=np.uint8)
    counts = raw[:32].view(np.int64).tolist()
    card_bytes = int(raw[32:40].view(np.uint64)[0])
    status = int(raw[40:44].view(np.uint32)[0])
    pos = 48
    bits = raw[pos:pos + T]; pos += T
    card = raw[pos:pos + card_bytes]; pos += card_bytes
    n = L * H * T * D * 2
    ko = raw[pos:pos + n].view(np.uint16).reshape(L, H, T, D); pos += n
    vo = raw[pos:pos + n].view(np.uint16).reshape(L, H, T, D); pos += n
    assert pos == raw.size and status == 0
    want_bits, want_counts = ref.assign_bits(scores, budget)
    assert counts == want_counts.tolist() and np.array_equal(bits, want_bits)
    rd = ref.make_desc(L, H, T, D, G, 8, 1, 0)
    want_card = ref.quantize_pack(rd, k16, v16, want_bits, want_counts)
    assert card_bytes == want_card.size and np.array_equal(card, want_card)
    wk, wv = ref.unpack_dequant(want_card, rd)
    assert np.array_equal(ko, wk) and np.array_equal(vo, wv)
