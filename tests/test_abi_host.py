"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and its pure-host entry points (card size, budget counts, argument checks)
agree with the layout description and the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2605_03884_amd as qkv
from oracle import ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "qkvcard.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qkv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"qkv_card_bytes", "qkv_assign_bits", "qkv_quantize_pack", "qkv_unpack_dequant"} <= set(names)
    L = qkv.lib()
    for n in names:
        assert hasattr(L, n), n
    assert qkv.version() >= 100
    assert qkv.error_string(0) == "ok" and "unknown" in qkv.error_string(-99)


def test_header_struct_is_256_bytes_with_documented_offsets():
    text = open(os.path.join(ROOT, "include", "qkvcard.h")).read()
    body = text[text.index("typedef struct qkv_card_header"):text.index("} qkv_card_header_t;")]
    size = {"uint8_t": 1, "uint32_t": 4, "uint64_t": 8, "int64_t": 8, "float": 4}
    off = 0
    for m in re.finditer(r"^\s*(\w+)\s+(\w+)(?:\[(\d+)\])?;\s*/\*\s*(\d+)", body, flags=re.M):
        ty, name, n, documented = m.group(1), m.group(2), int(m.group(3) or 1), int(m.group(4))
        assert off == documented, name
        assert off % min(size[ty], 8) == 0, name      # natural alignment: no hidden padding
        off += size[ty] * n
    assert off == 256


def golden_rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [part.split() for part in line.split("|")]


def test_card_bytes_golden_and_oracle():
    for shape, counts, total in golden_rows("card_sizes.txt"):
        L, H, T, D, G = map(int, shape)
        if D not in (64, 128, 256) or G not in (32, 64, 128):
            continue
        counts = list(map(int, counts))
        assert qkv.card_bytes(qkv.Desc.make(L, H, T, D, G), counts) == int(total[0])
    rng = np.random.default_rng(8)
    for _ in range(300):
        L, H = int(rng.integers(1, 40)), int(rng.integers(1, 17))
        D = int(rng.choice([64, 128, 256]))
        G = int(rng.choice([g for g in (32, 64, 128) if g <= D]))
        T = int(rng.integers(1, 40000))
        cuts = np.sort(rng.integers(0, T + 1, size=3))
        counts = [int(cuts[0]), int(cuts[1] - cuts[0]), int(cuts[2] - cuts[1]), int(T - cuts[2])]
        assert qkv.card_bytes(qkv.Desc.make(L, H, T, D, G), counts) == ref.card_bytes(ref.make_desc(L, H, T, D, G), counts)


def test_budget_counts_golden_and_oracle():
    for T, budget, counts in golden_rows("budget_counts.txt"):
        assert qkv.budget_counts(int(T[0]), float(budget[0])) == list(map(int, counts))
    rng = np.random.default_rng(2)
    for _ in range(2000):
        T = int(rng.integers(1, 1 << 22))
        bm = int(rng.integers(2000, 16001))
        assert qkv.budget_counts(T, bm / 1000.0) == ref.budget_counts(T, bm / 1000.0).tolist()
    for bad in (1.99, 16.5, float("nan"), float("inf")):
        with pytest.raises(qkv.QkvError) as e:
            qkv.budget_counts(100, bad)
        assert e.value.code == -4


def test_argument_errors_are_reported_before_any_gpu_work():
    L = qkv.lib()
    d = qkv.Desc.make(2, 2, 64, 128, 32)
    out = ctypes.c_uint64(0)
    c = (ctypes.c_int64 * 4)(64, 0, 0, 0)
    assert L.qkv_card_bytes(None, c, ctypes.byref(out)) == -1
    assert L.qkv_card_bytes(ctypes.byref(d), None, ctypes.byref(out)) == -1
    assert L.qkv_card_bytes(ctypes.byref(d), c, None) == -1
    for field, value, code in [("layers", 0, -2), ("kv_heads", -1, -2), ("tokens", 0, -2), ("head_dim", 96, -2),
                               ("group_size", 48, -3), ("group_size", 16, -3)]:
        bad = qkv.Desc.make(2, 2, 64, 128, 32)
        setattr(bad, field, value)
        assert L.qkv_card_bytes(ctypes.byref(bad), c, ctypes.byref(out)) == code, field
    assert L.qkv_card_bytes(ctypes.byref(qkv.Desc.make(1, 1, 64, 64, 128)), c, ctypes.byref(out)) == -3
    assert L.qkv_card_bytes(ctypes.byref(d), (ctypes.c_int64 * 4)(63, 0, 0, 0), ctypes.byref(out)) == -7
    assert L.qkv_card_bytes(ctypes.byref(d), (ctypes.c_int64 * 4)(65, -1, 0, 0), ctypes.byref(out)) == -7
    # 2 * L * H * T must stay below 2^32
    assert L.qkv_card_bytes(ctypes.byref(qkv.Desc.make(64, 64, 1 << 20, 128, 32)),
                            (ctypes.c_int64 * 4)(1 << 20, 0, 0, 0), ctypes.byref(out)) == -2
    # null device pointers never reach a kernel
    assert L.qkv_quantize_pack(ctypes.byref(d), None, None, None, c, None, 0, None) == -1
    assert L.qkv_unpack_dequant(None, 0, ctypes.byref(d), None, None, None, None) == -1
    assert L.qkv_assign_bits(None, 64, 4.0, None, c, None) == -1
    assert L.qkv_count_bits(None, 64, c, None) == -1
    assert L.qkv_card_peek(None, 0, None, None, None, None, None) == -1
    assert L.qkv_assign_plan(ctypes.byref(d), None, 4.0, None, c, None, 0, None) == -1
    assert L.qkv_assign_quantize_pack(ctypes.byref(d), None, None, None, 4.0, None, c, None, 0, None) == -1
    assert not hasattr(L, "qkv_stream_probe")          # the measurement aid lives in its own library
    fl = ctypes.c_uint32(0)
    assert L.qkv_card_flags(None, 0, ctypes.byref(fl), None) == -1 and L.qkv_card_flags(None, 0, None, None) == -1
    assert L.qkv_card_attend(None, 0, ctypes.byref(d), None, 8, ctypes.c_float(1.0), None, None, None, 0, None, None) == -1
    ws = ctypes.c_uint64(0)
    assert L.qkv_card_attend_workspace(ctypes.byref(d), 8, ctypes.byref(ws)) == 0 and ws.value > 0
    assert L.qkv_card_attend_workspace(ctypes.byref(d), 3, ctypes.byref(ws)) == -2      # not a multiple of kv_heads
    assert L.qkv_card_attend_workspace(ctypes.byref(d), 2 * 17, ctypes.byref(ws)) == -2  # more than 16 query heads per kv head
    ws64, ws256 = ctypes.c_uint64(0), ctypes.c_uint64(0)                                 # every supported head_dim
    assert L.qkv_card_attend_workspace(ctypes.byref(qkv.Desc.make(2, 2, 64, 64, 32)), 8, ctypes.byref(ws64)) == 0
    assert L.qkv_card_attend_workspace(ctypes.byref(qkv.Desc.make(2, 2, 64, 256, 32)), 8, ctypes.byref(ws256)) == 0
    assert 0 < ws64.value < ws256.value
    assert L.qkv_card_attend_workspace(ctypes.byref(qkv.Desc.make(2, 2, 64, 96, 32)), 8, ctypes.byref(ws)) == -2


def test_header_is_plain_c_and_the_library_links_from_c(tmp_path):
    """The boundary is a C ABI: the header compiles as strict C99 and a C program that links the library gets the
    host-side answers (version, closed-form card size, budget counts, error strings) without Python in between."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    qkv.lib()                                                   # builds the library if it is not there yet
    src = tmp_path / "use_qkvcard.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "qkvcard.h"
int main(void) {
  qkv_desc_t d;
  int64_t counts[4] = {6282, 1092, 682, 136}, got[4];
  uint64_t bytes = 0;
  memset(&d, 0, sizeof d);
  d.layers = 32; d.kv_heads = 8; d.head_dim = 128; d.group_size = 32; d.tokens = 8192;
  if (sizeof(qkv_card_header_t) != QKV_CARD_HEADER_BYTES) return 1;
  if (qkv_card_bytes(&d, counts, &bytes) != QKV_OK) return 2;
  if (qkv_budget_counts(8192, 3.0, got) != QKV_OK) return 3;
  if (memcmp(got, counts, sizeof got) != 0) return 4;
  if (qkv_budget_counts(8192, 1.0, got) != QKV_ERR_BUDGET) return 5;
  if (qkv_quantize_pack(&d, NULL, NULL, NULL, counts, NULL, 0, NULL) != QKV_ERR_NULL) return 6;
  printf("%d %llu %s\n", qkv_version(), (unsigned long long)bytes, qkv_error_string(QKV_ERR_CAPACITY));
  return 0;
}
''')
    exe = tmp_path / "use_qkvcard"
    libdir = os.path.dirname(qkv.lib_path())
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
                    "-o", str(exe), "-L", libdir, "-lqkvcard", "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(None, 2)
    assert int(out[0]) == qkv.version()
    assert int(out[1]) == 267297024                            # the 8K benchmark card, closed form of the layout
    assert out[2].strip() == "card buffer too small"
