"""ctypes marshalling for the C ABI declared in include/qkvcard.h (same names, same order)."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libqkvcard.so"

STATUS_BAD_BITS = 0x1
STATUS_BAD_COUNTS = 0x2
STATUS_BAD_HEADER = 0x4
STATUS_BAD_ORDER = 0x8
FLAG_KEYS_PER_CHANNEL = 0x1


class QkvError(RuntimeError):
    def __init__(self, code, where):
        super().__init__("%s: %s (%d)" % (where, error_string(code), code))
        self.code = code


class Desc(ctypes.Structure):
    """qkv_desc_t."""
    _fields_ = [
        ("layers", ctypes.c_int32),
        ("kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("group_size", ctypes.c_int32),
        ("tokens", ctypes.c_int64),
        ("model_id", ctypes.c_uint64),
        ("sender_id", ctypes.c_uint64),
        ("position_offset", ctypes.c_int64),
    ]

    @classmethod
    def make(cls, layers, kv_heads, tokens, head_dim, group_size, model_id=0, sender_id=0, position_offset=0):
        return cls(layers, kv_heads, head_dim, group_size, tokens, model_id, sender_id, position_offset)


class Controller(ctypes.Structure):
    """qkv_controller_t: the 512 parameters of the 6 -> 64 -> 1 network."""
    _fields_ = [("w1", ctypes.c_float * 6 * 64), ("b1", ctypes.c_float * 64), ("w2", ctypes.c_float * 64)]

    @classmethod
    def make(cls, w1, b1, w2):
        """w1 [64, 6], b1 [64], w2 [64]: host float32 tensors or arrays."""
        c = cls()
        flat = [float(x) for x in torch.as_tensor(w1, dtype=torch.float32).reshape(-1).tolist()]
        if len(flat) != 384 or len(b1) != 64 or len(w2) != 64:
            raise ValueError("controller parameters must be w1 [64, 6], b1 [64], w2 [64]")
        ctypes.memmove(c.w1, (ctypes.c_float * 384)(*flat), 384 * 4)
        ctypes.memmove(c.b1, (ctypes.c_float * 64)(*[float(x) for x in torch.as_tensor(b1, dtype=torch.float32).tolist()]), 256)
        ctypes.memmove(c.w2, (ctypes.c_float * 64)(*[float(x) for x in torch.as_tensor(w2, dtype=torch.float32).tolist()]), 256)
        return c


class Inject(ctypes.Structure):
    """qkv_inject_t."""
    _fields_ = [
        ("layer_begin", ctypes.c_int32),
        ("layer_count", ctypes.c_int32),
        ("k_layers", ctypes.POINTER(ctypes.c_void_p)),
        ("v_layers", ctypes.POINTER(ctypes.c_void_p)),
        ("head_stride", ctypes.c_int64),
        ("token_stride", ctypes.c_int64),
        ("rope_base", ctypes.c_double),
        ("rope_delta", ctypes.c_int64),
        ("keys_per_channel", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
    ]


_lib = None


def lib_path():
    return os.path.join(_HERE, _LIB_NAME)


def lib():
    """The loaded library.  Built once by paper_2605_03884_amd.build if it is not there; never replaced by a fallback."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    L = ctypes.CDLL(path)
    i64p = ctypes.POINTER(ctypes.c_int64)
    vp = ctypes.c_void_p
    L.qkv_version.restype = ctypes.c_int
    L.qkv_version.argtypes = []
    L.qkv_error_string.restype = ctypes.c_char_p
    L.qkv_error_string.argtypes = [ctypes.c_int]
    L.qkv_card_bytes.restype = ctypes.c_int
    L.qkv_card_bytes.argtypes = [ctypes.POINTER(Desc), i64p, ctypes.POINTER(ctypes.c_uint64)]
    L.qkv_budget_counts.restype = ctypes.c_int
    L.qkv_budget_counts.argtypes = [ctypes.c_int64, ctypes.c_double, i64p]
    L.qkv_assign_bits.restype = ctypes.c_int
    L.qkv_assign_bits.argtypes = [vp, ctypes.c_int64, ctypes.c_double, vp, i64p, vp]
    L.qkv_assign_plan.restype = ctypes.c_int
    L.qkv_assign_plan.argtypes = [ctypes.POINTER(Desc), vp, ctypes.c_double, vp, i64p, vp, ctypes.c_uint64, vp]
    L.qkv_assign_quantize_pack.restype = ctypes.c_int
    L.qkv_assign_quantize_pack.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, ctypes.c_double, vp, i64p, vp, ctypes.c_uint64, vp]
    L.qkv_controller_scores.restype = ctypes.c_int
    L.qkv_controller_scores.argtypes = [vp, ctypes.c_int64, ctypes.POINTER(Controller), vp, vp]
    L.qkv_assign_bits_greedy.restype = ctypes.c_int
    L.qkv_assign_bits_greedy.argtypes = [vp, ctypes.c_int64, ctypes.c_double, vp, vp, vp]
    L.qkv_count_bits.restype = ctypes.c_int
    L.qkv_count_bits.argtypes = [vp, ctypes.c_int64, i64p, vp]
    L.qkv_quantize_pack.restype = ctypes.c_int
    L.qkv_quantize_pack.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, i64p, vp, ctypes.c_uint64, vp]
    L.qkv_card_plan.restype = ctypes.c_int
    L.qkv_card_plan.argtypes = [ctypes.POINTER(Desc), vp, i64p, vp, ctypes.c_uint64, vp]
    L.qkv_card_fill.restype = ctypes.c_int
    L.qkv_card_fill.argtypes = [ctypes.POINTER(Desc), vp, vp, i64p, vp, ctypes.c_uint64, vp]
    L.qkv_inject_layers.restype = ctypes.c_int
    L.qkv_inject_layers.argtypes = [vp, ctypes.c_uint64, ctypes.POINTER(Desc), ctypes.POINTER(Inject), vp, vp]
    L.qkv_quantize_pack_kc.restype = ctypes.c_int
    L.qkv_quantize_pack_kc.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, i64p, vp, ctypes.c_uint64, vp]
    L.qkv_unpack_dequant_kc.restype = ctypes.c_int
    L.qkv_unpack_dequant_kc.argtypes = [vp, ctypes.c_uint64, ctypes.POINTER(Desc), vp, vp, vp, vp]
    L.qkv_requantize.restype = ctypes.c_int
    L.qkv_requantize.argtypes = [vp, ctypes.c_uint64, ctypes.POINTER(Desc), vp, i64p, vp, ctypes.c_uint64, vp, vp]
    L.qkv_unpack_dequant.restype = ctypes.c_int
    L.qkv_unpack_dequant.argtypes = [vp, ctypes.c_uint64, ctypes.POINTER(Desc), vp, vp, vp, vp]
    L.qkv_card_attend_workspace.restype = ctypes.c_int
    L.qkv_card_attend_workspace.argtypes = [ctypes.POINTER(Desc), ctypes.c_int32, ctypes.POINTER(ctypes.c_uint64)]
    L.qkv_card_attend.restype = ctypes.c_int
    L.qkv_card_attend.argtypes = [vp, ctypes.c_uint64, ctypes.POINTER(Desc), vp, ctypes.c_int32, ctypes.c_float, vp, vp,
                                  vp, ctypes.c_uint64, vp, vp]
    L.qkv_card_attend_kc.restype = ctypes.c_int
    L.qkv_card_attend_kc.argtypes = [vp, ctypes.c_uint64, ctypes.POINTER(Desc), vp, ctypes.c_int32, ctypes.c_float, vp, vp,
                                  vp, ctypes.c_uint64, vp, vp]
    L.qkv_card_attend_static.restype = ctypes.c_int
    L.qkv_card_attend_static.argtypes = [vp, ctypes.c_uint64, ctypes.POINTER(Desc), vp, ctypes.c_int32, ctypes.c_float, vp, vp,
                                         vp, vp]
    L.qkv_card_peek.restype = ctypes.c_int
    L.qkv_card_peek.argtypes = [vp, ctypes.c_uint64, ctypes.POINTER(Desc), i64p, ctypes.POINTER(ctypes.c_float),
                                ctypes.POINTER(ctypes.c_uint32), vp]
    L.qkv_card_flags.restype = ctypes.c_int
    L.qkv_card_flags.argtypes = [vp, ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint32), vp]
    _lib = L
    return L


def _check(rc, where):
    if rc != 0:
        raise QkvError(rc, where)


def _counts(counts):
    arr = (ctypes.c_int64 * 4)(*[int(c) for c in counts])
    return arr


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_ptr(t, dtype=None, name="tensor"):
    if not t.is_cuda:
        raise ValueError("%s must live in device memory" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must be %s" % (name, dtype))
    return ctypes.c_void_p(t.data_ptr())


def version():
    return lib().qkv_version()


def error_string(code):
    return lib().qkv_error_string(int(code)).decode()


def card_bytes(desc, counts):
    out = ctypes.c_uint64(0)
    _check(lib().qkv_card_bytes(ctypes.byref(desc), _counts(counts), ctypes.byref(out)), "qkv_card_bytes")
    return out.value


def budget_counts(tokens, avg_bits_budget):
    out = (ctypes.c_int64 * 4)()
    _check(lib().qkv_budget_counts(int(tokens), float(avg_bits_budget), out), "qkv_budget_counts")
    return list(out)


def assign_bits(scores, avg_bits_budget, bits=None, stream=None):
    """scores: device float32[T].  Returns (bits device uint8[T], counts list)."""
    T = scores.numel()
    if bits is None:
        bits = torch.empty(T, dtype=torch.uint8, device=scores.device)
    out = (ctypes.c_int64 * 4)()
    _check(lib().qkv_assign_bits(_dev_ptr(scores, torch.float32, "scores"), T, float(avg_bits_budget),
                                 _dev_ptr(bits, torch.uint8, "bits"), out, _stream(stream)), "qkv_assign_bits")
    return bits, list(out)


def assign_plan(desc, scores, avg_bits_budget, card, bits=None, stream=None):
    """scores: device float32[T]; card: device uint8 buffer (header, tables and pads are written); bits: device
    uint8[T] or None.  Returns the class counts (list)."""
    out = (ctypes.c_int64 * 4)()
    bp = ctypes.c_void_p(0) if bits is None else _dev_ptr(bits, torch.uint8, "bits")
    _check(lib().qkv_assign_plan(ctypes.byref(desc), _dev_ptr(scores, torch.float32, "scores"), float(avg_bits_budget), bp,
                                 out, _dev_ptr(card, torch.uint8, "card"), card.numel(), _stream(stream)),
           "qkv_assign_plan")
    return list(out)


def assign_quantize_pack(desc, k, v, scores, avg_bits_budget, card, bits=None, stream=None):
    """Scores, budget and K/V in; widths (if bits is given) and the whole card out.  Returns the class counts."""
    out = (ctypes.c_int64 * 4)()
    bp = ctypes.c_void_p(0) if bits is None else _dev_ptr(bits, torch.uint8, "bits")
    _check(lib().qkv_assign_quantize_pack(ctypes.byref(desc), _dev_ptr(k, torch.float16, "k"), _dev_ptr(v, torch.float16, "v"),
                                          _dev_ptr(scores, torch.float32, "scores"), float(avg_bits_budget), bp, out,
                                          _dev_ptr(card, torch.uint8, "card"), card.numel(), _stream(stream)),
           "qkv_assign_quantize_pack")
    return list(out)


def controller_scores(features, params, scores=None, stream=None):
    """features: device float32[T, 6]; params: Controller.  Returns scores, device float32[T]."""
    T = features.shape[0]
    if features.dim() != 2 or features.shape[1] != 6:
        raise ValueError("features must be [T, 6]")
    if scores is None:
        scores = torch.empty(T, dtype=torch.float32, device=features.device)
    _check(lib().qkv_controller_scores(_dev_ptr(features, torch.float32, "features"), T, ctypes.byref(params),
                                       _dev_ptr(scores, torch.float32, "scores"), _stream(stream)),
           "qkv_controller_scores")
    return scores


def assign_bits_greedy(scores, avg_bits_budget, bits=None, counts=None, stream=None):
    """scores: device float32[T].  Returns (bits device uint8[T], counts device int64[4]); nothing synchronises."""
    T = scores.numel()
    if bits is None:
        bits = torch.empty(T, dtype=torch.uint8, device=scores.device)
    if counts is None:
        counts = torch.empty(4, dtype=torch.int64, device=scores.device)
    _check(lib().qkv_assign_bits_greedy(_dev_ptr(scores, torch.float32, "scores"), T, float(avg_bits_budget),
                                        _dev_ptr(bits, torch.uint8, "bits"), _dev_ptr(counts, torch.int64, "counts"),
                                        _stream(stream)), "qkv_assign_bits_greedy")
    return bits, counts


def count_bits(bits, stream=None):
    out = (ctypes.c_int64 * 4)()
    _check(lib().qkv_count_bits(_dev_ptr(bits, torch.uint8, "bits"), bits.numel(), out, _stream(stream)),
           "qkv_count_bits")
    return list(out)


def quantize_pack(desc, k, v, bits, counts, card, stream=None):
    """k, v: device float16 [L, H, T, D]; bits: device uint8[T]; card: device uint8 buffer, written in place."""
    _check(lib().qkv_quantize_pack(ctypes.byref(desc), _dev_ptr(k, torch.float16, "k"), _dev_ptr(v, torch.float16, "v"),
                                   _dev_ptr(bits, torch.uint8, "bits"), _counts(counts),
                                   _dev_ptr(card, torch.uint8, "card"), card.numel(), _stream(stream)),
           "qkv_quantize_pack")
    return card


def quantize_pack_kc(desc, k, v, bits, counts, card, stream=None):
    """quantize_pack for a uniform card with the keys grouped per channel."""
    _check(lib().qkv_quantize_pack_kc(ctypes.byref(desc), _dev_ptr(k, torch.float16, "k"), _dev_ptr(v, torch.float16, "v"),
                                      _dev_ptr(bits, torch.uint8, "bits"), _counts(counts),
                                      _dev_ptr(card, torch.uint8, "card"), card.numel(), _stream(stream)),
           "qkv_quantize_pack_kc")
    return card


def requantize(card_in, desc, bits, counts, card_out, status=None, card_in_nbytes=None, stream=None):
    """The card that quantize_pack would build from unpack_dequant(card_in), at the new widths, card to card."""
    n = card_in.numel() if card_in_nbytes is None else int(card_in_nbytes)
    sp = ctypes.c_void_p(0) if status is None else _dev_ptr(status, None, "status")
    _check(lib().qkv_requantize(_dev_ptr(card_in, torch.uint8, "card_in"), n, ctypes.byref(desc),
                                _dev_ptr(bits, torch.uint8, "bits"), _counts(counts),
                                _dev_ptr(card_out, torch.uint8, "card_out"), card_out.numel(), sp, _stream(stream)),
           "qkv_requantize")
    return card_out


def card_plan(desc, bits, counts, card, stream=None):
    """First half of quantize_pack: header, tables and pads."""
    _check(lib().qkv_card_plan(ctypes.byref(desc), _dev_ptr(bits, torch.uint8, "bits"), _counts(counts),
                               _dev_ptr(card, torch.uint8, "card"), card.numel(), _stream(stream)), "qkv_card_plan")
    return card


def card_fill(desc, k, v, counts, card, stream=None):
    """Second half of quantize_pack: the K/V rows into a planned card."""
    _check(lib().qkv_card_fill(ctypes.byref(desc), _dev_ptr(k, torch.float16, "k"), _dev_ptr(v, torch.float16, "v"),
                               _counts(counts), _dev_ptr(card, torch.uint8, "card"), card.numel(), _stream(stream)),
           "qkv_card_fill")
    return card


def unpack_dequant(card, expect, k_out, v_out, status=None, card_nbytes=None, stream=None):
    """card: device uint8; k_out, v_out: device float16 [L, H, T, D]; status: device int32[1] or None."""
    n = card.numel() if card_nbytes is None else int(card_nbytes)
    sp = ctypes.c_void_p(0) if status is None else _dev_ptr(status, None, "status")
    _check(lib().qkv_unpack_dequant(_dev_ptr(card, torch.uint8, "card"), n, ctypes.byref(expect),
                                    _dev_ptr(k_out, torch.float16, "k_out"), _dev_ptr(v_out, torch.float16, "v_out"),
                                    sp, _stream(stream)), "qkv_unpack_dequant")
    return k_out, v_out


def unpack_dequant_kc(card, expect, k_out, v_out, status=None, card_nbytes=None, stream=None):
    """unpack_dequant for a uniform card with the keys grouped per channel."""
    n = card.numel() if card_nbytes is None else int(card_nbytes)
    sp = ctypes.c_void_p(0) if status is None else _dev_ptr(status, None, "status")
    _check(lib().qkv_unpack_dequant_kc(_dev_ptr(card, torch.uint8, "card"), n, ctypes.byref(expect),
                                       _dev_ptr(k_out, torch.float16, "k_out"), _dev_ptr(v_out, torch.float16, "v_out"),
                                       sp, _stream(stream)), "qkv_unpack_dequant_kc")
    return k_out, v_out


def inject_layers(card, expect, k_layers, v_layers, layer_begin=0, rope_base=0.0, rope_delta=0, status=None,
                  card_nbytes=None, stream=None, keys_per_channel=False):
    """Layers layer_begin .. layer_begin + len(k_layers) - 1 of the card into per-layer tensors.

    k_layers, v_layers: lists of device float16 tensors (views are fine) of shape [kv_heads, >= tokens, head_dim]
    whose element [h, t, :] is where token t of head h lands: rows contiguous, all layers with the same strides.
    A cache [kv_heads, capacity, head_dim] holding a prefix of P tokens is passed as cache[:, P:P + tokens]."""
    n = card.numel() if card_nbytes is None else int(card_nbytes)
    count = len(k_layers)
    if count != len(v_layers) or count < 1:
        raise ValueError("k_layers and v_layers must be lists of the same, non-zero length")
    ref_strides = k_layers[0].stride()
    for t in list(k_layers) + list(v_layers):
        if not t.is_cuda or t.dtype != torch.float16 or t.dim() != 3:
            raise ValueError("layer tensors must be device float16 [kv_heads, tokens, head_dim]")
        if t.shape[0] != expect.kv_heads or t.shape[1] < expect.tokens or t.shape[2] != expect.head_dim:
            raise ValueError("layer tensor shape %s does not hold the card's tokens" % (tuple(t.shape),))
        if t.stride() != ref_strides or t.stride(2) != 1:
            raise ValueError("layer tensors must share their strides and have contiguous rows")
    kp = (ctypes.c_void_p * count)(*[t.data_ptr() for t in k_layers])
    vp_ = (ctypes.c_void_p * count)(*[t.data_ptr() for t in v_layers])
    where = Inject(int(layer_begin), count, kp, vp_, ref_strides[0], ref_strides[1], float(rope_base), int(rope_delta),
                   1 if keys_per_channel else 0, 0)
    sp = ctypes.c_void_p(0) if status is None else _dev_ptr(status, None, "status")
    _check(lib().qkv_inject_layers(_dev_ptr(card, torch.uint8, "card"), n, ctypes.byref(expect), ctypes.byref(where),
                                   sp, _stream(stream)), "qkv_inject_layers")


def card_attend_workspace(expect, q_heads):
    out = ctypes.c_uint64(0)
    _check(lib().qkv_card_attend_workspace(ctypes.byref(expect), int(q_heads), ctypes.byref(out)),
           "qkv_card_attend_workspace")
    return out.value


def card_attend(card, expect, q, softmax_scale, out, lse=None, workspace=None, status=None, card_nbytes=None,
                stream=None):
    """card: device uint8; q: device float16 [L, Hq, D]; out: device float32 [L, Hq, D]; lse: float32 [L, Hq]; D = 64, 128 or 256."""
    n = card.numel() if card_nbytes is None else int(card_nbytes)
    q_heads = q.shape[1]
    if workspace is None:
        workspace = torch.empty(card_attend_workspace(expect, q_heads), dtype=torch.uint8, device=card.device)
    lp = ctypes.c_void_p(0) if lse is None else _dev_ptr(lse, torch.float32, "lse")
    sp = ctypes.c_void_p(0) if status is None else _dev_ptr(status, None, "status")
    _check(lib().qkv_card_attend(_dev_ptr(card, torch.uint8, "card"), n, ctypes.byref(expect),
                                 _dev_ptr(q, torch.float16, "q"), int(q_heads), float(softmax_scale),
                                 _dev_ptr(out, torch.float32, "out"), lp, _dev_ptr(workspace, torch.uint8, "workspace"),
                                 workspace.numel(), sp, _stream(stream)), "qkv_card_attend")
    return out, lse


def card_attend_kc(card, expect, q, softmax_scale, out, lse=None, workspace=None, status=None, card_nbytes=None,
                   stream=None):
    """card_attend for a card whose keys are grouped per channel (made by quantize_pack_kc)."""
    n = card.numel() if card_nbytes is None else int(card_nbytes)
    q_heads = q.shape[1]
    if workspace is None:
        workspace = torch.empty(card_attend_workspace(expect, q_heads), dtype=torch.uint8, device=card.device)
    lp = ctypes.c_void_p(0) if lse is None else _dev_ptr(lse, torch.float32, "lse")
    sp = ctypes.c_void_p(0) if status is None else _dev_ptr(status, None, "status")
    _check(lib().qkv_card_attend_kc(_dev_ptr(card, torch.uint8, "card"), n, ctypes.byref(expect),
                                    _dev_ptr(q, torch.float16, "q"), int(q_heads), float(softmax_scale),
                                    _dev_ptr(out, torch.float32, "out"), lp, _dev_ptr(workspace, torch.uint8, "workspace"),
                                    workspace.numel(), sp, _stream(stream)), "qkv_card_attend_kc")
    return out, lse


def card_attend_static(card, expect, q, softmax_scale, out, lse=None, status=None, card_nbytes=None, stream=None):
    """card_attend without a workspace: the partials live in the library's fixed scratch array (no allocation)."""
    n = card.numel() if card_nbytes is None else int(card_nbytes)
    lp = ctypes.c_void_p(0) if lse is None else _dev_ptr(lse, torch.float32, "lse")
    sp = ctypes.c_void_p(0) if status is None else _dev_ptr(status, None, "status")
    _check(lib().qkv_card_attend_static(_dev_ptr(card, torch.uint8, "card"), n, ctypes.byref(expect),
                                        _dev_ptr(q, torch.float16, "q"), int(q.shape[1]), float(softmax_scale),
                                        _dev_ptr(out, torch.float32, "out"), lp, sp, _stream(stream)), "qkv_card_attend_static")
    return out, lse


def card_flags(card, card_nbytes=None, stream=None):
    """The header's flags word (0 or FLAG_KEYS_PER_CHANNEL) of a valid card.  Synchronises the stream."""
    n = card.numel() if card_nbytes is None else int(card_nbytes)
    fl = ctypes.c_uint32(0)
    _check(lib().qkv_card_flags(_dev_ptr(card, torch.uint8, "card"), n, ctypes.byref(fl), _stream(stream)),
           "qkv_card_flags")
    return fl.value


def card_peek(card, card_nbytes=None, stream=None):
    """Returns (Desc, counts, avg_bits, status).  Synchronises the stream."""
    n = card.numel() if card_nbytes is None else int(card_nbytes)
    d = Desc()
    counts = (ctypes.c_int64 * 4)()
    avg = ctypes.c_float(0)
    st = ctypes.c_uint32(0)
    _check(lib().qkv_card_peek(_dev_ptr(card, torch.uint8, "card"), n, ctypes.byref(d), counts, ctypes.byref(avg),
                               ctypes.byref(st), _stream(stream)), "qkv_card_peek")
    return d, list(counts), avg.value, st.value
