"""CacheCard creation and receiver-side dequantization on MI355X.

Thin ctypes binding over libqkvcard.so (see include/qkvcard.h): argument marshalling only.
torch supplies device memory and the current HIP stream; every step runs in the library's
HIP kernels.  There is no CPU path: a missing library raises at first use.
"""
from .binding import (  # noqa: F401
    QkvError, Desc, Controller, Inject, lib, lib_path, version, error_string, card_bytes, budget_counts, assign_bits, count_bits, controller_scores,
    assign_bits_greedy, assign_plan, assign_quantize_pack,
    quantize_pack, requantize, quantize_pack_kc, unpack_dequant_kc, card_plan, card_fill, unpack_dequant, inject_layers, card_peek, card_flags, card_attend, card_attend_kc, card_attend_static, card_attend_workspace, STATUS_BAD_BITS, STATUS_BAD_COUNTS, STATUS_BAD_HEADER,
    STATUS_BAD_ORDER, FLAG_KEYS_PER_CHANNEL,
)
