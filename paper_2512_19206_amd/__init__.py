"""MixKVQ hot path for MI355X: decode attention over a mixed-precision quantized
KV cache.  Python names mirror the C ABI of include/mixkvq.h."""
from .binding import (BlockLayout, Cache, Config, MixKVQError, Sizes, block_layout, cache_sizes, load_library,
                      make_config, EXPORTS, LIB_PATH, PATH_NONE, PATH_MATRIX, PATH_VECTOR)


def mixkvq_select_channels(cache: Cache, q, k, sel=None, stream=None):
    return cache.select_channels(q, k, sel=sel, stream=stream)


def mixkvq_quantize_append(cache: Cache, k_new, v_new, sel=None, stream=None):
    return cache.quantize_append(k_new, v_new, sel=sel, stream=stream)


def mixkvq_decode_step(cache: Cache, k_new, v_new, q, out=None, lse=None, scale=0.0, accumulate_q=False, stream=None):
    return cache.decode_step(k_new, v_new, q, out=out, lse=lse, scale=scale, accumulate_q=accumulate_q, stream=stream)


def mixkvq_decode_attention(cache: Cache, q, out=None, lse=None, scale=0.0, accumulate_q=False, stream=None):
    return cache.decode_attention(q, out=out, lse=lse, scale=scale, accumulate_q=accumulate_q, stream=stream)


def mixkvq_decode_path(cache: Cache) -> int:
    return cache.decode_path()


def mixkvq_decode_attention_noalloc(cache: Cache, q, out, lse, scale=0.0, accumulate_q=False, stream=None):
    return cache.decode_attention_noalloc(q, out, lse, scale=scale, accumulate_q=accumulate_q, stream=stream)


def mixkvq_prefill(cache: Cache, q, k, v, sel=None, stream=None):
    return cache.prefill(q, k, v, sel=sel, stream=stream)
