"""MI355X-native Twilight decode hot path: hierarchical top-p pruning + sparse attention.

Python side = argument marshalling for the C ABI in include/twilight.h.
"""
from . import binding
from .binding import (TwilightError, twilight_kquant_append, twilight_select_pages, twilight_select_pages_static, twilight_append_select, twilight_ds_select_tokens, twilight_select_prune,
                      twilight_int4_score, twilight_int4_score_tokens, twilight_topp_prune_tokens,
                      twilight_topp_prune, twilight_sparse_decode, twilight_sparse_decode_per_head,
                      twilight_workspace_bytes,
                      twilight_prof_enable, twilight_prof_select, twilight_prof_collect, twilight_decode_plan, make_kv,
                      TW_WS_SELECT, TW_WS_PRUNE, TW_WS_DECODE, TW_WS_DECODE_PER_HEAD, TW_WS_PRUNE_TOKENS, TW_WS_DS_SELECT, TW_WS_SELECT_PRUNE)
from .cache import PagedKV, DecodeStep

__all__ = ["binding", "TwilightError", "twilight_kquant_append", "twilight_select_pages", "twilight_select_pages_static", "twilight_append_select", "twilight_ds_select_tokens", "TW_WS_DS_SELECT", "twilight_select_prune", "TW_WS_SELECT_PRUNE", "twilight_int4_score",
           "twilight_int4_score_tokens", "twilight_topp_prune_tokens", "TW_WS_PRUNE_TOKENS",
           "twilight_topp_prune", "twilight_sparse_decode", "twilight_sparse_decode_per_head", "twilight_workspace_bytes", "twilight_prof_enable",
           "twilight_prof_select", "twilight_prof_collect", "twilight_decode_plan", "make_kv", "PagedKV", "DecodeStep",
           "TW_WS_SELECT", "TW_WS_PRUNE", "TW_WS_DECODE", "TW_WS_DECODE_PER_HEAD"]
