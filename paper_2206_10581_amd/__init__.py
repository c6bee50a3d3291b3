"""MI355X-native tensor-train embedding lookup, backward pass and SGD update.

The arithmetic lives in libtt_emb.so (hand-written HIP for gfx950, C ABI in include/tt_emb.h);
this package only marshals arguments.  PyTorch supplies device memory and streams.
"""
from .binding import (TTEmbedding, TTEmbError, load_library, tt_emb_backward_update, tt_emb_create,
                      tt_emb_destroy, tt_emb_forward, tt_emb_forward_eval, tt_emb_get_stats, tt_emb_lookup_static,
                      tt_emb_materialize, tt_emb_prepare, tt_emb_profile_enable,
                      tt_emb_profile_peaks, tt_emb_profile_read, tt_emb_profile_slots,
                      tt_emb_set_adagrad, tt_emb_set_adam, tt_emb_set_reindex, tt_emb_strerror,
                      tt_emb_wait_backward, tt_emb_workspace_bytes)

__all__ = ["TTEmbedding", "TTEmbError", "load_library", "tt_emb_workspace_bytes", "tt_emb_create",
           "tt_emb_forward", "tt_emb_forward_eval", "tt_emb_materialize", "tt_emb_set_reindex",
           "tt_emb_set_adagrad", "tt_emb_set_adam", "tt_emb_wait_backward", "tt_emb_prepare",
           "tt_emb_backward_update", "tt_emb_get_stats", "tt_emb_destroy", "tt_emb_strerror",
           "tt_emb_profile_enable", "tt_emb_profile_slots", "tt_emb_profile_read",
           "tt_emb_profile_peaks", "tt_emb_lookup_static"]
