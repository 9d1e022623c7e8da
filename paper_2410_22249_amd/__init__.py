"""MI355X-native multi-table EmbeddingBag forward (C-ABI library + thin binding)."""
from .binding import (EMB_BF16, EMB_F16, EMB_F32, EMB_HINT_DEFAULT, EMB_HINT_STREAMING, EMB_MAX, EMB_MEAN, EMB_OK, MODES, DTYPES, EMB_U8ROW, EMB_FP8ROW,
                      EMB_SUM, EXPORTS, EmbBagError, emb_bag_profile_reuse,
                      emb_bag_profile_hot_rows, emb_bag_profile_hot_rows_workspace,
                      emb_bag_profile_hot_rows_noalloc,
                      emb_bag_desc, emb_bag_forward, emb_bag_forward_mixed, emb_bag_plan,
                      emb_bag_plan_forward, emb_bag_plan_forward_mixed, EMB_KERNEL_WAVE,
                      EMB_KERNEL_STREAM,
                      emb_bag_mixed_desc, make_mixed_desc, emb_bag_get_tuning, emb_bag_set_tuning,
                      emb_bag_set_tuning_table, emb_bag_tuning_entry, emb_bag_tuning,
                      emb_bag_tuning_defaults,
                      emb_bag_status_string, emb_bag_validate, emb_bag_version, lib, make_desc)
from . import metrics

__all__ = ["EMB_U8ROW", "EMB_FP8ROW", "DTYPES", "EMB_BF16", "EMB_F16", "EMB_F32", "EMB_HINT_DEFAULT", "EMB_HINT_STREAMING", "emb_bag_profile_reuse", "emb_bag_profile_hot_rows",
           "emb_bag_profile_hot_rows_workspace", "emb_bag_profile_hot_rows_noalloc", "EMB_MAX", "EMB_MEAN", "EMB_OK", "MODES", "EMB_SUM", "EXPORTS", "EmbBagError",
           "emb_bag_desc", "emb_bag_forward", "emb_bag_forward_mixed", "emb_bag_mixed_desc",
           "emb_bag_plan", "emb_bag_plan_forward", "emb_bag_plan_forward_mixed", "EMB_KERNEL_WAVE",
           "EMB_KERNEL_STREAM",
           "make_mixed_desc", "emb_bag_get_tuning", "emb_bag_set_tuning", "emb_bag_set_tuning_table",
           "emb_bag_tuning_entry", "emb_bag_tuning", "emb_bag_tuning_defaults",
           "emb_bag_status_string", "emb_bag_validate", "emb_bag_version", "lib", "make_desc",
           "metrics"]
