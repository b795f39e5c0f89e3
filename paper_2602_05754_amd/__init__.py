"""MI355X-native freeze-aware stage backward, masked AdamW and APF stability
statistics (the computation TimelyFreeze's freeze ratios speed up; Sec. 3.2.1,
App. D.1, Sec. 2.3).  Thin ctypes binding over the C-ABI library libtf.so;
every step of the path runs in hand-written gfx950 kernels.  There is no CPU
or PyTorch fallback: without the built library, calls raise."""
from .binding import (  # noqa: F401
    TF_BF16, TF_F32, Context, PtrTable, TfError, library_path, load_library,
    tf_masked_adamw, tf_num_frozen, tf_select_lowest, tf_stability_scores,
    tf_stability_update, tf_stage_backward, tf_strerror, tf_version, EXPORTED_SYMBOLS, KERNEL_KINDS,
    tf_autofreeze_norms, tf_autofreeze_scores, tf_autofreeze_select, tf_reconcile_mask, tf_reconcile_mask_static,
    tf_stage_backward_blocks, tf_stage_backward_shared, tf_stage_backward_microbatch, tf_microbatch_plan, tf_select_row_blocks, tf_row_blocks_to_bits,
    tf_pipeline_dag, tf_dag_start_times, tf_freeze_ratio_lp, tf_actual_freeze_ratio, TF_SCHEDULE_GPIPE, TF_SCHEDULE_1F1B, TF_SCHEDULE_INTERLEAVED_1F1B, TF_SCHEDULE_ZBV,
)
