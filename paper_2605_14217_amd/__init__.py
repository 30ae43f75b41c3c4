"""MI355X-native prefill-only adapter apply (segmented multi-adapter LoRA, DiReFT and LoReFT).

The compute lives in ``libpreft.so`` (hand-written HIP for gfx950, C ABI declared in
``include/preft.h``); this package is the thin Python binding with the same names.
Importing the package does not load the library; the first call does, and raises if the
library has not been built (``python -m paper_2605_14217_amd.build``).
"""
from .binding import (  # noqa: F401
    PREFT_ALL_TOKENS, PREFT_PREFILL_ONLY, PREFT_SCHEDULE_READY, PREFT_BF16, PREFT_F32,
    PREFT_TEST_VARIANT, PREFT_TEST_WAVES, PREFT_TEST_ROWBLOCKS, PREFT_TEST_COLSPLIT, PREFT_TEST_RESIDENT,
    test_flags, set_test_flags, PREFT_ESCHEDULE, PREFT_ETOOLARGE, PREFT_STATIC_SCRATCH_BYTES,
    PreftError, load_library, pointer_table, preft_direft_apply, preft_direft_apply_static, preft_direft_apply_layers, preft_lora_apply, preft_lora_apply_packed, preft_loreft_apply,
    preft_loreft_prepare, preft_schedule,
    preft_schedule_counts, preft_strerror, preft_version, preft_workspace_bytes, preft_workspace_bytes_z,
    new_workspace, preft_slots_create, preft_slots_destroy, preft_slots_store, preft_slots_acquire,
    preft_slots_pool, preft_slots_resident, preft_slots_stats, PREFT_ECAPACITY,
)
