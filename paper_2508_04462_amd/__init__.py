"""MI355X-native verification step of CARD (query-and-correct speculative decoding).

The work is done by libcard.so (hand-written HIP for gfx950 behind the C ABI of
include/card.h).  This package only marshals arguments; PyTorch supplies device
memory and streams.  The library is opened at the first call of any entry point and
that call fails loudly (ImportError) if it has not been built
(python -m paper_2508_04462_amd.build): there is no other implementation behind it.
"""
from .binding import (  # noqa: F401
    CARD_OK,
    CARD_EINVAL,
    CARD_ERANGE,
    CARD_ECAPACITY,
    CARD_EDEVICE,
    CARD_ESTALE,
    CARD_ETOOBIG,
    TENSOR_IDS,
    CardError,
    CardModelCfg,
    CardKV,
    CardVerifyResult,
    CardSampling,
    CardStep,
    CardTreeRows,
    CARD_STEP_NO_CORRECT,
    lib,
    lib_path,
    card_strerror,
    card_packed_weight_bytes,
    card_workspace_bytes,
    card_kv_pool_bytes,
    card_stream_frag_index,
    card_weights_pack_tensor,
    card_verify,
    card_verify_debug_logits,
    card_verify_static,
    card_draft_level,
    card_cache_select,
    card_tree_mask_level,
    card_step_begin,
    card_step_begin_sampled,
    card_step_end,
    card_verify_sampled,
    card_static_scratch_bytes,
    card_static_scratch_reset,
    card_kv_gather,
    card_profile_enable,
    card_profile_disable,
    card_workspace_init,
    card_profile_collect,
    card_profile_timeline,
    card_cache_create,
    card_cache_destroy,
    card_cache_write,
    card_cache_query,
    card_cache_correct,
    card_cache_epoch,
    card_cache_depth,
    card_cache_read_level,
)
from .runtime import Target, CandidateCache, make_cfg  # noqa: F401
from .loop import ConcurrentLoop, PlantedAgreement  # noqa: F401
