"""MI355X (gfx950) library for "stairs" assisted greedy generation -- Python binding.

Argument marshalling only: every step of the method runs in the HIP kernels of libstairs.so
(sources under csrc/, C ABI in include/stairs.h).  There is no CPU fallback: importing the
binding without the built library raises.
"""
from .binding import (  # noqa: F401
    LIB_PATH, StairsError, Stairs, StairsStats, lib, stairs_init, stairs_free, stairs_prefill,
    draft_propose, stairs_verify, stairs_verify_tokens, stairs_generate, stairs_decode, stairs_decode_adaptive, stairs_get_tokens, stairs_set_eos, stairs_reserve_batch, stairs_generate_batch,
    stairs_gemm_host, stairs_gemm_device, stairs_time_kernel, stairs_copy_probe, stairs_strerror, stairs_last_error, build_library,
    EXPORTED_SYMBOLS, stairs_decode_sampled, stairs_generate_sampled, draft_propose_sampled, stairs_verify_sampled, StairsEncDec, stairs_encdec_init, stairs_encode, stairs_encdec_generate, stairs_rel_bucket,
)
