"""MI355X (gfx950) hot path of signSGD / Signum with majority vote
(arxiv 1802.04434, Algorithms 1-3): thin Python binding over the C-ABI HIP
library declared in include/signsgd.h.

Argument marshalling only: every step of the path runs in the library's
kernels.  torch is used for device memory and the current stream.  There is
no CPU fallback: if the built library is missing, every call raises.
"""
from .binding import (  # noqa: F401
    BF16, F32, MAX_WORKERS, STEP_DEFAULT, STEP_SUM_UPDATE, STEP_WARMUP, SignSGDError,
    last_hip_error, library_path, load_library, majority_vote, new_bits, packed_bytes,
    packed_words, sign_apply, signum_pack, signum_pack_warmup, signum_vote_step,
    signum_vote_step_ex, stream_copy, sum_apply, vote_sum, warmup_length,
    density, density_static, new_density_workspace, welford_sigma, welford_update,
    quorum_vote, signum_pack_ternary, signum_vote_step_ternary, ternary_apply,
)
