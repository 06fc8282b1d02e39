"""MI355X-native training-time-test (TTT) attention: thin Python face of the C-ABI HIP library."""
from .binding import (  # noqa: F401
    TTT_BF16, TTT_F32, TTT_MAX_STEPS, TTT_PASS_BWD, TTT_PASS_BWD_ACCUM, TTT_PASS_FWD,
    TttAttnError, TttAttnParams, load_library, make_params,
    ttt_attn_bwd, ttt_attn_fwd, ttt_attn_last_error, ttt_attn_workspace_bytes,
)
from .runner import TttAttnRunner  # noqa: F401
