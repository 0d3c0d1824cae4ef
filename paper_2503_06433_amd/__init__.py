"""MI355X (gfx950) hot path of re-sharded LLM inference: a decoder layer in the
pipeline-parallel (prefill) and tensor-parallel (decode) layouts and the KV-cache
movement between them through a host tier.  All compute runs in the HIP library
`libseesaw_rt.so`; this package only marshals arguments (see binding.py)."""
from .binding import (  # noqa: F401
    SS_F32, SS_BF16, SS_F16, SS_PP, SS_TP, SS_ATTN, SS_MLP, SS_BOTH, SS_NO_RESIDUAL, SS_OUT, SS_IN,
    SS_HOST, SS_DEVICE, SS_OK, SS_EINVAL, SS_ENOMEM, SS_ENOENT, SS_EHIP,
    SeesawError, ModelCfg, RuntimeCfg, ShardDesc, OfflineCfg, OfflineStats, Context, load_library, library_path,
)
