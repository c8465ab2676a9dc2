"""fp64 CPU oracle (test infrastructure only; never imported by the product path)."""
from .rolling_attention import (  # noqa: F401
    RollingCacheOracle,
    RingTableSim,
    rope_angles,
    rope_rotate,
    round_to_bf16,
    visible_history,
)
from .nft_loss import nft_loss, normalized_reward  # noqa: F401,E402
