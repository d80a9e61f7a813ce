"""CPU oracle (test infrastructure only; see fcco_oracle.py)."""
from .fcco_oracle import V0, V1, V2, V3, check_indices, ema_update, fcco_step, gamma_cosine  # noqa: F401
