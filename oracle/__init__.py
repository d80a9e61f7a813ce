"""CPU oracle (test infrastructure only; see fcco_oracle.py)."""
from .fcco_oracle import (ADAMW, LAMB, LION, SGDM, V0, V1, V2, V3, check_indices, ema_update, fcco_step,  # noqa: F401
                          gamma_cosine, normalize_rows, parameter_update, temperature_update)
