"""MI355X-native decode path for Direct Multi-Token Decoding: ctypes binding over libdmtd.so."""
from .binding import (DMTD_ECAPACITY, DMTD_EHIP, DMTD_EINVAL, DMTD_ESTATE, DMTD_OK, DmtdError, Engine, ModelConfig,
                      load_library)

__all__ = ["Engine", "ModelConfig", "DmtdError", "load_library", "DMTD_OK", "DMTD_EINVAL", "DMTD_ESTATE",
           "DMTD_ECAPACITY", "DMTD_EHIP"]
