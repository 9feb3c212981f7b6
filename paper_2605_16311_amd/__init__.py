"""MI355X-native Sign-Muon optimizer hot path (libsignmuon + ctypes binding)."""
from .binding import (  # noqa: F401
    Context, SignMuonError, StepPlan, kernel_name, signmuon_majority_vote, signmuon_momentum, signmuon_momentum_noalloc,
    signmuon_polar_ns, signmuon_sign_pack, signmuon_step,
)
from . import binding  # noqa: F401
