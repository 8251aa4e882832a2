"""MI355X-native hot path of EvoJAX-style neuroevolution: one PGPE generation on the GPU.

The product is the C-ABI library built from csrc/ (see include/evo.h); this package is
its thin ctypes binding, plus a small host-side training shell (trainer.py).  There is no CPU
fallback."""
from .api import *  # noqa: F401,F403
from .api import PGPE, EvoError  # noqa: F401
