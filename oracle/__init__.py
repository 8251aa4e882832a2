"""CPU ORACLE: a plain, slow, fp64 statement of what one PGPE generation computes.

Test infrastructure only.  Nothing in the product path (the HIP library and its Python
binding) imports this package; it is used by tests/, by the smoke check and by the bench's
cpu_baseline leg.  It shares no code with the HIP path.
"""
from . import philox, pgpe, policy, tasks, seq2seq, generation  # noqa: F401
