"""fp64 CPU oracle of the Expected-Attention compress path: test infrastructure, not product.

Importable only from tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg."""
from . import ea_oracle, ea_scalar  # noqa: F401
