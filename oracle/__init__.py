"""CPU oracle of the hierarchical-ZeRO shard-update path.

Test infrastructure, not product: only ``tests/``, ``__graft_entry__.smoke()``
and the CPU-baseline leg of ``bench.py`` may import it.  ``planner`` is plain
Python integers; ``numeric`` drives a plain scalar C file.  Neither imports,
links or reads anything of the GPU library.
"""
from . import planner  # noqa: F401
from . import numeric  # noqa: F401


def build():
    """Compile the C part of the oracle."""
    return numeric.build(force=True)
