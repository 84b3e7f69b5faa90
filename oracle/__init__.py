"""CPU oracle for the Barnes-Hut t-SNE path (test infrastructure only).

Importable from tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg; the product package never imports it.
"""
from .oracle import *  # noqa: F401,F403
from . import ivf  # noqa: F401,E402  (approximate neighbour search; numpy only)
