"""CPU oracle of the IntSGD step -- test infrastructure only.

Importable from tests/, the smoke check and bench.py's cpu_baseline leg; the
product package never imports it.
"""
from .oracle import *  # noqa: F401,F403
