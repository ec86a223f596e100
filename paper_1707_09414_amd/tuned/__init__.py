"""Tuning tables measured on hardware, shipped with the package.

``mi355x.txt`` (if present) is what ``bcast_tune`` wrote on an MI355X for the
rank counts of the benchmark workloads; ``load_default_table`` installs it into
the library's process-wide table so that AUTO plans and chain plans with
``chunk_bytes == 0`` use measured choices."""
from __future__ import annotations

from pathlib import Path
from typing import Optional

DEFAULT_TABLE = Path(__file__).resolve().parent / "mi355x.txt"


def load_default_table() -> Optional[str]:
    """Install the shipped table; returns its path, or None if there is none."""
    from .. import binding

    if DEFAULT_TABLE.exists():
        binding.bcast_tune_load(str(DEFAULT_TABLE))
        return str(DEFAULT_TABLE.name)
    return None
