"""Seeded synthetic inputs (record layouts + capture-archive generator) used by tests,
bench and the smoke check.  Holds no step of the method itself."""
from . import layout  # noqa: F401
from .archive import Archive, make_config, CONFIG_NAMES  # noqa: F401
from .problem import MatProblem  # noqa: F401
