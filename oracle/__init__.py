"""CPU oracle for the AdaSD verification path -- TEST INFRASTRUCTURE ONLY.

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It never imports the GPU package and the
GPU package never imports it.
"""
from .pyoracle import Oracle, build_oracle, load_oracle, new_state  # noqa: F401
