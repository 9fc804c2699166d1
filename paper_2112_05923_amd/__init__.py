"""MI355X-native rollout hot path of one pod (actor forward, Gaussian sampling,
vectorised stock-trading step, critic forward, GAE) behind a C-ABI library.

`inputs` holds the seeded synthetic workloads; `podrollout` is the thin ctypes
binding of the HIP library (loaded lazily, so importing this package on a
machine without the built library still works for the input generators).
"""
from . import inputs  # noqa: F401
