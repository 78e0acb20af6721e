"""MI355X-native blended decoder-layer step (BlendServe's per-GPU hot path).

`load()` returns the ctypes binding of the C-ABI library; importing this package
does not touch the GPU, so the seeded input generators in `.workloads` can be
used on a machine without one.
"""


def load():
    from . import binding
    return binding.load()
