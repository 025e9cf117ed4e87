"""MI355X-native hot path of the value-function-guided greedy scheduler of
arXiv 2011.14486 (Algorithm 1): enumerate -> featurize -> V(s) -> argmin -> commit.

``binding`` wraps the C-ABI library libvf.so (HIP, gfx950); ``inputs`` holds the seeded
synthetic workloads; ``build`` compiles the library in-tree.
"""
from . import inputs  # noqa: F401


def load():
    """Loads libvf.so and returns the binding module; raises if the library is missing."""
    from . import binding
    binding.lib()
    return binding
