"""MI355X-native pruned prefill for 2D+3D vision-language-action backbones.

The compute path lives in the HIP library under ``csrc/`` and is reached
through :mod:`paper_2604_09244_amd.binding`.  ``workloads`` holds the seeded
synthetic input generators (no method arithmetic).  Importing the package
loads nothing native; ``binding.load()`` does, and fails loudly when the
library has not been built.
"""
__version__ = "0.1.0"
