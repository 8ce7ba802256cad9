"""MI355X-native paged GQA decode + KV append for SpeechLM serving.

The package holds the HIP kernels (``csrc/``), the build helper, the thin
``ctypes`` binding to the C-ABI library (``binding``) and the seeded synthetic
workload generators (``synth``).  Nothing is imported eagerly: ``synth`` is
usable without the HIP library, and ``binding`` fails loudly if the library
has not been built.
"""

__all__ = ["binding", "build", "synth"]
