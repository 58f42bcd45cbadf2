"""MI355X-native SACP gradient-synchronisation path (Poseidon, arXiv 1512.06216).

`binding` wraps the C-ABI HIP library; `inputs` holds the seeded synthetic workloads.
Importing the package does not load the library; the first call into `binding` does,
and fails loudly if it has not been built.
"""
__all__ = ["binding", "inputs"]
