"""MI355X-native scoring / selection / online update of the AutoByte meta-network.

``paper_2112_13509_amd.binding`` is the thin ctypes layer over the C-ABI library built from
``csrc/``; ``paper_2112_13509_amd.workloads`` draws seeded synthetic inputs.  Importing the package
loads nothing; the binding loads the HIP library on first use and raises if it is missing.
"""
__all__ = ["binding", "workloads"]
