"""MI355X-native Adam-mini optimizer step (arXiv 2406.16793).

``binding`` is the thin ctypes layer over the C ABI declared in
``include/adam_mini.h``; ``partition`` turns named tensor shapes into block
descriptors (the paper's "Partition for Transformers", Appendix B); ``workloads`` holds the seeded synthetic
benchmark configurations.  Importing the package does not load the HIP library;
the first use of ``binding`` does, and raises if it has not been built.
"""
__all__ = ["binding", "device_state", "partition", "workloads"]
