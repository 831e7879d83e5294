"""MI355X-native hybrid-batch attention (prefill chunks and decodes in one launch).

``paper_2410_18038_amd.pod`` is the thin binding over the C-ABI library built from
``csrc/``; ``paper_2410_18038_amd.workloads`` makes seeded synthetic batches.  The
binding loads the HIP library on first use and raises if it has not been built.
"""
__all__ = ["pod", "workloads", "build"]
