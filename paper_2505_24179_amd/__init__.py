"""MI355X-native SALE prefill attention path (arXiv 2505.24179).

`paper_2505_24179_amd.sale` is the binding over the C-ABI library (it raises
at import if the built library is missing); `paper_2505_24179_amd.inputs`
makes the seeded synthetic workloads.  Nothing is imported eagerly here so the
input generator stays usable on a machine without the built library.
"""

__all__ = ["inputs", "sale"]
