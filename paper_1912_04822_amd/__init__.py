"""MI355X-native atom-to-grid path of libmolgrid (arXiv 1912.04822).

``paper_1912_04822_amd.molgrid`` is the thin Python binding over the C-ABI HIP
library (``csrc/``); ``paper_1912_04822_amd.autograd`` wires forward and backward into
``torch.autograd``; ``paper_1912_04822_amd.workloads`` draws seeded synthetic inputs.  Importing the
package does not load the HIP library; the binding does so on first use and
raises if it is missing.
"""

__all__ = ["molgrid", "autograd", "workloads"]
