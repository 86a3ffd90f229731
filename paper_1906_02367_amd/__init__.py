"""MI355X-native compression hot path of Qsparse-local-SGD (arXiv:1906.02367).

`paper_1906_02367_amd.binding` is the Python face of the C-ABI library (it loads the HIP
library and fails loudly if it has not been built); `paper_1906_02367_amd.workloads` holds the
seeded synthetic inputs.  Nothing is imported eagerly so that the input generators can be used
on a machine without the GPU library.
"""
__all__ = ["binding", "workloads", "build"]
