"""MI355X-native streaming step of Inf-MLLM (arxiv 2409.09086): hand-written HIP for gfx950
behind a C ABI, with a thin ctypes binding.  Importing the package loads nothing native;
``paper_2409_09086_amd.binding`` loads the shared library on first use and fails loudly if it is
missing."""

__all__ = ["binding", "workloads"]
