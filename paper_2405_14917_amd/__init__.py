"""MI355X-native per-layer quantisation pass of SliM-LLM (salience-driven mixed-precision
group quantisation): hand-written gfx950 HIP kernels behind a C ABI (`libslim.so`), with a
thin ctypes binding in `paper_2405_14917_amd.binding`.

Importing the package does not load the native library; `binding.load()` does, and raises
if it has not been built.
"""

__all__ = ["binding", "synth", "build"]
