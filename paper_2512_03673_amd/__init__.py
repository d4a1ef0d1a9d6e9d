"""libconvrot: the ConvLinear4bit forward path (ConvRot, arXiv 2512.03673) for AMD MI355X.

``binding`` wraps the C ABI of ``libconvrot.so`` (hand-written HIP for gfx950, built by
``python -m paper_2512_03673_amd.build``); ``workloads`` draws the seeded synthetic inputs.
The binding is imported lazily so that the input generator works without torch or the library.
"""
__all__ = ["binding", "workloads", "build"]
