"""WERSA attention hot path for MI355X (gfx950): thin Python binding over the C-ABI library.

`binding` needs torch and the built shared library; `workloads` (synthetic inputs) needs
neither and is imported on its own by the CPU-side tests.
"""
