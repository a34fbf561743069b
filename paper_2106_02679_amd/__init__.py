"""MI355X-native layered gradient accumulation over a GPT layer stack (arxiv 2106.02679, section 3).

The product is `liblga.so` (HIP kernels + C ABI, sources in csrc/, contract in include/lga.h);
`binding` is its thin ctypes wrapper.  Build with `python -m paper_2106_02679_amd.build`.
"""
