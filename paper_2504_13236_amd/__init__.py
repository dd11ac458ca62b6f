"""MI355X-native tile-operation library for GPT-2 block training (arxiv 2504.13236).

  paper_2504_13236_amd.build   compiles csrc/*.hip into libnntile_mi.so (gfx950)
  paper_2504_13236_amd.capi    ctypes binding: one function per C entry point
  paper_2504_13236_amd.tiled   device memory for tiles (PyTorch) and array <-> tile marshalling

Importing capi or tiled needs the built library; nothing here computes on the CPU.
"""
__version__ = "0.1"
