"""MI355X (gfx950) hot path of Hydra decoding behind a C ABI.

    paper_2402_05109_amd.build     compiles csrc/*.hip into libhydra.so (in-tree)
    paper_2402_05109_amd.binding   ctypes binding, same names as include/hydra.h
    paper_2402_05109_amd.session   decode-loop driver that owns the device buffers

Importing `binding` fails loudly when libhydra.so has not been built; there is
no fallback path.
"""
