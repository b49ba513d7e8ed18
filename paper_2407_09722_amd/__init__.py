"""MI355X-native hot path of multi-token assisted decoding (MTAD / MMTAD, arXiv 2407.09722).

csrc/      hand-written HIP kernels for gfx950 and the C ABI (include/mtad.h) -> libmtad.so
binding    ctypes binding with the C names (argument marshalling only)
engine     torch allocations + the call sequence of one iteration
build      in-tree build of libmtad.so
"""
