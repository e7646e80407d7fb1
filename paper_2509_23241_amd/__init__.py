"""MI355X-native stage hot path of V-TiMePReSt / I-TiMePReSt.

The product is the HIP library `lib/libtimeprest_stage.so` (C ABI declared in
`include/timeprest_stage.h`).  `binding` marshals arguments into it; `runner` holds the
torch-side plumbing (device buffers, streams) used by the tests and the benchmark; `build`
compiles the library.  There is no CPU fallback: importing `binding` fails loudly if the
library has not been built.
"""
