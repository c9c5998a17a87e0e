"""MI355X-native expert materialization + expert FFN (FluxMoE hot path).

The compute lives in libfluxmoe.so (hand-written HIP for gfx950 behind a C ABI, declared in
include/fluxmoe.h); `binding` marshals arguments to it.  Importing this package does not
load the library; the first binding call does, and fails loudly if it was not built.
"""
