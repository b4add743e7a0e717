"""MI355X (gfx950) library for the routed forward pass through quantization experts (MoQE).

`binding` exposes the C ABI of include/moqe.h; `experts` builds packed experts with it.
Importing `binding` fails if libmoqe.so has not been built: there is no fallback path.
"""
