"""MI355X-native chunked mixed-precision AdamW update (the GPU optimizer step of
AutoHete-style heterogeneous training).  The product is libautohete.so (HIP, gfx950) behind
the C ABI in include/autohete.h; `binding` marshals arguments to it and nothing else."""
