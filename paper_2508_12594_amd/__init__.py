"""MI355X-native FLARE token mixer (encode-decode low-rank attention) behind a C ABI.

`synth` draws the seeded synthetic workloads; `binding` marshals arguments into
libflare.so (hand-written HIP kernels for gfx950); `autograd` wraps the two calls in a
torch.autograd.Function.  Importing the package loads nothing
native; the first call into `binding` does, and raises if the library is missing.
"""
__all__ = ["synth", "binding", "autograd"]
