"""MI355X-native inverse of a causally masked convolution and its backpropagation.

`binding` wraps the C ABI of libinvconv.so (hand-written HIP, gfx950);
`inputs` generates the seeded synthetic workloads; `build` compiles the library.
"""
from .binding import (InvconvError, bwd_workspace_bytes, invconv_bwd, invconv_fwd,  # noqa: F401
                      invconv_logdet)
