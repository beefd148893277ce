"""Write-Gated KV hot path for AMD MI355X: thin Python binding over libwgkv.so.

All work happens in the HIP kernels of the C-ABI library (include/wgkv.h); this
package only marshals arguments.  PyTorch supplies device memory and the stream.
There is no CPU fallback: importing works anywhere, calling needs the built
library and a GPU.
"""
from .binding import (Config, Pool, WgkvError, gate_mlp_scores, gate_scores, load_library, library_path,  # noqa: F401
                      soft_attn_backward, soft_attn_forward, sparsity_loss, stream_read_probe,
                      EXPORTED_SYMBOLS, F32, BF16)
