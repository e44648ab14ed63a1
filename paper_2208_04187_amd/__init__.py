"""DIVISION activation codec for AMD MI355X: HIP kernels behind a C ABI.

compress / decompress of cached activation maps as in "DIVISION: Memory
Efficient Training via Dual Activation Precision" (Sec. 4.1 and Sec. 4.2).
"""
from .binding import (DIVISION_BF16, DIVISION_F32, DivisionError, division_compress,  # noqa: F401
                      division_compress_batch, division_decompress, division_decompress_batch, division_kernel_name, division_packed_bytes, division_packed_layout, lib)
from .autograd import DivisionDropout, DivisionMaxPool2d, DivisionReLU, division_saved_tensors  # noqa: F401,E402
from .binding import (division_dropout_forward, division_mask_backward, division_mask_bytes,  # noqa: F401,E402
                      division_relu_forward)
from .binding import division_maxpool_backward, division_maxpool_forward  # noqa: F401,E402
from .binding import (division_compress_3d, division_decompress_3d, division_kernel_name_3d,  # noqa: F401,E402
                      division_packed_bytes_3d, division_packed_layout_3d)
from .binding import division_compress_maps, division_decompress_maps  # noqa: F401,E402
from .binding import division_relu_compress, division_relu_compress_fused  # noqa: F401,E402
