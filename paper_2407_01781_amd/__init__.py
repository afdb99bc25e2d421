"""MI355X-native hot path of fVDB's sparse 3-D networks: index-grid build, kernel map,
sparse convolution forward and backward, transposed convolution, pooling and upsampling (HIP library +
ctypes binding)."""
from .binding import (FxError, IndexGrid, KernelMap, build_index_grid, build_index_grid_from_points, build_kernel_map, build_kernel_map_onto, get_option, set_option, use_torch_allocator,  # noqa: F401
                      pool2, pool2_bwd, profile_enable, profile_read, profile_reset, sparse_conv_bwd_data,
                      sparse_conv_bwd_weight, sparse_conv_fwd, sparse_conv_fwd_noalloc, sparse_conv_leaf_bwd_data, sparse_conv_leaf_bwd_weight, sparse_conv_leaf_fwd, sparse_conv_transpose_fwd,
                      upsample2, upsample2_bwd, version)
