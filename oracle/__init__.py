"""CPU oracle for the ternary 3D convolution (test infrastructure, not the product).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
"""
from .tern_oracle import (  # noqa: F401
    ConvGeom,
    conv3d,
    conv3d_points,
    fcn_forward,
    max_threads,
    out_dims,
    pack,
    set_threads,
    threshold,
    unpack,
)
from .prepare_oracle import (activation_code, bn_affine, ternarize_filters,  # noqa: F401,E402
                             ternarize_filters_sparse)
from .unet_oracle import (  # noqa: F401,E402
    centre_crop,
    concat_channels,
    conv3d_real,
    count_codes,
    pool_digits,
    pool_sum,
    unet_forward,
    upsample_nearest,
)
