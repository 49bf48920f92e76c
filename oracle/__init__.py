"""CPU oracle for the W8A8 / W4A8 quantized linear layer -- TEST INFRASTRUCTURE.

A plain, slow, obviously-correct implementation of what the hot path computes,
written from the paper's definitions (its Eq. 1-2 quantizer, the per-token /
per-channel / group-wise granularities of its Preliminary section, the
symmetric setting of its Experimental Setup, and Y = XW of its Eq. 3), plus the
two operand transforms of its W4A8 variants (SmoothQuant, Eq. 3; Hadamard rotation, Eq. 4)
and the other quantizer forms of its Preliminary section (Eq. 2 as printed, per-tensor
granularity, a calibrated static activation scale), and an RMSNorm and a SwiGLU in front of the activation
quantizer (textbook definitions; the paper does not spell out the normalisation or the gated MLP of its decoder
layers).

Only tests, the smoke check and the benchmark's cpu_baseline leg may use this
package.  It shares no code with the HIP path and imports nothing from it.

Parity pins: every function here is pinned by tests/test_oracle_*.py against
hand-derived vectors (tests/golden/), closed forms, brute force in exact
Python arithmetic and an exact float64-BLAS integer product.  No function is
"parity unpinned".
"""
from .quantizers import (  # noqa: F401
    quant_act_per_token,
    quant_weight_int8,
    quant_weight_int4,
    pack_int4,
    unpack_int4,
    quant_eq2_literal,
    quant_act_opt,
    quant_weight_opt,
    act_scale_calibrate,
    scale_from_amax,
    RANGE_SYMMETRIC,
    RANGE_EQ2,
    SCOPE_FINE,
    SCOPE_TENSOR,
    SCOPE_STATIC,
)
from .linear import igemm, igemm_grouped, linear_w8a8, linear_w4a8  # noqa: F401
from .transforms import (  # noqa: F401
    channel_absmax,
    smooth_scales,
    smooth_act,
    smooth_weight,
    hadamard_block,
    fwht_blocks,
    rmsnorm_act,
    swiglu_act,
    exp_f32_steps,
)
