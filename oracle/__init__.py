"""CPU oracle (test infrastructure only).  See prom_oracle.c for what it computes.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the HIP product path never does.
"""
from .prom_oracle import (  # noqa: F401
    build, requant, requant_prelu, pw_accum, pw_conv, dw_conv, block, block_prelu, gconv3x3, gconv3x3_accum,
    max_threads,
    set_threads,
)
from .quant_oracle import (quantize_pw_absmean, quantize_dw_absmax, quantize_gconv_absmax,
                           quantize_activation_absmax, pw_conv_dynamic_quant)  # noqa: F401,E402
