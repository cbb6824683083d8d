"""CPU oracle for the Matryoshka-sliced quantized linear layer.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
module; it is used by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  It shares no code with the HIP path.
"""
from .mq_oracle import (  # noqa: F401
    slice_codes,
    sliced_index,
    dequant,
    linear,
    linear_rows,
    linear_stack,
)
from .mq_quant_oracle import quant_matgptq, quant_errors, matgptq_quantize  # noqa: F401,E402
