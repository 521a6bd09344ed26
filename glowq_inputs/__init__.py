"""Seeded synthetic inputs for the GlowQ group forward.

This package only draws random numbers and lists workload shapes.  It holds
none of the method's arithmetic (no quantiser, no packing, no factorisation,
no forward): the CPU oracle and the HIP library both consume the bytes made
here, and neither of them is imported from here.
"""
from .synth import (  # noqa: F401
    CONFIGS,
    UnitShape,
    config_units,
    gen_module_weight,
    gen_activations,
    gen_restore_mask,
    gen_direct_unit,
    gen_direct_layerwise_B,
    to_act_bits,
    from_act_bits,
)
