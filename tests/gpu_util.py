"""Shared helper of the GPU parity tests: build the variant, run it through the C ABI, download."""
from paper_2205_13603_amd import binding as B, devmem


def run_variant(op, space, trace, inputs, out_dtype, out_shape, instances=1):
    """Returns the output as float64 / int32 numpy, or None in a precompile-only run (no GPU)."""
    v = B.Variant(op, space, trace)
    if not devmem.gpu_available():
        return None
    dev = [devmem.to_device(a, instances) for a in inputs]
    out = devmem.empty_output(out_shape, out_dtype, instances, poison=True)
    v.launch([d.data_ptr() for d in dev], out.data_ptr(), instances=instances, stream=devmem.current_stream())
    return devmem.to_host(out, out_dtype)


def run_variant_distinct(op, space, trace, per_instance_inputs, out_dtype, out_shape):
    """Like run_variant, but every instance has its own inputs: per_instance_inputs[r] = list of arrays."""
    import numpy as np
    v = B.Variant(op, space, trace)
    if not devmem.gpu_available():
        return None
    R = len(per_instance_inputs)
    dev = [devmem.to_device(np.stack([per_instance_inputs[r][k] for r in range(R)])) for k in range(len(per_instance_inputs[0]))]
    out = devmem.empty_output(out_shape, out_dtype, R, poison=True)
    v.launch([d.data_ptr() for d in dev], out.data_ptr(), instances=R, stream=devmem.current_stream())
    return devmem.to_host(out, out_dtype)
