"""Shared helper of the GPU parity tests: build the variant, run it through the C ABI, download.

Precompile mode (`MS_PRECOMPILE=1` on a machine without a GPU): the helpers only build the variant, so that the
in-tree kernel cache ends up holding every kernel the GPU tests launch, and return None.  `PRECOMPILED_ONLY` records
that this happened; conftest.py then reports the test as skipped, never as passed: nothing was launched or compared.
"""
import numpy as np

from paper_2205_13603_amd import binding as B, devmem

PRECOMPILED_ONLY = False
# Every variant is launched twice into freshly poisoned outputs and the two results must agree bit for bit:
# a variant with a race between its wavefronts (a missing barrier, a buffer refilled too early) is not reproducible.
LAUNCH_TWICE = True


def _precompiled():
    global PRECOMPILED_ONLY
    PRECOMPILED_ONLY = True
    return None


def _workspace(v, instances):
    """Device buffer for variants that need one (reductions split across workgroups), else None."""
    need = v.workspace_bytes() * instances
    if not need:
        return None, None
    import torch
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)  # NaN patterns: a partial result that is read before it is written shows
    return ws, ws.data_ptr()


def _launch_checked(v, dev, out_shape, out_dtype, instances):
    keep, ws = _workspace(v, instances)
    outs = []
    for _ in range(2 if LAUNCH_TWICE else 1):
        out = devmem.empty_output(out_shape, out_dtype, instances, poison=True)
        v.launch([d.data_ptr() for d in dev], out.data_ptr(), instances=instances, stream=devmem.current_stream(), workspace=ws)
        outs.append(devmem.to_host(out, out_dtype))
    if len(outs) == 2:
        same = np.array_equal(outs[0], outs[1], equal_nan=True) if outs[0].dtype.kind == "f" else np.array_equal(outs[0], outs[1])
        assert same, "two launches of one variant on the same inputs differ (%d elements): a race inside the kernel" % int(
            np.sum(outs[0] != outs[1]))
    del keep
    return outs[0]


def run_variant(op, space, trace, inputs, out_dtype, out_shape, instances=1):
    """Returns the output as float64 / int32 numpy, or None in a precompile-only run (no GPU)."""
    v = B.Variant(op, space, trace)
    if not devmem.gpu_available():
        return _precompiled()
    dev = [devmem.to_device(a, instances) for a in inputs]
    return _launch_checked(v, dev, out_shape, out_dtype, instances)


def run_variant_distinct(op, space, trace, per_instance_inputs, out_dtype, out_shape):
    """Like run_variant, but every instance has its own inputs: per_instance_inputs[r] = list of arrays."""
    v = B.Variant(op, space, trace)
    if not devmem.gpu_available():
        return _precompiled()
    R = len(per_instance_inputs)
    dev = [devmem.to_device(np.stack([per_instance_inputs[r][k] for r in range(R)])) for k in range(len(per_instance_inputs[0]))]
    return _launch_checked(v, dev, out_shape, out_dtype, R)
