"""Device memory and stream plumbing through PyTorch (no arithmetic here)."""
import numpy as np
import torch


def gpu_available():
    return torch.cuda.is_available()


def require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
    return torch.device("cuda:0")


def to_device(arr, instances=1):
    """Upload a numpy array (uint16 = bf16 bit patterns); `instances` > 1 stacks that many copies."""
    a = np.ascontiguousarray(arr)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    t = torch.from_numpy(a).to(require_gpu())
    if instances > 1:
        t = t.unsqueeze(0).expand(instances, *t.shape).contiguous()
    return t


_OUT_DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.int16, "i32": torch.int32}


def empty_output(shape, dtype, instances=1, poison=False):
    """Uninitialised output; poison=True pre-fills with NaN (floats) or a sentinel (i32)."""
    shp = tuple(shape) if instances == 1 else (instances,) + tuple(shape)
    t = torch.empty(shp, dtype=_OUT_DTYPES[dtype], device=require_gpu())
    if poison:
        t.fill_({"bf16": 0x7FC0, "i32": -123456789}.get(dtype, float("nan")))
    return t


def to_host(t, dtype):
    """Download; returns float64 for float outputs (bf16 decoded from bits), int32 for i32."""
    torch.cuda.synchronize()
    a = t.cpu().numpy()
    if dtype == "bf16":
        return (a.view(np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if dtype == "i32":
        return a
    return a.astype(np.float64)


def current_stream():
    return torch.cuda.current_stream().cuda_stream
