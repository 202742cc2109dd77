"""PyTorch glue: device memory and streams only.  All data movement happens in
libamap.so; nothing here computes, and there is no CPU fallback."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B

_TORCH_DT = {2: torch.int16, 4: torch.int32}
_NP_DT = {2: np.uint16, 4: np.uint32}
_NP_SIGNED = {2: np.int16, 4: np.int32}


def require_gpu() -> torch.device:
    if not torch.cuda.is_available():
        raise RuntimeError("amap needs a GPU: the HIP path has no CPU fallback")
    return torch.device("cuda:0")


def to_device(bits: np.ndarray) -> torch.Tensor:
    """Opaque element bits (uint16 / uint32 ndarray) -> device tensor of the same bits."""
    es = bits.dtype.itemsize
    return torch.from_numpy(np.ascontiguousarray(bits).view(_NP_SIGNED[es])).to(require_gpu())


def to_host(t: torch.Tensor) -> np.ndarray:
    es = t.element_size()
    return t.cpu().numpy().view(_NP_DT[es])


def empty_dst(m, fill=None) -> torch.Tensor:
    info = B.amap_describe(m)
    shape = tuple(info.shape[k] for k in range(info.rank))
    t = torch.empty(shape, dtype=_TORCH_DT[info.elem_size], device=require_gpu())
    if fill is not None:
        t.fill_(fill)
    return t


def current_stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def execute(m, srcs, dst=None, kernel_id=None, stream=None) -> torch.Tensor:
    """dst <- map(srcs) on the current stream; returns dst (allocated if None)."""
    if dst is None:
        dst = empty_dst(m)
    ptrs = [0 if s is None else s.data_ptr() for s in srcs]
    B.amap_execute(ptrs, dst.data_ptr(), m, current_stream() if stream is None else stream, kernel_id)
    return dst


def execute_multi(maps, srcs, dsts=None, stream=None):
    """dsts[i] <- maps[i](srcs), all maps in shared launches; returns the dst tensors."""
    if dsts is None:
        dsts = [empty_dst(m) for m in maps]
    B.amap_execute_multi([0 if s is None else s.data_ptr() for s in srcs], [d.data_ptr() for d in dsts], maps,
                         current_stream() if stream is None else stream)
    return dsts


def gemm_fused(a_src: torch.Tensor, a_map, w: torch.Tensor, out=None, stream=None, out_map=None) -> torch.Tensor:
    """out = A x W with A read through a_map; with out_map the product is stored through
    that map (out then has out_map's dst shape)."""
    info = B.amap_describe(a_map)
    n = w.shape[1]
    if out is None:
        shape = (info.shape[0], n) if out_map is None else B.dst_shape(out_map)
        out = torch.empty(shape, dtype=torch.int16, device=require_gpu())
    st = current_stream() if stream is None else stream
    if out_map is None:
        B.amap_gemm_fused(a_src.data_ptr(), a_map, w.data_ptr(), n, out.data_ptr(), st)
    else:
        B.amap_gemm_fused_store(a_src.data_ptr(), a_map, w.data_ptr(), n, out_map, out.data_ptr(), st)
    return out
