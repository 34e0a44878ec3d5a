"""Host <-> device plumbing shared by the GPU tests: numpy in, numpy out, through the C ABI."""
import numpy as np
import torch

from paper_2410_12707_amd import binding as B


def torch_dtype(np_dtype) -> torch.dtype:
    """float32 -> float32, float16 -> float16, uint16 (bf16 bit patterns) -> bfloat16."""
    return {np.dtype(np.float32): torch.float32, np.dtype(np.float16): torch.float16,
            np.dtype(np.uint16): torch.bfloat16}[np.dtype(np_dtype)]


def to_device(x: np.ndarray, offset_elems: int = 0) -> torch.Tensor:
    """float32 and float16 keep their type; uint16 bit patterns become a bfloat16 tensor.
    offset_elems > 0 places the tensor that many elements past a fresh allocation (a misaligned base)."""
    x = np.ascontiguousarray(x).reshape(-1)
    tdt = torch_dtype(x.dtype)
    host = torch.from_numpy(x.view(np.int16)).view(torch.bfloat16) if x.dtype == np.uint16 else torch.from_numpy(x)
    buf = torch.empty(x.size + offset_elems, dtype=tdt, device="cuda")
    view = buf[offset_elems:]
    view.copy_(host)
    return view


def to_host(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def bits(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.float32:
        return a.view(np.uint32)
    return a.view(np.uint16) if a.dtype != np.uint16 else a


def gpu_compress(x: np.ndarray, k: int, offset_elems: int = 0, want_err: bool = True):
    d = to_device(x, offset_elems)
    idx = torch.full((max(k, 1),), -7, dtype=torch.int32, device="cuda")
    val = torch.zeros(max(k, 1), dtype=d.dtype, device="cuda")
    err = torch.full((1,), -1.0, dtype=torch.float32, device="cuda") if want_err else None
    ws = B.new_workspace(d.numel(), 1, d.dtype)
    B.adatopk_compress(d, k, idx, val, err, ws)
    torch.cuda.synchronize()
    return to_host(idx)[:k], to_host(val)[:k], (to_host(err)[0] if want_err else None)


def gpu_decompress(idx: np.ndarray, val: np.ndarray, n: int, offset_elems: int = 0, sorted_call: bool = False) -> np.ndarray:
    k = int(idx.size)
    di = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).cuda() if k else torch.zeros(1, dtype=torch.int32, device="cuda")
    dv = to_device(val) if k else torch.zeros(1, dtype=torch_dtype(val.dtype), device="cuda")
    buf = torch.full((n + offset_elems + 8,), 7.0, dtype=dv.dtype, device="cuda")  # poisoned; 8 guard elements
    out = buf[offset_elems:offset_elems + n]
    (B.adatopk_decompress_sorted if sorted_call else B.adatopk_decompress)(di, dv, k, out)
    torch.cuda.synchronize()
    guard = to_host(buf[offset_elems + n:])
    assert np.all(bits(guard) == bits(to_host(torch.full((8,), 7.0, dtype=dv.dtype)))), "decompress wrote past n"
    if offset_elems:
        head = to_host(buf[:offset_elems])
        assert np.all(bits(head) == bits(to_host(torch.full((offset_elems,), 7.0, dtype=dv.dtype)))), "wrote before base"
    return to_host(out)


def gpu_compress_segmented(xs, ks, want_err: bool = True):
    ds = [to_device(x) for x in xs]
    S = len(xs)
    off = np.zeros(S + 1, dtype=np.int64)
    off[1:] = np.cumsum(np.asarray(ks, dtype=np.int64))
    tot = int(off[S])
    tdt = ds[0].dtype if S else torch.float32
    idx = torch.full((max(tot, 1),), -7, dtype=torch.int32, device="cuda")
    val = torch.zeros(max(tot, 1), dtype=tdt, device="cuda")
    err = torch.full((max(S, 1),), -1.0, dtype=torch.float32, device="cuda") if want_err else None
    ws = B.new_workspace(sum(d.numel() for d in ds), max(S, 1), tdt)
    B.adatopk_compress_segmented(ds, ks, idx, val, off.tolist(), err, ws)
    torch.cuda.synchronize()
    return to_host(idx)[:tot], to_host(val)[:tot], off, (to_host(err)[:S] if want_err else None)


def gpu_decompress_segmented(idx: np.ndarray, val: np.ndarray, off, ns):
    """One segmented decompress call into poisoned buffers with guard elements; returns the S tensors."""
    S = len(ns)
    tot = int(off[S])
    tdt = torch_dtype(val.dtype)
    di = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).cuda() if tot else torch.zeros(1, dtype=torch.int32, device="cuda")
    dv = to_device(val) if tot else torch.zeros(1, dtype=tdt, device="cuda")
    bufs = [torch.full((n + 8,), 7.0, dtype=tdt, device="cuda") for n in ns]
    B.adatopk_decompress_segmented(di, dv, [int(v) for v in off], [b[:n] for b, n in zip(bufs, ns)])
    torch.cuda.synchronize()
    poison = bits(to_host(torch.full((8,), 7.0, dtype=tdt)))
    outs = []
    for b, n in zip(bufs, ns):
        assert np.all(bits(to_host(b[n:])) == poison), "segmented decompress wrote past a tensor"
        outs.append(to_host(b[:n]))
    return outs


def same_err(e_gpu, e_ref, rtol=1e-5) -> bool:
    e_gpu, e_ref = float(e_gpu), float(e_ref)
    if np.isnan(e_ref) or np.isinf(e_ref):
        return (np.isnan(e_gpu) and np.isnan(e_ref)) or (e_gpu == e_ref)
    return abs(e_gpu - e_ref) <= rtol * abs(e_ref)
