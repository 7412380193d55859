"""Helpers shared by the GPU parity tests: moving bits between torch (device) and
numpy (oracle) without changing them."""
import numpy as np
import torch


def storage_np(t: torch.Tensor) -> np.ndarray:
    """Underlying storage of a (possibly strided) tensor as a flat numpy array on the host."""
    n = t.untyped_storage().nbytes() // t.element_size()
    flat = torch.as_strided(t, (n,), (1,), 0)
    return flat.cpu().numpy()


def u8(t):
    return t.cpu().numpy().view(np.uint8)


def u16(t):
    return t.contiguous().cpu().numpy().view(np.uint16)


def u32(t):
    return t.contiguous().cpu().numpy().view(np.uint32)


def u64(t):
    return t.contiguous().cpu().numpy().view(np.uint64)


def oracle_dims(O, w, S=None, L=None, H=None):
    return O.make_dims(S or w.S, L or w.L, H or w.H, w.n, w.k, w.d, w.delta, w.qmax,
                       cand_stride=w.cand_k.stride()[:5], act_stride=w.act_k.stride()[:4])


def codec_for(w, **kw):
    from paper_2604_15356_amd.codec import KVDeltaCodec
    return KVDeltaCodec(w.S, w.L, w.H, w.n, w.k, w.d, w.delta, w.qmax,
                        cand_stride=w.cand_k.stride()[:5], act_stride=w.act_k.stride()[:4], **kw)


def near_tie_report(sym_gpu, sym_f64, u_f64, tau):
    """Classifies symbol differences between an fp32 decision and the fp64 oracle.
    Returns (n_diff, n_explained): a difference is explained if it is one step (or
    in/out of the escape range by one step) and u lies within tau of a half-integer."""
    diff = sym_gpu != sym_f64
    n_diff = int(diff.sum())
    if n_diff == 0:
        return 0, 0
    u = u_f64[diff]
    frac = np.abs(u - np.floor(u) - 0.5)
    a = sym_gpu[diff].astype(np.int64)
    b = sym_f64[diff].astype(np.int64)
    one_step = (np.abs(a - b) == 1) | ((a == 255) & (b >= 253)) | ((b == 255) & (a >= 253)) \
        | ((a == 255) & (b <= 1)) | ((b == 255) & (a <= 1))
    return n_diff, int(((frac < tau) & one_step).sum())
