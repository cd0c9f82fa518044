"""Plumbing shared by the GPU parity tests: host <-> device copies and oracle-side views."""
import numpy as np
import torch

from oracle import keepkv_oracle as O
from paper_2504_09936_amd import workloads as W


def kk():
    from paper_2504_09936_amd import binding
    return binding


def layout_of(w):
    b = kk()
    return b.Layout(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, b.BF16 if w.dtype == "bf16" else b.F32, w.scale)


def to_device(a, dtype):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return torch.from_numpy(W.to_bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t):
    if t.dtype == torch.bfloat16:
        return W.from_bf16_bits(t.view(torch.int16).cpu().numpy().view(np.uint16))
    return t.cpu().numpy()


def new_cache(w, capacity=None, K=None, V=None, votes=None, lens=None):
    b = kk()
    lay = layout_of(w)
    c = b.Cache(lay, capacity or w.capacity)
    if K is not None:
        n = K.shape[2]
        c.k[:, :, :n] = to_device(K, w.dtype)
        c.v[:, :, :n] = to_device(V, w.dtype)
        c.votes[:, :, :n] = 1 if votes is None else torch.from_numpy(np.asarray(votes, dtype=np.int32)).cuda()
        c.len[:] = n if lens is None else torch.from_numpy(np.asarray(lens, dtype=np.int32)).cuda()
    return lay, c


def download(c):
    """GPU cache -> oracle Cache holding the same values (float64 / int64)."""
    B, H, cap, D = c.k.shape
    o = O.Cache(B, H, cap, D)
    o.k[:] = to_host(c.k)
    o.v[:] = to_host(c.v)
    o.votes[:] = c.votes.cpu().numpy()
    o.log_S[:] = c.log_s.cpu().numpy().astype(np.float64)
    o.n_obs[:] = n_obs(c).cpu().numpy()
    o.len[:] = c.len.cpu().numpy()
    return o


def n_obs(c):
    """Observation count of every slot of a GPU cache (the library stores its origin: count = t_obs - born)."""
    return c.t_obs.unsqueeze(-1) - c.born


def set_n_obs(c, n, index=None):
    """Give the slots `index` (default: all) of a GPU cache the observation counts `n` (scalar, array or tensor):
    born = t_obs - n with the heads' current step counters."""
    if not torch.is_tensor(n):
        n = torch.as_tensor(np.asarray(n, dtype=np.int32)).cuda()
    t = c.t_obs.unsqueeze(-1).expand_as(c.born)
    if index is None:
        c.born[:] = t - n
    else:
        c.born[index] = t[index] - n


def workspace(lay, capacity, budget):
    assert kk().workspace_bytes(lay, capacity, budget) > 0
    return kk().new_workspace(lay, capacity, budget)


def storage_err_rows(got, ref, dtype, slack=5e-6, return_forgiven=False):
    """Per-vector relative error of a result stored in `dtype` against the fp64 reference `ref` rounded to
    that storage.  Two correct evaluations round an element to neighbouring bf16 values when the exact
    value lies within the arithmetic's own error of the midpoint between them (one bf16 ulp is up to
    2^-7 of the element, so a single such element can exceed the vector tolerance by itself): an element
    that is adjacent to the rounded reference while the reference is within `slack` of the vector's norm
    of their midpoint counts as equal.  `slack` is the f32 accumulation error of the kernels relative to the
    vector (a few 1e-7 observed; 5e-6 allowed).  With `return_forgiven` the number of elements the rule
    applied to is returned as well, so that a test can bound it."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    r = np.asarray(W.round_storage(ref, dtype), np.float64)
    forgiven = 0
    if dtype == "bf16":
        norm = np.linalg.norm(ref, axis=-1, keepdims=True)
        adjacent = (got != r) & (np.abs(got - r) <= 2.0 ** -7 * np.abs(r) * 1.001)
        at_midpoint = np.abs(ref - 0.5 * (got + r)) <= slack * norm
        forgiven = int((adjacent & at_midpoint).sum())
        got = np.where(adjacent & at_midpoint, r, got)
    err = rel_err_rows(got, r)
    return (err, forgiven) if return_forgiven else err


def rel_err_rows(got, ref):
    """Per-vector ||got - ref||_2 / ||ref||_2 over the last axis (0 where both are 0)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    num = np.linalg.norm(got - ref, axis=-1)
    den = np.linalg.norm(ref, axis=-1)
    return np.where(den > 0, num / np.where(den > 0, den, 1), num)


def f32(x):
    """The float32 value of a Python float, as a Python float (what the C ABI receives)."""
    return float(np.float32(x))
