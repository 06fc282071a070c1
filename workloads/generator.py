"""Counter-based seeded tensor generator, bit-identical on CPU and GPU.

Every element is a pure function of (stream key, flat element index), so any
slice of any tensor can be regenerated alone: the GPU bench fills whole
[S, H, T, d] tensors on the device while a CPU test regenerates just the
(sequence, head) units it wants to hand to the oracle, and both hold the same
bits.  Only integer ops, table lookups and single IEEE float ops are used, so
the result does not depend on the device or on its math library.

Streams:  64-bit hash of (key + counter) -> four 16-bit uniforms -> lookup in a
65536-entry table of standard-normal quantiles.

This module holds none of the method's arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Sequence, Tuple

import torch

from .configs import WorkloadConfig, c_full, stream_key

_TABLES: Dict[str, torch.Tensor] = {}

# tensor ids for stream_key
_T_G_Q, _T_G_K, _T_G_V = 1, 2, 3
_T_U_Q, _T_U_K, _T_U_V = 4, 5, 6
_T_W_QK, _T_W_V = 7, 8
_T_CHI = 9
_T_SIGN = 10
_T_BOOST = 11


def _signed64(x: int) -> int:
    x &= (1 << 64) - 1
    return x - (1 << 64) if x >= (1 << 63) else x


_C_GOLD = _signed64(0x9E3779B97F4A7C15)
_C_M1 = _signed64(0xBF58476D1CE4E5B9)
_C_M2 = _signed64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """logical shift right of an int64 tensor"""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _hash64(key: int, ctr: torch.Tensor) -> torch.Tensor:
    """splitmix64: z = key + (ctr+1)*golden, then the output mix.  int64
    arithmetic wraps mod 2^64 on every torch device."""
    z = (ctr + 1) * _C_GOLD + _signed64(key)
    z = (z ^ _lsr(z, 30)) * _C_M1
    z = (z ^ _lsr(z, 27)) * _C_M2
    return z ^ _lsr(z, 31)


def _uniform16(key: int, start: int, count: int, device) -> torch.Tensor:
    """16-bit uniforms number start .. start+count-1 of stream `key` (int64)."""
    first = start // 4
    last = (start + count + 3) // 4
    ctr = torch.arange(first, last, dtype=torch.int64, device=device)
    z = _hash64(key, ctr)
    # the four 16-bit lanes of every hash word, written into a tensor allocated beforehand (no
    # concatenation kernel: element-wise writes only)
    u = torch.empty(z.shape[0], 4, dtype=torch.int64, device=device)
    u[:, 0] = z & 0xFFFF
    u[:, 1] = _lsr(z, 16) & 0xFFFF
    u[:, 2] = _lsr(z, 32) & 0xFFFF
    u[:, 3] = _lsr(z, 48) & 0xFFFF
    u = u.reshape(-1)
    off = start - 4 * first
    return u[off: off + count]


def _normal_table(device) -> torch.Tensor:
    dev = str(torch.device(device))
    if dev not in _TABLES:
        p = (torch.arange(65536, dtype=torch.float64) + 0.5) / 65536.0
        _TABLES[dev] = torch.special.ndtri(p).to(torch.float32).to(device)
    return _TABLES[dev]


def normal_tensor(key: int, shape: Sequence[int], device="cpu", start: int = 0) -> torch.Tensor:
    """fp32 standard-normal draws (65536-level quantile table), elements
    start .. start+prod(shape)-1 of the stream."""
    n = 1
    for s in shape:
        n *= int(s)
    u = _uniform16(key, start, n, device)
    return _normal_table(device)[u].reshape(*shape)


def sign_tensor(key: int, shape: Sequence[int], device="cpu", start: int = 0) -> torch.Tensor:
    """fp32 +-1 draws."""
    n = 1
    for s in shape:
        n *= int(s)
    u = _uniform16(key, start, n, device)
    return ((u & 1) * 2 - 1).to(torch.float32).reshape(*shape)


def student_t_tensor(key_z: int, key_chi: int, shape: Sequence[int], device="cpu", start: int = 0) -> torch.Tensor:
    """Student-t with 3 degrees of freedom scaled to unit variance:
    z / sqrt(chi2_3 / 3) / sqrt(3), chi2_3 from three more normals."""
    n = 1
    for s in shape:
        n *= int(s)
    z = normal_tensor(key_z, (n,), device, start)
    c = normal_tensor(key_chi, (n, 3), device, 3 * start)
    chi = (c[:, 0] * c[:, 0] + c[:, 1] * c[:, 1]) + c[:, 2] * c[:, 2]
    t = z / torch.sqrt(chi / 3.0)
    return (t * 0.57735026918962576).reshape(*shape)


def _to_dtype(x: torch.Tensor, cfg: WorkloadConfig) -> torch.Tensor:
    return x if cfg.dtype == "f32" else x.to(torch.bfloat16)


def _units(cfg: WorkloadConfig, units: Optional[Sequence[int]]):
    if units is None:
        return None
    return [int(u) for u in units]


def _stack(parts, tail_shape, device, dtype=torch.float32):
    """the parts along a new leading axis, written one by one into a tensor allocated beforehand"""
    out = torch.empty(len(parts), *tail_shape, dtype=dtype, device=device)
    for i, p in enumerate(parts):
        out[i] = p
    return out


def _per_token(key: int, cfg: WorkloadConfig, n_tok: int, width: int, device, units, kind="normal"):
    """[S,H,n_tok,width] tensor of stream `key`, or [len(units),n_tok,width]
    for the listed flat unit ids u = s*H + h (same bits as the full tensor)."""
    gen = normal_tensor if kind == "normal" else sign_tensor
    if units is None:
        return gen(key, (cfg.n_seq, cfg.n_head, n_tok, width), device)
    per = n_tok * width
    parts = [gen(key, (n_tok, width), device, start=u * per) for u in units]
    return _stack(parts, (n_tok, width), device)


def _per_head(key: int, cfg: WorkloadConfig, rows: int, width: int, device, units):
    """[1,H,rows,width] (broadcast over sequences) or [len(units),rows,width]."""
    w = normal_tensor(key, (cfg.n_head, rows, width), device)
    if units is None:
        return w.unsqueeze(0)
    idx = torch.tensor([u % cfg.n_head for u in units], dtype=torch.int64, device=device)
    return w[idx]


_INV_SQRT8 = 0.35355339059327373


def _add_lowrank(g: torch.Tensor, u: torch.Tensor, w: torch.Tensor) -> torch.Tensor:
    """g + (1/sqrt 8) * u @ w written as eight rank-1 updates of single IEEE
    multiplies and adds (no fused multiply-add, no library matmul), so the bits
    do not depend on the device."""
    acc = g
    for r in range(u.shape[-1]):
        term = u[..., r: r + 1] * w[..., r: r + 1, :]
        term = term * _INV_SQRT8
        acc = acc + term
    return acc


@dataclass
class StepInputs:
    q: torch.Tensor       # [S,H,n_k,d] (or [U,n_k,d] when units were listed)
    k_cur: torch.Tensor
    v_cur: torch.Tensor


def _qkv(cfg: WorkloadConfig, layer: int, scale: int, n_tok: int, device, units) -> Tuple[torch.Tensor, ...]:
    d, s = cfg.head_dim, cfg.seed
    gq = _per_token(stream_key(s, _T_G_Q, layer, scale), cfg, n_tok, d, device, units)
    gk = _per_token(stream_key(s, _T_G_K, layer, scale), cfg, n_tok, d, device, units)
    gv = _per_token(stream_key(s, _T_G_V, layer, scale), cfg, n_tok, d, device, units)
    if cfg.recipe == "iid_small":
        # N(0,1)/sqrt(64): tiny logits, near-uniform softmax, many near-ties.
        q, k, v = gq * 0.125, gk * 0.125, gv * 0.125
    elif cfg.recipe == "lowrank8":
        # Q and K share one rank-8 subspace per (layer, head) so the logits have
        # std ~4 and attention is peaked; V gets its own.
        w = _per_head(stream_key(s, _T_W_QK, layer), cfg, 8, d, device, units)
        wv = _per_head(stream_key(s, _T_W_V, layer), cfg, 8, d, device, units)
        uq = _per_token(stream_key(s, _T_U_Q, layer, scale), cfg, n_tok, 8, device, units)
        uk = _per_token(stream_key(s, _T_U_K, layer, scale), cfg, n_tok, 8, device, units)
        uv = _per_token(stream_key(s, _T_U_V, layer, scale), cfg, n_tok, 8, device, units)
        q, k, v = _add_lowrank(gq, uq, w), _add_lowrank(gk, uk, w), _add_lowrank(gv, uv, wv)
    elif cfg.recipe == "student_t3":
        # heavy-tailed keys stress near-ties and fp32 underflow of exp().
        kz = stream_key(s, _T_G_K, layer, scale)
        kc = stream_key(s, _T_CHI, layer, scale)
        if units is None:
            k = student_t_tensor(kz, kc, (cfg.n_seq, cfg.n_head, n_tok, d), device)
        else:
            per = n_tok * d
            k = _stack([student_t_tensor(kz, kc, (n_tok, d), device, start=u * per) for u in units], (n_tok, d), device)
        q, v = gq, gv
    else:
        raise ValueError(cfg.recipe)
    return _to_dtype(q, cfg), _to_dtype(k, cfg), _to_dtype(v, cfg)


def make_step_inputs(cfg: WorkloadConfig, layer: int, scale: int, device="cpu",
                     units: Optional[Sequence[int]] = None) -> StepInputs:
    """Q, K, V of the h_k*w_k tokens of `scale` (1-based) in `layer`."""
    q, k, v = _qkv(cfg, layer, scale, cfg.n_tokens(scale), device, _units(cfg, units))
    return StepInputs(q, k, v)


def make_prefix(cfg: WorkloadConfig, layer: int, device="cpu",
                units: Optional[Sequence[int]] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """K, V of the text prefix (scale id 0): ordinary evictable cache rows."""
    _, k, v = _qkv(cfg, layer, 0, cfg.prefix, device, _units(cfg, units))
    return k, v


@dataclass
class FinalScaleCase:
    q: torch.Tensor        # [S,H,n_q,d]
    k_cur: torch.Tensor
    v_cur: torch.Tensor
    k_hist: torch.Tensor   # [S,H,hist_len,d]
    v_hist: torch.Tensor
    boosted: torch.Tensor  # bool [S,H,hist_len]: the dominant keys


def make_final_scale_case(cfg: WorkloadConfig, device="cpu", units: Optional[Sequence[int]] = None,
                          n_q: Optional[int] = None, hist_len: Optional[int] = None) -> FinalScaleCase:
    """Last scale only: n_q current tokens against a generated history of
    C_full(K) rows.  Q = G + w with a per-(seq, head) +-1 vector w; a seeded ~1 %
    of history keys get + (4/sqrt d) w, which lifts their logit by 4 for every
    query: dominant tokens."""
    units = _units(cfg, units)
    d, s = cfg.head_dim, cfg.seed
    n_q = cfg.n_tokens(cfg.n_scale) if n_q is None else n_q
    hist_len = c_full(cfg, cfg.n_scale) if hist_len is None else hist_len
    gq = _per_token(stream_key(s, _T_G_Q, 0, 99), cfg, n_q, d, device, units)
    kc = _per_token(stream_key(s, _T_G_K, 0, 99), cfg, n_q, d, device, units)
    vc = _per_token(stream_key(s, _T_G_V, 0, 99), cfg, n_q, d, device, units)
    kh = _per_token(stream_key(s, _T_G_K, 0, 98), cfg, hist_len, d, device, units)
    vh = _per_token(stream_key(s, _T_G_V, 0, 98), cfg, hist_len, d, device, units)
    w = _per_token(stream_key(s, _T_SIGN, 0, 99), cfg, 1, d, device, units, kind="sign")
    if units is None:
        u = _uniform16(stream_key(s, _T_BOOST, 0, 98), 0, cfg.n_seq * cfg.n_head * hist_len, device)
        u = u.reshape(cfg.n_seq, cfg.n_head, hist_len)
    else:
        u = _stack([_uniform16(stream_key(s, _T_BOOST, 0, 98), x * hist_len, hist_len, device) for x in units],
                   (hist_len,), device, torch.int64)
    boosted = u < 655
    q = gq + w
    bump = w * (4.0 / float(d) ** 0.5)
    kh = torch.where(boosted.unsqueeze(-1), kh + bump, kh)
    return FinalScaleCase(_to_dtype(q, cfg), _to_dtype(kc, cfg), _to_dtype(vc, cfg),
                          _to_dtype(kh, cfg), _to_dtype(vh, cfg), boosted)


@dataclass
class AsiCase:
    q_samp: torch.Tensor   # [S,H,n_samp,d] sampled queries of the current map
    k_all: torch.Tensor    # [S,H,hist_len + cur_len,d]: every earlier row, then the current map's keys
    hist_len: int
    cur_len: int
    rows: Tuple[int, ...]  # positions of the sampled queries in the current map


def asi_sample_rows(n_k: int, n_samp: int) -> Tuple[int, ...]:
    """min(n_samp, n_k) query positions spread evenly over the current map (raster order)."""
    n = min(n_samp, n_k)
    return tuple((2 * j + 1) * n_k // (2 * n) for j in range(n))


def assemble_asi_case(k_history: Sequence[torch.Tensor], q_cur: torch.Tensor, k_cur: torch.Tensor,
                      n_samp: int = 16) -> AsiCase:
    """Inputs of the Attention Selectivity Index (Eq. 2) for one (layer, scale) pair from
    tensors that already exist: k_history = the keys of the prefix and of every earlier map,
    in cache order; q_cur / k_cur = the current map's queries and keys.  Rows only are moved."""
    n_k = q_cur.shape[-2]
    rows = asi_sample_rows(n_k, n_samp)
    q_samp = q_cur.index_select(-2, torch.tensor(rows, device=q_cur.device)).contiguous()
    parts = list(k_history) + [k_cur]
    k_all = torch.empty(*k_cur.shape[:-2], sum(p.shape[-2] for p in parts), k_cur.shape[-1], dtype=k_cur.dtype,
                        device=k_cur.device)
    at = 0
    for p in parts:
        k_all[..., at: at + p.shape[-2], :] = p
        at += p.shape[-2]
    return AsiCase(q_samp, k_all, k_all.shape[-2] - n_k, n_k, rows)


def make_asi_case(cfg: WorkloadConfig, layer: int, scale: int, device="cpu", n_samp: int = 16,
                  units: Optional[Sequence[int]] = None) -> AsiCase:
    """The same for a workload config: the uncompressed cache entering `scale` (prefix and maps
    1..scale-1), the current map's keys behind it, and n_samp of its queries."""
    hist = [make_prefix(cfg, layer, device, units)[0]]
    hist += [make_step_inputs(cfg, layer, j, device, units).k_cur for j in range(1, scale)]
    x = make_step_inputs(cfg, layer, scale, device, units)
    return assemble_asi_case(hist, x.q, x.k_cur, n_samp)
