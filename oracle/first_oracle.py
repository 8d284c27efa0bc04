"""CPU oracle for FiRST's router-gated prefill and decode.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module;
the product path (the HIP library) never does and shares no code with it.

What it computes, written out plainly with PyTorch CPU ops in fp64 (weights are upcast
exactly from their storage type; pass ``cdt=torch.float32`` for the paper's "full
precision"):

  * hidden-state recurrence  H_i = H_{i-1} + phi_i(H_{i-1})            (Section 2, Eq. 1)
  * gated recurrence         H_i = H_{i-1} + round(rho_i) * phi_i(..)  (Section 3, Eq. 2
                                                                        and the rounded form)
  * router R_i: bias-free linear D->1 on the input of layer i, sigmoid per token, mean
    over the sequence -> rho_i; keep iff rho_i >= 0.5                  (Section 4.1, 4.3)
  * prefill never skips; decisions are cached and every decode token follows them; a
    skipped layer neither reads nor appends KV                         (Section 4.3, items 1-2)

phi_i is a pre-norm Llama block (RMSNorm, GQA attention with rotate-half RoPE, SwiGLU MLP,
no biases).  The paper does not restate those; the readings taken are:
  - router input is the raw residual stream entering layer i (the embedded prompt for the
    first layer), all real prompt tokens enter the mean, equality at 0.5 keeps;
  - K (after RoPE) and V are rounded to the model's storage type when stored, and
    attention always reads the stored values (also for the token being processed);
  - rho is rounded to fp32 before the threshold; logits are rounded to fp32 before the
    greedy argmax; exact ties go to the lowest index.

Pins (tests/test_oracle_pins.py): independent no-cache recompute with library attention,
all-skip closed form, pruned-model equivalence, zero-router tie, prefill independent of the
routers, RoPE relative-position property, a scalar pure-Python twin on a toy model, and the
paper's printed router-parameter fractions; KV elision (`elide_kv`) through the same pruned
model and a byte count done by hand.  The paper prints no worked numeric example, so absolute
logit values are pinned only through those.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch

KV_DTYPES = {"bf16": torch.bfloat16, "fp32": torch.float32}


# --------------------------------------------------------------------------- building blocks
def rmsnorm(x: torch.Tensor, g: torch.Tensor, eps: float) -> torch.Tensor:
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    ms = (x * x).mean(dim=-1, keepdim=True)
    return x / torch.sqrt(ms + eps) * g


def rope(x: torch.Tensor, pos: torch.Tensor, base: float) -> torch.Tensor:
    """Rotate-half rotary embedding.  x [n, H, hd], pos [n] (integer positions).
    Pair (d, d + hd/2) is rotated by angle pos * base^(-2d/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    d = torch.arange(half, dtype=torch.float64)
    theta = torch.pow(torch.tensor(base, dtype=torch.float64), -2.0 * d / hd)
    ang = pos.to(torch.float64)[:, None] * theta[None, :]          # [n, half]
    c = torch.cos(ang).to(x.dtype)[:, None, :]
    s = torch.sin(ang).to(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * c - x2 * s, x2 * c + x1 * s], dim=-1)


def router_score(H: torch.Tensor, w: torch.Tensor) -> torch.Tensor:
    """rho = mean_j sigmoid(w . H[j])  for one sequence (Section 4.1).  H [n, D], w [D]."""
    z = H @ w
    s = 1.0 / (1.0 + torch.exp(-z))
    return s.mean()


def keep_decision(rho: torch.Tensor) -> int:
    """round(rho): 1 iff rho >= 0.5, decided on the fp32 value (Section 3, Section 4.3)."""
    return 1 if float(rho.to(torch.float32)) >= 0.5 else 0


def compact_kept(mask) -> List[int]:
    """Ascending indices of the kept layers."""
    return [i for i, m in enumerate(list(mask)) if int(m) != 0]


def greedy_token(logits32: torch.Tensor) -> int:
    """argmax over fp32 logits, lowest index on exact ties."""
    m = logits32.max()
    return int(torch.nonzero(logits32 == m)[0, 0])


def attention_rows(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, q_pos: torch.Tensor,
                   group: int) -> torch.Tensor:
    """softmax(q.k / sqrt(hd)) v with a causal limit per query row.
    q [nq, Hq, hd]; K, V [nk, Hkv, hd] (positions 0..nk-1); query row r sees keys 0..q_pos[r].
    Query head h reads KV head h // group."""
    nq, Hq, hd = q.shape
    nk = K.shape[0]
    out = torch.empty_like(q)
    key_pos = torch.arange(nk)
    allowed = key_pos[None, :] <= q_pos[:, None]                   # [nq, nk]
    for h in range(Hq):
        g = h // group
        s = (q[:, h, :] @ K[:, g, :].T) / math.sqrt(hd)            # [nq, nk]
        s = s.masked_fill(~allowed, float("-inf"))
        s = s - s.max(dim=-1, keepdim=True).values
        p = torch.exp(s)
        p = p / p.sum(dim=-1, keepdim=True)
        out[:, h, :] = p @ V[:, g, :]
    return out


def mlp(y: torch.Tensor, w_gate, w_up, w_down) -> torch.Tensor:
    """SwiGLU: W_down( silu(W_gate y) * (W_up y) )."""
    g = y @ w_gate.T
    u = y @ w_up.T
    return ((g / (1.0 + torch.exp(-g))) * u) @ w_down.T


# --------------------------------------------------------------------------- state
@dataclass
class OracleState:
    """Per-sequence state after prefill: KV of every layer, router outputs, cached mask."""
    K: List[torch.Tensor]            # per layer [len_i, Hkv, hd] in the KV storage type
    V: List[torch.Tensor]
    rho: torch.Tensor                # [L] fp32
    mask: torch.Tensor               # [L] uint8, 1 = keep
    n_prompt: int
    pos: int                         # position the next decode token will occupy
    hidden: torch.Tensor             # H_L of the last prompt position (compute dtype)
    logits: torch.Tensor             # first-token logits, fp32
    token: int                       # first generated token (full model)
    router_in: Optional[List[torch.Tensor]] = None   # optional: H_{i-1} per layer

    def set_mask(self, mask) -> None:
        """Benchmark override of the cached decisions."""
        self.mask = torch.as_tensor(mask, dtype=torch.uint8).clone()


def _layer(desc, lw, cdt):
    return {k: v.to(cdt) for k, v in lw.items()}


def block(desc, lw, H: torch.Tensor, pos: torch.Tensor, K_prev, V_prev, cdt):
    """phi_i applied to rows H [n, D] at positions pos, given the already stored
    K_prev/V_prev [n_prev, Hkv, hd] (or None).  Returns (H + phi(H), K_all, V_all) where
    K_all/V_all are in the KV storage type and include the rows just appended."""
    kvt = KV_DTYPES[desc.dtype]
    Hq, Hkv, hd = desc.n_q_heads, desc.n_kv_heads, desc.head_dim
    w = _layer(desc, lw, cdt)
    n = H.shape[0]
    n_prev = 0 if K_prev is None else K_prev.shape[0]
    if int(pos[0]) != n_prev:
        raise ValueError("KV of this layer has a hole: it was skipped by an earlier decode token")
    x = rmsnorm(H, w["attn_norm"], desc.rms_eps)
    q = (x @ w["wq"].T).view(n, Hq, hd)
    k = (x @ w["wk"].T).view(n, Hkv, hd)
    v = (x @ w["wv"].T).view(n, Hkv, hd)
    q = rope(q, pos, desc.rope_base)
    k = rope(k, pos, desc.rope_base)
    k_st, v_st = k.to(kvt), v.to(kvt)
    K_all = k_st if K_prev is None else torch.cat([K_prev, k_st], dim=0)
    V_all = v_st if V_prev is None else torch.cat([V_prev, v_st], dim=0)
    a = attention_rows(q, K_all.to(cdt), V_all.to(cdt), pos, Hq // Hkv)
    u = H + a.reshape(n, Hq * hd) @ w["wo"].T
    y = rmsnorm(u, w["mlp_norm"], desc.rms_eps)
    out = u + mlp(y, w["w_gate"], w["w_up"], w["w_down"])
    return out, K_all, V_all


def lm_logits(desc, weights, h: torch.Tensor, cdt) -> torch.Tensor:
    """W_lm . RMSNorm(h; g_final), rounded to fp32."""
    x = rmsnorm(h, weights["final_norm"].to(cdt), desc.rms_eps)
    V = weights["lm_head"].shape[0]
    out = torch.empty(V, dtype=torch.float32)
    step = 1 << 15                                     # upcast the head in row slabs
    for r0 in range(0, V, step):
        out[r0:r0 + step] = (weights["lm_head"][r0:r0 + step].to(cdt) @ x).to(torch.float32)
    return out


# --------------------------------------------------------------------------- prefill + route
def prefill_route(desc, weights, router: torch.Tensor, ids: torch.Tensor,
                  cdt=torch.float64, keep_router_inputs: bool = False,
                  progress=None, elide_kv: bool = False) -> OracleState:
    """Runs every layer on the prompt (no skipping), scores router i on the stream entering
    layer i, thresholds, and returns the first token from the full model (Section 4.3).

    elide_kv: router i is evaluated on the input of layer i (Section 4.1), so mask_i is fixed
    before layer i runs, and decode never touches the KV of a layer whose mask is 0 (Section
    4.3: the prefill decision is reused by every later token).  With elide_kv the K/V a skipped
    layer formed for its own prompt attention is therefore dropped once the layer is done
    (K[i] = V[i] = None); nothing else changes."""
    n = int(ids.numel())
    pos = torch.arange(n)
    H = weights["embed"][ids.long()].to(cdt)                        # H_0
    Ks, Vs, rhos, mask, taps = [], [], [], [], []
    for i in range(desc.n_layers):
        rho = router_score(H, router[i].to(cdt))
        rhos.append(rho.to(torch.float32))
        mask.append(keep_decision(rho))
        if keep_router_inputs:
            taps.append(H.clone())
        H, K, V = block(desc, weights["layers"][i], H, pos, None, None, cdt)
        stored = not (elide_kv and mask[i] == 0)
        Ks.append(K if stored else None)
        Vs.append(V if stored else None)
        if progress is not None:
            progress(f"oracle prefill layer {i + 1}/{desc.n_layers}")
    logits = lm_logits(desc, weights, H[n - 1], cdt)
    return OracleState(K=Ks, V=Vs, rho=torch.stack(rhos), mask=torch.tensor(mask, dtype=torch.uint8),
                       n_prompt=n, pos=n, hidden=H[n - 1].clone(), logits=logits,
                       token=greedy_token(logits), router_in=taps if keep_router_inputs else None)


# --------------------------------------------------------------------------- decode
def decode_step(desc, weights, st: OracleState, token: int, cdt=torch.float64,
                return_hidden: bool = False):
    """One token through the kept layers only; skipped layers leave h and their KV alone."""
    p = st.pos
    pos = torch.tensor([p])
    h = weights["embed"][int(token)].to(cdt)[None, :]
    for i in range(desc.n_layers):
        if int(st.mask[i]) == 0:
            continue
        h, st.K[i], st.V[i] = block(desc, weights["layers"][i], h, pos, st.K[i], st.V[i], cdt)
    st.pos = p + 1
    logits = lm_logits(desc, weights, h[0], cdt)
    tok = greedy_token(logits)
    if return_hidden:
        return logits, tok, h[0]
    return logits, tok


def generate(desc, weights, st: OracleState, n_steps: int, cdt=torch.float64, forced=None):
    """n_steps decode steps starting from the prefill token.  forced: optional list of input
    tokens (teacher forcing); otherwise each step feeds its own argmax."""
    logits_all, toks = [], []
    t = st.token
    for s in range(n_steps):
        if forced is not None:
            t = int(forced[s])
        lg, nt = decode_step(desc, weights, st, t, cdt)
        logits_all.append(lg)
        toks.append(nt)
        t = nt
    return torch.stack(logits_all), toks


# --------------------------------------------------------------------------- KV elision accounting
def kv_layers_stored(masks) -> List[int]:
    """Layers whose prompt KV must be persisted for a set of live sequences: those kept by at
    least one of them (a slice of the cache belongs to a layer, all sequences share it)."""
    masks = [list(m) for m in masks]
    return [i for i in range(len(masks[0])) if any(int(m[i]) for m in masks)]


def kv_bytes(desc, n_layers_stored: int, n_tokens: int) -> int:
    """Bytes of K and V for n_tokens positions in n_layers_stored layers, in the KV storage type."""
    elem = torch.empty(0, dtype=KV_DTYPES[desc.dtype]).element_size()
    return 2 * n_layers_stored * n_tokens * desc.n_kv_heads * desc.head_dim * elem

