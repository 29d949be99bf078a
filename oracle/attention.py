"""fp64 CPU oracle for the attention computations of the semi-PD hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path imports this package;
only tests, the smoke check and the bench's `cpu_baseline` leg call it.  It
shares no code with the HIP library and keeps its own (plain) page layout.

Everything here is the textbook definition written out, in float64:

* prefill  (paper, Background "LLM Processing Phases": the prefill phase
  processes the whole input context and produces the initial KV cache): causal
  softmax attention over the prompt, and a copy of K, V into the request's pages.
* decode   (same section: the next token is produced from the last token and
  the KV cache): one query row attends over all cached tokens, which are found
  through the block table (System Design, "Unified Memory Manager": paged
  storage accessed through the block-table index).
* MLA      (Evaluation, Setup "Model": DeepSeek-V2-Lite; the paper names the
  model only): decode over the 576-dim latent cache with an absorbed query,
  and the un-absorbed multi-head form it must equal.

A library matmul is used as a step; there is no blocking, no online softmax,
no reordering.  All pins live in tests/ (marker: not gpu).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _softmax_rows(s: np.ndarray) -> np.ndarray:
    """Row-wise softmax of a 2-D score matrix; -inf entries get weight 0."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


# --------------------------------------------------------------------------- dense definitions
def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float) -> np.ndarray:
    """O[i,h] = sum_{j<=i} softmax_j(scale * Q[i,h].K[j,g]) V[j,g],  g = h // (H/Hkv).

    q [L,H,dqk], k [L,Hkv,dqk], v [L,Hkv,dv] -> O [L,H,dv]; float64.
    Grouped-query attention: query head h reads KV head h // (H/Hkv).
    """
    q, k, v = (np.asarray(a, dtype=F64) for a in (q, k, v))
    L, H, _ = q.shape
    Hkv = k.shape[1]
    if L == 0:
        raise ValueError("empty prompt")
    if H % Hkv != 0 or k.shape[0] != L or v.shape[0] != L or v.shape[1] != Hkv:
        raise ValueError("shape mismatch")
    group = H // Hkv
    future = np.triu(np.ones((L, L), dtype=bool), k=1)      # j > i
    out = np.empty((L, H, v.shape[2]), dtype=F64)
    for h in range(H):
        g = h // group
        s = scale * (q[:, h, :] @ k[:, g, :].T)
        s[future] = -np.inf
        out[:, h, :] = _softmax_rows(s) @ v[:, g, :]
    return out


def prefill_attention(q, k, v, cu_seqlens, scale: float) -> np.ndarray:
    """Causal attention applied independently to each request of a packed batch.

    q [T,H,dqk], k [T,Hkv,dqk], v [T,Hkv,dv]; request r owns rows
    cu_seqlens[r]:cu_seqlens[r+1].  No request sees another's tokens.
    """
    q = np.asarray(q, dtype=F64)
    out = np.empty((q.shape[0], q.shape[1], np.asarray(v).shape[2]), dtype=F64)
    for r in range(len(cu_seqlens) - 1):
        a, b = int(cu_seqlens[r]), int(cu_seqlens[r + 1])
        out[a:b] = causal_attention(q[a:b], np.asarray(k)[a:b], np.asarray(v)[a:b], scale)
    return out


def chunk_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float) -> np.ndarray:
    """A chunk of a prompt attending to everything before it and causally to itself
    (paper, Evaluation "Baselines": the chunked-prefill variants process a prompt piece by piece,
    each piece over the cache built so far).

    q [C,H,dqk] are the chunk's C query rows, k [n,Hkv,dqk], v [n,Hkv,dv] the n = prefix + C rows of
    the request so far, the chunk's own rows last.  Row i of the chunk sits at position prefix + i:
        O[i,h] = sum_{j <= prefix+i} softmax_j(scale * Q[i,h].K[j,g]) V[j,g].
    """
    q, k, v = (np.asarray(a, dtype=F64) for a in (q, k, v))
    C, H, _ = q.shape
    n, Hkv = k.shape[0], k.shape[1]
    if C == 0 or n < C:
        raise ValueError("chunk longer than its context, or empty")
    prefix = n - C
    group = H // Hkv
    future = np.arange(n)[None, :] > (prefix + np.arange(C))[:, None]      # j > prefix + i
    out = np.empty((C, H, v.shape[2]), dtype=F64)
    for h in range(H):
        g = h // group
        s = scale * (q[:, h, :] @ k[:, g, :].T)
        s[future] = -np.inf
        out[:, h, :] = _softmax_rows(s) @ v[:, g, :]
    return out


def decode_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float) -> np.ndarray:
    """o[h] = softmax_t(scale * q[h].K[t,g]) V[t,g] over all n cached tokens (no mask).

    q [H,dqk], k [n,Hkv,dqk], v [n,Hkv,dv] -> o [H,dv]; float64.
    """
    q, k, v = (np.asarray(a, dtype=F64) for a in (q, k, v))
    H, Hkv, n = q.shape[0], k.shape[1], k.shape[0]
    if n == 0:
        raise ValueError("empty context")
    group = H // Hkv
    out = np.empty((H, v.shape[2]), dtype=F64)
    for h in range(H):
        g = h // group
        s = scale * (k[:, g, :] @ q[h])
        out[h] = _softmax_rows(s[None, :])[0] @ v[:, g, :]
    return out


# --------------------------------------------------------------------------- paged storage
class PagedKV:
    """The oracle's own paged K/V store: page p, slot s holds one token's K and V rows.

    Layout here is the plainest one, pool_k[page, slot, kv_head, dim]; it is
    independent of the HIP library's layout.  Values are kept as whatever dtype
    the caller supplies (bf16 bit patterns for bit-exact copy checks, or floats).
    """

    def __init__(self, num_pages: int, page_tokens: int, n_kv_heads: int, dim_k: int, dim_v: int,
                 dtype=F64):
        self.P = page_tokens
        self.k = np.zeros((num_pages, page_tokens, n_kv_heads, dim_k), dtype=dtype)
        self.v = np.zeros((num_pages, page_tokens, n_kv_heads, dim_v), dtype=dtype)

    def write(self, block_table, start: int, k: np.ndarray, v: np.ndarray) -> None:
        """Token j of (k, v) lands at logical position start + j of the request."""
        for j in range(k.shape[0]):
            pos = start + j
            page, slot = int(block_table[pos // self.P]), pos % self.P
            self.k[page, slot] = k[j]
            self.v[page, slot] = v[j]

    def gather(self, block_table, n: int):
        """Logical K[0:n], V[0:n] of a request, read through its block table."""
        ks = np.empty((n,) + self.k.shape[2:], dtype=self.k.dtype)
        vs = np.empty((n,) + self.v.shape[2:], dtype=self.v.dtype)
        for t in range(n):
            page, slot = int(block_table[t // self.P]), t % self.P
            ks[t] = self.k[page, slot]
            vs[t] = self.v[page, slot]
        return ks, vs


def paged_decode_attention(q, store: PagedKV, block_table, n: int, scale: float) -> np.ndarray:
    """Decode attention whose K, V are gathered from pages through the block table."""
    k, v = store.gather(block_table, n)
    return decode_attention(q, k, v, scale)


# --------------------------------------------------------------------------- MLA (latent cache)
def mla_absorb_query(q_nope: np.ndarray, q_rope: np.ndarray, w_uk: np.ndarray) -> np.ndarray:
    """Qabs[h] = [ q_nope[h] . W_UK[h] ; q_rope[h] ]  -> [H, kv_lora + rope].

    q_nope [H,nope], q_rope [H,rope], w_uk [H,nope,kv_lora].
    """
    q_nope, q_rope, w_uk = (np.asarray(a, dtype=F64) for a in (q_nope, q_rope, w_uk))
    absorbed = np.einsum("hn,hnc->hc", q_nope, w_uk)
    return np.concatenate([absorbed, q_rope], axis=-1)


def mla_decode_latent(qabs: np.ndarray, latent: np.ndarray, scale: float, kv_lora: int) -> np.ndarray:
    """Absorbed-form decode over the latent cache.

    latent row c_t = [ckv_t (kv_lora) ; krope_t (rope)], shared by all heads:
      s[h,t]  = scale * qabs[h] . c_t
      o_lat[h] = sum_t softmax_t(s[h,:]) * ckv_t            -> [H, kv_lora]
    """
    qabs, latent = np.asarray(qabs, dtype=F64), np.asarray(latent, dtype=F64)
    if latent.shape[0] == 0:
        raise ValueError("empty context")
    s = scale * (qabs @ latent.T)                 # [H, n]
    return _softmax_rows(s) @ latent[:, :kv_lora]


def mla_expand_kv(latent: np.ndarray, w_uk: np.ndarray, w_uv: np.ndarray, kv_lora: int):
    """Un-absorbed per-head K, V:  K[t,h] = [W_UK[h] ckv_t ; krope_t],  V[t,h] = ckv_t W_UV[h]."""
    latent, w_uk, w_uv = (np.asarray(a, dtype=F64) for a in (latent, w_uk, w_uv))
    ckv, krope = latent[:, :kv_lora], latent[:, kv_lora:]
    H = w_uk.shape[0]
    k_nope = np.einsum("hnc,tc->thn", w_uk, ckv)
    k = np.concatenate([k_nope, np.broadcast_to(krope[:, None, :], (latent.shape[0], H, krope.shape[1]))], axis=-1)
    v = np.einsum("tc,hcd->thd", ckv, w_uv)
    return k, v


def mla_decode_unabsorbed(q_nope, q_rope, latent, w_uk, w_uv, scale: float, kv_lora: int) -> np.ndarray:
    """Ordinary multi-head decode on the expanded K, V (what the absorbed form must equal)."""
    k, v = mla_expand_kv(latent, w_uk, w_uv, kv_lora)
    q = np.concatenate([np.asarray(q_nope, dtype=F64), np.asarray(q_rope, dtype=F64)], axis=-1)
    return decode_attention(q, k, v, scale)


class PagedLatent:
    """The oracle's paged latent store for MLA: pool[page, slot, latent_dim]."""

    def __init__(self, num_pages: int, page_tokens: int, latent_dim: int, dtype=F64):
        self.P = page_tokens
        self.c = np.zeros((num_pages, page_tokens, latent_dim), dtype=dtype)

    def write(self, block_table, start: int, latent: np.ndarray) -> None:
        for j in range(latent.shape[0]):
            pos = start + j
            self.c[int(block_table[pos // self.P]), pos % self.P] = latent[j]

    def gather(self, block_table, n: int) -> np.ndarray:
        out = np.empty((n, self.c.shape[2]), dtype=self.c.dtype)
        for t in range(n):
            out[t] = self.c[int(block_table[t // self.P]), t % self.P]
        return out
