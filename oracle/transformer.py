"""CPU oracle, part 1: the combined scoring-and-proposal model  p_1 .. p_k.

TEST INFRASTRUCTURE ONLY.  Plain numpy in float64, no caching, no blocking, no
fusion: every call recomputes the whole network from the token ids.  Nothing in
the product path may import this package; it shares no code with the HIP library.

What the paper fixes (Section 6, Figure 3, footnote in Section 7.1):
  * the base model is an encoder-decoder Transformer; its decoder output at
    position t, h_t, depends only on the source x and on the target tokens
    y_1..y_t (Section 3: all positions can be scored in one pass);
  * between h_t and the vocabulary projection sits one feed-forward layer with
    k outputs, each with a residual connection from h_t:
        o_{t,i} = h_t + FFN_i(h_t),   i = 1..k   (p_1 goes through a head too);
  * the original vocabulary projection is applied to each o_{t,i}; head i at
    position t scores token y_{t+i}:  p_i(y_{t+i} | y_{<=t}, x).

What the paper leaves open, and the readings taken here:
  * the k heads are k independent FFNs d_model -> d_ff -> d_model with ReLU
    (first layers concatenated form the "hidden layer of size k*d_hidden",
    second layers are the "k output layers" of Figure 3);
  * pre-LayerNorm sublayers (x + Sublayer(LN(x))), a final LayerNorm on both
    stacks, eps = 1e-6, biased variance, learned gain and bias;
  * learned position tables, one per side, added to sqrt(d_model)-scaled
    embeddings; one embedding matrix E for source, target and the output
    projection (logits = o @ E^T, no bias);
  * the decoder input at position 0 is the zero vector (shifted-right targets,
    no BOS id); attention projections have no bias, FFN layers do;
  * scaled dot-product attention with 1/sqrt(d_head), softmax over visible keys;
  * the image model of Section 7.2 is named as an Image Transformer with 1D local
    attention and no more is said.  Reading (the published layer of that name):
    target positions are cut into consecutive query blocks of ``local_q``
    positions; position t sees, causally, its own block and the ``local_m``
    positions before the block:  j visible to t  iff  b(t) - local_m <= j <= t,
    b(t) = floor(t / local_q) * local_q.  local_q = 0 means full causal attention.
    Block lengths are not given: they are parameters here.

Parity status: every function here is pinned by tests/test_oracle_model.py
(library attention/LayerNorm/decoder-layer routines, closed forms, causality,
zero-head identity).  Trained-model quality numbers of Tables 1, 2 and 4 are
"parity unpinned": they need datasets and weights that do not exist here.
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Sequence

import numpy as np


def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float) -> np.ndarray:
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def softmax_rows(s: np.ndarray, visible: np.ndarray) -> np.ndarray:
    """Softmax over the last axis restricted to ``visible`` keys (others get weight 0)."""
    s = np.where(visible, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def multi_head_attention(xq: np.ndarray, xkv: np.ndarray, wq, wk, wv, wo,
                         n_heads: int, visible: np.ndarray) -> np.ndarray:
    """xq [Tq,d], xkv [Tk,d], visible [Tq,Tk] bool -> [Tq,d]."""
    tq, d = xq.shape
    tk = xkv.shape[0]
    dh = d // n_heads
    q = (xq @ wq).reshape(tq, n_heads, dh)
    k = (xkv @ wk).reshape(tk, n_heads, dh)
    v = (xkv @ wv).reshape(tk, n_heads, dh)
    out = np.empty((tq, n_heads, dh), dtype=np.float64)
    for h in range(n_heads):
        s = q[:, h, :] @ k[:, h, :].T / math.sqrt(dh)
        out[:, h, :] = softmax_rows(s, visible) @ v[:, h, :]
    return out.reshape(tq, d) @ wo


def self_attention_visibility(t1: int, local_q: int = 0, local_m: int = 0) -> np.ndarray:
    """[t1, t1] bool: may decoder position t (row) look at position j (column)?

    Full causal attention: j <= t.  1D local attention (Section 7.2, see the module
    header): additionally j >= floor(t / local_q) * local_q - local_m."""
    vis = np.zeros((t1, t1), dtype=bool)
    for t in range(t1):
        lo = 0
        if local_q > 0:
            lo = max(0, (t // local_q) * local_q - local_m)
        for j in range(lo, t + 1):
            vis[t, j] = True
    return vis


def feed_forward(x, w1, b1, w2, b2):
    return np.maximum(x @ w1 + b1, 0.0) @ w2 + b2


class CombinedModel:
    """The network of Section 6: Transformer + k residual FFN heads + shared projection."""

    def __init__(self, weights: Dict[str, np.ndarray], n_enc: int, n_dec: int,
                 n_heads: int, k: int, ln_eps: float = 1e-6, local_q: int = 0, local_m: int = 0):
        self.w = {n: np.asarray(a, dtype=np.float64) for n, a in weights.items()}
        self.n_enc, self.n_dec, self.n_heads, self.k, self.eps = n_enc, n_dec, n_heads, k, ln_eps
        self.local_q, self.local_m = local_q, local_m
        self.d = self.w["emb"].shape[1]
        self.vocab = self.w["emb"].shape[0]

    # -- small helpers -------------------------------------------------------
    def _ln(self, x, prefix):
        return layer_norm(x, self.w[prefix + ".g"], self.w[prefix + ".b"], self.eps)

    def _attn(self, xq, xkv, prefix, visible):
        w = self.w
        return multi_head_attention(xq, xkv, w[prefix + ".wq"], w[prefix + ".wk"],
                                    w[prefix + ".wv"], w[prefix + ".wo"], self.n_heads, visible)

    def _ffn(self, x, prefix):
        w = self.w
        return feed_forward(x, w[prefix + ".w1"], w[prefix + ".b1"], w[prefix + ".w2"], w[prefix + ".b2"])

    # -- encoder over the source x = (x_1..x_n)  (Section 2) -------------------
    def encode(self, src_ids: Sequence[int]) -> np.ndarray:
        src = np.asarray(src_ids, dtype=np.int64)
        n = src.shape[0]
        x = math.sqrt(self.d) * self.w["emb"][src] + self.w["pos_src"][:n]
        all_visible = np.ones((n, n), dtype=bool)
        for l in range(self.n_enc):
            y = self._ln(x, f"enc.{l}.ln1")
            x = x + self._attn(y, y, f"enc.{l}.self", all_visible)
            x = x + self._ffn(self._ln(x, f"enc.{l}.ln2"), f"enc.{l}.ffn")
        return self._ln(x, "enc.lnf")

    # -- decoder over y_{<=t}: returns h_0..h_t --------------------------------
    def decoder_states(self, memory: np.ndarray, prefix: Sequence[int]) -> np.ndarray:
        """``prefix`` = (y_1..y_t).  Position 0 takes the zero vector, position s takes
        y_s; h_s may look at positions <= s only."""
        y = np.asarray(prefix, dtype=np.int64)
        t1 = y.shape[0] + 1
        u = np.zeros((t1, self.d), dtype=np.float64)
        if t1 > 1:
            u[1:] = math.sqrt(self.d) * self.w["emb"][y]
        x = u + self.w["pos_tgt"][:t1]
        causal = self_attention_visibility(t1, self.local_q, self.local_m)
        mem_visible = np.ones((t1, memory.shape[0]), dtype=bool)
        for l in range(self.n_dec):
            a = self._ln(x, f"dec.{l}.ln1")
            x = x + self._attn(a, a, f"dec.{l}.self", causal)
            x = x + self._attn(self._ln(x, f"dec.{l}.ln2"), memory, f"dec.{l}.cross", mem_visible)
            x = x + self._ffn(self._ln(x, f"dec.{l}.ln3"), f"dec.{l}.ffn")
        return self._ln(x, "dec.lnf")

    # -- the inserted multi-output layer + shared projection (Section 6) -------
    def head_outputs(self, h: np.ndarray, k: Optional[int] = None) -> np.ndarray:
        """h [..., d] -> o [..., k, d] with o_i = h + FFN_i(h)."""
        k = self.k if k is None else k
        w = self.w
        outs = []
        for i in range(k):
            outs.append(h + feed_forward(h, w["head.w1"][i], w["head.b1"][i],
                                         w["head.w2"][i], w["head.b2"][i]))
        return np.stack(outs, axis=-2)

    def logits(self, h: np.ndarray, k: Optional[int] = None) -> np.ndarray:
        """h [..., d] -> z [..., k, V];  z[..., i-1, :] are the scores of p_i."""
        return self.head_outputs(h, k) @ self.w["emb"].T

    # -- the model as the decoding algorithms see it ---------------------------
    def next_logits(self, memory: np.ndarray, prefix: Sequence[int], k: Optional[int] = None) -> np.ndarray:
        """z[i-1, v] = score of y_{j+i} = v under p_i( . | y_{<=j}, x), j = len(prefix).
        Full recomputation of the decoder over the prefix."""
        h = self.decoder_states(memory, prefix)
        return self.logits(h[-1], k)

    def all_position_logits(self, memory: np.ndarray, prefix: Sequence[int],
                            first: int = 0, k: Optional[int] = None) -> np.ndarray:
        """z[s-first, i-1, v] for positions s = first..len(prefix) from ONE decoder pass
        (the parallel scoring the method relies on, Section 3).  By causality this
        equals calling next_logits on each prefix y_{<=s}; tests check that."""
        h = self.decoder_states(memory, prefix)
        return self.logits(h[first:], k)
