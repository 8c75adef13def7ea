"""A seeded toy transformer in fp64 -- TEST INFRASTRUCTURE ONLY.

Used to pin the oracle against the paper's central equivalence (Sec. 3.1,
Sec. 3.3 "attention masking effect", Sec. 3.4): serving a prompt from
independently encoded prompt modules gives, for the uncached tokens, exactly
what one pass over the whole prompt gives when the attention mask confines each
module to itself.  The equivalence only holds through several layers if the
position IDs, the mask, the concatenation and the append of new-token states
are all right, which is what makes it a useful pin.

The model is attention-only (QKV and output projections with a residual); an
MLP would act per token and cannot affect the equivalence.
"""
from __future__ import annotations

import numpy as np

from . import assemble, attn, full_masked, rope


class ToyModel:
    def __init__(self, seed: int, n_layers: int = 2, n_q_heads: int = 2, n_kv_heads: int = 2,
                 head_dim: int = 16, vocab: int = 97, base: float = 10000.0):
        rng = np.random.default_rng(seed)
        self.L, self.Hq, self.Hkv, self.d, self.base = n_layers, n_q_heads, n_kv_heads, head_dim, base
        self.dm = n_q_heads * head_dim
        s = 1.0 / np.sqrt(self.dm)
        self.emb = rng.standard_normal((vocab, self.dm))
        self.Wq = rng.standard_normal((n_layers, self.dm, n_q_heads * head_dim)) * s
        self.Wk = rng.standard_normal((n_layers, self.dm, n_kv_heads * head_dim)) * s
        self.Wv = rng.standard_normal((n_layers, self.dm, n_kv_heads * head_dim)) * s
        self.Wo = rng.standard_normal((n_layers, n_q_heads * head_dim, self.dm)) * s

    def _qkv(self, layer: int, h: np.ndarray):
        n = h.shape[0]
        q = (h @ self.Wq[layer]).reshape(n, self.Hq, self.d)
        k = (h @ self.Wk[layer]).reshape(n, self.Hkv, self.d)
        v = (h @ self.Wv[layer]).reshape(n, self.Hkv, self.d)
        return q, k, v

    # ---- path A: the whole prompt in one pass under the module-local mask
    def forward_full_masked(self, tokens, pos, module_of) -> np.ndarray:
        h = self.emb[np.asarray(tokens)]
        for layer in range(self.L):
            q, k, v = self._qkv(layer, h)
            o, _ = full_masked(q, k, v, pos, module_of, self.base)
            h = h + o.reshape(len(tokens), -1) @ self.Wo[layer]
        return h

    # ---- path B, step 1: prompt-module encoding (Sec. 3.3)
    def encode_module(self, tokens, start_pos: int):
        """Run the module alone at its schema positions; return per-layer (K encoded, V)."""
        n = len(tokens)
        pos = np.arange(start_pos, start_pos + n, dtype=np.int32)
        same = np.zeros(n, dtype=np.int32)
        h = self.emb[np.asarray(tokens)]
        states = []
        for layer in range(self.L):
            q, k, v = self._qkv(layer, h)
            o, k_enc = full_masked(q, k, v, pos, same, self.base)
            states.append((k_enc, v))
            h = h + o.reshape(n, -1) @ self.Wo[layer]
        return states

    # ---- scaffolding (Sec. 3.3): several modules encoded together, sharing one attention span
    def encode_scaffold(self, members):
        """members: list of (tokens, start_pos).  The members' tokens run as ONE module at their own schema
        positions; returns, per member, per-layer (K encoded, V) cut out of the joint result."""
        toks = np.concatenate([np.asarray(t) for t, _ in members])
        pos = np.concatenate([np.arange(s0, s0 + len(t)) for t, s0 in members]).astype(np.int32)
        same = np.zeros(len(toks), dtype=np.int32)
        h = self.emb[toks]
        joint = []
        for layer in range(self.L):
            q, k, v = self._qkv(layer, h)
            o, k_enc = full_masked(q, k, v, pos, same, self.base)
            joint.append((k_enc, v))
            h = h + o.reshape(len(toks), -1) @ self.Wo[layer]
        out, row = [], 0
        for t, _ in members:
            out.append([(k[row:row + len(t)], v[row:row + len(t)]) for k, v in joint])
            row += len(t)
        return out

    # ---- path B, step 2: cached inference (Sec. 3.4)
    def forward_cached(self, module_states, module_starts, new_tokens, new_pos) -> np.ndarray:
        """module_states[m][layer] = (K_enc, V); modules are concatenated in the order given."""
        new_pos = np.asarray(new_pos, dtype=np.int32)
        h = self.emb[np.asarray(new_tokens)]
        for layer in range(self.L):
            q, k, v = self._qkv(layer, h)
            aK, aV, aPos = assemble([s[layer][0] for s in module_states],
                                    [s[layer][1] for s in module_states], module_starts)
            k_enc = rope(k, new_pos, self.base)
            K_all = np.concatenate([aK, k_enc], axis=0)
            V_all = np.concatenate([aV, v], axis=0)
            pos_all = np.concatenate([aPos, new_pos])
            o = attn(q, new_pos, K_all, V_all, pos_all, self.base)
            h = h + o.reshape(len(new_tokens), -1) @ self.Wo[layer]
        return h
