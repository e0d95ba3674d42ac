"""Independent pins for the CPU oracle: small, literal re-derivations that do not
use the oracle's code or its formulation.

 * trie_dedup: a literal prefix trie (the structure Sec. 3.3 says the tensor
   method replaces): walk each candidate through a dict-of-dicts, remember which
   candidate created each node.
 * beam_causal_attention: ordinary causal attention of ONE unpacked candidate
   over context + its own earlier tokens, numpy float64, softmax via matmul.
 * greedy_rollout: autoregressive greedy decoding with a toy deterministic LM.
"""
from __future__ import annotations

import numpy as np


def trie_dedup(beam):
    """Returns (prefix_tree, n_nodes, node_id[i][j], parent_of_node, token_of_node, depth_of_node);
    nodes are numbered in order of creation while inserting candidates 0, 1, ... in turn."""
    W, L = len(beam), len(beam[0])
    root = {}
    owner, parent, token, depth = [], [], [], []
    prefix_tree = [[None] * L for _ in range(W)]
    node_id = [[None] * L for _ in range(W)]
    for i in range(W):
        cur, cur_id = root, -1
        for j in range(L):
            t = int(beam[i][j])
            if t not in cur:
                cur[t] = (len(owner), {})
                owner.append(i)
                parent.append(cur_id)
                token.append(t)
                depth.append(j)
            nid, nxt = cur[t]
            prefix_tree[i][j] = owner[nid]
            node_id[i][j] = nid
            cur, cur_id = nxt, nid
    return prefix_tree, len(owner), node_id, parent, token, depth


def n_distinct_prefixes(beam):
    return len({tuple(int(x) for x in row[: j + 1]) for row in beam for j in range(len(row))})


def beam_causal_attention(q_u, k_u, v_u, k_ctx, v_ctx, scale):
    """q_u,k_u,v_u: [L,D] float64 of one unpacked candidate; k_ctx,v_ctx: [C,D].
    Token j attends to all C context keys and to its own tokens 0..j.  Returns [L,D]."""
    L = q_u.shape[0]
    C = k_ctx.shape[0]
    K = np.concatenate([k_ctx, k_u], axis=0)
    V = np.concatenate([v_ctx, v_u], axis=0)
    S = scale * (q_u @ K.T)                              # [L, C+L]
    allowed = np.ones((L, C + L), dtype=bool)
    allowed[:, C:] = np.tril(np.ones((L, L), dtype=bool))
    S = np.where(allowed, S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    Pm = np.exp(S)
    Pm /= Pm.sum(axis=1, keepdims=True)
    return Pm @ V


def greedy_accept(beam, am_of_node, node_id, root_token=None):
    """Pure-Python token matching for one sequence.  am_of_node[n] = LLM prediction after node n."""
    W, L = len(beam), len(beam[0])
    n_accept = []
    for w in range(W):
        n = 0
        for j in range(L):
            if j == 0:
                ok = root_token is None or int(beam[w][0]) == int(root_token)
            else:
                ok = int(am_of_node[node_id[w][j - 1]]) == int(beam[w][j])
            if not ok:
                break
            n += 1
        n_accept.append(n)
    best_len = max(n_accept)
    best_beam = n_accept.index(best_len)
    return n_accept, best_beam, best_len


def toy_lm_next(prefix, V, salt=0):
    """Deterministic toy LM: next token is a hash of the whole prefix."""
    h = 1469598103934665603 ^ salt
    for t in prefix:
        h = ((h ^ (int(t) + 1)) * 1099511628211) % (1 << 64)
    return int(h % V)


def greedy_rollout(start_prefix, n_steps, V, salt=0):
    seq = list(start_prefix)
    out = []
    for _ in range(n_steps):
        t = toy_lm_next(seq, V, salt)
        out.append(t)
        seq.append(t)
    return out


class ToyAttentionLM:
    """A one-layer attention "LLM" in numpy float64, for end-to-end checks of the whole step.

    Token t contributes key Ek[t] and value Ev[t] (per head); the model's output at the last token
    of a sequence is plain softmax attention of Eq[last token] over the keys of ALL tokens of the
    sequence (itself included), heads concatenated, times a readout matrix.  It is a deterministic
    function of the sequence, so greedy decoding with it is well defined."""

    def __init__(self, V, H, D, seed):
        rng = np.random.default_rng(seed)
        self.V, self.H, self.D = V, H, D
        self.Eq = rng.standard_normal((V, H, D)).astype(np.float32)
        self.Ek = rng.standard_normal((V, H, D)).astype(np.float32)
        self.Ev = rng.standard_normal((V, H, D)).astype(np.float32)
        self.Wout = rng.standard_normal((H * D, V)).astype(np.float32)
        self.scale = 1.0 / np.sqrt(D)

    def logits_from_attn(self, out_hd):
        """out_hd [..., H, D] (attention output at a token) -> logits [..., V]."""
        o = np.asarray(out_hd, np.float64)
        return o.reshape(o.shape[:-2] + (self.H * self.D,)) @ self.Wout.astype(np.float64)

    def next_logits(self, seq):
        seq = np.asarray(seq, np.int64)
        q = self.Eq[seq[-1]].astype(np.float64)              # [H, D]
        k = self.Ek[seq].astype(np.float64)                  # [T, H, D]
        v = self.Ev[seq].astype(np.float64)
        out = np.empty((self.H, self.D))
        for h in range(self.H):
            s = (k[:, h, :] @ q[h]) * self.scale
            w = np.exp(s - s.max())
            out[h] = (w / w.sum()) @ v[:, h, :]
        return self.logits_from_attn(out)

    def greedy(self, prompt, n_new):
        seq = list(prompt)
        for _ in range(n_new):
            seq.append(int(np.argmax(self.next_logits(seq))))
        return seq
