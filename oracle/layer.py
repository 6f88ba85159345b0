"""Plain fp64 definition of one pre-norm GQA transformer layer run over a batch
of independent token blocks, as used by parallel context compaction.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
CPU-baseline leg of the benchmark.  It shares no code with the HIP library
and must never be reachable from the product path.

What it follows.  The method (paper Sec. IV, "Parallel Compaction") cuts the
conversation snapshot into N contiguous blocks, hands every block to its own
worker concurrently and concatenates the per-block results in block order.
In the independent-chunk arrangement discussed in the same section each worker
sees only its own block, so on the device the N workers are one ragged batch
in which no token attends outside its block.  The paper treats the model as a
black box (Sec. IV-A lists Llama-3.x dense and gpt-oss MoE backbones), so the
layer itself is the textbook one: RMSNorm -> QKV -> rotary embedding -> causal
softmax attention with grouped KV heads -> output projection + residual ->
RMSNorm -> SwiGLU feed-forward (dense, or top-k routed experts) + residual.

Everything is written as the definition: the full score matrix per (block,
head), ordinary matrix products, a full sort for top-k.  No tiling, no online
softmax, no fusion.  All arithmetic is float64; inputs arrive already rounded
to the storage type of the case under test and are only widened here.

Parity pins (tests/test_oracle_*.py): softmax rows sum to one; identical keys
give the running mean of the values; a two-token case worked by hand
(tests/golden/two_token_attention.txt); batched == one block at a time;
prefill(L+1) == prefill(L) + one decode step; causality; rotary invariants and
a complex-number restatement; RMSNorm scale invariance; GQA == MHA with
duplicated KV weights; SwiGLU special cases; router brute force and the
identical-experts == dense equivalence; and a whole-layer cross-check against
library fp64 routines (torch CPU rms_norm / scaled_dot_product_attention /
silu).  Conventions that no mathematics fixes -- the rotate-half pairing of
rotary dimensions and the contiguous grouping of query heads onto KV heads --
are pinned only to the library routines' conventions.  The prefix-aware
layout is pinned by lone runs on truncated histories; the depth of layers
(Stack) by library layers applied in turn, an inserted identity layer, and
decode == longer prefill through the whole depth.
"""
import math

import numpy as np

F64 = np.float64


def _f64(a):
    return np.asarray(a, dtype=F64)


# ---------------------------------------------------------------------------
# elementary pieces
# ---------------------------------------------------------------------------
def rmsnorm(x, g, eps):
    """n = x / sqrt(mean_d(x^2) + eps) * g, per token (last axis)."""
    x = _f64(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * _f64(g)


def rope(x, pos, theta):
    """Rotary embedding, rotate-half pairing.

    x [T, H, hd]; pos [T] integer positions.  For i < hd/2 the pair
    (x_i, x_{i+hd/2}) is rotated by the angle pos * theta**(-2i/hd).
    """
    x = _f64(x)
    hd = x.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=F64)
    freq = np.power(F64(theta), -2.0 * i / hd)
    phi = _f64(pos)[:, None] * freq[None, :]            # [T, half]
    c = np.cos(phi)[:, None, :]
    s = np.sin(phi)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def softmax_rows(s):
    """Row softmax with the row maximum subtracted; -inf entries get weight 0."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_probs(q, k, visible):
    """Softmax weights of R query rows over J keys for one head.

    q [R, hd], k [J, hd]; visible[r] = number of leading keys row r may see
    (key j is masked out when j >= visible[r]).  Scale 1/sqrt(hd).
    """
    q, k = _f64(q), _f64(k)
    hd = q.shape[-1]
    s = (q @ k.T) / math.sqrt(hd)                       # full [R, J] scores
    j = np.arange(k.shape[0])[None, :]
    s = np.where(j < np.asarray(visible)[:, None], s, -np.inf)
    return softmax_rows(s)


def attention_head(q, k, v, visible):
    """o_r = sum_j a_rj v_j for one head."""
    return attention_probs(q, k, visible) @ _f64(v)


def gqa_attention(q, k, v, visible):
    """q [R, Hq, hd], k/v [J, Hkv, hd] -> o [R, Hq, hd].

    Query head h reads KV head h // (Hq // Hkv) (contiguous groups).
    """
    R, Hq, hd = q.shape
    Hkv = k.shape[1]
    group = Hq // Hkv
    o = np.empty((R, Hq, hd), dtype=F64)
    for h in range(Hq):
        o[:, h, :] = attention_head(q[:, h, :], k[:, h // group, :],
                                    v[:, h // group, :], visible)
    return o


def linear(x, w):
    """x W^T with W stored [out, in]."""
    return _f64(x) @ _f64(w).T


def silu(z):
    return z / (1.0 + np.exp(-z))


def swiglu_ffn(m, w_gate, w_up, w_down):
    """(silu(m Wg^T) * (m Wu^T)) Wd^T; weights are [out, in]."""
    m = _f64(m)
    return (silu(m @ _f64(w_gate).T) * (m @ _f64(w_up).T)) @ _f64(w_down).T


def router_logits(m, w_router):
    return _f64(m) @ _f64(w_router).T


def topk_route(logits, k):
    """Indices of the k largest logits per row (descending; equal logits ->
    lower expert index first) and the softmax over just those k logits."""
    logits = _f64(logits)
    order = np.argsort(-logits, axis=-1, kind="stable")  # full sort
    idx = order[:, :k]
    sel = np.take_along_axis(logits, idx, axis=-1)
    return idx.astype(np.int32), softmax_rows(sel)


def moe_ffn(m, idx, gate, w_exp_gate_up, w_exp_down):
    """sum_{e in idx[r]} gate[r,e] * FFN_e(m_r).  No capacity limit, no drops.

    w_exp_gate_up [E, 2F, d] (rows 0..F-1 gate, F..2F-1 up), w_exp_down [E, d, F].
    """
    m = _f64(m)
    F = w_exp_gate_up.shape[1] // 2
    out = np.zeros((m.shape[0], w_exp_down.shape[1]), dtype=F64)
    for e in np.unique(idx):
        rows, slot = np.nonzero(idx == e)
        y = swiglu_ffn(m[rows], w_exp_gate_up[e, :F], w_exp_gate_up[e, F:],
                       w_exp_down[e])
        out[rows] += gate[rows, slot][:, None] * y
    return out


# ---------------------------------------------------------------------------
# the layer
# ---------------------------------------------------------------------------
class Layer:
    """Weights in the layout of the library boundary, all [out, in] row-major.

    cfg keys: d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, n_experts
    (0 = dense), top_k, rms_eps, rope_theta.
    w keys: g_attn [d], w_qkv [Dq+2Dkv, d], w_o [d, Dq], g_ffn [d], and either
    w_gate_up [2F, d], w_down [d, F] (dense) or w_router [E, d],
    w_exp_gate_up [E, 2F, d], w_exp_down [E, d, F] (MoE).
    """

    def __init__(self, cfg, w):
        self.cfg = dict(cfg)
        self.w = w
        c = self.cfg
        self.d = c["d_model"]
        self.Hq, self.Hkv, self.hd = c["n_q_heads"], c["n_kv_heads"], c["head_dim"]
        self.Dq, self.Dkv = self.Hq * self.hd, self.Hkv * self.hd
        self.F = c["ffn_dim"]
        self.E = c.get("n_experts", 0)
        self.k = c.get("top_k", 0)
        self.eps = c["rms_eps"]
        self.theta = c["rope_theta"]

    # -- attention half -----------------------------------------------------
    def qkv(self, x, pos):
        """RMSNorm, QKV projection and rotary embedding for the rows of x."""
        n = rmsnorm(x, self.w["g_attn"], self.eps)
        p = n @ _f64(self.w["w_qkv"]).T
        T = p.shape[0]
        q = p[:, :self.Dq].reshape(T, self.Hq, self.hd)
        k = p[:, self.Dq:self.Dq + self.Dkv].reshape(T, self.Hkv, self.hd)
        v = p[:, self.Dq + self.Dkv:].reshape(T, self.Hkv, self.hd)
        return rope(q, pos, self.theta), rope(k, pos, self.theta), v

    # -- feed-forward half --------------------------------------------------
    def ffn(self, h, forced_idx=None):
        """Second RMSNorm, feed-forward, residual.  Returns (y, idx, gate, router logits).

        forced_idx [R, k] (routed layers only) replaces the top-k selection: row r
        is sent to exactly those experts, gated by the softmax over ITS logits at
        those experts.  The parity tests use it where two experts' logits are
        closer than the storage rounding of the path under test, so that both
        choices are correct: the layer is then evaluated for the choice made.
        """
        m = rmsnorm(h, self.w["g_ffn"], self.eps)
        if self.E == 0:
            F = self.F
            wgu = self.w["w_gate_up"]
            return h + swiglu_ffn(m, wgu[:F], wgu[F:], self.w["w_down"]), None, None, None
        logits = router_logits(m, self.w["w_router"])
        if forced_idx is None:
            idx, gate = topk_route(logits, self.k)
        else:
            idx = np.asarray(forced_idx, dtype=np.int32).reshape(logits.shape[0], self.k)
            gate = softmax_rows(np.take_along_axis(logits, idx.astype(np.int64), axis=-1))
        y = h + moe_ffn(m, idx, gate, self.w["w_exp_gate_up"], self.w["w_exp_down"])
        return y, idx, gate, logits

    # -- one block ----------------------------------------------------------
    def prefill_block(self, x, pos0=0, rows=None, forced_idx=None):
        """Causal forward over one block's own L tokens.

        x [L, d].  Positions are pos0 .. pos0+L-1.  K and V are produced for
        every token; attention and everything after it are evaluated for the
        query rows in `rows` (default: all).  Returns dict with y [R, d],
        K, V [L, Hkv, hd] (K after rotation), rows, idx, gate, logits and h (the
        rows after the attention half).  forced_idx [R, k]: see ffn.
        """
        x = _f64(x)
        L = x.shape[0]
        pos = pos0 + np.arange(L)
        q, k, v = self.qkv(x, pos)
        rows = np.arange(L) if rows is None else np.asarray(rows, dtype=np.int64)
        o = gqa_attention(q[rows], k, v, visible=rows + 1)     # row i sees j <= i
        h = x[rows] + o.reshape(len(rows), self.Dq) @ _f64(self.w["w_o"]).T
        y, idx, gate, logits = self.ffn(h, forced_idx)
        return dict(y=y, K=k, V=v, rows=rows, idx=idx, gate=gate, logits=logits, h=h)

    def decode_block(self, x, K, V, pos0=0, forced_idx=None):
        """One new token for one block whose cache holds len = K.shape[0] rows.

        The token sits at position pos0 + len, its K/V row is appended, and it
        attends rows 0..len inclusive.  Returns dict with y [d], K, V grown by
        one row, idx, gate.
        """
        x = _f64(x).reshape(1, self.d)
        n_cached = K.shape[0]
        q, k, v = self.qkv(x, np.array([pos0 + n_cached]))
        K = np.concatenate([K, k], axis=0)
        V = np.concatenate([V, v], axis=0)
        o = gqa_attention(q, K, V, visible=np.array([n_cached + 1]))
        h = x + o.reshape(1, self.Dq) @ _f64(self.w["w_o"]).T
        y, idx, gate, logits = self.ffn(h, forced_idx)
        return dict(y=y[0], K=K, V=V, h=h[0],
                    idx=None if idx is None else idx[0],
                    gate=None if gate is None else gate[0],
                    logits=None if logits is None else logits[0])

    def extend_block(self, x, K, V, pos0=0, rows=None, forced_idx=None):
        """The next chunk of a block whose cache already holds len = K.shape[0]
        rows (a prefill cut into chunks, Sec. IV-B: the server prefills long
        prompts chunk by chunk; also a worker's own block behind a cached prefix).

        x [C, d] sits at positions pos0 + len .. pos0 + len + C - 1; its K/V rows
        are appended and chunk row i attends cache rows 0 .. len + i.  Returns a
        dict like prefill_block, K and V grown by C rows.
        """
        x = _f64(x)
        C = x.shape[0]
        n_cached = K.shape[0]
        q, k, v = self.qkv(x, pos0 + n_cached + np.arange(C))
        K = np.concatenate([K, k], axis=0)
        V = np.concatenate([V, v], axis=0)
        rows = np.arange(C) if rows is None else np.asarray(rows, dtype=np.int64)
        o = gqa_attention(q[rows], K, V, visible=n_cached + rows + 1)
        h = x[rows] + o.reshape(len(rows), self.Dq) @ _f64(self.w["w_o"]).T
        y, idx, gate, logits = self.ffn(h, forced_idx)
        return dict(y=y, K=K, V=V, rows=rows, idx=idx, gate=gate, logits=logits, h=h)

    # -- the batch of blocks ------------------------------------------------
    def prefill(self, x, cu_seqlens, pos_offset=None, rows=None, forced_idx=None):
        """Block b = rows cu[b]..cu[b+1]-1 of the packed x [T, d]; blocks are
        independent.  rows: optional list (per block) of block-local query rows.
        forced_idx: optional list (per block) of [R_b, k] expert choices (see ffn).
        Returns one prefill_block dict per block, in block order."""
        out = []
        for b in range(len(cu_seqlens) - 1):
            xb = x[cu_seqlens[b]:cu_seqlens[b + 1]]
            out.append(self.prefill_block(
                xb, 0 if pos_offset is None else int(pos_offset[b]),
                None if rows is None else rows[b],
                None if forced_idx is None else forced_idx[b]))
        return out

    def decode_step(self, x, Ks, Vs, pos_offset=None, forced_idx=None):
        """x [N, d]: one token per block, each against its own cache.
        forced_idx: optional [N, k] expert choices (see ffn)."""
        out = []
        for b in range(len(Ks)):
            out.append(self.decode_block(
                x[b], Ks[b], Vs[b], 0 if pos_offset is None else int(pos_offset[b]),
                None if forced_idx is None else forced_idx[b]))
        return out

    def forward(self, x_prefill, cu_seqlens, x_decode, pos_offset=None, rows=None):
        """Prefill of every block, then S batched decode steps with the given
        step inputs x_decode [S, N, d].  Returns (prefill dicts, y_decode
        [S, N, d], final K list, final V list, per step and block the tuple
        (idx, gate, router logits, h))."""
        pre = self.prefill(x_prefill, cu_seqlens, pos_offset, rows)
        Ks = [p["K"] for p in pre]
        Vs = [p["V"] for p in pre]
        S = 0 if x_decode is None else x_decode.shape[0]
        N = len(Ks)
        y_dec = np.zeros((S, N, self.d), dtype=F64)
        routes = []
        for s in range(S):
            st = self.decode_step(x_decode[s], Ks, Vs, pos_offset)
            for b in range(N):
                y_dec[s, b] = st[b]["y"]
                Ks[b], Vs[b] = st[b]["K"], st[b]["V"]
            routes.append([(st[b]["idx"], st[b]["gate"], st[b]["logits"], st[b]["h"]) for b in range(N)])
        return pre, y_dec, Ks, Vs, routes

    # -- prefix-aware layout ------------------------------------------------
    def decode_block_prefix(self, x, Kp, Vp, prefix_len, Kt, Vt, forced_idx=None):
        """One new token of worker k in the prefix-aware target-at-end layout
        (paper Sec. IV, Dispatch: worker k's prompt is blocks 1..k in order, so
        every worker's prefix extends the previous one's and its cache is
        shared).  The worker sees the first `prefix_len` rows of the shared
        cache (Kp, Vp: the whole history, computed once) followed by its own
        private tail (Kt, Vt: the tokens it has generated so far).  The new
        token sits at position prefix_len + len(tail); its K/V row is appended
        to the tail.  Returns dict with y [d], Kt, Vt grown by one row."""
        x = _f64(x).reshape(1, self.d)
        n_tail = Kt.shape[0]
        q, k, v = self.qkv(x, np.array([prefix_len + n_tail]))
        Kt = np.concatenate([Kt, k], axis=0)
        Vt = np.concatenate([Vt, v], axis=0)
        K = np.concatenate([Kp[:prefix_len], Kt], axis=0)
        V = np.concatenate([Vp[:prefix_len], Vt], axis=0)
        o = gqa_attention(q, K, V, visible=np.array([K.shape[0]]))
        h = x + o.reshape(1, self.Dq) @ _f64(self.w["w_o"]).T
        y, idx, gate, logits = self.ffn(h, forced_idx)
        return dict(y=y[0], Kt=Kt, Vt=Vt, h=h[0],
                    idx=None if idx is None else idx[0],
                    gate=None if gate is None else gate[0],
                    logits=None if logits is None else logits[0])

    def forward_prefix(self, x_history, cu_seqlens, x_decode, rows=None):
        """Prefix-aware pass: the history is prefilled once as ONE causal
        sequence (every worker's prompt is a prefix of it, so its cache rows are
        the workers' shared prefix), then worker b decodes S tokens against rows
        0 .. cu[b+1]-1 of that cache plus its own tail.  x_decode [S, N, d].
        Returns (prefill dict of the whole history, y_decode [S, N, d],
        tail K list, tail V list)."""
        pre = self.prefill_block(_f64(x_history), 0, rows)
        Kp, Vp = pre["K"], pre["V"]
        N = len(cu_seqlens) - 1
        S = 0 if x_decode is None else x_decode.shape[0]
        Kt = [np.zeros((0, self.Hkv, self.hd), dtype=F64) for _ in range(N)]
        Vt = [np.zeros((0, self.Hkv, self.hd), dtype=F64) for _ in range(N)]
        y_dec = np.zeros((S, N, self.d), dtype=F64)
        for s in range(S):
            for b in range(N):
                st = self.decode_block_prefix(x_decode[s, b], Kp, Vp, int(cu_seqlens[b + 1]), Kt[b], Vt[b])
                y_dec[s, b] = st["y"]
                Kt[b], Vt[b] = st["Kt"], st["Vt"]
        return pre, y_dec, Kt, Vt

    def forward_sampled(self, x_prefill, cu_seqlens, x_decode, rows, steps, pos_offset=None):
        """The same pass, evaluated only at sampled places (for workloads too
        large to check everywhere).  Because the decode-step inputs are given
        rather than generated, the K/V rows of every decode token follow from
        x_decode alone; they are appended to each block's cache up front, and
        attention + feed-forward are then evaluated for the prefill query rows
        `rows[b]` and for the decode steps in `steps` (step s of block b sees
        cache rows 0 .. L_b + s).  Returns (prefill dicts, {s: y [N, d]},
        K list, V list, {s: (idx, gate, logits, h)})."""
        pre = self.prefill(x_prefill, cu_seqlens, pos_offset, rows)
        S, N = x_decode.shape[0], len(pre)
        Ks, Vs, qs = [], [], []
        for b in range(N):
            L = pre[b]["K"].shape[0]
            p0 = 0 if pos_offset is None else int(pos_offset[b])
            q, k, v = self.qkv(_f64(x_decode[:, b]), p0 + L + np.arange(S))
            Ks.append(np.concatenate([pre[b]["K"], k], axis=0))
            Vs.append(np.concatenate([pre[b]["V"], v], axis=0))
            qs.append(q)
        y_dec, routes = {}, {}
        for s in steps:
            o = np.stack([gqa_attention(qs[b][s:s + 1], Ks[b], Vs[b],
                                        visible=np.array([pre[b]["K"].shape[0] + s + 1]))[0]
                          for b in range(N)])
            h = _f64(x_decode[s]) + o.reshape(N, self.Dq) @ _f64(self.w["w_o"]).T
            y, idx, gate, logits = self.ffn(h)
            y_dec[s] = y
            routes[s] = (idx, gate, logits, h)
        return pre, y_dec, Ks, Vs, routes


class Stack:
    """A depth of L layers run over the batch of blocks (the full model the
    paper's workers run, Sec. IV-A, minus embedding and output head): the
    output rows of layer l are the input rows of layer l + 1, in prefill (all
    rows of every block) and in each decode step (one row per block); every
    layer keeps its own K/V cache per block.  Nothing else connects the layers.
    """

    def __init__(self, cfg, weights):
        """weights: one weight dict per layer."""
        self.layers = [Layer(cfg, w) for w in weights]

    def forward(self, x_prefill, cu_seqlens, x_decode, pos_offset=None, forced=None):
        """Returns (y_prefill [T, d] of the last layer, y_decode [S, N, d] of the
        last layer, per-layer K lists, per-layer V lists).  forced (routed layers):
        per layer a pair (packed [T, k] prefill expert choices, [S, N, k] decode
        ones), see Layer.ffn; self.routes then holds per layer the router logits
        (packed [T, E] prefill, [S, N, E] decode) of the pass."""
        x = _f64(x_prefill)
        N = len(cu_seqlens) - 1
        Ks, Vs = [], []
        self.routes = []
        for li, lay in enumerate(self.layers):
            fi = None if forced is None else [forced[li][0][cu_seqlens[b]:cu_seqlens[b + 1]] for b in range(N)]
            pre = lay.prefill(x, cu_seqlens, pos_offset, forced_idx=fi)
            self.routes.append(dict(pre_logits=None if lay.E == 0 else np.concatenate([p["logits"] for p in pre]),
                                    pre_idx=None if lay.E == 0 else np.concatenate([p["idx"] for p in pre]),
                                    dec_logits=[], dec_idx=[]))
            Ks.append([p["K"] for p in pre])
            Vs.append([p["V"] for p in pre])
            x = np.concatenate([p["y"] for p in pre], axis=0)
        y_pre = x
        S = 0 if x_decode is None else x_decode.shape[0]
        y_dec = np.zeros((S, N, self.layers[0].d), dtype=F64)
        for s in range(S):
            xs = _f64(x_decode[s])
            for li, lay in enumerate(self.layers):
                st = lay.decode_step(xs, Ks[li], Vs[li], pos_offset,
                                     None if forced is None else forced[li][1][s])
                for b in range(N):
                    Ks[li][b], Vs[li][b] = st[b]["K"], st[b]["V"]
                if lay.E:
                    self.routes[li]["dec_logits"].append(np.stack([st[b]["logits"] for b in range(N)]))
                    self.routes[li]["dec_idx"].append(np.stack([st[b]["idx"] for b in range(N)]))
                xs = np.stack([st[b]["y"] for b in range(N)])
            y_dec[s] = xs
        return y_pre, y_dec, Ks, Vs

    def forward_prefix(self, x_history, cu_seqlens, x_decode):
        """The depth of layers in the prefix-aware target-at-end layout (Sec. IV,
        Dispatch): every layer prefills the whole history as one causal block
        (its cache is shared by the workers), then in each decode step worker b's
        token goes through all layers, attending in layer l rows 0 .. cu[b+1]-1
        of that layer's shared cache plus its own tail in that layer.  Returns
        (y_decode [S, N, d] of the last layer, per-layer shared (K, V), per-layer
        per-worker tail K lists, tail V lists)."""
        x = _f64(x_history)
        N = len(cu_seqlens) - 1
        shared = []
        for lay in self.layers:
            pre = lay.prefill_block(x)
            shared.append((pre["K"], pre["V"]))
            x = pre["y"]
        S = x_decode.shape[0]
        lay0 = self.layers[0]
        Kt = [[np.zeros((0, lay0.Hkv, lay0.hd)) for _ in range(N)] for _ in self.layers]
        Vt = [[np.zeros((0, lay0.Hkv, lay0.hd)) for _ in range(N)] for _ in self.layers]
        y_dec = np.zeros((S, N, lay0.d), dtype=F64)
        for s in range(S):
            xs = _f64(x_decode[s])
            for li, lay in enumerate(self.layers):
                ys = np.zeros_like(xs)
                for b in range(N):
                    st = lay.decode_block_prefix(xs[b], shared[li][0], shared[li][1], int(cu_seqlens[b + 1]),
                                                 Kt[li][b], Vt[li][b])
                    Kt[li][b], Vt[li][b] = st["Kt"], st["Vt"]
                    ys[b] = st["y"]
                xs = ys
            y_dec[s] = xs
        return y_dec, shared, Kt, Vt
