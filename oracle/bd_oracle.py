"""CPU oracle for the block-denoising decode path of the block-diffusion VLM.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP path is checked
against.  Only tests, the smoke check and the benchmark's cpu_baseline leg may import it; the
product path never does.  It shares no code with the HIP library: no kernels, headers, tables
or helpers.  It receives its inputs (weights, prompt, drafts) as arrays.

Arithmetic: numpy, float64 by default (`dtype=` selects float32).  Every matrix product is a
single library matmul over the whole operand; attention builds the dense score matrix over all
visible keys and takes an ordinary softmax; nothing is tiled, fused or reordered.

What it follows (the paper, by section):
  * Sec. 3.4 "Inference": decoding proceeds block by block re-using a KV cache; inside a block
    masked positions are revealed by confidence-aware parallel decoding with threshold tau;
    each block is seeded by one autoregressive prediction from the cached causal context.
  * Sec. 3.3 attention-mask rules: noisy (block) tokens attend bidirectionally inside their
    block and to all preceding clean context; clean context is token-level causal.
  * Appendix "Details of Speculative Decoding", Alg. 1: the draft forward (bidirectional in the
    block, whole prefix visible, cache not updated, hidden state i-1 predicts position i), the
    verify forward (causal in the block, cache updated), the left-to-right accept rule and the
    cache crop.
  * "Decoding threshold" paragraph: at tau = 1.0 exactly one token is revealed per step.
The paper only names the backbone; its layer equations (pre-RMSNorm, grouped-query attention,
1-D rotary embedding with half-split pairing, SwiGLU, no biases, separate LM head) are the
standard ones for that backbone family and are fixed by the configuration text.

Pins (tests/test_oracle_*.py): an independent full-sequence PyTorch model with a literally built
dense mask (forward, prefill, KV-cache equivalence), greedy AR equivalence at B=1, sequential
single-token equivalence of a block commit, rotary closed forms, unmask-rule invariants and
closed forms, accept-rule cases, speculative decoding == greedy AR.
Readings of points the paper leaves open that no pin can fix (forced seed, strict '>' against
tau, tie-breaks toward the lowest index, mask id = vocab-1): parity unpinned for those choices;
they are listed in the design notes.
"""
from __future__ import annotations

import numpy as np

BIDIR = 0    # in-block keys all visible            (Alg. 1, draft mask)
CAUSAL = 1   # in-block key j visible to row i iff j <= i   (Alg. 1, verify mask)


def _decode_e4m3(codes: np.ndarray) -> np.ndarray:
    """OCP e4m3fn byte -> value: sign, 4 exponent bits (bias 7), 3 mantissa bits, no infinities."""
    c = codes.astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 0x7).astype(np.float64)
    sub = m / 8.0 * 2.0 ** -6
    nor = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    v = np.where(e == 0, sub, nor)
    v = np.where((e == 0xF) & ((c & 0x7) == 0x7), np.nan, v)
    return sign * v


class BlockDiffusionOracle:
    """State = per-layer KV cache of the committed context, its length n, and the carry row."""

    def __init__(self, shape, weights, dtype=np.float64):
        self.s = shape
        self.w = weights
        self.dt = np.dtype(dtype)
        self.mask_id = shape.vocab - 1
        self.reset()

    # ---- plumbing -------------------------------------------------------------------------
    def reset(self):
        self.n = 0
        self.K = [np.zeros((0, self.s.n_kv_heads, self.s.head_dim), self.dt) for _ in range(self.s.n_layers)]
        self.V = [np.zeros((0, self.s.n_kv_heads, self.s.head_dim), self.dt) for _ in range(self.s.n_layers)]
        self.carry = None          # logits row that predicts the token at position n

    def _mat(self, name):
        """Weight matrix [out, in] as real values in the compute dtype."""
        w = self.w[name]
        if w.dtype == np.uint8:    # e4m3 codes with one scale per output channel
            return (_decode_e4m3(w) * self.w[name + ".scale"].astype(np.float64)[:, None]).astype(self.dt)
        return w.astype(self.dt, copy=False)

    def embed(self, ids):
        return self._mat_rows("embed", np.asarray(ids, dtype=np.int64))

    def _mat_rows(self, name, rows):
        return self.w[name][rows].astype(self.dt)

    # ---- layer pieces ---------------------------------------------------------------------
    def rmsnorm(self, x, gain):
        ms = np.mean(x * x, axis=-1, keepdims=True)
        return x / np.sqrt(ms + self.dt.type(self.s.rms_eps)) * gain.astype(self.dt)

    def rope(self, x, pos):
        """x [M, heads, d]; rotate pair (x_i, x_{i+d/2}) by angle pos * theta^(-2i/d)."""
        d = self.s.head_dim
        half = d // 2
        inv = np.asarray(self.s.rope_theta, np.float64) ** (-np.arange(half, dtype=np.float64) * 2.0 / d)
        ang = np.asarray(pos, np.float64)[:, None] * inv[None, :]          # [M, half]
        c = np.cos(ang).astype(self.dt)[:, None, :]
        s = np.sin(ang).astype(self.dt)[:, None, :]
        a, b = x[..., :half], x[..., half:]
        return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)

    def attention(self, q, keys, vals, n_prefix, mode, vis_block=None):
        """q [M,n_q,d] (rotated), keys/vals [n_prefix+M, n_kv, d] -> [M, n_q*d].

        Visibility (Sec. 3.3 mask rules; Alg. 1 draft / verify masks): every prefix key is visible
        to every row; in-block key j is visible to row i always (BIDIR) or iff j <= i (CAUSAL).
        vis_block [M, M] (Alg. 2: the quadratic mask) replaces the in-block rule when given.
        """
        M = q.shape[0]
        T = keys.shape[0]
        G = self.s.n_q_heads // self.s.n_kv_heads
        vis = np.ones((M, T), dtype=bool)
        if vis_block is not None:
            vis[:, n_prefix:] = np.asarray(vis_block, bool)
        elif mode == CAUSAL:
            i = np.arange(M)[:, None]
            j = np.arange(T)[None, :] - n_prefix
            vis = (j < 0) | (j <= i)
        out = np.empty((M, self.s.n_q_heads, self.s.head_dim), self.dt)
        scale = self.dt.type(1.0) / np.sqrt(self.dt.type(self.s.head_dim))
        for h in range(self.s.n_q_heads):
            g = h // G
            sc = (q[:, h, :] @ keys[:, g, :].T) * scale                     # [M, T]
            sc = np.where(vis, sc, -np.inf)
            sc = sc - sc.max(axis=1, keepdims=True)
            p = np.exp(sc)
            p = p / p.sum(axis=1, keepdims=True)
            out[:, h, :] = p @ vals[:, g, :]
        return out.reshape(M, -1)

    def forward(self, x, mode, want_logits_rows=None, pos=None, vis_block=None):
        """One decoder forward over M new rows at positions n..n+M-1 against the cached prefix.

        Returns (logits [rows, vocab], new K per layer, new V per layer); the cache is untouched.
        pos / vis_block (Alg. 2): explicit position ids of the rows and an explicit [M, M] in-block mask.
        """
        s = self.s
        x = np.asarray(x, self.dt)
        M = x.shape[0]
        pos = np.arange(self.n, self.n + M) if pos is None else np.asarray(pos)
        newK, newV = [], []
        for l in range(s.n_layers):
            p = f"l{l}."
            xh = self.rmsnorm(x, self.w[p + "attn_norm"])
            q = (xh @ self._mat(p + "wq").T).reshape(M, s.n_q_heads, s.head_dim)
            k = (xh @ self._mat(p + "wk").T).reshape(M, s.n_kv_heads, s.head_dim)
            v = (xh @ self._mat(p + "wv").T).reshape(M, s.n_kv_heads, s.head_dim)
            q = self.rope(q, pos)
            k = self.rope(k, pos)
            keys = np.concatenate([self.K[l][:self.n], k], axis=0)
            vals = np.concatenate([self.V[l][:self.n], v], axis=0)
            o = self.attention(q, keys, vals, self.n, mode, vis_block)
            x = x + o @ self._mat(p + "wo").T
            hh = self.rmsnorm(x, self.w[p + "ffn_norm"])
            gate = hh @ self._mat(p + "w_gate").T
            up = hh @ self._mat(p + "w_up").T
            act = gate / (1.0 + np.exp(-gate)) * up
            x = x + act @ self._mat(p + "w_down").T
            newK.append(k)
            newV.append(v)
        xf = self.rmsnorm(x, self.w["final_norm"])
        if want_logits_rows is not None:
            xf = xf[want_logits_rows]
        logits = xf @ self._mat("lm_head").T
        return logits, newK, newV

    def _append(self, newK, newV):
        for l in range(self.s.n_layers):
            self.K[l] = np.concatenate([self.K[l][:self.n], newK[l]], axis=0)
            self.V[l] = np.concatenate([self.V[l][:self.n], newV[l]], axis=0)
        self.n += newK[0].shape[0]

    # ---- confidence -----------------------------------------------------------------------
    @staticmethod
    def cand_conf(logits):
        """argmax id (lowest id on ties) and its softmax probability, per row."""
        cand = np.argmax(logits, axis=-1)
        z = logits - logits.max(axis=-1, keepdims=True)
        conf = 1.0 / np.exp(z).sum(axis=-1)
        return cand.astype(np.int32), conf

    # ---- the calls of the boundary --------------------------------------------------------
    def prefill(self, embeds, ids, chunk=None):
        """Alg. 1 prefill: causal forward over the prompt (continuous embeddings, then embedded
        ids); keeps K,V of every layer; the last row's logits become the carry.
        chunk=None runs it in one forward; an integer processes that many rows at a time
        (identical by the KV-cache equivalence the tests pin)."""
        self.reset()
        parts = []
        if embeds is not None and len(embeds):
            parts.append(np.asarray(embeds, self.dt))
        if ids is not None and len(ids):
            parts.append(self.embed(ids))
        x = np.concatenate(parts, axis=0)
        step = x.shape[0] if chunk is None else int(chunk)
        for a in range(0, x.shape[0], step):
            xb = x[a:a + step]
            logits, nk, nv = self.forward(xb, CAUSAL, want_logits_rows=[xb.shape[0] - 1])
            self._append(nk, nv)
            self.carry = logits[0]

    def denoise_step(self, tokens, mask, tau, fixed_k=0):
        """One denoising step on a block (Sec. 3.4; Alg. 1 draft step; threshold paragraph).

        tokens int[B], mask bool[B] (True = still masked) are updated in place.
        Returns dict(n_unmasked, conf[B], logits or None).
        """
        B = len(tokens)
        n_un = 0
        conf_out = np.zeros(B, np.float64)
        cand0, conf0 = self.cand_conf(self.carry[None, :])
        conf_out[0] = conf0[0]
        if mask[0]:                                   # seed from the cached causal context
            tokens[0] = cand0[0]
            mask[0] = False
            n_un += 1
        if B == 1 or not mask.any():
            return dict(n_unmasked=n_un, conf=conf_out, logits=None)
        d = np.where(mask, self.mask_id, tokens)
        logits, _, _ = self.forward(self.embed(d), BIDIR)             # cache not updated
        cand, conf = self.cand_conf(logits)
        conf_out[1:] = conf[:-1]                      # row i-1 predicts block position i
        masked = [i for i in range(1, B) if mask[i]]
        if fixed_k and fixed_k > 0:
            order = sorted(masked, key=lambda i: (-conf[i - 1], i))
            chosen = order[:min(fixed_k, len(order))]
        else:
            chosen = [i for i in masked if conf[i - 1] > tau]
            if not chosen:
                chosen = [min(masked, key=lambda i: (-conf[i - 1], i))]
        for i in chosen:
            tokens[i] = cand[i - 1]
            mask[i] = False
        n_un += len(chosen)
        return dict(n_unmasked=n_un, conf=conf_out, logits=logits)

    def commit_block(self, tokens):
        """Causal forward over the finished block, K/V appended, last row -> carry."""
        tokens = np.asarray(tokens)
        if np.any(tokens == self.mask_id):
            raise ValueError("commit of a block that still holds the mask token")
        logits, nk, nv = self.forward(self.embed(tokens), CAUSAL)
        self._append(nk, nv)
        self.carry = logits[-1]
        return logits

    def verify_block(self, draft, commit=True):
        """Alg. 1 verify + accept on B drafted ids: a_j = argmax of causal row j; draft 0 is held
        against the carry's argmax, draft j+1 against a_j; n_accept = longest matching prefix."""
        draft = np.asarray(draft)
        B = len(draft)
        logits, nk, nv = self.forward(self.embed(draft), CAUSAL)
        a, _ = self.cand_conf(logits)
        pred = np.concatenate([self.cand_conf(self.carry[None, :])[0], a[:-1]])
        n_accept = 0
        while n_accept < B and pred[n_accept] == draft[n_accept]:
            n_accept += 1
        if commit:
            self._append(nk, nv)
            self.carry = logits[-1]
        return dict(ar_pred=a, n_accept=n_accept, logits=logits)

    def crop(self, new_len):
        """Alg. 1 Crop: forget cache positions >= new_len (the carry is no longer defined)."""
        if not 0 <= new_len <= self.n:
            raise ValueError("crop beyond cache length")
        self.n = new_len
        self.carry = None

    # ---- decoding loops -------------------------------------------------------------------
    def decode_block(self, B, tau, fixed_k=0):
        """Seed, denoise until no mask is left, commit.  Returns (tokens, denoise forwards)."""
        tokens = np.full(B, self.mask_id, np.int32)
        mask = np.ones(B, bool)
        fwd = 0
        while mask.any():
            r = self.denoise_step(tokens, mask, tau, fixed_k)
            fwd += r["logits"] is not None
        self.commit_block(tokens)
        return tokens, fwd

    def greedy_ar(self, n_tokens):
        """Ordinary causal decoding, one token per forward (the B=1 special case spelled out)."""
        out = []
        for _ in range(n_tokens):
            t = int(np.argmax(self.carry))
            logits, nk, nv = self.forward(self.embed([t]), CAUSAL)
            self._append(nk, nv)
            self.carry = logits[-1]
            out.append(t)
        return np.array(out, np.int32)

    def linear_speculative(self, n_tokens, B):
        """Alg. 1 loop: draft all masks in one bidirectional pass, verify causally, accept the
        matching prefix plus the AR correction, crop.  Returns (tokens, forwards)."""
        x_n = int(np.argmax(self.carry))            # first token after the prompt, not yet cached
        out = [x_n]
        fwd = 0
        while len(out) < n_tokens:
            d = np.full(B, self.mask_id, np.int32)
            d[0] = x_n
            logits, _, _ = self.forward(self.embed(d), BIDIR)
            fwd += 1
            xh, _ = self.cand_conf(logits)
            d[1:] = xh[:-1]                          # shift by one
            n0 = self.n
            logits_v, nk, nv = self.forward(self.embed(d), CAUSAL)
            fwd += 1
            self._append(nk, nv)
            a, _ = self.cand_conf(logits_v)
            mism = [j for j in range(B - 1) if a[j] != d[j + 1]]
            k = (mism[0] + 1) if mism else B
            out.extend(int(t) for t in a[:k])
            self.crop(n0 + k)                        # keep cache rows of d_0 .. d_{k-1}
            x_n = int(a[k - 1])
        return np.array(out[:n_tokens], np.int32), fwd


    # ---- Alg. 2: quadratic speculative decoding --------------------------------------------------
    @staticmethod
    def quad_mask(B):
        """In-block visibility of the B(B+1) rows of Alg. 2 (group i = [d_i, MASK x B]): the first token of
        group i sees the first tokens of groups <= i; every other token sees all tokens of its own group and
        nothing of other groups.  (The cached prefix is visible to every row.)"""
        W = B + 1
        r = np.arange(B * W)
        gi, gj = r // W, r % W
        first = gj == 0
        vis = first[:, None] & first[None, :] & (gi[None, :] <= gi[:, None])
        vis |= (~first)[:, None] & (gi[None, :] == gi[:, None])
        return vis

    def quad_draft(self, B):
        """Alg. 2 step 1: B mask tokens after the context, bidirectional pass without cache update; draft i is the
        argmax of the hidden state one position earlier (draft 0: of the last context row, i.e. the carry)."""
        d = np.full(B, self.mask_id, np.int32)
        out = np.empty(B, np.int32)
        out[0] = int(np.argmax(self.carry))
        if B > 1:
            logits, _, _ = self.forward(self.embed(d), BIDIR)
            out[1:] = self.cand_conf(logits)[0][:-1]
        return out

    def quad_step(self, d):
        """Alg. 2 loop body on the draft block d[0..B-1] (d[0] is the exact next token): one forward over the B
        groups [d_i, MASK x B] with position ids n+i .. n+i+B and the quadratic mask.  P[i][j] = argmax of group i,
        entry j, predicts position n+i+j+1 (shift by one).  k = 1 + number of leading drafts d_1.. equal to the
        autoregressive predictions P[0][0], P[1][0], ..; d_0..d_{k-1} are accepted, the cache keeps the keys and
        values of those groups' first tokens, and the next draft block is P[k-1][0..B-1] (tokens n+k .. n+k+B-1, the
        first of them exact)."""
        d = np.asarray(d, np.int32)
        B = len(d)
        W = B + 1
        q = np.full(B * W, self.mask_id, np.int32)
        q[::W] = d
        r = np.arange(B * W)
        pos = self.n + r // W + r % W
        logits, nk, nv = self.forward(self.embed(q), None, pos=pos, vis_block=self.quad_mask(B))
        P = self.cand_conf(logits)[0].reshape(B, W)
        k = 1
        while k < B and P[k - 1, 0] == d[k]:
            k += 1
        rows = [i * W for i in range(k)]
        self._append([x[rows] for x in nk], [x[rows] for x in nv])
        self.carry = logits[(k - 1) * W]
        return dict(k=k, accepted=d[:k].copy(), next_draft=P[k - 1, :B].astype(np.int32), logits=logits, P=P)

    def quadratic_speculative(self, n_tokens, B):
        """Alg. 2: draft once, then one forward per iteration.  Returns (tokens, forwards)."""
        d = self.quad_draft(B)
        fwd = int(B > 1)
        out = []
        while len(out) < n_tokens:
            r = self.quad_step(d)
            fwd += 1
            out.extend(int(t) for t in r["accepted"])
            d = r["next_draft"]
        return np.array(out[:n_tokens], np.int32), fwd


def annealed_block_size(u, b_max):
    """Block-size annealing closed form (Sec. 3.3): sizes 2,4,..,b_max; progress u in [0,1]."""
    sizes = []
    b = 2
    while b <= b_max:
        sizes.append(b)
        b *= 2
    return sizes[min(int(np.floor(u * len(sizes))), len(sizes) - 1)]
