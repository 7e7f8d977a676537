"""Pins of the CPU oracle against things other than itself (no GPU).

Forward / mask / cache: an independent dense-mask full-sequence PyTorch model
(tests/dense_torch_model.py).  Unmask, accept and schedule rules: the invariants, closed forms
and degenerate cases the paper fixes (Sec. 3.4; Alg. 1; 'Decoding threshold' paragraph).
"""
import copy
import math

import numpy as np
import pytest
import torch

from oracle.bd_oracle import BIDIR, CAUSAL, BlockDiffusionOracle, annealed_block_size
from paper_2604_06832_amd import inputs
from tests import dense_torch_model as ref

SMALL = inputs.ModelShape(n_layers=3, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn=88, vocab=97)
TOL = 1e-9


def _model(shape=SMALL, seed=0, lm_scale=1.0, std=0.25):
    # std 0.25 on the small shape keeps logits O(1) so argmaxes are well separated
    return inputs.make_weights(shape, seed, "f32", std=std, norm_gain_jitter=0.2, lm_head_scale=lm_scale,
                               threads=1)


def _prefilled(shape=SMALL, L_e=7, L_i=6, **kw):
    w = _model(shape, **kw)
    emb, ids = inputs.make_prompt(shape, L_e, L_i, seed=5)
    o = BlockDiffusionOracle(shape, w)
    o.prefill(emb, ids)
    x_prompt = torch.cat([torch.from_numpy(emb).double(), ref.embed_rows(w, ids)], 0)
    return o, w, x_prompt


# ---- forward, masks, cache (T1, T3, T4, T8) --------------------------------------------------------

@pytest.mark.parametrize("mode", [BIDIR, CAUSAL])
@pytest.mark.parametrize("shape", [SMALL, inputs.TINY])
def test_block_forward_equals_dense_mask_model(mode, shape):
    o, w, xp = _prefilled(shape, std=0.25 if shape is SMALL else 0.02)
    L = xp.shape[0]
    B = 5
    blk = np.array([3, shape.mask_token_id, 11, shape.mask_token_id, 2])
    logits, nk, nv = o.forward(o.embed(blk), mode)
    x = torch.cat([xp, ref.embed_rows(w, blk)], 0)
    want, kvs = ref.full_forward(shape, w, x, ref.dense_mask(L, B, bidir=(mode == BIDIR)), return_kv=True)
    np.testing.assert_allclose(logits, want[L:].numpy(), atol=TOL, rtol=1e-9)
    for l in range(shape.n_layers):
        np.testing.assert_allclose(o.K[l], kvs[l][0][:L].numpy(), atol=TOL)
        np.testing.assert_allclose(o.V[l], kvs[l][1][:L].numpy(), atol=TOL)
        np.testing.assert_allclose(nk[l], kvs[l][0][L:].numpy(), atol=TOL)
        np.testing.assert_allclose(nv[l], kvs[l][1][L:].numpy(), atol=TOL)


def test_prefill_carry_is_last_prompt_row_of_causal_model():
    o, w, xp = _prefilled()
    L = xp.shape[0]
    want = ref.full_forward(SMALL, w, xp, ref.dense_mask(L, 0, False))
    np.testing.assert_allclose(o.carry, want[-1].numpy(), atol=TOL)
    assert o.n == L


def test_chunked_prefill_equals_one_shot():
    w = _model()
    emb, ids = inputs.make_prompt(SMALL, 9, 8, seed=3)
    a = BlockDiffusionOracle(SMALL, w); a.prefill(emb, ids)
    b = BlockDiffusionOracle(SMALL, w); b.prefill(emb, ids, chunk=4)
    np.testing.assert_allclose(a.carry, b.carry, atol=TOL)
    for l in range(SMALL.n_layers):
        np.testing.assert_allclose(a.K[l], b.K[l], atol=TOL)
        np.testing.assert_allclose(a.V[l], b.V[l], atol=TOL)


def test_block_commit_equals_sequential_single_token_steps():
    o, w, _ = _prefilled()
    blk = np.array([5, 9, 1, 44, 17, 80])
    a = copy.deepcopy(o)
    la = a.commit_block(blk)
    b = copy.deepcopy(o)
    rows = [b.commit_block(blk[i:i + 1])[0] for i in range(len(blk))]
    np.testing.assert_allclose(la, np.stack(rows), atol=TOL)
    assert a.n == b.n == o.n + len(blk)
    for l in range(SMALL.n_layers):
        np.testing.assert_allclose(a.K[l], b.K[l], atol=TOL)
        np.testing.assert_allclose(a.V[l], b.V[l], atol=TOL)


def test_layer0_kv_do_not_depend_on_inblock_mask_but_deeper_layers_do():
    o, _, _ = _prefilled()
    blk = np.array([5, SMALL.mask_token_id, 1, SMALL.mask_token_id])
    _, k0, v0 = o.forward(o.embed(blk), BIDIR)
    _, k1, v1 = o.forward(o.embed(blk), CAUSAL)
    np.testing.assert_array_equal(k0[0], k1[0])
    np.testing.assert_array_equal(v0[0], v1[0])
    assert np.abs(k0[1] - k1[1]).max() > 1e-6


def test_denoise_does_not_touch_cache():
    o, _, _ = _prefilled()
    K0 = [k.copy() for k in o.K]; n0 = o.n; c0 = o.carry.copy()
    t = np.full(4, SMALL.mask_token_id, np.int32); m = np.ones(4, bool)
    o.denoise_step(t, m, 0.9)
    assert o.n == n0 and all(np.array_equal(a, b) for a, b in zip(K0, o.K)) and np.array_equal(c0, o.carry)


def test_shift_by_one_and_seed_from_carry():
    # candidate for block position i comes from row i-1 of the bidirectional forward over
    # [seed, M, M, M]; position 0 from the prompt's last causal row.  tau < 1/V reveals all at once.
    o, w, xp = _prefilled()
    L = xp.shape[0]
    B = 4
    t = np.full(B, SMALL.mask_token_id, np.int32); m = np.ones(B, bool)
    causal = ref.full_forward(SMALL, w, xp, ref.dense_mask(L, 0, False))
    seed = int(torch.argmax(causal[-1]))
    o.denoise_step(t, m, tau=0.5 / SMALL.vocab)
    blk = np.array([seed] + [SMALL.mask_token_id] * (B - 1))
    x = torch.cat([xp, ref.embed_rows(w, blk)], 0)
    want = ref.full_forward(SMALL, w, x, ref.dense_mask(L, B, True))[L:]
    assert t[0] == seed
    assert list(t[1:]) == [int(torch.argmax(want[i - 1])) for i in range(1, B)]
    assert not m.any()


# ---- rotary closed forms --------------------------------------------------------------------------

def test_rope_closed_forms():
    o = BlockDiffusionOracle(SMALL, _model())
    rng = np.random.default_rng(0)
    q = rng.standard_normal((1, 1, 16)); k = rng.standard_normal((1, 1, 16))
    # position 0 is the identity; norms are preserved; <R_p q, R_p' k> depends on p - p' only
    np.testing.assert_allclose(o.rope(q, [0]), q, atol=1e-15)
    np.testing.assert_allclose(np.linalg.norm(o.rope(q, [123])), np.linalg.norm(q), rtol=1e-12)
    d1 = (o.rope(q, [40]) * o.rope(k, [33])).sum()
    d2 = (o.rope(q, [1007]) * o.rope(k, [1000])).sum()
    np.testing.assert_allclose(d1, d2, rtol=1e-9)
    # channel pair (0, d/2) turns by exactly p radians (frequency theta^0 = 1); pair (d/2-1, d-1)
    # by p * theta^(-(d-2)/d)
    e = np.zeros((1, 1, 16)); e[0, 0, 0] = 1.0
    r = o.rope(e, [2.0])
    np.testing.assert_allclose([r[0, 0, 0], r[0, 0, 8]], [math.cos(2.0), math.sin(2.0)], atol=1e-15)
    e = np.zeros((1, 1, 16)); e[0, 0, 7] = 1.0
    a = 3.0 * SMALL.rope_theta ** (-14.0 / 16.0)
    r = o.rope(e, [3.0])
    np.testing.assert_allclose([r[0, 0, 7], r[0, 0, 15]], [math.cos(a), math.sin(a)], atol=1e-15)
    # against the complex form used by the pin model
    x = rng.standard_normal((5, 3, 16))
    want = ref.rope_complex(torch.from_numpy(x), torch.arange(5) + 11, SMALL.rope_theta).numpy()
    np.testing.assert_allclose(o.rope(x, np.arange(5) + 11), want, atol=1e-12)


# ---- B = 1 is ordinary autoregressive decoding (T2) ---------------------------------------------------

def test_block_size_one_reproduces_greedy_ar_without_cache():
    o, w, xp = _prefilled()
    got = []
    for _ in range(6):
        tok, fwd = o.decode_block(1, tau=0.9)
        assert fwd == 0                      # seed only: no denoising forward at B = 1
        got.append(int(tok[0]))
    x = xp
    want = []
    for _ in range(6):                       # full recompute, no cache, plain causal mask
        T = x.shape[0]
        lg = ref.full_forward(SMALL, w, x, ref.dense_mask(T, 0, False))
        t = int(torch.argmax(lg[-1])); want.append(t)
        x = torch.cat([x, ref.embed_rows(w, [t])], 0)
    assert got == want
    o2, _, _ = _prefilled()
    assert list(o2.greedy_ar(6)) == want


# ---- unmask rule (T5, T6, T7, T12) ------------------------------------------------------------------

def _spread_oracle():
    # LM head scaled so confidences spread over (0,1) and the threshold branch really fires
    return _prefilled(lm_scale=6.0)[0]


def test_confidence_is_softmax_max_and_uniform_logits_give_one_over_vocab():
    lg = np.random.default_rng(1).standard_normal((7, 97)) * 3
    cand, conf = BlockDiffusionOracle.cand_conf(lg)
    p = torch.softmax(torch.from_numpy(lg), -1)
    np.testing.assert_allclose(conf, p.max(-1).values.numpy(), rtol=1e-12)
    assert list(cand) == list(p.argmax(-1).numpy())
    cand, conf = BlockDiffusionOracle.cand_conf(np.zeros((2, 97)))
    assert list(cand) == [0, 0] and np.allclose(conf, 1 / 97)
    lg = np.zeros((1, 9)); lg[0, [2, 6]] = 1.5           # tie -> lowest id
    assert BlockDiffusionOracle.cand_conf(lg)[0][0] == 2


def test_every_step_unmasks_at_least_one_and_revealed_positions_stay():
    o = _spread_oracle()
    B = 8
    t = np.full(B, SMALL.mask_token_id, np.int32); m = np.ones(B, bool)
    steps = 0
    while m.any():
        t0, m0 = t.copy(), m.copy()
        r = o.denoise_step(t, m, tau=0.6)
        steps += 1
        assert r["n_unmasked"] >= 1 and r["n_unmasked"] == int(m0.sum() - m.sum())
        assert np.array_equal(t[~m0], t0[~m0])           # no remasking, no rewriting
        assert not np.any(m & ~m0)
        assert np.all(t[~m] != SMALL.mask_token_id)
    assert steps <= B - 1


def test_revealed_set_shrinks_as_threshold_rises():
    o = _spread_oracle()
    B = 8
    prev = None
    sizes = []
    for tau in [0.0, 0.05, 0.2, 0.4, 0.6, 0.8, 0.9, 0.99, 1.0]:
        oo = copy.deepcopy(o)
        t = np.full(B, SMALL.mask_token_id, np.int32); m = np.ones(B, bool)
        oo.denoise_step(t, m, tau)
        S = set(np.flatnonzero(~m))
        if prev is not None:
            assert S <= prev
        prev = S
        sizes.append(len(S))
    assert sizes[0] == B and sizes[-1] == 2               # all at tau<1/V; seed + one at tau=1
    assert len(set(sizes)) > 2                            # the threshold branch really discriminates


def test_tau_one_reveals_exactly_one_per_step_and_low_tau_reveals_all():
    o = _spread_oracle()
    B = 6
    oo = copy.deepcopy(o)
    _, fwd = oo.decode_block(B, tau=1.0)
    assert fwd == B - 1
    oo = copy.deepcopy(o)
    _, fwd = oo.decode_block(B, tau=0.5 / SMALL.vocab)
    assert fwd == 1


def test_threshold_is_strict_and_fallback_takes_highest_confidence():
    o = _spread_oracle()
    B = 5
    t = np.full(B, SMALL.mask_token_id, np.int32); m = np.ones(B, bool)
    probe = copy.deepcopy(o)
    r = probe.denoise_step(t.copy(), m.copy(), tau=2.0)    # nothing can clear tau=2 -> fallback
    conf = r["conf"]
    best = 1 + int(np.argmax(conf[1:]))
    t2, m2 = t.copy(), m.copy()
    copy.deepcopy(o).denoise_step(t2, m2, tau=2.0)
    assert list(np.flatnonzero(~m2)) == [0, best]
    # tau exactly equal to a confidence does not reveal that position (strict '>')
    order = np.argsort(-conf[1:]) + 1
    t3, m3 = t.copy(), m.copy()
    copy.deepcopy(o).denoise_step(t3, m3, tau=float(conf[order[1]]))
    assert list(np.flatnonzero(~m3)) == sorted([0, int(order[0])])


@pytest.mark.parametrize("B,K", [(4, 1), (32, 4), (8, 3), (16, 16), (5, 2)])
def test_fixed_schedule_forward_count(B, K):
    shape = inputs.ModelShape(n_layers=1, hidden=32, n_q_heads=2, n_kv_heads=1, head_dim=16, ffn=40, vocab=53)
    w = inputs.make_weights(shape, 0, "f32", std=0.3, threads=1)
    emb, ids = inputs.make_prompt(shape, 3, 3, 0)
    o = BlockDiffusionOracle(shape, w); o.prefill(emb, ids)
    t = np.full(B, shape.mask_token_id, np.int32); m = np.ones(B, bool)
    fwd = 0
    first = True
    while m.any():
        before = int(m.sum())
        r = o.denoise_step(t, m, tau=0.9, fixed_k=K)
        fwd += 1
        want = min(K, before - (1 if first else 0)) + (1 if first else 0)
        assert r["n_unmasked"] == want
        first = False
    assert fwd == math.ceil((B - 1) / K)
    # the K revealed positions are the K most confident masked ones
    o2 = BlockDiffusionOracle(shape, w); o2.prefill(emb, ids)
    t = np.full(B, shape.mask_token_id, np.int32); m = np.ones(B, bool)
    r = o2.denoise_step(t, m, 0.9, fixed_k=K)
    got = set(np.flatnonzero(~m)) - {0}
    want = set((np.argsort(-r["conf"][1:], kind="stable")[:min(K, B - 1)] + 1).tolist())
    assert got == want


# ---- verify / accept / speculative loop (T9, T10) ------------------------------------------------------

def test_verify_accept_cases():
    o, _, _ = _prefilled()
    B = 6
    draft = copy.deepcopy(o).greedy_ar(B)
    r = copy.deepcopy(o).verify_block(draft)
    assert r["n_accept"] == B
    for j in range(B):
        bad = draft.copy()
        bad[j] = (bad[j] + 1) % (SMALL.vocab - 1)
        oo = copy.deepcopy(o)
        r = oo.verify_block(bad)
        assert r["n_accept"] == j
        assert oo.n == o.n + B
        # the AR prediction at the first rejected position is the greedy token
        if j > 0:
            assert r["ar_pred"][j - 1] == draft[j]
    oo = copy.deepcopy(o)
    oo.verify_block(draft, commit=False)
    assert oo.n == o.n


def test_corrupted_draft_accept_length_is_first_replaced_position():
    o, _, _ = _prefilled()
    B = 16
    clean = copy.deepcopy(o).greedy_ar(B)
    draft, hit = inputs.corrupt_draft(SMALL, clean, seed=1, p=0.2)
    changed = np.flatnonzero(draft != clean)
    want = int(changed[0]) if len(changed) else B
    assert copy.deepcopy(o).verify_block(draft)["n_accept"] == want


@pytest.mark.parametrize("B", [2, 4, 7])
def test_linear_speculative_emits_greedy_ar_sequence(B):
    o, _, _ = _prefilled()
    want = copy.deepcopy(o).greedy_ar(20)
    got, fwd = copy.deepcopy(o).linear_speculative(20, B)
    assert list(got) == list(want)
    assert fwd % 2 == 0 and fwd <= 2 * 19           # two forwards per block, >= 1 new token each


# ---- Alg. 2: quadratic speculative decoding -------------------------------------------------------------

@pytest.mark.parametrize("B", [1, 2, 3, 5, 7])
def test_quadratic_mask_structure(B):
    """Counting form of the mask rules: the first token of group i sees exactly the i+1 first tokens up to its own
    (and no mask token, not even of its own group); any other token sees exactly the B+1 tokens of its group."""
    vis = BlockDiffusionOracle.quad_mask(B)
    W = B + 1
    assert vis.shape == (B * W, B * W)
    for i in range(B):
        row = vis[i * W]
        assert row.sum() == i + 1 and all(row[g * W] for g in range(i + 1))
        for j in range(1, W):
            row = vis[i * W + j]
            assert row.sum() == W and row[i * W:(i + 1) * W].all()
    # brute force against the four rules spelled out per pair
    for a in range(B * W):
        for b in range(B * W):
            ai, aj, bi, bj = a // W, a % W, b // W, b % W
            want = (bj == 0 and bi <= ai) if aj == 0 else (bi == ai)
            assert vis[a, b] == want


@pytest.mark.parametrize("B", [1, 2, 3, 5])
def test_quadratic_speculative_emits_greedy_ar_sequence(B):
    """Whatever the proposals are worth, the accepted tokens are the greedy autoregressive continuation: every
    accepted draft was compared with the prediction of a causal row that saw exactly the accepted tokens before it."""
    o, _, _ = _prefilled()
    want = copy.deepcopy(o).greedy_ar(14)
    got, fwd = copy.deepcopy(o).quadratic_speculative(14, B)
    assert list(got) == list(want)
    assert fwd <= 14 + 1                                # one forward per iteration (+ the draft), >= 1 token each


def test_quadratic_step_first_tokens_are_a_causal_pass():
    """The first tokens of the groups, taken alone, form an ordinary causal forward over d: same logits, same keys and
    values (their mask rows see the prefix and the earlier first tokens only, their positions are n, n+1, ..)."""
    o, _, _ = _prefilled()
    B = 4
    d = copy.deepcopy(o).greedy_ar(B)
    d[2] = (d[2] + 1) % (SMALL.vocab - 1)               # a wrong draft: accepted length 2
    a = copy.deepcopy(o)
    r = a.quad_step(d)
    b = copy.deepcopy(o)
    v = b.verify_block(d, commit=False)
    np.testing.assert_allclose(r["logits"][::B + 1], v["logits"], atol=TOL)
    assert r["k"] == 2 and list(r["accepted"]) == list(d[:2])
    assert r["next_draft"][0] == v["ar_pred"][1]        # the exact token after the accepted ones
    b.commit_block(d[:2])
    assert a.n == b.n
    for l in range(SMALL.n_layers):
        np.testing.assert_allclose(a.K[l], b.K[l], atol=TOL)
        np.testing.assert_allclose(a.V[l], b.V[l], atol=TOL)
    np.testing.assert_allclose(a.carry, b.carry, atol=TOL)


def test_quadratic_groups_do_not_leak_into_each_other():
    """No token other than a group's first sees another group: group 0 is untouched by the other drafts, and the
    proposals of group i change with d_i's own context only through the first tokens before it."""
    o, _, _ = _prefilled()
    B = 3
    d = np.array([5, 11, 23], np.int32)
    r = copy.deepcopy(o).quad_step(d)
    d2 = np.array([5, 40, 77], np.int32)
    r2 = copy.deepcopy(o).quad_step(d2)
    W = B + 1
    np.testing.assert_allclose(r["logits"][:W], r2["logits"][:W], atol=TOL)          # group 0: identical
    assert np.abs(r["logits"][W:2 * W] - r2["logits"][W:2 * W]).max() > 1e-3          # group 1 follows its own d_1
    d3 = np.array([5, 11, 77], np.int32)
    r3 = copy.deepcopy(o).quad_step(d3)
    np.testing.assert_allclose(r["logits"][:2 * W], r3["logits"][:2 * W], atol=TOL)  # groups 0, 1 ignore d_2
    # positions: group i sits at n+i .. n+i+B, so group 0 alone is the block [d_0, MASK x B] at position n whose first
    # token sees only itself and whose mask tokens see the whole block
    blk = np.full(W, o.mask_id, np.int32)
    blk[0] = d[0]
    vis = np.ones((W, W), bool)
    vis[0, 1:] = False
    oo = copy.deepcopy(o)
    lg, _, _ = oo.forward(oo.embed(blk), None, vis_block=vis)
    np.testing.assert_allclose(r["logits"][:W], lg, atol=TOL)


def _quad_group_rollout(w, xp, d, i, B):
    """Logits of group i of an Alg. 2 step from the dense full-sequence model alone: the sequence
    [prompt, d_0 .. d_{i-1}, d_i, MASK x B] at positions 0, 1, .. (so group i sits at L+i .. L+i+B, the rollout
    from the acceptance point i of the appendix's 'Quadratic' paragraph) under the literally built mask: prompt
    and first tokens token-causal (rule b), the B mask rows see the prompt (rule a) and the B+1 tokens of their
    own group (rule c) and none of d_0 .. d_{i-1} (rule d)."""
    L = xp.shape[0]
    W = B + 1
    ids = np.concatenate([np.asarray(d[:i + 1], np.int64), np.full(B, SMALL.mask_token_id, np.int64)])
    x = torch.cat([xp, ref.embed_rows(w, ids)], 0)
    T = L + i + W
    A = torch.zeros(T, T, dtype=torch.bool)
    for r in range(T):
        for c in range(T):
            if r <= L + i:
                A[r, c] = c <= r
            else:
                A[r, c] = c < L or c >= L + i
    return ref.full_forward(SMALL, w, x, A)[L + i:].numpy()


@pytest.mark.parametrize("B", [2, 3, 5])
def test_quadratic_step_groups_are_rollouts_from_each_acceptance_point(B):
    """Every row of the B(B+1)-row forward, mask rows of the later groups included, against the dense model: this
    fixes the position ids n+i+j of group i, the four mask rules, and with them every proposal P[i][j]."""
    o, w, xp = _prefilled()
    W = B + 1
    d = copy.deepcopy(o).greedy_ar(B)
    if B > 2:
        d[B - 1] = (d[B - 1] + 3) % (SMALL.vocab - 1)      # the last draft is wrong: k = B - 1
    r = copy.deepcopy(o).quad_step(d)
    want_P = np.empty((B, W), np.int64)
    for i in range(B):
        want = _quad_group_rollout(w, xp, d, i, B)
        np.testing.assert_allclose(r["logits"][i * W:(i + 1) * W], want, atol=TOL, rtol=1e-9)
        want_P[i] = want.argmax(-1)
    assert np.array_equal(r["P"], want_P)
    k = 1
    while k < B and want_P[k - 1, 0] == d[k]:
        k += 1
    assert r["k"] == k == (B - 1 if B > 2 else B)
    assert list(r["next_draft"]) == list(want_P[k - 1, :B])


@pytest.mark.parametrize("B", [1, 2, 4, 6])
def test_quadratic_first_draft_is_the_dense_model_over_prompt_and_masks(B):
    """Alg. 2 step 1: z = [prompt, MASK x B], prompt rows causal, mask rows see everything; draft i is the argmax of
    row L-1+i (draft 0 comes from the last prompt row), and the cache keeps the prompt only."""
    o, w, xp = _prefilled()
    L = xp.shape[0]
    x = torch.cat([xp, ref.embed_rows(w, np.full(B, SMALL.mask_token_id, np.int64))], 0)
    lg = ref.full_forward(SMALL, w, x, ref.dense_mask(L, B, bidir=True)).numpy()
    oo = copy.deepcopy(o)
    got = oo.quad_draft(B)
    assert list(got) == list(lg[L - 1:L - 1 + B].argmax(-1))
    assert oo.n == L


def test_quadratic_pins_catch_same_positions_for_every_group(monkeypatch):
    """Planted mistake: positions n+j in every group (instead of n+i+j).  The first-token and greedy-equivalence pins
    cannot see it in group 0; the rollout pin must."""
    o, w, xp = _prefilled()
    B, W = 3, 4
    d = copy.deepcopy(o).greedy_ar(B)
    bad = copy.deepcopy(o)
    orig = bad.forward

    def forward_same_pos(x, mode, want_logits_rows=None, pos=None, vis_block=None):
        if pos is not None:
            r = np.arange(len(pos))
            pos = bad.n + r % W
        return orig(x, mode, want_logits_rows, pos, vis_block)

    monkeypatch.setattr(bad, "forward", forward_same_pos)
    r = bad.quad_step(d)
    np.testing.assert_allclose(r["logits"][:W], _quad_group_rollout(w, xp, d, 0, B), atol=TOL)   # group 0 unaffected
    assert np.abs(r["logits"][W:2 * W] - _quad_group_rollout(w, xp, d, 1, B)).max() > 1e-4
    # and a mask row that wrongly sees an earlier group's first token is caught too
    leaky = copy.deepcopy(o)
    vis = BlockDiffusionOracle.quad_mask(B).copy()
    vis[W + 1, 0] = True
    monkeypatch.setattr(BlockDiffusionOracle, "quad_mask", staticmethod(lambda b: vis))
    r2 = leaky.quad_step(d)
    assert np.abs(r2["logits"][W:2 * W] - _quad_group_rollout(w, xp, d, 1, B)).max() > 1e-6


def test_crop_restores_earlier_state():
    o, _, _ = _prefilled()
    a = copy.deepcopy(o); a.commit_block(np.array([1, 2, 3, 4])); a.crop(o.n + 2); a.commit_block(np.array([9]))
    b = copy.deepcopy(o); b.commit_block(np.array([1, 2])); b.commit_block(np.array([9]))
    np.testing.assert_allclose(a.carry, b.carry, atol=TOL)
    with pytest.raises(ValueError):
        a.crop(a.n + 1)


def test_commit_rejects_mask_token():
    o, _, _ = _prefilled()
    with pytest.raises(ValueError):
        o.commit_block(np.array([1, SMALL.mask_token_id]))


# ---- small closed forms -----------------------------------------------------------------------------

def test_block_size_annealing_closed_form():
    assert [annealed_block_size(u, 32) for u in (0, 0.2, 0.4, 0.6, 0.8, 1.0)] == [2, 4, 8, 16, 32, 32]
    assert annealed_block_size(0.19, 32) == 2 and annealed_block_size(0.99, 32) == 32


def test_block_size_annealing_golden_table():
    # hand-evaluated values of the paper's closed form (tests/golden/annealing_schedule.txt)
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "annealing_schedule.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 16
    for b_max, u, want in rows:
        assert annealed_block_size(float(u), int(b_max)) == int(want), (b_max, u, want)


# ---- planted mistakes must be caught ------------------------------------------------------------------

@pytest.mark.parametrize("mutation", ["rope_sign", "no_gain", "wrong_group", "causal_offbyone", "no_scale"])
def test_pins_catch_planted_mistakes(mutation, monkeypatch):
    o, w, xp = _prefilled()
    L = xp.shape[0]
    if mutation == "rope_sign":
        orig = o.rope
        monkeypatch.setattr(o, "rope", lambda x, pos: orig(x, -np.asarray(pos)))
    elif mutation == "no_gain":
        monkeypatch.setattr(o, "rmsnorm", lambda x, g: x / np.sqrt(np.mean(x * x, -1, keepdims=True) + 1e-6))
    elif mutation == "wrong_group":
        orig = o.attention
        monkeypatch.setattr(o, "attention", lambda q, k, v, n, mode, vb=None: orig(q, k[:, ::-1], v[:, ::-1], n, mode, vb))
    elif mutation == "causal_offbyone":
        orig = o.attention
        monkeypatch.setattr(o, "attention", lambda q, k, v, n, mode, vb=None: orig(q, k, v, n + (mode == CAUSAL), mode, vb))
    elif mutation == "no_scale":
        orig = o.attention
        monkeypatch.setattr(o, "attention", lambda q, k, v, n, mode, vb=None: orig(q * 4.0, k, v, n, mode, vb))
    blk = np.array([3, 8, 11, 4])
    logits, _, _ = o.forward(o.embed(blk), CAUSAL)
    x = torch.cat([xp, ref.embed_rows(w, blk)], 0)
    want = ref.full_forward(SMALL, w, x, ref.dense_mask(L, 4, False))[L:].numpy()
    assert np.abs(logits - want).max() > 1e-4
