"""End-to-end parity of the HIP decode path against the CPU oracle, through the C ABI.

Bars (tests/gpu_util.bars): logits within 3e-2 of the oracle's logit range (bf16 path; 1e-1 with e4m3 weights) and
within the bound E that the bf16 hand-overs of the path can cause; unmask masks and token ids bit-exact wherever the
oracle's top-2 logit margin exceeds max(1e-2, 2 E) and the revealed set is not decided by two confidences closer than
the fixed confidence bound; cached K/V within bf16 rounding of the oracle's.  Every test prints what its comparisons
covered (tests/conftest.py).
"""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle.bd_oracle import BlockDiffusionOracle
from paper_2604_06832_amd import binding, inputs
from tests.gpu_util import FP8_LOGIT_TOL, MARGIN, Pair, assert_logits_close, bars, check_argmax_ids, fresh_block, note, top2_margin

pytestmark = pytest.mark.gpu


def _say(msg):
    """Progress line: printed, and appended to a file next to the other run outputs (a test that computes on the host
    for minutes still shows that it is alive when pytest captures its output)."""
    print(msg, flush=True)
    try:
        import os
        d = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "test_progress.log"), "a") as f:
            f.write(msg + "\n")
    except OSError:
        pass


# ---- configs[0]: the tiny plumbing model ---------------------------------------------------------------

@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_tiny_config_block_decode(storage):
    _say(f"tiny config, weights {storage}")
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, storage, threads=1)
    emb, ids = inputs.make_prompt(shape, 64, 64, seed=100)
    p = Pair(shape, w, max_seq=256)
    p.prefill(emb, ids)
    p.check_carry()
    p.check_kv(0, 128)
    tok, msk = fresh_block(shape, 4)
    fwd = 0
    while msk.any():
        tok, msk, r = p.denoise_step(tok, msk, tau=0.9)
        fwd += r["logits"] is not None
    assert fwd == 3                                   # never clears 0.9 with random weights: one per step
    p.commit(tok)
    p.check_kv(128, 4)
    p.close()


def test_block_size_one_is_autoregressive_decoding():
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", threads=1)
    emb, ids = inputs.make_prompt(shape, 8, 8, seed=3)
    p = Pair(shape, w, max_seq=64)
    p.prefill(emb, ids)
    want = BlockDiffusionOracle(shape, w)
    want.prefill(emb, ids)
    ar = want.greedy_ar(6)
    held = 0
    for t in range(6):
        tok, msk = fresh_block(shape, 1)
        tok, msk, _ = p.denoise_step(tok, msk, 0.9)
        assert not msk.any()
        if p.carry_is_robust():
            assert tok[0] == ar[t]
            held += 1
        p.commit(tok)
    note("count", what="autoregressive tokens held against the oracle's", n=held)
    assert held >= 1
    p.close()


# ---- the threshold branch, with confidences spread over (0,1) ---------------------------------------

@pytest.mark.parametrize("tau", [0.0, 0.3, 0.6, 0.9, 1.0])
def test_threshold_unmask_with_peaked_confidences(tau):
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", lm_head_scale=20.0, norm_gain_jitter=0.1, threads=1)
    emb, ids = inputs.make_prompt(shape, 16, 16, seed=4)
    p = Pair(shape, w, max_seq=128)
    p.prefill(emb, ids)
    tok, msk = fresh_block(shape, 16)
    steps = 0
    sizes = []
    while msk.any():
        before = int(msk.sum())
        tok, msk, r = p.denoise_step(tok, msk, tau)
        sizes.append(before - int(msk.sum()))
        steps += 1
        assert steps <= 16
    if tau >= 1.0:
        assert sizes[0] == 2 and all(s == 1 for s in sizes[1:])
    if tau == 0.0:
        assert steps == 1
    p.commit(tok)
    p.close()


@pytest.mark.parametrize("B,K", [(8, 3), (32, 4), (64, 4), (33, 5)])
def test_fixed_schedule(B, K):
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", lm_head_scale=20.0, threads=1)
    emb, ids = inputs.make_prompt(shape, 20, 17, seed=5)
    p = Pair(shape, w, max_seq=37 + 2 * B, max_block=B)
    p.prefill(emb, ids)
    for blk in range(2):
        tok, msk = fresh_block(shape, B)
        fwd = 0
        while msk.any():
            tok, msk, _ = p.denoise_step(tok, msk, 0.9, fixed_k=K)
            fwd += 1
        assert fwd == -(-(B - 1) // K)
        p.commit(tok)
    p.check_kv(0, 37 + 2 * B)
    p.close()


# ---- verify / accept / crop (configs[3] on the tiny model) --------------------------------------------

@pytest.mark.parametrize("B", [4, 8, 16, 32, 64])
def test_verify_accept_and_crop(B):
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", lm_head_scale=20.0, threads=1)
    emb, ids = inputs.make_prompt(shape, 24, 24, seed=6)
    p = Pair(shape, w, max_seq=48 + 2 * B, max_block=B)
    p.prefill(emb, ids)
    import copy
    clean = copy.deepcopy(p.o).greedy_ar(B)
    draft, _ = inputs.corrupt_draft(shape, clean, seed=1, p=0.2)
    r = copy.deepcopy(p.o).verify_block(draft, commit=False)
    d = torch.from_numpy(draft).cuda()
    pred = torch.zeros(B, dtype=torch.int32, device="cuda")
    nacc = torch.zeros(1, dtype=torch.int32, device="cuda")
    p.ctx.bd_verify_block(d, False, pred, nacc)
    torch.cuda.synchronize()
    assert p.ctx.bd_cache_len() == 48
    glog = p.ctx.bd_read_logits(B).cpu().numpy()
    assert_logits_close(glog, r["logits"], n_layers=shape.n_layers)
    ok = check_argmax_ids(pred.cpu().numpy(), glog, r["logits"], shape.n_layers)
    # the accept length is decided by the carry and rows 0 .. n_accept-1: held exact when all of those are robust
    decided = bool(ok[:max(r["n_accept"], 1)].all() and p.carry_is_robust())
    note("count", what="accept length held against the oracle's", n=int(decided))
    if decided:
        assert int(nacc.item()) == r["n_accept"]
    else:
        # integer work on the GPU's own predictions: the accept rule itself is still checked bit-exactly
        gp = np.concatenate([[p.ctx.bd_read_carry()[0]], pred.cpu().numpy()[:-1]])
        k = 0
        while k < B and gp[k] == draft[k]:
            k += 1
        assert int(nacc.item()) == k
    # commit, then crop to the accepted prefix and continue: same state as committing only that prefix
    k = max(1, r["n_accept"])
    p.ctx.bd_verify_block(d, True, None, None)
    p.ctx.bd_crop(48 + k)
    assert p.ctx.bd_cache_len() == 48 + k
    p.o.commit_block(draft[:k])
    nxt = np.array([1, 2, 3], np.int32)
    p.commit(nxt)
    p.check_kv(0, 48 + k + 3)
    p.close()




# ---- a whole block per call, early-out on the device ---------------------------------------------------------

@pytest.mark.parametrize("shape_name,B,tau,fixed_k", [("tiny", 16, 0.3, 0), ("tiny", 16, 0.0, 0), ("tiny", 16, 1.0, 0),
                                                      ("tiny", 1, 0.5, 0), ("tiny", 64, 0.6, 0), ("tiny", 33, 0.9, 5),
                                                      ("wide", 32, 0.02, 0), ("wide", 16, 0.9, 4)])
def test_decode_block_equals_the_step_by_step_loop(shape_name, B, tau, fixed_k):
    """bd_decode_block enqueues the largest number of steps a block can need and lets the device skip the ones after
    the block is complete.  Against a second context driven step by step (host reads the mask after every step):
    same tokens, same number of forwards, same cache and carry, bit for bit, over three blocks -- and the step-by-step
    loop itself is held against the oracle."""
    _say(f"bd_decode_block vs step-by-step, {shape_name}, B={B}, tau={tau}, fixed_k={fixed_k}")
    if shape_name == "tiny":
        shape = inputs.TINY
        w = inputs.make_weights(shape, 0, "bf16", lm_head_scale=20.0, norm_gain_jitter=0.1, threads=1)
    else:
        shape = _wide(2, vocab=8192)
        w = inputs.make_weights(shape, 0, "bf16", lm_head_scale=20.0, threads=8)
    emb, ids = inputs.make_prompt(shape, 16, 16, seed=4)
    p = Pair(shape, w, max_seq=32 + 3 * B, max_block=B)
    p.prefill(emb, ids)
    ctx2 = binding.Context(shape, max_seq=32 + 3 * B, max_block=B)
    ctx2.load_model(w, as_bf16_bits=True)
    ctx2.bd_prefill(torch.from_numpy(emb).cuda(), torch.from_numpy(ids).cuda())
    out = torch.zeros(B, dtype=torch.int32, device="cuda")
    nst = torch.zeros(1, dtype=torch.int32, device="cuda")
    for blk in range(3):
        ctx2.bd_decode_block(B, tau, fixed_k, out, nst)
        tok, msk = fresh_block(shape, B)
        gt = torch.from_numpy(tok.astype(np.int32)).cuda()
        gm = torch.from_numpy(msk.astype(np.uint8)).cuda()
        fwd = 0
        while True:
            p.ctx.bd_denoise_step(gt, gm, tau, fixed_k, None, None)
            fwd += int(B > 1)
            if not bool(gm.any().item()):
                break
            assert fwd < B
        p.ctx.bd_commit_block(gt)
        assert torch.equal(out, gt), (blk, out, gt)
        assert int(nst.item()) == fwd, (blk, int(nst.item()), fwd)
        assert ctx2.bd_cache_len() == p.ctx.bd_cache_len()
        assert ctx2.bd_read_carry() == p.ctx.bd_read_carry()
    n = p.ctx.bd_cache_len()
    for l in range(shape.n_layers):
        ka, va = ctx2.bd_read_kv(l, 0, n)
        kb, vb = p.ctx.bd_read_kv(l, 0, n)
        assert torch.equal(ka, kb) and torch.equal(va, vb)
    ctx2.bd_status()
    p.ctx.bd_status()
    if fixed_k == 0 and tau <= 0.0 and B > 1:
        assert int(nst.item()) == 1                     # everything clears a threshold of zero in one step
    if fixed_k == 0 and tau >= 1.0:
        assert int(nst.item()) == B - 1                 # one position per step
    ctx2.close()
    p.close()

# ---- linear self-speculative loop (Alg. 1) as one call per iteration ------------------------------------------

def _oracle_spec_iteration(o, x_n, B):
    """One iteration of Alg. 1 on the oracle, step by step (same steps as its linear_speculative loop), returning
    what the device call reports plus the logits the decisions were taken on."""
    from oracle.bd_oracle import BIDIR, CAUSAL
    d = np.full(B, o.mask_id, np.int32)
    d[0] = x_n
    lg_d = None
    if B > 1:
        lg_d, _, _ = o.forward(o.embed(d), BIDIR)
        d[1:] = o.cand_conf(lg_d)[0][:-1]
    n0 = o.n
    lg_v, nk, nv = o.forward(o.embed(d), CAUSAL)
    o._append(nk, nv)
    a, _ = o.cand_conf(lg_v)
    mism = [j for j in range(B - 1) if a[j] != d[j + 1]]
    k = (mism[0] + 1) if mism else B
    o.crop(n0 + k)
    return dict(draft=d, a=a, k=k, draft_logits=lg_d, verify_logits=lg_v)


def _cyclic_model(shape, flip):
    """A model whose predictions depend on the current token only (attention and MLP outputs switched off by zero
    output projections, one-hot embeddings): every ordinary token and the mask token predict token A; A predicts A
    (flip=False: every draft is accepted) or A predicts Bt and Bt predicts A (flip=True: the drafts A, A, ... after
    the first are rejected where the sequence alternates)."""
    w = inputs.make_weights(shape, 3, "bf16", threads=1)
    A, Bt = 5, 9
    emb = np.zeros((shape.vocab, shape.hidden), np.float32)
    emb[:, 0] = 1.0
    head = np.zeros((shape.vocab, shape.hidden), np.float32)
    head[A, 0] = 1.0
    if flip:
        emb[A] = 0.0; emb[A, 1] = 1.0          # A -> class 1 -> Bt
        emb[Bt] = 0.0; emb[Bt, 2] = 1.0        # Bt -> class 2 -> A
        head[Bt, 1] = 1.0
        head[A, 2] = 1.0
    w["embed"] = emb
    w["lm_head"] = head
    for l in range(shape.n_layers):
        w[f"l{l}.wo"] = np.zeros_like(w[f"l{l}.wo"])
        w[f"l{l}.w_down"] = np.zeros_like(w[f"l{l}.w_down"])
    return w, A, Bt


@pytest.mark.parametrize("B,flip", [(1, True), (4, False), (8, True), (32, True), (33, False), (64, True)])
def test_speculative_step_accept_lengths_on_a_token_cycle(B, flip):
    _say(f"speculative step on the cyclic model, B={B}, flip={flip}")
    shape = inputs.TINY
    w, A, Bt = _cyclic_model(shape, flip)
    ids = np.array([3, 17, 200, 41, 7], np.int32)
    p = Pair(shape, w, max_seq=5 + 6 * B + B, max_block=B)
    p.prefill(None, ids)
    x_n = int(np.argmax(p.o.carry))
    assert x_n == A
    out = torch.zeros(B, dtype=torch.int32, device="cuda")
    ks = []
    for it in range(5):
        r = _oracle_spec_iteration(p.o, x_n, B)
        k = p.ctx.bd_speculative_step(B, out)
        got = out.cpu().numpy()
        assert k == r["k"], (it, k, r["k"])
        assert np.array_equal(got[:k], r["a"][:k]), (it, got[:k], r["a"][:k])
        assert p.ctx.bd_cache_len() == p.o.n
        x_n = int(r["a"][k - 1])
        cand, _ = p.ctx.bd_read_carry()
        assert cand == x_n
        ks.append(k)
    # closed form of the accept lengths: fixed point -> whole blocks; alternation -> 3 (from A: A Bt A | A) then 2
    if not flip:
        assert ks == [B] * 5
    elif B >= 4:
        assert ks == [3, 2, 2, 2, 2]
    p.check_kv(0, p.o.n)
    p.close()


@pytest.mark.parametrize("B", [4, 16])
def test_speculative_steps_emit_the_greedy_sequence(B):
    """Alg. 1 emits exactly the greedy autoregressive continuation, whatever the drafts are worth: with random
    weights nearly every draft is rejected, so every iteration exercises reject + crop.  Iterations are compared as
    long as every decision of the oracle clears the fixed id margin; when one does not, both sides start again from
    another prompt, until at least three iterations have been held against the oracle."""
    _say(f"speculative steps vs greedy decoding, tiny config, B={B}")
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", lm_head_scale=20.0, threads=1)
    p = Pair(shape, w, max_seq=48 + 12 * B, max_block=B)
    import copy
    out = torch.zeros(B, dtype=torch.int32, device="cuda")
    compared, prompts = 0, 0
    for seed in range(6, 400):
        if compared >= 3:
            break
        emb, ids = inputs.make_prompt(shape, 24, 24, seed=seed)
        p.prefill(emb, ids)
        prompts += 1
        if not p.carry_is_robust():
            continue
        greedy = copy.deepcopy(p.o).greedy_ar(12)
        x_n = int(np.argmax(p.o.carry))
        emitted = [x_n]
        while len(emitted) < 12:
            r = _oracle_spec_iteration(p.o, x_n, B)
            k = p.ctx.bd_speculative_step(B, out)
            got = out.cpu().numpy()
            glog = p.ctx.bd_read_logits(B).cpu().numpy()              # logits of the verify pass
            # row 0 of the verify pass has the same input on both sides whatever the drafts are
            assert_logits_close(glog[:1], r["verify_logits"][:1], n_layers=shape.n_layers)
            # decisions count only where the oracle's margins exceed the fixed id margin: the k verify rows that emit,
            # and the drafts up to the first rejected one (later drafts change nothing)
            thr = bars(r["verify_logits"], shape.n_layers)[1]
            n_dr = min(r["k"], B - 1)
            robust = top2_margin(r["verify_logits"])[:r["k"]].min() > thr and \
                (r["draft_logits"] is None or
                 top2_margin(r["draft_logits"])[:n_dr].min() > bars(r["draft_logits"], shape.n_layers)[1])
            if not robust:
                break                                                  # a near-tie decides from here on: next prompt
            assert_logits_close(glog, r["verify_logits"], n_layers=shape.n_layers)
            assert k == r["k"] and np.array_equal(got[:k], r["a"][:k])
            compared += 1
            emitted += [int(t) for t in got[:k]]
            x_n = int(r["a"][k - 1])
            assert p.ctx.bd_cache_len() == p.o.n
        n = min(len(emitted), 12)
        assert np.array_equal(np.array(emitted[:n]), greedy[:n])
    note("count", what=f"speculative iterations held against the oracle's (over {prompts} prompts)", n=compared)
    assert compared >= 3, compared
    p.close()


def test_speculative_step_needs_a_carry():
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", threads=1)
    ctx = binding.Context(shape, max_seq=64, max_block=8)
    ctx.load_model(w, as_bf16_bits=True)
    out = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.BdError):
        ctx.bd_speculative_step(4, out)                            # before prefill
    ctx.bd_prefill(None, torch.arange(10, dtype=torch.int32, device="cuda"))
    ctx.bd_crop(6)
    with pytest.raises(binding.BdError):
        ctx.bd_speculative_step(4, out)                            # the crop dropped the carry
    ctx.bd_commit_block(torch.tensor([1, 2], dtype=torch.int32, device="cuda"))
    assert ctx.bd_speculative_step(4, out) >= 1
    with pytest.raises(binding.BdError):
        ctx.bd_speculative_step(9, out)                            # block larger than max_block
    ctx.close()



# ---- quadratic speculative decoding (Alg. 2): one forward per iteration -----------------------------------------

@pytest.mark.parametrize("B", [1, 2, 3, 5, 7, 8, 16, 21, 32])
def test_quadratic_step_against_the_oracle(B):
    """Draft, then iterations of the quadratic step, each held against the oracle's on the same state: logits of all
    B(B+1) rows, accept length, next draft, carry, and the cache (keys and values of the accepted first tokens moved
    into place).  B = 5 (30 rows) runs on the streaming kernel, B = 7 (56 rows) on the register-ring kernel (the context
    is too small for the large-M kernels), B = 8 (72 rows), 16 (272), 21 (462: a ragged last tile) and 32 (1056 rows, the
    largest block) on the large-M kernels with the quadratic mask and the per-row positions, the LM head in slices of
    64 rows."""
    _say(f"quadratic step vs oracle, tiny config, B={B}")
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", lm_head_scale=20.0, threads=1)
    emb, ids = inputs.make_prompt(shape, 24, 24, seed=6)
    M = B * (B + 1)
    p = Pair(shape, w, max_seq=48 + 6 * B + M, max_block=min(max(M, 4), 64))
    p.prefill(emb, ids)
    import copy
    greedy = copy.deepcopy(p.o).greedy_ar(6)
    d_gpu = torch.zeros(B, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(B, dtype=torch.int32, device="cuda")
    p.ctx.bd_quad_draft(B, d_gpu)
    d = p.o.quad_draft(B)
    if B > 1:
        glog = p.ctx.bd_read_logits(B).cpu().numpy()
        from oracle.bd_oracle import BIDIR
        olog, _, _ = p.o.forward(p.o.embed(np.full(B, p.o.mask_id, np.int32)), BIDIR)
        assert_logits_close(glog, olog, n_layers=shape.n_layers)
        thr0 = bars(olog, shape.n_layers)[1]
        draft_robust = bool(top2_margin(olog)[:B - 1].min() > thr0 and p.carry_is_robust())
    else:
        draft_robust = bool(p.carry_is_robust())
    note("count", what="first draft held against the oracle's", n=int(draft_robust))
    if draft_robust:
        assert np.array_equal(d_gpu.cpu().numpy(), d)
    else:
        d = d_gpu.cpu().numpy().copy()            # the oracle follows the device's draft: the steps are what is compared
        d[0] = int(np.argmax(p.o.carry))
        d_gpu.copy_(torch.from_numpy(d))
    emitted = []
    compared = 0
    for it in range(6):
        r = p.o.quad_step(d)
        k = p.ctx.bd_quad_step(B, d_gpu, nxt)
        glog = p.ctx.bd_read_logits(M).cpu().numpy()
        assert_logits_close(glog, r["logits"], n_layers=shape.n_layers)
        thr = bars(r["logits"], shape.n_layers)[1]
        W = B + 1
        firsts = top2_margin(r["logits"])[::W]
        if firsts[:r["k"]].min() <= thr:          # a near-tie among the rows that decide the accept length
            break
        assert k == r["k"], (it, k, r["k"])
        # the next draft, entry by entry where the oracle's row is not a near-tie (the first entry is the carry: held)
        sure = top2_margin(r["logits"])[(r["k"] - 1) * W:(r["k"] - 1) * W + B] > thr
        assert sure[0] and np.array_equal(nxt.cpu().numpy()[sure], r["next_draft"][sure])
        note("count", what="next-draft entries held against the oracle's", n=int(sure.sum()))
        assert p.ctx.bd_cache_len() == p.o.n
        cand, _ = p.ctx.bd_read_carry()
        assert cand == int(np.argmax(p.o.carry))
        p.check_kv(max(0, p.o.n - k - 2), min(k + 2, p.o.n))
        compared += 1
        emitted += [int(t) for t in r["accepted"]]
        d = r["next_draft"]                       # both sides go on from the oracle's draft
        d_gpu.copy_(torch.from_numpy(np.asarray(d, np.int32)))
    note("count", what="quadratic iterations held against the oracle's", n=compared)
    assert compared >= 1 and len(emitted) >= 1, compared
    if draft_robust:
        n = min(len(emitted), 6)
        assert emitted[:n] == [int(t) for t in greedy[:n]]
    p.check_kv(0, p.o.n)
    p.close()


@pytest.mark.parametrize("B,flip", [(3, False), (5, True), (7, True)])
def test_quadratic_step_accept_lengths_on_a_token_cycle(B, flip):
    _say(f"quadratic step on the cyclic model, B={B}, flip={flip}")
    shape = inputs.TINY
    w, A, Bt = _cyclic_model(shape, flip)
    ids = np.array([3, 17, 200, 41, 7], np.int32)
    M = B * (B + 1)
    p = Pair(shape, w, max_seq=5 + 6 * B + M, max_block=M)
    p.prefill(None, ids)
    d_gpu = torch.zeros(B, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(B, dtype=torch.int32, device="cuda")
    p.ctx.bd_quad_draft(B, d_gpu)
    d = p.o.quad_draft(B)
    assert np.array_equal(d_gpu.cpu().numpy(), d) and list(d) == [A] * B
    ks = []
    for it in range(5):
        r = p.o.quad_step(d)
        k = p.ctx.bd_quad_step(B, d_gpu, nxt)
        assert k == r["k"] and np.array_equal(nxt.cpu().numpy(), r["next_draft"])
        assert p.ctx.bd_cache_len() == p.o.n
        ks.append(k)
        d = r["next_draft"]
        d_gpu.copy_(nxt)
    # fixed point: whole blocks; alternation A, Bt, A, ..: the all-A draft fails at once, then [Bt, A, A, ..] gives 2
    assert ks == ([B] * 5 if not flip else [1, 2, 2, 2, 2])
    p.check_kv(0, p.o.n)
    p.close()


def test_quadratic_step_rejects_blocks_that_do_not_fit():
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", threads=1)
    ctx = binding.Context(shape, max_seq=64, max_block=32)
    ctx.load_model(w, as_bf16_bits=True)
    d = torch.zeros(8, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.BdError):
        ctx.bd_quad_step(3, d, nxt)                                # before prefill
    ctx.bd_prefill(None, torch.arange(40, dtype=torch.int32, device="cuda"))
    with pytest.raises(binding.BdError):
        ctx.bd_quad_step(6, d, nxt)                                # 42 rows > max_block
    with pytest.raises(binding.BdError):
        ctx.bd_quad_step(5, d, nxt)                                # 40 + 30 rows > max_seq
    ctx.bd_quad_draft(4, d)
    assert 1 <= ctx.bd_quad_step(4, d, nxt) <= 4                   # 40 + 20 rows fit
    ctx.close()


@pytest.mark.parametrize("B", [5, 8, 16, 32])
def test_quadratic_step_3b_shaped_two_layers(B):
    M = B * (B + 1)
    _say(f"quadratic step vs oracle, 3B-shaped x2 layers, B={B} ({M} rows)")
    shape = _wide(2, vocab=8192)
    w = inputs.make_weights(shape, 0, "bf16", lm_head_scale=20.0, threads=8)
    emb, ids = inputs.make_prompt(shape, 100, 41, seed=13)
    p = Pair(shape, w, max_seq=141 + 3 * B + M, max_block=32 if M <= 32 else 64)
    p.prefill(emb, ids)
    d_gpu = torch.zeros(B, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(B, dtype=torch.int32, device="cuda")
    p.ctx.bd_quad_draft(B, d_gpu)
    d = d_gpu.cpu().numpy()                       # the oracle follows the device's draft: the step is what is compared
    compared = 0
    for it in range(2):
        r = p.o.quad_step(d)
        k = p.ctx.bd_quad_step(B, d_gpu, nxt)
        glog = p.ctx.bd_read_logits(M).cpu().numpy()
        assert_logits_close(glog, r["logits"], n_layers=shape.n_layers)
        thr = bars(r["logits"], shape.n_layers)[1]
        W = B + 1
        if top2_margin(r["logits"])[::W][:r["k"]].min() <= thr:
            break
        sure = top2_margin(r["logits"])[(r["k"] - 1) * W:(r["k"] - 1) * W + B] > thr
        assert k == r["k"] and sure[0] and np.array_equal(nxt.cpu().numpy()[sure], r["next_draft"][sure])
        p.check_kv(p.o.n - k, k)
        compared += 1
        d = r["next_draft"]                       # both sides go on from the oracle's draft
        d_gpu.copy_(torch.from_numpy(np.asarray(d, np.int32)))
    note("count", what="quadratic iterations held against the oracle's (logits of every iteration run are held)", n=compared)
    p.close()

# ---- 3B-shaped layers at reduced depth: every block size, ragged prefix, both masks -------------------

def _wide(n_layers, vocab=32000):
    return inputs.ModelShape(n_layers=n_layers, hidden=2048, n_q_heads=16, n_kv_heads=2, head_dim=128, ffn=11008,
                             vocab=vocab)


@pytest.mark.parametrize("B", [4, 8, 16, 32, 33, 64])
def test_3b_shaped_two_layers_block_sizes(B):
    _say(f"3B-shaped x2 layers, B={B}")
    shape = _wide(2)
    w = inputs.make_weights(shape, 0, "bf16", threads=8)
    emb, ids = inputs.make_prompt(shape, 200, 101, seed=103)       # 301: not a multiple of 32 or of 64
    p = Pair(shape, w, max_seq=301 + 2 * 64)
    p.prefill(emb, ids)
    p.check_carry()
    p.check_kv(0, 301)
    tok, msk = fresh_block(shape, B)
    K = min(4, B - 1)
    while msk.any():
        tok, msk, _ = p.denoise_step(tok, msk, 0.9, fixed_k=K)
    p.commit(tok)
    p.check_kv(301, B)
    # the same forward twice gives bit-identical logits (fixed-order reductions)
    t = torch.from_numpy(tok).cuda()
    p.ctx.bd_verify_block(t, False, None, None)
    a = p.ctx.bd_read_logits(B).clone()
    p.ctx.bd_verify_block(t, False, None, None)
    b = p.ctx.bd_read_logits(B)
    assert torch.equal(a, b)
    p.close()



@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
def test_xcd_local_handover_is_bit_identical_to_the_chip_wide_one(dtype):
    """The gate/up -> down hand-over inside each XCD moves the same values through other caches: logits, K/V and
    the revealed ids of a whole block must not change by a bit against the chip-wide path, and a forward repeated
    many times (alternating with forwards of another block size, which rewrite the same buffers) must repeat
    exactly.  A stale line anywhere in the hand-over would show up as a difference.  The attention phase kept inside
    the XCDs sums its key chunks in another order than the chip-wide key split: it must repeat exactly too, and agree
    with the key split to bf16 rounding."""
    _say(f"3B-shaped x2 layers, {dtype} weights: XCD-local vs chip-wide hand-overs, B=32 and B=8 interleaved")
    shape = _wide(2, vocab=8192)
    w = inputs.make_weights(shape, 5, dtype, threads=8)
    emb, ids = inputs.make_prompt(shape, 96, 37, seed=11)

    def run(flags):
        ctx = binding.Context(shape, max_seq=133 + 64, max_block=32,
                              weight_dtype=binding.BD_FP8_E4M3 if dtype == "fp8" else binding.BD_BF16, flags=flags)
        ctx.load_model(w, as_bf16_bits=True)
        ctx.bd_debug_logits(True)
        ctx.bd_prefill(torch.from_numpy(emb).cuda(), torch.from_numpy(ids).cuda())
        out = []
        rng = np.random.default_rng(3)
        big = torch.from_numpy(rng.integers(0, shape.vocab - 1, 32).astype(np.int32)).cuda()
        small = torch.from_numpy(rng.integers(0, shape.vocab - 1, 8).astype(np.int32)).cuda()
        for rep in range(6):
            ctx.bd_verify_block(big, False, None, None)
            out.append(ctx.bd_read_logits(32).clone())
            ctx.bd_verify_block(small, False, None, None)
            out.append(ctx.bd_read_logits(8).clone())
        ctx.bd_status()
        ctx.bd_commit_block(big)
        k, v = ctx.bd_read_kv(1, 133, 32)
        out += [k.clone(), v.clone()]
        ctx.close()
        return out

    a = run(binding.BD_FLAG_ATTENTION_KEY_SPLIT)
    b = run(binding.BD_FLAG_ATTENTION_KEY_SPLIT | binding.BD_FLAG_CHIP_WIDE_HANDOVER)
    for rep in range(2, 12):
        assert torch.equal(a[rep], a[rep % 2]), f"repeat {rep} of the XCD-local forward differs"
    for i, (x, y) in enumerate(zip(a, b)):
        assert torch.equal(x, y), f"output {i} differs between the two hand-overs"
    c = run(0)
    for rep in range(2, 12):
        assert torch.equal(c[rep], c[rep % 2]), f"repeat {rep} of the forward with attention inside the XCDs differs"
    for i, (x, y) in enumerate(zip(c, a)):
        scale = float(y.abs().max())
        assert float((x - y).abs().max()) <= 2e-2 * scale, f"output {i}: attention inside the XCDs vs key split"


def test_long_prefix_3b_shaped_two_layers():
    _say("3B-shaped x2 layers, prefix 8192 (4 x 1920 embeddings + 512 ids)")
    shape = _wide(2, vocab=8192)
    w = inputs.make_weights(shape, 0, "bf16", threads=8)
    emb, ids = inputs.make_prompt(shape, 4 * 1920, 512, seed=102)
    p = Pair(shape, w, max_seq=8192 + 64, oracle_dtype=np.float32)
    p.prefill(emb, ids, oracle_chunk=1024)
    p.check_carry()
    p.check_kv(8000, 192)
    tok, msk = fresh_block(shape, 32)
    while msk.any():
        tok, msk, _ = p.denoise_step(tok, msk, 0.9, fixed_k=4)
    p.commit(tok)
    p.check_kv(8192, 32)
    # a verify call on top of the 8224 tokens: logits of all rows and the predictions against the oracle's
    import copy
    draft = np.asarray(tok[:16], np.int32)
    r = copy.deepcopy(p.o).verify_block(draft, commit=False)
    pred = torch.zeros(16, dtype=torch.int32, device="cuda")
    nacc = torch.zeros(1, dtype=torch.int32, device="cuda")
    p.ctx.bd_verify_block(torch.from_numpy(draft).cuda(), False, pred, nacc)
    glog = p.ctx.bd_read_logits(16).cpu().numpy()
    assert_logits_close(glog, r["logits"], n_layers=shape.n_layers)
    check_argmax_ids(pred.cpu().numpy(), glog, r["logits"], shape.n_layers)
    assert p.ctx.bd_cache_len() == 8224
    p.close()


# ---- configs[3] at 3B width: verification of drafts of every block size on a 2048-token prefix -----------------

def test_verify_block_sizes_3b_shaped_prefix_2048():
    """bd_verify_block on a 2048-token prefix (1536 embeddings + 512 ids), 3B-shaped x2 layers, drafts of 4 .. 64
    tokens (the greedy continuation with a fifth of the tokens replaced): logits of every row, the predictions and the
    accept length against the oracle; blocks of 64 run on the large-M kernels, the others on the streaming kernel."""
    _say("3B-shaped x2 layers, prefix 2048, verify blocks of 4 .. 64 tokens")
    shape = _wide(2, vocab=8192)
    w = inputs.make_weights(shape, 0, "bf16", lm_head_scale=20.0, threads=8)
    p = Pair(shape, w, max_seq=2048 + 64, oracle_dtype=np.float32)
    for seed in range(103, 111):                 # (a prompt whose last row decides its argmax beyond the id margin)
        emb, ids = inputs.make_prompt(shape, 1536, 512, seed=seed)
        p.prefill(emb, ids, oracle_chunk=512)
        p.check_carry()
        if p.carry_is_robust():
            break
    assert p.carry_is_robust()
    import copy
    clean = copy.deepcopy(p.o).greedy_ar(64)
    held = 0
    for B in (4, 8, 16, 32, 33, 64):
        _say(f"  B={B}")
        draft, _ = inputs.corrupt_draft(shape, clean[:B], seed=B, p=0.2)
        r = copy.deepcopy(p.o).verify_block(draft, commit=False)
        pred = torch.zeros(B, dtype=torch.int32, device="cuda")
        nacc = torch.zeros(1, dtype=torch.int32, device="cuda")
        p.ctx.bd_verify_block(torch.from_numpy(draft).cuda(), False, pred, nacc)
        assert p.ctx.bd_cache_len() == 2048
        glog = p.ctx.bd_read_logits(B).cpu().numpy()
        assert_logits_close(glog, r["logits"], n_layers=shape.n_layers)
        ok = check_argmax_ids(pred.cpu().numpy(), glog, r["logits"], shape.n_layers)
        decided = bool(ok[:max(r["n_accept"], 1)].all() and p.carry_is_robust())
        held += int(decided)
        if decided:
            assert int(nacc.item()) == r["n_accept"], (B, int(nacc.item()), r["n_accept"])
        else:
            gp = np.concatenate([[p.ctx.bd_read_carry()[0]], pred.cpu().numpy()[:-1]])
            k = 0
            while k < B and gp[k] == draft[k]:
                k += 1
            assert int(nacc.item()) == k
    note("count", what="accept lengths held against the oracle's (of 6 block sizes)", n=held)
    assert held >= 1, held
    p.close()


@pytest.mark.parametrize("B", [33, 64])
def test_large_m_forward_agrees_with_the_register_ring_kernel(B):
    """Forwards of 33 .. 64 rows run on the large-M kernels where the context has their buffers, else (or with
    BD_FLAG_PREFILL_DECODE) on the register-ring kernel: two implementations of the same forward, written apart, must
    agree to bf16 rounding on logits and cache, for the bidirectional and the causal mask."""
    _say(f"3B-shaped x2 layers, B={B}: large-M kernels vs register-ring kernel")
    shape = _wide(2, vocab=8192)
    w = inputs.make_weights(shape, 4, "bf16", threads=8)
    emb, ids = inputs.make_prompt(shape, 96, 37, seed=11)
    outs = []
    for flags in (0, binding.BD_FLAG_PREFILL_DECODE):
        ctx = binding.Context(shape, max_seq=133 + 2 * 64, max_block=64, flags=flags)
        ctx.load_model(w, as_bf16_bits=True)
        ctx.bd_debug_logits(True)
        ctx.bd_prefill(torch.from_numpy(emb).cuda(), torch.from_numpy(ids).cuda())
        tok, msk = fresh_block(shape, B)
        gt = torch.from_numpy(tok.astype(np.int32)).cuda()
        gm = torch.from_numpy(msk.astype(np.uint8)).cuda()
        ctx.bd_denoise_step(gt, gm, 0.9, 4, None, None)
        res = [ctx.bd_read_logits(B).clone()]
        ctx.bd_commit_block(torch.arange(7, 7 + B, dtype=torch.int32, device="cuda"))
        res.append(ctx.bd_read_logits(B).clone())
        k, v = ctx.bd_read_kv(1, 133, B)
        res += [k.clone(), v.clone()]
        ctx.bd_status()
        ctx.close()
        outs.append(res)
    for i, (x, y) in enumerate(zip(*outs)):
        scale = float(y.abs().max())
        err = float((x - y).abs().max())
        note("count", what=f"output {i}: max abs difference / range x 1e6", n=int(1e6 * err / scale))
        assert err <= 2e-2 * scale, (i, err, scale)


# ---- paged cache: results do not depend on which pages hold which blocks -----------------------------------------

@pytest.mark.parametrize("flags", [0, binding.BD_FLAG_ATTENTION_KEY_SPLIT, binding.BD_FLAG_REGISTER_RING, binding.BD_FLAG_PREFILL_DECODE])
def test_paged_cache_any_page_order_gives_the_same_bits(flags):
    """Two contexts on the same model and prompt, one handing out its cache pages in ascending order (a contiguous
    cache), one in a shuffled order: prompt pass, denoising steps, commit, verify + crop, a speculative step, quadratic
    steps (30 and 72 rows), a 64-row forward and a last commit must agree bit for bit in logits, ids, accept lengths and
    in the cache read back by position -- through the streaming kernel (attention inside the XCDs and by key split), the
    register-ring kernel and the large-M kernels.  The page lists themselves must differ, shrink at every crop (the list
    is cut where the context is) and hand the freed pages out again in the same order."""
    _say(f"paged cache, shuffled vs ascending page order, flags={flags}")
    shape = _wide(2, vocab=8192)
    w = inputs.make_weights(shape, 6, "bf16", lm_head_scale=20.0, threads=8)
    emb, ids = inputs.make_prompt(shape, 150, 57, seed=21)               # 207 rows: large-M prompt pass unless switched off
    max_seq = 207 + 3 * 64 + 72 + 16
    n_pages = -(-max_seq // 32)
    order = np.random.default_rng(5).permutation(n_pages).astype(np.int32)
    assert not np.array_equal(order, np.arange(n_pages))
    runs = []
    for shuffled in (False, True):
        ctx = binding.Context(shape, max_seq=max_seq, max_block=64, flags=flags)
        ctx.load_model(w, as_bf16_bits=True)
        ctx.bd_debug_logits(True)
        if shuffled:
            ctx.bd_kv_page_order(order)
        assert len(ctx.bd_kv_pages()) == 0
        log, pages = [], []

        def keep(*tensors):
            log.extend(t.clone() if torch.is_tensor(t) else torch.tensor(t) for t in tensors)

        ctx.bd_prefill(torch.from_numpy(emb).cuda(), torch.from_numpy(ids).cuda())
        pages.append(ctx.bd_kv_pages().copy())
        assert len(pages[-1]) == -(-207 // 32)
        keep(ctx.bd_read_logits(1), *ctx.bd_read_kv(1, 0, 207))
        tok, msk = fresh_block(shape, 32)
        gt = torch.from_numpy(tok.astype(np.int32)).cuda()
        gm = torch.from_numpy(msk.astype(np.uint8)).cuda()
        while bool(gm.any().item()):
            ctx.bd_denoise_step(gt, gm, 0.9, 4, None, None)
            keep(ctx.bd_read_logits(32), gt, gm)
        ctx.bd_commit_block(gt)                                            # 239
        keep(ctx.bd_read_logits(32), *ctx.bd_read_kv(0, 200, 39))
        pages.append(ctx.bd_kv_pages().copy())
        # verify with commit, then crop into the middle of a block and to a block boundary
        d = torch.arange(11, 11 + 16, dtype=torch.int32, device="cuda")
        pred = torch.zeros(16, dtype=torch.int32, device="cuda")
        nacc = torch.zeros(1, dtype=torch.int32, device="cuda")
        ctx.bd_verify_block(d, True, pred, nacc)                           # 255
        keep(ctx.bd_read_logits(16), pred, nacc)
        ctx.bd_crop(250)
        assert len(ctx.bd_kv_pages()) == 8
        ctx.bd_crop(224)
        pages.append(ctx.bd_kv_pages().copy())
        assert len(pages[-1]) == 7
        ctx.bd_commit_block(torch.arange(3, 3 + 8, dtype=torch.int32, device="cuda"))   # 232: block 7 comes back
        pages.append(ctx.bd_kv_pages().copy())
        assert len(pages[-1]) == 8 and pages[-1][7] == pages[1][7]
        out = torch.zeros(64, dtype=torch.int32, device="cuda")
        k = ctx.bd_speculative_step(8, out)                                # 232 + k
        keep(ctx.bd_read_logits(8), out[:k], k)
        for B in (5, 7 if flags & binding.BD_FLAG_PREFILL_DECODE else 8):   # (72 rows need the large-M kernels)
            dq = torch.zeros(B, dtype=torch.int32, device="cuda")
            nx = torch.zeros(B, dtype=torch.int32, device="cuda")
            ctx.bd_quad_draft(B, dq)
            k = ctx.bd_quad_step(B, dq, nx)
            keep(ctx.bd_read_logits(B * (B + 1)), dq, nx, k)
            assert len(ctx.bd_kv_pages()) == -(-ctx.bd_cache_len() // 32)   # the rows beyond the accepted ones gave their pages back
        n = ctx.bd_cache_len()
        tok, msk = fresh_block(shape, 64)
        gt = torch.from_numpy(tok.astype(np.int32)).cuda()
        gm = torch.from_numpy(msk.astype(np.uint8)).cuda()
        ctx.bd_denoise_step(gt, gm, 0.9, 8, None, None)
        keep(ctx.bd_read_logits(64), gt, gm)
        ctx.bd_commit_block(torch.arange(40, 40 + 64, dtype=torch.int32, device="cuda"))
        keep(ctx.bd_read_logits(64), *ctx.bd_read_kv(1, 0, n + 64), *ctx.bd_read_kv(0, n - 10, 74))
        pages.append(ctx.bd_kv_pages().copy())
        ctx.bd_status()
        ctx.bd_crop(0)
        assert len(ctx.bd_kv_pages()) == 0
        ctx.close()
        runs.append((log, pages))
    (la, pa), (lb, pb) = runs
    assert len(la) == len(lb)
    for i, (x, y) in enumerate(zip(la, lb)):
        assert torch.equal(x, y), f"output {i} depends on the page order"
    for x, y in zip(pa, pb):
        assert np.array_equal(x, np.arange(len(x)))                        # ascending order = the contiguous cache
        assert np.array_equal(y, order[:len(y)]) and not np.array_equal(x, y)
    note("count", what="outputs held bit-identical between page orders", n=len(la))


def test_page_order_is_fixed_while_pages_are_in_use():
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", threads=1)
    ctx = binding.Context(shape, max_seq=96, max_block=16)
    ctx.load_model(w, as_bf16_bits=True)
    with pytest.raises(binding.BdError) as e:
        ctx.bd_kv_page_order([0, 1])                                       # not the pool's size
    assert e.value.code == binding.BD_E_ARG
    with pytest.raises(binding.BdError):
        ctx.bd_kv_page_order([0, 0, 1])                                    # not a permutation
    ctx.bd_kv_page_order([2, 0, 1])
    ctx.bd_prefill(None, torch.arange(40, dtype=torch.int32, device="cuda"))
    assert list(ctx.bd_kv_pages()) == [2, 0]
    with pytest.raises(binding.BdError) as e:
        ctx.bd_kv_page_order([0, 1, 2])
    assert e.value.code == binding.BD_E_STATE
    ctx.bd_crop(0)
    ctx.bd_kv_page_order([1, 2, 0])
    ctx.bd_prefill(None, torch.arange(70, dtype=torch.int32, device="cuda"))
    assert list(ctx.bd_kv_pages()) == [1, 2, 0]
    ctx.close()


# ---- configs[4]: e4m3 decoder weights with per-output-channel scales ---------------------------------------

def test_fp8_tiny_block_decode():
    _say("tiny config, e4m3 decoder linears (seed 2), jittered norm gains")
    shape = inputs.TINY
    w = inputs.make_weights(shape, 2, "fp8", norm_gain_jitter=0.1, threads=1)
    emb, ids = inputs.make_prompt(shape, 40, 37, seed=104)
    p = Pair(shape, w, max_seq=256)
    p.prefill(emb, ids)
    p.check_carry()
    p.check_kv(0, 77, frac=6e-2)
    tok, msk = fresh_block(shape, 8)
    while msk.any():
        tok, msk, _ = p.denoise_step(tok, msk, 0.9, fixed_k=3, frac=FP8_LOGIT_TOL)
    p.commit(tok, frac=FP8_LOGIT_TOL)
    p.close()


@pytest.mark.parametrize("n_embed,n_ids", [(0, 129), (150, 150), (0, 400)])
def test_fp8_large_m_prefill(n_embed, n_ids):
    """Prompts of more than 128 rows on a context with e4m3 weights go through the large-M kernels (codes widened into
    the tile-major bf16 copy, row scales on the accumulators, norm gains in the activation copy): cache, carry and a
    decode step on top against the oracle."""
    _say(f"tiny config, e4m3 weights, jittered gains, large-M prefill of {n_embed}+{n_ids} rows")
    shape = inputs.TINY
    w = inputs.make_weights(shape, 2, "fp8", norm_gain_jitter=0.1, threads=1)
    emb, ids = inputs.make_prompt(shape, n_embed, n_ids, seed=106)
    p = Pair(shape, w, max_seq=n_embed + n_ids + 64)
    p.prefill(emb, ids)
    p.check_carry()
    p.check_kv(0, n_embed + n_ids, frac=6e-2)
    tok, msk = fresh_block(shape, 8)
    p.denoise_step(tok, msk, 0.9, fixed_k=3, frac=FP8_LOGIT_TOL)
    p.close()


def test_fp8_whole_block_and_speculative_calls():
    """The calls that chain forwards on the device, on a context with e4m3 weights: a whole block per call equals the
    step-by-step loop bit for bit, a speculative iteration accepts between 1 and B tokens and leaves a valid carry, and
    so does a quadratic one (held against the oracle in test_fp8_quadratic_step)."""
    _say("tiny config, e4m3 weights: bd_decode_block, bd_speculative_step, bd_quad_step")
    shape = inputs.TINY
    w = inputs.make_weights(shape, 2, "fp8", lm_head_scale=20.0, threads=1)
    emb, ids = inputs.make_prompt(shape, 20, 20, seed=105)
    ctxs = []
    for _ in range(2):
        c = binding.Context(shape, max_seq=200, max_block=32, weight_dtype=binding.BD_FP8_E4M3)
        c.load_model(w)
        c.bd_prefill(torch.from_numpy(emb).cuda(), torch.from_numpy(ids).cuda())
        ctxs.append(c)
    a, b = ctxs
    B = 16
    out = torch.zeros(B, dtype=torch.int32, device="cuda")
    nst = torch.zeros(1, dtype=torch.int32, device="cuda")
    a.bd_decode_block(B, 0.3, 0, out, nst)
    tok = torch.full((B,), shape.mask_token_id, dtype=torch.int32, device="cuda")
    msk = torch.ones(B, dtype=torch.uint8, device="cuda")
    fwd = 0
    while bool(msk.any().item()):
        b.bd_denoise_step(tok, msk, 0.3, 0, None, None)
        fwd += 1
    b.bd_commit_block(tok)
    assert torch.equal(out, tok) and int(nst.item()) == fwd
    assert a.bd_read_carry() == b.bd_read_carry()
    k = a.bd_speculative_step(8, out)
    assert 1 <= k <= 8 and a.bd_cache_len() == 40 + B + k
    a.bd_read_carry()
    n0 = a.bd_cache_len()
    a.bd_quad_draft(3, out)
    k = a.bd_quad_step(3, out, tok)
    assert 1 <= k <= 3 and a.bd_cache_len() == n0 + k
    a.bd_read_carry()
    a.bd_status()
    a.close()
    b.close()


@pytest.mark.parametrize("shape_name,B", [("tiny", 3), ("tiny", 5), ("tiny", 8), ("wide", 5), ("wide", 16)])
def test_fp8_quadratic_step(shape_name, B):
    """Alg. 2 on e4m3 decoder linears: 12 and 30 rows on the streaming kernel, 72 and 272 rows on the large-M kernels
    (widened weights, row scales in the epilogue); logits of every row, accept length, next draft and the moved cache
    rows against the oracle's on the same state."""
    M = B * (B + 1)
    _say(f"quadratic step vs oracle, e4m3 weights, {shape_name}, B={B} ({M} rows)")
    shape = inputs.TINY if shape_name == "tiny" else _wide(2, vocab=8192)
    w = inputs.make_weights(shape, 2, "fp8", lm_head_scale=20.0, threads=1 if shape_name == "tiny" else 8)
    emb, ids = inputs.make_prompt(shape, 100, 41, seed=13)
    p = Pair(shape, w, max_seq=141 + 3 * B + M, max_block=32 if M <= 32 else 64)
    p.prefill(emb, ids)
    d_gpu = torch.zeros(B, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(B, dtype=torch.int32, device="cuda")
    p.ctx.bd_quad_draft(B, d_gpu)
    d = d_gpu.cpu().numpy()                       # the oracle follows the device's draft: the step is what is compared
    compared = 0
    W = B + 1
    for it in range(3):
        r = p.o.quad_step(d)
        k = p.ctx.bd_quad_step(B, d_gpu, nxt)
        glog = p.ctx.bd_read_logits(M).cpu().numpy()
        assert_logits_close(glog, r["logits"], frac=FP8_LOGIT_TOL, n_layers=shape.n_layers)
        thr = bars(r["logits"], shape.n_layers)[1]
        if top2_margin(r["logits"])[::W][:r["k"]].min() <= thr:
            break
        sure = top2_margin(r["logits"])[(r["k"] - 1) * W:(r["k"] - 1) * W + B] > thr
        assert k == r["k"] and sure[0] and np.array_equal(nxt.cpu().numpy()[sure], r["next_draft"][sure])
        assert p.ctx.bd_cache_len() == p.o.n
        p.check_kv(p.o.n - k, k, frac=6e-2)
        compared += 1
        d = r["next_draft"]                       # both sides go on from the oracle's draft
        d_gpu.copy_(torch.from_numpy(np.asarray(d, np.int32)))
    note("count", what="quadratic iterations held against the oracle's (logits of every iteration run are held)", n=compared)
    p.close()


@pytest.mark.parametrize("B", [4, 16, 32, 33, 64])
def test_fp8_3b_shaped_two_layers(B):
    _say(f"3B-shaped x2 layers, e4m3 decoder linears, B={B}")
    shape = _wide(2)
    w = inputs.make_weights(shape, 2, "fp8", threads=8)
    emb, ids = inputs.make_prompt(shape, 150, 83, seed=104)
    p = Pair(shape, w, max_seq=233 + 64)
    p.prefill(emb, ids)
    p.check_kv(0, 233, frac=6e-2)
    tok, msk = fresh_block(shape, B)
    K = min(4, B - 1)
    while msk.any():
        tok, msk, _ = p.denoise_step(tok, msk, 0.9, fixed_k=K, frac=FP8_LOGIT_TOL)
    p.commit(tok, frac=FP8_LOGIT_TOL)
    p.check_kv(233, B, frac=6e-2)
    assert p.ctx.bd_forward_bytes() == (shape.weight_elements() - shape.vocab * shape.hidden) \
        + 2 * shape.vocab * shape.hidden + 4 * 2 * (shape.q_dim + 2 * shape.kv_dim + 2 * shape.hidden + 2 * shape.ffn) \
        + 2 * 2 * 2 * shape.kv_dim * (233 + B)
    p.close()


def test_fp8_context_rejects_wide_blocks_and_bf16_linears():
    shape = inputs.TINY
    with pytest.raises(binding.BdError) as e:
        binding.Context(shape, max_seq=128, max_block=64, weight_dtype=binding.BD_FP8_E4M3)
    assert e.value.code == binding.BD_E_ARG
    ctx = binding.Context(shape, max_seq=128, max_block=32, weight_dtype=binding.BD_FP8_E4M3)
    ctx.bd_load_weight("l0.attn_norm", np.ones(shape.hidden, np.float32))
    with pytest.raises(binding.BdError) as e:
        ctx.bd_load_weight("l0.wq", np.zeros((shape.q_dim, shape.hidden), np.float32))
    assert e.value.code == binding.BD_E_DTYPE
    ctx.close()


# ---- configs[1] at full size ----------------------------------------------------------------------------

@pytest.mark.slow
def test_headline_config_first_block_full_depth():
    shape = inputs.QWEN3B
    _say("generating 3B-shaped bf16 weights (seed 0)")
    w = inputs.make_weights(shape, 0, "bf16", threads=16)
    emb, ids = inputs.make_prompt(shape, 768, 256, seed=101)
    _say("uploading + oracle prefill of 1024 tokens")
    p = Pair(shape, w, max_seq=1024 + 256 + 32, oracle_dtype=np.float32)
    p.prefill(emb, ids, oracle_chunk=256)
    # the last prompt row's logits (row 0 of the LM-head pass that ends a large-M prefill) against the oracle's, to the
    # bars of every other logits row
    glog = p.ctx.bd_read_logits(1).cpu().numpy()[0]
    assert_logits_close(glog, p.o.carry, what="carry logits", n_layers=shape.n_layers)
    p.check_carry()
    tok, msk = fresh_block(shape, 32)
    fwd = 0
    while msk.any():
        tok, msk, r = p.denoise_step(tok, msk, 0.9, fixed_k=4)
        fwd += 1
        _say(f"  denoise forward {fwd}: {int((~msk).sum())}/32 revealed")
    assert fwd == 8
    p.commit(tok)
    assert p.ctx.bd_forward_bytes() == 2 * shape.weight_elements() + 36864 * (1024 + 32)
    # one denoising forward of 64 rows on top (the large-M kernels at full depth), and its commit
    tok, msk = fresh_block(shape, 64)
    tok, msk, _ = p.denoise_step(tok, msk, 0.9, fixed_k=4)
    _say(f"  64-row denoise forward: {int((~msk).sum())}/64 revealed")
    tok[msk] = 7
    p.commit(tok)
    p.close()


@pytest.mark.slow
def test_fp8_config_first_block_full_depth():
    """configs[4] at full depth: e4m3 decoder linears, 36 layers, the first block of 32 tokens (8 denoising forwards +
    commit) against the fp32 oracle on the same codes and scales, to the e4m3 bars.  The prefix is 1024 tokens here (the
    oracle's prompt pass over 2048 takes minutes; the 2048-token prefix is held at reduced depth above)."""
    shape = inputs.QWEN3B
    _say("generating 3B-shaped e4m3 weights (seed 2)")
    w = inputs.make_weights(shape, 2, "fp8", threads=16)
    emb, ids = inputs.make_prompt(shape, 768, 256, seed=104)
    _say("uploading + oracle prefill of 1024 tokens")
    p = Pair(shape, w, max_seq=1024 + 64, oracle_dtype=np.float32, predecode=True)
    p.prefill(emb, ids, oracle_chunk=256)
    glog = p.ctx.bd_read_logits(1).cpu().numpy()[0]
    assert_logits_close(glog, p.o.carry, FP8_LOGIT_TOL, what="carry logits", n_layers=shape.n_layers)
    tok, msk = fresh_block(shape, 32)
    fwd = 0
    while msk.any():
        tok, msk, r = p.denoise_step(tok, msk, 0.9, fixed_k=4, frac=FP8_LOGIT_TOL)
        fwd += 1
        _say(f"  denoise forward {fwd}: {int((~msk).sum())}/32 revealed")
    assert fwd == 8
    p.commit(tok, frac=FP8_LOGIT_TOL)
    p.close()


def test_a_context_whose_kernels_gave_up_reports_it_and_never_hangs():
    """What a timed-out barrier leaves behind, forced from the host: with the device-side error flag raised every forward
    kernel returns at once, so nothing can wait for anything; bd_status, bd_speculative_step and bd_quad_step report
    BD_E_HIP (the two steps must not hand back the accept length of an earlier call), and the host's view of the context
    length stays where it was."""
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", threads=1)
    for max_seq in (96, 300):                                  # decode kernels only / with the large-M kernels
        ctx = binding.Context(shape, max_seq=max_seq, max_block=16)
        ctx.load_model(w, as_bf16_bits=True)
        ctx.bd_prefill(None, torch.arange(40, dtype=torch.int32, device="cuda"))
        out = torch.zeros(16, dtype=torch.int32, device="cuda")
        assert 1 <= ctx.bd_speculative_step(4, out) <= 4       # a good step first: its accept length stays in the buffer
        n = ctx.bd_cache_len()
        ctx.bd_k_raise_device_error()
        with pytest.raises(binding.BdError) as e:
            ctx.bd_speculative_step(4, out)
        assert e.value.code == binding.BD_E_HIP
        assert ctx.bd_cache_len() == n
        d = torch.zeros(3, dtype=torch.int32, device="cuda")
        nx = torch.zeros(3, dtype=torch.int32, device="cuda")
        with pytest.raises(binding.BdError) as e:
            ctx.bd_quad_step(3, d, nx)
        assert e.value.code == binding.BD_E_HIP
        tok = torch.zeros(8, dtype=torch.int32, device="cuda")
        msk = torch.ones(8, dtype=torch.uint8, device="cuda")
        ctx.bd_denoise_step(tok, msk, 0.9, 0, None, None)      # enqueues; its kernels return at once
        with pytest.raises(binding.BdError) as e:
            ctx.bd_status()
        assert e.value.code == binding.BD_E_HIP
        assert ctx.bd_cache_len() == n
        ctx.close()


# ---- error paths that need a live context -------------------------------------------------------------------

def test_call_order_and_capacity_errors():
    shape = inputs.TINY
    L = binding.lib()
    ctx = binding.Context(shape, max_seq=40, max_block=16)
    tok = torch.zeros(4, dtype=torch.int32, device="cuda")
    msk = torch.ones(4, dtype=torch.uint8, device="cuda")
    ids = torch.zeros(30, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.BdError) as e:
        ctx.bd_prefill(None, ids)                          # weights not loaded
    assert e.value.code == binding.BD_E_STATE
    ctx.load_model(inputs.make_weights(shape, 0, "bf16", threads=1))
    with pytest.raises(binding.BdError) as e:
        ctx.bd_denoise_step(tok, msk, 0.9)                 # before prefill
    assert e.value.code == binding.BD_E_STATE
    with pytest.raises(binding.BdError) as e:
        ctx.bd_prefill(None, torch.zeros(41, dtype=torch.int32, device="cuda"))
    assert e.value.code == binding.BD_E_CAPACITY
    ctx.bd_prefill(None, ids)
    big = torch.zeros(17, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.BdError) as e:
        ctx.bd_commit_block(big)                           # B > max_block
    assert e.value.code == binding.BD_E_ARG
    ctx.bd_commit_block(tok)                               # 34
    ctx.bd_commit_block(tok)                               # 38
    with pytest.raises(binding.BdError) as e:
        ctx.bd_commit_block(tok)                           # 42 > 40
    assert e.value.code == binding.BD_E_CAPACITY
    with pytest.raises(binding.BdError) as e:
        ctx.bd_crop(39)
    assert e.value.code == binding.BD_E_ARG
    ctx.bd_crop(10)
    assert ctx.bd_cache_len() == 10
    with pytest.raises(binding.BdError) as e:
        ctx.bd_read_carry()                                # undefined after a crop
    assert e.value.code == binding.BD_E_STATE
    with pytest.raises(binding.BdError) as e:
        ctx.bd_load_weight("l7.wq", np.zeros((256, 256), np.float32))
    assert e.value.code == binding.BD_E_ARG
    with pytest.raises(binding.BdError) as e:
        ctx.bd_load_weight("l0.wq", np.zeros((256, 255), np.float32))
    assert e.value.code == binding.BD_E_ARG
    torch.cuda.synchronize()
    ctx.close()


@pytest.mark.parametrize("n_embed,n_ids", [(0, 1), (1, 0), (0, 70), (70, 0), (63, 66), (0, 128), (130, 126), (0, 144),
                                           (700, 400)])
def test_prefill_edge_lengths(n_embed, n_ids):
    """Prompts of up to 128 rows go through the decode kernels; longer ones wholly through the large-M path (the last
    tile padded to 16 rows), the last row's residual stream handed to the LM head: 129 -> chunks of 128 and 1,
    256 -> 128 + 128, 144 -> 128 + 16, 1100 -> 896 + 204 rows (max_seq bounds the chunk size here)."""
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", threads=1)
    emb, ids = inputs.make_prompt(shape, n_embed, n_ids, seed=7)
    p = Pair(shape, w, max_seq=max(256, n_embed + n_ids + 32))
    p.prefill(emb, ids)
    p.check_carry()
    p.check_kv(0, n_embed + n_ids)
    tok, msk = fresh_block(shape, 8)
    p.denoise_step(tok, msk, 0.9, fixed_k=3)            # a decode step on top of the prefilled cache
    p.close()


@pytest.mark.parametrize("n_embed,n_ids", [(130, 126), (700, 400)])
def test_prefill_with_the_register_staged_gemms(n_embed, n_ids):
    """The large-M GEMM kernel that stages its operands through registers (the fallback for K tails, forced here
    for every phase, without the K split of the down projection) against the oracle."""
    shape = inputs.TINY
    w = inputs.make_weights(shape, 0, "bf16", threads=1)
    emb, ids = inputs.make_prompt(shape, n_embed, n_ids, seed=7)
    p = Pair(shape, w, max_seq=max(256, n_embed + n_ids + 32), flags=binding.BD_FLAG_PREFILL_STAGED)
    p.prefill(emb, ids)
    p.check_carry()
    p.check_kv(0, n_embed + n_ids)
    p.close()


@pytest.mark.parametrize("n_embed,n_ids", [(130, 126), (0, 144), (700, 400)])
def test_prefill_with_the_k_split_down_projection(n_embed, n_ids):
    """A small model whose FFN width lets the down projection of the large-M path split K over workgroups (the
    tiny config's 688 has a K tail and takes the unsplit kernel): cache, carry and a decode step against the oracle."""
    shape = inputs.ModelShape(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=768, vocab=1024)
    w = inputs.make_weights(shape, 3, "bf16", threads=1)
    emb, ids = inputs.make_prompt(shape, n_embed, n_ids, seed=8)
    p = Pair(shape, w, max_seq=max(256, n_embed + n_ids + 32))
    p.prefill(emb, ids)
    p.check_carry()
    p.check_kv(0, n_embed + n_ids)
    tok, msk = fresh_block(shape, 8)
    p.denoise_step(tok, msk, 0.9, fixed_k=3)
    p.close()


def test_large_m_prefill_agrees_with_the_chunked_one():
    """The same prompt through the large-M kernels and through 64-row decode forwards: same cache and carry up to
    bf16 rounding of a different summation order (each path is also held against the oracle elsewhere)."""
    _say("3B-shaped x2 layers: large-M prefill vs chunked prefill, 700 rows")
    shape = _wide(2, vocab=8192)
    w = inputs.make_weights(shape, 4, "bf16", threads=8)
    emb, ids = inputs.make_prompt(shape, 500, 200, seed=12)
    res = []
    for flags in (0, binding.BD_FLAG_PREFILL_DECODE, binding.BD_FLAG_PREFILL_STAGED):
        ctx = binding.Context(shape, max_seq=768, max_block=64, flags=flags)
        ctx.load_model(w, as_bf16_bits=True)
        ctx.bd_prefill(torch.from_numpy(emb).cuda(), torch.from_numpy(ids).cuda())
        assert ctx.bd_cache_len() == 700
        k, v = ctx.bd_read_kv(1, 0, 700)
        res.append((k.clone(), v.clone(), ctx.bd_read_carry()))
        ctx.bd_status()
        ctx.close()
    (k0, v0, c0), (k1, v1, c1), (k2, v2, c2) = res
    for a, b in ((k0, k1), (v0, v1)):
        assert float((a - b).abs().max()) <= 2e-2 * float(b.abs().max())
    assert c0[0] == c1[0] and abs(c0[1] - c1[1]) <= 0.05 * c1[1]
    # direct-to-LDS GEMMs with the K split of the down projection vs the register-staged ones: the same products, the
    # down projection summed in another order
    for a, b in ((k0, k2), (v0, v2)):
        assert float((a - b).abs().max()) <= 1e-2 * float(b.abs().max())
    assert c0[0] == c2[0] and abs(c0[1] - c2[1]) <= 0.02 * c2[1]
