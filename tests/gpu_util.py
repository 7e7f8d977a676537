"""Helpers of the GPU parity tests: run the HIP path and the oracle side by side on the same seeded inputs."""
import numpy as np
import torch

from oracle.bd_oracle import BlockDiffusionOracle
from paper_2604_06832_amd import binding, inputs

BF16_LOGIT_TOL = 3e-2      # max-abs logit error as a fraction of the oracle's logit range (bf16 path)
FP8_LOGIT_TOL = 1e-1       # the same bar for the path with e4m3 decoder weights
MARGIN = 1e-2              # ids are compared where the oracle's top-2 logit margin exceeds this

# What every comparison of the current test really covered (filled by the helpers below, summarised per test by
# tests/conftest.py): kind -> list of records.
REPORT = []


def note(kind, **kw):
    REPORT.append((kind, kw))


BAND_MISMATCH = 0.15       # share of the rows between the 1e-2 margin and the derived id margin that may differ


def assert_band(n_band, n_diff, what):
    assert n_diff <= BAND_MISMATCH * n_band + 1, f"{what}: {n_diff} of {n_band} rows inside the error band differ"


def top2_margin(logits):
    part = np.partition(logits, -2, axis=-1)
    return part[..., -1] - part[..., -2]


def bars(want_logits, n_layers):
    """The fixed bars of one comparison, from the oracle's side alone (nothing measured on the GPU enters):

    E  bound on the absolute logit error that the GPU path's arithmetic can cause.  The path hands eight tensors per
       layer from kernel to kernel in bf16 (the two normalised copies of the residual stream, Q, K, V, the attention
       probabilities, the attention output, the SwiGLU output), each rounding with relative error <= 2^-9; the
       errors are independent, add in quadrature through the 8 L hand-overs and reach the logits scaled like the
       logits themselves (standard deviation sigma of the oracle's logits): rms 2^-9 sqrt(8 L) sigma.  E is 8 times
       that (the largest of ~10^6 logits of a forward): E = 2^-6 sqrt(8 L) sigma.
    id margin  an argmax can differ between two logit rows that agree within E only where the top-2 margin is below
       2 E; ids are held bit-exact wherever the oracle's margin exceeds max(1e-2, 2 E).  At 3B scale E > 5e-3, so
       the 1e-2 margin alone cannot be met by any bf16 path (the design notes list this reading); the rows in the
       band between 1e-2 and 2 E are counted, reported and held statistically: at most BAND_MISMATCH of them (plus
       one) may differ, which a wrong mask, index or operand (every row off) cannot pass.
    C  bound on the relative error of a confidence: log conf = max logit - log sum exp; for V >> 1 the error of the
       sum averages out, leaving the error of single logits, for which 4 sigma (C = E / 2) covers the <= 64 rows of
       a forward.  A ranking of two confidences can differ only where they are closer than 2 C.
    """
    sigma = float(np.std(np.asarray(want_logits, np.float64)))
    E = 2.0 ** -6 * float(np.sqrt(8.0 * n_layers)) * sigma
    return E, max(MARGIN, 2.0 * E), 0.5 * E


def assert_logits_close(got, want, frac=BF16_LOGIT_TOL, what="logits", n_layers=None):
    """The stated bar (max-abs error within frac of the oracle's logit range) and, when the depth is given, the
    bound E derived from the arithmetic (see bars()), which is the tighter of the two in every configuration here."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    rng = float(want.max() - want.min())
    err = float(np.abs(got - want).max())
    note("logits", err=err, range=rng, rows=int(got.shape[0]) if got.ndim > 1 else 1)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    assert err <= frac * rng, f"{what}: max-abs error {err:.4g} > {frac} * range {rng:.4g}"
    if n_layers is not None:
        E = bars(want, n_layers)[0]
        assert err <= E, f"{what}: max-abs error {err:.4g} > derived bound {E:.4g}"
    return err / rng


def check_argmax_ids(got_ids, got_logits, want_logits, n_layers):
    """Fused argmax: (a) bit-exact against the argmax (lowest id on ties) of the GPU's own stored logits;
    (b) equal to the oracle's wherever the oracle's top-2 margin exceeds the fixed id margin of bars().
    Returns the rows that were compared."""
    got_ids = np.asarray(got_ids)
    assert np.array_equal(got_ids, np.argmax(got_logits, axis=-1)), "fused argmax != argmax of own logits"
    _, idm, _ = bars(want_logits, n_layers)
    marg = top2_margin(want_logits)
    ok = marg > idm
    band = (marg > MARGIN) & ~ok
    want = np.argmax(want_logits, axis=-1)
    note("ids", compared=int(ok.sum()), rows=int(ok.size), band=int(band.sum()),
         band_mismatch=int((got_ids != want)[band].sum()))
    assert np.array_equal(got_ids[ok], want[ok]), (got_ids[ok], want[ok])
    assert_band(int(band.sum()), int((got_ids != want)[band].sum()), "argmax ids")
    return ok


class Pair:
    """A HIP context and an oracle holding the same model and prompt."""

    def __init__(self, shape, weights, max_seq, max_block=64, oracle_dtype=np.float64, gpu_weights=None, flags=0,
                 predecode=False):
        self.shape = shape
        self.L = shape.n_layers
        fp8 = weights["l0.wq"].dtype == np.uint8
        if predecode and fp8:
            # The oracle turns e4m3 codes and scales into real values every time it touches a matrix; at full depth
            # that takes longer than the forwards.  Here it does so once, with its own routine, and then runs on the values.
            dec = BlockDiffusionOracle(shape, weights, dtype=oracle_dtype)
            if gpu_weights is None:
                gpu_weights = weights
            weights = {k: (dec._mat(k) if v.dtype == np.uint8 else v) for k, v in weights.items() if not k.endswith(".scale")}
        self.o = BlockDiffusionOracle(shape, weights, dtype=oracle_dtype)
        # (e4m3 contexts too small for the large-M kernels take forwards of up to 32 rows only)
        self.ctx = binding.Context(shape, max_seq=max_seq, max_block=min(max_block, 32) if fp8 and max_seq <= 128 else max_block,
                                   weight_dtype=binding.BD_FP8_E4M3 if fp8 else binding.BD_BF16, flags=flags)
        self.ctx.load_model(gpu_weights if gpu_weights is not None else weights,
                            as_bf16_bits=gpu_weights is None and _is_bf16(weights))
        self.ctx.bd_debug_logits(True)

    def close(self):
        self.ctx.close()

    def prefill(self, emb, ids, oracle_chunk=None):
        self.o.prefill(emb, ids, chunk=oracle_chunk)
        e = torch.from_numpy(emb).cuda() if emb is not None and len(emb) else None
        i = torch.from_numpy(ids).cuda() if ids is not None and len(ids) else None
        self.ctx.bd_prefill(e, i)
        self.ctx.bd_status()
        assert self.ctx.bd_cache_len() == self.o.n

    def carry_is_robust(self):
        """The oracle's carry decides its argmax by more than the fixed id margin."""
        return top2_margin(self.o.carry) > bars(self.o.carry, self.L)[1]

    def check_carry(self):
        """Carry = (argmax id, its softmax probability) of the last causal row, to the fixed bars of bars()."""
        cand, conf = self.ctx.bd_read_carry()
        ocand, oconf = self.o.cand_conf(self.o.carry[None, :])
        E, idm, C = bars(self.o.carry, self.L)
        robust = top2_margin(self.o.carry) > idm
        note("carry", compared=bool(robust), cerr=abs(conf - float(oconf[0])) / float(oconf[0]))
        if robust:
            assert cand == int(ocand[0]), (cand, int(ocand[0]))
        assert abs(conf - float(oconf[0])) <= 2.0 * C * float(oconf[0]) + 1e-7, (conf, float(oconf[0]), C)

    def check_kv(self, pos0, count, frac=2e-2):
        for l in range(self.shape.n_layers):
            k, v = self.ctx.bd_read_kv(l, pos0, count)
            ok, ov = self.o.K[l][pos0:pos0 + count], self.o.V[l][pos0:pos0 + count]
            for g, w, nm in ((k, ok, "K"), (v, ov, "V")):
                g = g.cpu().numpy().astype(np.float64)
                scale = float(np.abs(w).max())
                err = float(np.abs(g - w).max())
                assert err <= frac * scale, f"layer {l} {nm}: err {err:.4g} > {frac} * {scale:.4g}"

    def denoise_step(self, tokens, mask, tau, fixed_k=0, frac=BF16_LOGIT_TOL):
        """One step on both sides from the same (tokens, mask); returns the oracle's new state.
        Compares logits, confidences, revealed set and ids to the fixed bars of bars()."""
        B = len(tokens)
        ot, om = tokens.copy(), mask.copy()
        r = self.o.denoise_step(ot, om, tau, fixed_k)
        gt = torch.from_numpy(tokens.astype(np.int32)).cuda()
        gm = torch.from_numpy(mask.astype(np.uint8)).cuda()
        nun = torch.zeros(1, dtype=torch.int32, device="cuda")
        conf = torch.zeros(B, dtype=torch.float32, device="cuda")
        self.ctx.bd_denoise_step(gt, gm, tau, fixed_k, nun, conf)
        self.ctx.bd_status()
        gtok, gmask = gt.cpu().numpy(), gm.cpu().numpy().astype(bool)
        if r["logits"] is None:
            assert np.array_equal(gtok[~gmask], ot[~om]) and np.array_equal(gmask, om)
            assert int(nun.item()) == r["n_unmasked"]
            return ot, om, r
        glog = self.ctx.bd_read_logits(B).cpu().numpy()
        assert_logits_close(glog, r["logits"], frac, n_layers=self.L)
        E, idm, C = bars(r["logits"], self.L)
        oconf = r["conf"]
        gconf = conf.cpu().numpy()
        cerr = float(np.max(np.abs(gconf - oconf) / np.maximum(oconf, 1e-30)))
        assert cerr <= 2.0 * C, f"confidence relative error {cerr:.4g} > {2 * C:.4g}"
        # (a) integer work: the GPU's revealed set must be exactly what the rule gives on the GPU's own
        #     confidences (both sides decide in the same precision)
        masked = [i for i in range(1, B) if mask[i]]
        sel = _apply_rule(gconf, masked, tau, fixed_k)
        want_mask = mask.copy()
        want_mask[0] = False
        want_mask[sel] = False
        assert np.array_equal(gmask, want_mask), (gmask, want_mask)
        assert int(nun.item()) == int(mask[0]) + len(sel)
        # (b) against the oracle's set, wherever that set is not decided by two confidences closer than 2 C + 1e-3
        cm = np.array([oconf[i] for i in masked])
        tol = 2.0 * C + 1e-3
        unique = True
        srt = np.sort(cm)[::-1]
        if fixed_k > 0:
            k = min(fixed_k, len(masked))
            if k < len(masked) and (srt[k - 1] - srt[k]) < tol * srt[k - 1]:
                unique = False
        else:
            if np.any(np.abs(cm - tau) < tol * max(tau, 1e-6)):
                unique = False
            if not np.any(cm > tau) and len(srt) > 1 and (srt[0] - srt[1]) < tol * srt[0]:
                unique = False
        # ids written at revealed positions: exactly the argmax of the GPU's own logits row i-1
        gam = np.argmax(glog, axis=-1)
        for i in np.flatnonzero(mask & ~gmask):
            if i > 0:
                assert gtok[i] == gam[i - 1], (i, gtok[i], gam[i - 1])
        assert np.array_equal(gtok[~mask], tokens[~mask])          # already revealed positions untouched
        # candidate ids of every row against the oracle's, wherever its margin exceeds the fixed id margin
        marg = top2_margin(r["logits"])
        oam = np.argmax(r["logits"], axis=-1)
        rows_ok = marg > idm
        band = (marg > MARGIN) & ~rows_ok
        assert np.array_equal(gam[rows_ok], oam[rows_ok]), (gam[rows_ok], oam[rows_ok])
        note("step", cerr=cerr, set_compared=bool(unique), set_equal=bool(np.array_equal(gmask, om)),
             id_rows=int(rows_ok.sum()), band=int(band.sum()), band_mismatch=int((gam != oam)[band].sum()), rows=int(B))
        assert_band(int(band.sum()), int((gam != oam)[band].sum()), "candidate ids")
        if unique:
            assert np.array_equal(gmask, om), (gmask, om)
            assert int(nun.item()) == r["n_unmasked"]
            for i in np.flatnonzero(mask & ~om):
                if i == 0:
                    if self.carry_is_robust():
                        assert gtok[0] == ot[0]
                elif rows_ok[i - 1]:
                    assert gtok[i] == ot[i], (i, gtok[i], ot[i])
        return ot, om, r

    def commit(self, tokens, frac=BF16_LOGIT_TOL):
        n0 = self.o.n
        ol = self.o.commit_block(tokens)
        self.ctx.bd_commit_block(torch.from_numpy(np.asarray(tokens, np.int32)).cuda())
        self.ctx.bd_status()
        assert self.ctx.bd_cache_len() == self.o.n == n0 + len(tokens)
        glog = self.ctx.bd_read_logits(len(tokens)).cpu().numpy()
        assert_logits_close(glog, ol, frac, "commit logits", n_layers=self.L)
        self.check_carry()
        return ol


def _apply_rule(conf, masked, tau, fixed_k):
    """The unmask rule on given per-position confidences (integer work once the confidences are fixed)."""
    if not masked:
        return []
    if fixed_k > 0:
        order = sorted(masked, key=lambda i: (-conf[i], i))
        return order[:min(fixed_k, len(order))]
    chosen = [i for i in masked if conf[i] > np.float32(tau)]
    if not chosen:
        chosen = [min(masked, key=lambda i: (-conf[i], i))]
    return chosen


def _is_bf16(weights):
    w = weights["lm_head"]
    return w.dtype == np.float32 and not np.any(w.view(np.uint32) & np.uint32(0xFFFF))


def fresh_block(shape, B):
    return np.full(B, shape.mask_token_id, np.int32), np.ones(B, bool)
