"""Helpers of the GPU parity tests: run the HIP path and the oracle side by side on the same seeded inputs."""
import numpy as np
import torch

from oracle.bd_oracle import BlockDiffusionOracle
from paper_2604_06832_amd import binding, inputs

BF16_LOGIT_TOL = 3e-2      # max-abs logit error as a fraction of the oracle's logit range (bf16 path)
MARGIN = 1e-2              # ids are compared where the oracle's top-2 logit margin exceeds this


def top2_margin(logits):
    part = np.partition(logits, -2, axis=-1)
    return part[..., -1] - part[..., -2]


def assert_logits_close(got, want, frac=BF16_LOGIT_TOL, what="logits"):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    rng = float(want.max() - want.min())
    err = float(np.abs(got - want).max())
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    assert err <= frac * rng, f"{what}: max-abs error {err:.4g} > {frac} * range {rng:.4g}"
    return err / rng


class Pair:
    """A HIP context and an oracle holding the same model and prompt."""

    def __init__(self, shape, weights, max_seq, max_block=64, oracle_dtype=np.float64, gpu_weights=None):
        self.shape = shape
        self.o = BlockDiffusionOracle(shape, weights, dtype=oracle_dtype)
        self.ctx = binding.Context(shape, max_seq=max_seq, max_block=max_block)
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
        torch.cuda.synchronize()
        assert self.ctx.bd_cache_len() == self.o.n

    def check_carry(self):
        cand, conf = self.ctx.bd_read_carry()
        ocand, oconf = self.o.cand_conf(self.o.carry[None, :])
        if top2_margin(self.o.carry) > MARGIN:
            assert cand == int(ocand[0]), (cand, int(ocand[0]))
        assert abs(conf - float(oconf[0])) <= 0.05 * float(oconf[0]) + 1e-6

    def check_kv(self, pos0, count, frac=2e-2):
        for l in range(self.shape.n_layers):
            k, v = self.ctx.bd_read_kv(l, pos0, count)
            ok, ov = self.o.K[l][pos0:pos0 + count], self.o.V[l][pos0:pos0 + count]
            for g, w, nm in ((k, ok, "K"), (v, ov, "V")):
                g = g.cpu().numpy().astype(np.float64)
                scale = float(np.abs(w).max())
                err = float(np.abs(g - w).max())
                assert err <= frac * scale, f"layer {l} {nm}: err {err:.4g} > {frac} * {scale:.4g}"

    def denoise_step(self, tokens, mask, tau, fixed_k=0, frac=BF16_LOGIT_TOL, rank_tol=1e-3):
        """One step on both sides from the same (tokens, mask); returns the oracle's new state.
        Compares logits, confidences, revealed set and ids, with the near-tie exemptions."""
        B = len(tokens)
        ot, om = tokens.copy(), mask.copy()
        r = self.o.denoise_step(ot, om, tau, fixed_k)
        gt = torch.from_numpy(tokens.astype(np.int32)).cuda()
        gm = torch.from_numpy(mask.astype(np.uint8)).cuda()
        nun = torch.zeros(1, dtype=torch.int32, device="cuda")
        conf = torch.zeros(B, dtype=torch.float32, device="cuda")
        self.ctx.bd_denoise_step(gt, gm, tau, fixed_k, nun, conf)
        torch.cuda.synchronize()
        gtok, gmask = gt.cpu().numpy(), gm.cpu().numpy().astype(bool)
        if r["logits"] is None:
            assert np.array_equal(gtok[~gmask], ot[~om]) and np.array_equal(gmask, om)
            assert int(nun.item()) == r["n_unmasked"]
            return ot, om, r
        glog = self.ctx.bd_read_logits(B).cpu().numpy()
        assert_logits_close(glog, r["logits"], frac)
        oconf = r["conf"]
        gconf = conf.cpu().numpy()
        np.testing.assert_allclose(gconf, oconf, rtol=0.08, atol=1e-7)
        # is the revealed set uniquely determined?  (near-ties in the confidence ranking / at the threshold)
        masked = [i for i in range(1, B) if mask[i]]
        cm = np.array([oconf[i] for i in masked])
        unique = True
        if fixed_k > 0:
            k = min(fixed_k, len(masked))
            srt = np.sort(cm)[::-1]
            if k < len(masked) and (srt[k - 1] - srt[k]) < rank_tol * srt[k - 1]:
                unique = False
        else:
            if np.any(np.abs(cm - tau) < rank_tol * max(tau, 1e-6)):
                unique = False
            srt = np.sort(cm)[::-1]
            if not np.any(cm > tau) and len(srt) > 1 and (srt[0] - srt[1]) < rank_tol * srt[0]:
                unique = False
        if unique:
            assert np.array_equal(gmask, om), (gmask, om)
            assert int(nun.item()) == r["n_unmasked"]
            marg = top2_margin(r["logits"])
            for i in np.flatnonzero(mask & ~om):
                if i == 0:
                    if top2_margin(self.o.carry) > MARGIN:
                        assert gtok[0] == ot[0]
                elif marg[i - 1] > MARGIN:
                    assert gtok[i] == ot[i], (i, gtok[i], ot[i])
        else:
            assert int(nun.item()) == r["n_unmasked"]
        return ot, om, r

    def commit(self, tokens, frac=BF16_LOGIT_TOL):
        n0 = self.o.n
        ol = self.o.commit_block(tokens)
        self.ctx.bd_commit_block(torch.from_numpy(np.asarray(tokens, np.int32)).cuda())
        torch.cuda.synchronize()
        assert self.ctx.bd_cache_len() == self.o.n == n0 + len(tokens)
        glog = self.ctx.bd_read_logits(len(tokens)).cpu().numpy()
        assert_logits_close(glog, ol, frac, "commit logits")
        self.check_carry()
        return ol


def _is_bf16(weights):
    w = weights["l0.wq"]
    return w.dtype == np.float32 and not np.any(w.view(np.uint32) & np.uint32(0xFFFF))


def fresh_block(shape, B):
    return np.full(B, shape.mask_token_id, np.int32), np.ones(B, bool)
