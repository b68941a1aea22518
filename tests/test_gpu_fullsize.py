"""Full-size parity (GPU): the 7B-shaped engine in exactly the configuration bench.py times (28 layers,
batch 256, 128-token pages, steady-state contexts of thousands of tokens, device-generated weights),
checked on sampled rows the oracle can compute one by one: for a chosen slot the oracle is handed the
slot's cached keys/values (read back from the device pages, all layers) and the same weights (the blob
copied back and un-permuted), computes that slot's logits for the step, and the sampler is replayed on
the engine's logits.  The other 254 rows are checked through properties that hold at any size."""
import os
import sys

import numpy as np
import pytest

import paper_2509_19128_amd as pl
import synth
from oracle import decoder, sampler

from gpu_util import close

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

pytestmark = pytest.mark.gpu


class _Rows:
    """The embedding table restricted to the rows the oracle will look up."""

    def __init__(self, rows):
        self.rows = rows

    def astype(self, dtype, copy=False):
        return self

    def __getitem__(self, tok):
        return self.rows[int(tok)]


class _LazyWeights(dict):
    """Oracle-format weights un-permuted from the engine's blob one layer at a time."""

    def __init__(self, eng, blob, embed_rows):
        super().__init__()
        self.eng, self.blob, self.layer, self.cur = eng, blob, None, {}
        top = eng.unpack_weights(blob, synth.bf16_bits_to_f32, names={"gf", "lm_head"})
        self.fixed = {"gf": top["gf"], "lm_head": top["lm_head"], "embed": _Rows(embed_rows)}

    def __getitem__(self, name):
        if name in self.fixed:
            return self.fixed[name]
        layer = name.split(".")[0]
        if layer != self.layer:
            names = {f"{layer}.{t}" for t in ("g1", "w_qkv", "w_o", "g2", "w_gu", "w_d")}
            self.cur = self.eng.unpack_weights(self.blob, synth.bf16_bits_to_f32, names=names)
            self.layer = layer
        return self.cur[name]


def test_7b_bench_configuration_sampled_rows_against_oracle():
    import torch
    import bench

    spec = dict(bench.WORKLOADS["7b"], pool_tokens=1_300_000)
    m = synth.CONFIGS["7b"]
    B = spec["batch"]
    seed = 1234 + 3
    eng = pl.Engine.from_model(m, max_batch=B, max_context=spec["prompt"] + spec["gmax"],
                               kv_pool_tokens=spec["pool_tokens"], n_weight_buffers=2, seed=seed, device=0)
    blob_d = bench.device_weight_blob(eng, torch, seed=1237)
    torch.cuda.synchronize()
    eng.load_weights(blob_d.data_ptr(), eng.weight_nbytes())
    blob = blob_d.view(torch.int16).cpu().numpy().view(np.uint16)
    del blob_d
    torch.cuda.empty_cache()
    bench.fill_kv_pool(eng, torch, seed=1239)
    wl = bench.Workload(eng, spec, m, seed=seed)
    wl.admit_steady_state()

    first = eng.decode_step()
    n = first["n"]
    assert n == B
    pos1 = first["position"].copy()
    tok1 = first["token"].copy()
    emitted1 = first["emitted"].astype(bool)
    assert np.isfinite(first["logprob"]).all() and (first["logprob"] <= 0).all()
    # rows to check: one generating sequence with a mid-sized context, one with a short one
    gen = np.nonzero(emitted1)[0]
    order = gen[np.argsort(pos1[gen])]
    picks = [int(order[len(order) // 2]), int(order[len(order) // 8])]
    caches = {}
    for r in picks:
        ctx = int(pos1[r]) + 1                      # positions cached after the first step
        c = decoder.Cache(m, np.float32)
        for layer in range(m.n_layers):
            k, v = eng.debug_read_kv(int(first["slot"][r]), layer, ctx)
            c.k[layer], c.v[layer] = k, v
        caches[r] = c

    second = eng.decode_step()
    logits = eng.debug_get_logits(second["n"])
    assert np.array_equal(second["position"], pos1 + 1)
    assert np.isfinite(logits).all()
    # properties at full size, all rows: the recorded log-prob is log-softmax of the row's logits at the
    # drawn token; the draw is the oracle sampler's draw on the same logits (sampled rows)
    ls = sampler.log_softmax(logits)
    for r in range(second["n"]):
        assert abs(ls[r, second["token"][r]] - second["logprob"][r]) <= 1e-4 * max(1.0, abs(second["logprob"][r]))
    for r in list(range(0, B, 37)) + picks:
        tok, _ = sampler.sample_row(logits[r], 1.0, seed, int(second["seq_id"][r]), int(second["position"][r]))
        assert tok == second["token"][r], r

    # sampled rows against the oracle
    embed = eng.unpack_weights(blob, synth.bf16_bits_to_f32, names={"embed"})["embed"]
    rows = {int(tok1[r]): embed[int(tok1[r])].copy() for r in picks}
    del embed
    W = _LazyWeights(eng, blob, rows)
    for r in picks:
        ref = decoder.step(m, W, int(tok1[r]), int(pos1[r]) + 1, caches[r], np.float32)
        err = logits[r] - ref
        rel = float(err.std() / ref.std())
        print(f"row {r}: context {int(pos1[r]) + 1}, logit rms {ref.std():.3f}, error rms {err.std():.4f} ({100 * rel:.2f} %), max {np.abs(err).max():.4f}")
        # 28 layers of bf16 rounding stages (see the one-layer slice test): the per-layer noise of about
        # 0.6 % of the logit scale adds in quadrature over depth
        assert rel <= 0.006 * np.sqrt(m.n_layers) * 1.5, (r, rel)
        scale = max(1.0, float(ref.std()) / 0.32) * np.sqrt(m.n_layers)
        assert close(logits[r], ref, 2e-2 * scale, 1e-2)[0], r
        assert int(np.argmax(logits[r])) in np.argsort(ref)[-5:]
    eng.close()
