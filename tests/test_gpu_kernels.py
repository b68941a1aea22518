"""Kernel-level parity (GPU): the HIP kernels, called through the C ABI, against the CPU oracle on the
same seeded inputs."""
import numpy as np
import pytest
import torch

import paper_2509_19128_amd as pl
import synth
from oracle import decoder, sampler

from gpu_util import close, dev_bf16, to_np

pytestmark = pytest.mark.gpu

# spec tolerance for bf16 results
ATOL, RTOL = 2e-2, 1e-2


def _paged_inputs(rng, ctx, Hq, Hkv, hd, page_tokens, check_rows):
    """Random page pool on the device; rows in `check_rows` get host-known K/V written into their pages."""
    n = len(ctx)
    pages_per_seq = (int(max(ctx)) + page_tokens - 1) // page_tokens
    need = [(int(c) + page_tokens - 1) // page_tokens for c in ctx]
    n_pages = sum(need) + 3
    perm = rng.permutation(n_pages).astype(np.int32)
    table = np.zeros((n, pages_per_seq), np.int32)
    k = 0
    for b in range(n):
        table[b, :need[b]] = perm[k:k + need[b]]
        k += need[b]
    page_elems = Hkv * 2 * page_tokens * hd
    g = torch.Generator(device="cuda").manual_seed(int(rng.integers(1 << 30)))
    pool = torch.randn(n_pages * page_elems, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    known = {}
    for b in check_rows:
        c = int(ctx[b])
        K = synth.bf16_round(rng.standard_normal((c, Hkv, hd)).astype(np.float32))
        V = synth.bf16_round(rng.standard_normal((c, Hkv, hd)).astype(np.float32))
        img = np.zeros(need[b] * page_elems, np.uint16)
        pl.pl_kv_pack_host(img, np.arange(need[b], dtype=np.int32), K, V, 0, Hkv, hd, page_tokens)
        dst = pool.view(torch.int16).view(n_pages, page_elems)
        dst[torch.from_numpy(table[b, :need[b]].astype(np.int64)).cuda()] = torch.from_numpy(
            img.view(np.int16).reshape(need[b], page_elems)).cuda()
        known[b] = (K, V)
    return pool, table, pages_per_seq, known


def _run_attention(q_np, pool, table, ctx, Hq, Hkv, hd, page_tokens, pages_per_seq, max_ctx):
    n = len(ctx)
    q = dev_bf16(q_np)
    out = torch.zeros(n, Hq, hd, device="cuda", dtype=torch.bfloat16)
    ws = torch.empty(max(pl.pl_attention_workspace_bytes(n, Hq, Hkv, hd, max_ctx), 16), device="cuda", dtype=torch.uint8)
    tb = torch.from_numpy(table).cuda()
    cl = torch.from_numpy(np.asarray(ctx, np.int32)).cuda()
    torch.cuda.synchronize()
    pl.pl_attention_decode(q.data_ptr(), pool.data_ptr(), tb.data_ptr(), cl.data_ptr(), out.data_ptr(), ws.data_ptr(),
                           n, Hq, Hkv, hd, page_tokens, pages_per_seq, max_ctx, 0)
    torch.cuda.synchronize()
    return to_np(out)


@pytest.mark.parametrize("Hq,Hkv,hd,page_tokens", [(28, 4, 128, 64), (8, 2, 32, 64), (12, 2, 128, 32),
                                                    (40, 8, 128, 128), (16, 1, 64, 64)])
def test_attention_matches_oracle_on_ragged_contexts(Hq, Hkv, hd, page_tokens):
    rng = np.random.default_rng(hd + Hq)
    ctx = np.array([1, 31, 32, 33, 64, 127, 129, 700, 1500, 0, 5], np.int32)   # a zero-length row is skipped
    pool, table, pps, known = _paged_inputs(rng, np.maximum(ctx, 1), Hq, Hkv, hd, page_tokens, range(len(ctx)))
    q = synth.bf16_round(rng.standard_normal((len(ctx), Hq, hd)).astype(np.float32))
    got = _run_attention(q, pool, table, ctx, Hq, Hkv, hd, page_tokens, pps, int(ctx.max()))
    for b, c in enumerate(ctx):
        if c == 0:
            assert np.all(got[b] == 0)
            continue
        K, V = known[b]
        ref = decoder.attend_one(q[b].astype(np.float64), K[:c].astype(np.float64), V[:c].astype(np.float64))
        ok, err = close(got[b], ref, ATOL, RTOL)
        assert ok, (b, c, err)


def test_attention_closed_forms_on_device():
    """q = 0 gives the mean of V; one cached token gives its value."""
    rng = np.random.default_rng(5)
    Hq, Hkv, hd, pt = 28, 4, 128, 64
    ctx = np.array([300, 1], np.int32)
    pool, table, pps, known = _paged_inputs(rng, ctx, Hq, Hkv, hd, pt, [0, 1])
    q = synth.bf16_round(rng.standard_normal((2, Hq, hd)).astype(np.float32))
    q[0] = 0
    got = _run_attention(q, pool, table, ctx, Hq, Hkv, hd, pt, pps, 300)
    for h in range(Hq):
        assert close(got[0, h], known[0][1][:, h // 7].mean(0), ATOL, RTOL)[0]
        assert close(got[1, h], known[1][1][0, h // 7], 1e-6, 4e-3)[0]


def test_attention_full_microbench_shape_on_sampled_rows():
    """The launch shape of the attention microbenchmark (batch 512, 28 q / 4 kv heads, head_dim 128,
    log-normal contexts clipped to [128, 16384]); 12 sampled rows, shortest and longest included, are
    checked against the oracle, the others only for being finite."""
    rng = np.random.default_rng(1236)
    Hq, Hkv, hd, pt = 28, 4, 128, 64
    ctx = synth.attention_microbench_lengths(1236).astype(np.int32)
    rows = sorted(set([int(ctx.argmin()), int(ctx.argmax())] + rng.choice(512, 10, replace=False).tolist()))
    pool, table, pps, known = _paged_inputs(rng, ctx, Hq, Hkv, hd, pt, rows)
    q = synth.bf16_round(rng.standard_normal((512, Hq, hd)).astype(np.float32))
    got = _run_attention(q, pool, table, ctx, Hq, Hkv, hd, pt, pps, 16384)
    assert np.isfinite(got).all()
    for b in rows:
        K, V = known[b]
        ref = decoder.attend_one(q[b].astype(np.float64), K.astype(np.float64), V.astype(np.float64))
        ok, err = close(got[b], ref, ATOL, RTOL)
        assert ok, (b, int(ctx[b]), err)


def test_attention_chunk_boundaries_in_the_benchmark_launch_shape():
    """Batch 256, 28 q / 4 kv heads, head_dim 128, 128-token pages, contexts up to 512 + 16384: the launch
    shape of the 7B benchmark, where one workgroup handles up to 8192 tokens.  Contexts on both sides of
    one and two full chunks, and the maximum, against the oracle; the merge of two and three chunks is on
    the path of the last five."""
    rng = np.random.default_rng(99)
    Hq, Hkv, hd, pt = 28, 4, 128, 128
    edges = [8191, 8192, 8193, 16383, 16384, 16385, 16896, 1, 128, 129]
    ctx = np.concatenate([edges, rng.integers(200, 3000, 256 - len(edges))]).astype(np.int32)
    rows = list(range(len(edges)))
    pool, table, pps, known = _paged_inputs(rng, ctx, Hq, Hkv, hd, pt, rows)
    q = synth.bf16_round(rng.standard_normal((256, Hq, hd)).astype(np.float32))
    got = _run_attention(q, pool, table, ctx, Hq, Hkv, hd, pt, pps, 16896)
    assert np.isfinite(got).all()
    for b in rows:
        K, V = known[b]
        ref = decoder.attend_one(q[b].astype(np.float64), K.astype(np.float64), V.astype(np.float64))
        ok, err = close(got[b], ref, ATOL, RTOL)
        assert ok, (b, int(ctx[b]), err)


def test_attention_of_a_sequence_does_not_depend_on_its_neighbours():
    """The chunk length is a function of the launch shape only, and the merge order is fixed: the same
    sequence gives bit-identical output whatever the other rows' contexts are and wherever it sits in
    the work list (which is sorted by length)."""
    rng = np.random.default_rng(321)
    Hq, Hkv, hd, pt, n = 28, 4, 128, 128, 64
    ctx_a = rng.integers(100, 12000, n).astype(np.int32)
    ctx_b = rng.integers(100, 12000, n).astype(np.int32)
    keep = [3, 17, 40]
    ctx_a[keep] = ctx_b[keep] = [9000, 700, 16896]
    both = np.maximum(ctx_a, ctx_b)
    pool, table, pps, _ = _paged_inputs(rng, both, Hq, Hkv, hd, pt, [])
    q = synth.bf16_round(rng.standard_normal((n, Hq, hd)).astype(np.float32))
    out_a = _run_attention(q, pool, table, ctx_a, Hq, Hkv, hd, pt, pps, 16896)
    out_b = _run_attention(q, pool, table, ctx_b, Hq, Hkv, hd, pt, pps, 16896)
    for b in keep:
        assert np.array_equal(out_a[b], out_b[b]), b
    assert not np.array_equal(out_a[0], out_b[0])        # the other rows did change


def test_attention_rejects_bad_arguments():
    t = torch.zeros(1 << 16, device="cuda", dtype=torch.bfloat16)
    p = t.data_ptr()
    good = dict(n=2, Hq=8, Hkv=2, hd=32, pt=32, pps=4, mx=128)
    for bad in [dict(Hq=7), dict(hd=48), dict(pt=48), dict(pt=16), dict(mx=129), dict(mx=0), dict(n=0), dict(n=2000), dict(Hq=40, Hkv=2)]:
        a = dict(good, **bad)
        with pytest.raises(pl.PlError) as ex:
            pl.pl_attention_decode(p, p, p, p, p, p, a["n"], a["Hq"], a["Hkv"], a["hd"], a["pt"], a["pps"], a["mx"], 0)
        assert ex.value.code == pl.PL_E_INVAL, bad
    with pytest.raises(pl.PlError):
        pl.pl_attention_decode(0, p, p, p, p, p, 2, 8, 2, 32, 32, 4, 128, 0)
    assert pl.pl_attention_workspace_bytes(0, 8, 2, 32, 128) == 0


GEMM_SHAPES = [(4, 384, 256, 1), (4, 4096, 1024, 4), (3, 256, 1024, 2), (33, 320, 256, 1), (64, 2048, 1536, 3),
               (130, 1536, 8960, 7), (256, 4608, 3584, 7), (200, 3584, 18944, 8), (256, 3584, 18944, 9), (256, 2560, 3584, 1),
               (300, 640, 512, 2), (256, 33792, 256, 1), (130, 34000 // 32 * 32, 256, 1),
               (256, 43552, 256, 1), (129, 32768, 512, 1), (200, 3584, 3584, 4), (256, 2048, 1536, 3)]   # the last four take the paired 128 x 256 tiles


@pytest.mark.parametrize("M,N,K,splits", GEMM_SHAPES)
def test_gemm_partials_sum_to_the_product(M, N, K, splits):
    rng = np.random.default_rng(M * 7 + N)
    x = synth.bf16_round(rng.standard_normal((M, K)).astype(np.float32))
    w = synth.bf16_round((rng.standard_normal((N, K)) * 0.05).astype(np.float32))
    xd, wd = dev_bf16(x), dev_bf16(pl.operand_order(w))
    y = torch.full((splits, M, N), float("nan"), device="cuda", dtype=torch.float32)
    pl.pl_gemm_bf16(xd.data_ptr(), wd.data_ptr(), y.data_ptr(), M, N, K, 0, splits, 0)
    torch.cuda.synchronize()
    got = to_np(y).astype(np.float64).sum(0)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    ok, err = close(got, ref, 1e-4 * np.sqrt(K) * 0.05, 1e-4)      # fp32 accumulation of exact bf16 products
    assert ok, err


@pytest.mark.parametrize("M,F,K", [(4, 1024, 256), (64, 2240, 1536), (256, 1280, 3584), (129, 320, 512), (200, 16640, 256),
                                   (200, 18944, 256)])
def test_gemm_swiglu_epilogue(M, F, K):
    rng = np.random.default_rng(F + M)
    x = synth.bf16_round(rng.standard_normal((M, K)).astype(np.float32))
    wg = synth.bf16_round((rng.standard_normal((F, K)) * 0.05).astype(np.float32))
    wu = synth.bf16_round((rng.standard_normal((F, K)) * 0.05).astype(np.float32))
    inter = np.stack([wg.reshape(F // 32, 32, K), wu.reshape(F // 32, 32, K)], axis=1).reshape(2 * F, K)
    y = torch.full((M, F), float("nan"), device="cuda", dtype=torch.bfloat16)
    xd, wd = dev_bf16(x), dev_bf16(pl.operand_order(inter))          # keep the device tensors alive across the launch
    pl.pl_gemm_bf16(xd.data_ptr(), wd.data_ptr(), y.data_ptr(), M, 2 * F, K, 1, 1, 0)
    torch.cuda.synchronize()
    x64 = x.astype(np.float64)
    ref = decoder.silu(x64 @ wg.astype(np.float64).T) * (x64 @ wu.astype(np.float64).T)
    ok, err = close(to_np(y), ref, 2e-3, RTOL)
    assert ok, err


CFG_TILES = {0: (32, 256), 1: (64, 256), 2: (128, 256), 3: (64, 128), 4: (128, 128), 5: (256, 128), 6: (64, 64),
             7: (128, 64), 8: (32, 128), 9: (128, 64), 10: (256, 64)}


@pytest.mark.parametrize("cfg", sorted(CFG_TILES))
def test_every_gemm_tile_configuration_against_fp64(cfg):
    """Each tile configuration of the kernel on shapes with several row tiles, a ragged last row tile,
    a column range that starts and ends inside the matrix, with and without a K split; the SwiGLU
    product also with its K split (partials + reduction)."""
    rows, cols = CFG_TILES[cfg]
    rng = np.random.default_rng(100 + cfg)
    M, N, K = min(2 * rows + 7, 300), 5 * 128, 768
    x = synth.bf16_round(rng.standard_normal((M, K), dtype=np.float32))
    w = synth.bf16_round(rng.standard_normal((N, K), dtype=np.float32) * 0.05)
    xd, wd = dev_bf16(x), dev_bf16(pl.operand_order(w))
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    for splits, nb, ne, paired in [(1, 0, N, False), (3, 128, N - 64, False), (1, 64, N, True)]:
        y = torch.full((splits, M, N), float("nan"), device="cuda", dtype=torch.float32)
        pl.pl_debug_gemm_cfg(cfg, xd.data_ptr(), wd.data_ptr(), y.data_ptr(), 0, M, N, K, 0, splits, nb, ne, paired, 0)
        torch.cuda.synchronize()
        got = to_np(y)
        assert np.isnan(got[:, :, :nb]).all() and np.isnan(got[:, :, ne:]).all()       # nothing outside the range
        tol = 1e-4 * (np.sqrt(K) * 0.05 + np.abs(ref[:, nb:ne]))
        assert (np.abs(got[:, :, nb:ne].astype(np.float64).sum(0) - ref[:, nb:ne]) <= tol).all(), (splits, nb, ne)
    if cfg in (6, 7, 8):                              # one 32-column tile per wavefront: no gate/up pair
        with pytest.raises(pl.PlError):
            pl.pl_debug_gemm_cfg(cfg, xd.data_ptr(), wd.data_ptr(), xd.data_ptr(), 0, M, N, K, 1, 1, 0, N, False, 0)
        return
    F = N // 2
    gate = ref.reshape(M, N // 64, 2, 32)[:, :, 0].reshape(M, F)
    up = ref.reshape(M, N // 64, 2, 32)[:, :, 1].reshape(M, F)
    want = gate / (1.0 + np.exp(-gate)) * up
    for splits, nb, ne in [(1, 0, N), (3, 0, N), (2, 128, N - 64)]:
        mid = torch.full((M, F), float("nan"), device="cuda", dtype=torch.bfloat16)
        ws = torch.empty(splits * M * (ne - nb), device="cuda", dtype=torch.float32)
        pl.pl_debug_gemm_cfg(cfg, xd.data_ptr(), wd.data_ptr(), mid.data_ptr(), ws.data_ptr(), M, N, K, 1, splits, nb, ne, False, 0)
        torch.cuda.synchronize()
        got = to_np(mid)
        assert np.isnan(got[:, :nb // 2]).all() and np.isnan(got[:, ne // 2:]).all()
        ok, err = close(got[:, nb // 2:ne // 2], want[:, nb // 2:ne // 2], 2e-3, RTOL)
        assert ok, (splits, nb, ne, err)


@pytest.mark.parametrize("F,K", [(18944, 3584), (18976, 768)])
def test_swiglu_product_of_a_256_row_engine_is_the_same_for_every_row_count(F, K):
    """An engine of 256 slots at a wide SwiGLU product: passes of 129..256 rows take the launch that gives every
    compute unit a main tile and a K slice of the leftover columns, narrower passes separate launches with
    the same slices.  Every row count against fp64, and the rows of a narrower pass bit-equal to the same
    rows of the widest one.  The second shape ends in a ragged column tile."""
    N, M_max = 2 * F, 256
    splits, n_main, rem_splits, ws_elems = pl.pl_debug_gemm_plan(M_max, N, K, 1)
    assert splits == 1 and 0 < n_main < N and rem_splits > 1 and ws_elems == rem_splits * M_max * (N - n_main)
    rng = np.random.default_rng(F + K)
    x = synth.bf16_round(rng.standard_normal((M_max, K), dtype=np.float32))
    w = synth.bf16_round(rng.standard_normal((N, K), dtype=np.float32) * 0.05)
    xd, wd = dev_bf16(x), dev_bf16(pl.operand_order(w))
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    gate = ref.reshape(M_max, N // 64, 2, 32)[:, :, 0].reshape(M_max, F)
    up = ref.reshape(M_max, N // 64, 2, 32)[:, :, 1].reshape(M_max, F)
    want = gate / (1.0 + np.exp(-gate)) * up
    ws = torch.empty(ws_elems, device="cuda", dtype=torch.float32)
    widest = None
    for M in (256, 255, 200, 129, 128, 65, 64, 20, 1):
        mid = torch.full((M, F), float("nan"), device="cuda", dtype=torch.bfloat16)
        ws.fill_(float("nan"))
        pl.pl_debug_gemm_planned(xd.data_ptr(), wd.data_ptr(), mid.data_ptr(), ws.data_ptr(), M_max, M, N, K, 1, 0)
        torch.cuda.synchronize()
        got = to_np(mid)
        ok, err = close(got, want[:M], 2e-3, RTOL)
        assert ok, (M, err)
        if widest is None:
            widest = got
        else:
            assert np.array_equal(got, widest[:M]), M
    with pytest.raises(pl.PlError):
        pl.pl_debug_gemm_planned(xd.data_ptr(), wd.data_ptr(), mid.data_ptr(), 0, M_max, 200, N, K, 1, 0)


@pytest.mark.parametrize("M_max,N,K", [(256, 4608, 3584), (256, 3584, 18944), (64, 2048, 1536), (128, 7168, 5120)])
def test_plain_products_of_an_engine_are_the_same_for_every_row_count(M_max, N, K):
    """QKV- and down-shaped products as an engine of M_max slots launches them: the tile shape follows the rows
    of the call, the K split is fixed, so every slice of the partial sums of a narrow pass is bit-equal to the
    same rows of the widest pass; their sum is the product."""
    splits, n_main, rem_splits, ws_elems = pl.pl_debug_gemm_plan(M_max, N, K, 0)
    assert n_main == N and ws_elems == 0
    rng = np.random.default_rng(N + K)
    x = synth.bf16_round(rng.standard_normal((M_max, K), dtype=np.float32))
    w = synth.bf16_round(rng.standard_normal((N, K), dtype=np.float32) * 0.05)
    xd, wd = dev_bf16(x), dev_bf16(pl.operand_order(w))
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    widest = None
    for M in sorted({M_max, M_max - 1, 200, 129, 128, 65, 64, 33, 32, 5, 1}, reverse=True):
        if M > M_max:
            continue
        y = torch.full((splits, M, N), float("nan"), device="cuda", dtype=torch.float32)
        pl.pl_debug_gemm_planned(xd.data_ptr(), wd.data_ptr(), y.data_ptr(), 0, M_max, M, N, K, 0, 0)
        torch.cuda.synchronize()
        got = to_np(y)
        if widest is None:
            widest = got
            ok, err = close(got.astype(np.float64).sum(0), ref, 1e-4 * np.sqrt(K) * 0.05, 1e-4)
            assert ok, err
        else:
            assert np.array_equal(got, widest[:, :M]), M


def test_gemm_rejects_bad_shapes():
    t = torch.zeros(600 * 512, device="cuda", dtype=torch.bfloat16)
    for args in [(4, 64, 192, 0, 1), (0, 64, 256, 0, 1), (4, 64, 512, 0, 3), (4, 96, 256, 1, 1), (4, 64, 512, 1, 2),
                 (4, 64, 256, 2, 1), (600, 64, 256, 0, 1), (4, 48, 256, 0, 1)]:
        with pytest.raises(pl.PlError) as ex:
            pl.pl_gemm_bf16(t.data_ptr(), t.data_ptr(), t.data_ptr(), args[0], args[1], args[2], args[3], args[4], 0)
        assert ex.value.code == pl.PL_E_INVAL


def _gpu_sample(logits, seq_id, pos, temps, forced, seed):
    n, V = logits.shape
    lg = torch.from_numpy(logits).cuda()
    sid = torch.from_numpy(np.asarray(seq_id, np.uint64).view(np.int64)).cuda()
    ps = torch.from_numpy(np.asarray(pos, np.int32)).cuda()
    it = torch.from_numpy((np.float32(1.0) / np.asarray(temps, np.float32)).astype(np.float32)).cuda()
    fr = torch.from_numpy(np.asarray(forced, np.int32)).cuda()
    tok = torch.zeros(n, device="cuda", dtype=torch.int32)
    lp = torch.zeros(n, device="cuda", dtype=torch.float32)
    ws = torch.empty(pl.pl_sample_workspace_bytes(n, V), device="cuda", dtype=torch.uint8)
    pl.pl_sample(lg.data_ptr(), n, V, sid.data_ptr(), ps.data_ptr(), it.data_ptr(), fr.data_ptr(), seed,
                 tok.data_ptr(), lp.data_ptr(), ws.data_ptr(), 0)
    torch.cuda.synchronize()
    return tok.cpu().numpy(), lp.cpu().numpy()


@pytest.mark.parametrize("n,V", [(7, 4096), (4, 152064), (3, 151936), (5, 8)])
def test_sampler_tokens_bit_exact_and_logprobs_close(n, V):
    rng = np.random.default_rng(V + n)
    logits = (rng.standard_normal((n, V)) * 2).astype(np.float32)
    seq_id = rng.integers(0, 2**63, size=n, dtype=np.uint64) * np.uint64(2) + np.uint64(1)
    pos = rng.integers(0, 16384, size=n).astype(np.int32)
    temps = np.array([1.0, 0.7, 1.3, 1.0, 0.5, 2.0, 1.0][:n], np.float32)
    forced = np.full(n, -1, np.int32)
    forced[n - 1] = V // 3
    seed = 0x1234567890ABCDEF
    tok, lp = _gpu_sample(logits, seq_id, pos, temps, forced, seed)
    for r in range(n):
        t_ref, lp_ref = sampler.sample_row(logits[r], float(temps[r]), seed, int(seq_id[r]), int(pos[r]), int(forced[r]))
        assert tok[r] == t_ref, (r, tok[r], t_ref)
        assert abs(lp[r] - lp_ref) <= 1e-4 * max(1.0, abs(lp_ref))


def test_sampler_ties_resolve_to_the_lowest_index_like_the_oracle():
    """Constant logits: the winner is decided by the noise alone, and with 2^23 distinct uniforms over
    152064 entries equal maxima do occur; both sides must pick the lowest index."""
    n, V = 96, 152064
    logits = np.zeros((n, V), np.float32)
    seq_id = np.arange(n, dtype=np.uint64) + np.uint64(1 << 33)
    pos = np.arange(n, dtype=np.int32) * 3
    tok, lp = _gpu_sample(logits, seq_id, pos, np.ones(n, np.float32), np.full(n, -1, np.int32), 42)
    ties = 0
    for r in range(n):
        g = sampler.gumbel_from_bits(__import__("oracle.philox", fromlist=["x"]).sampler_bits(42, int(seq_id[r]), int(pos[r]), V))
        ties += int((g == g.max()).sum() > 1)
        assert tok[r] == int(np.argmax(g))
        assert abs(lp[r] + np.log(V)) < 1e-4
    print("rows with tied maxima:", ties)
