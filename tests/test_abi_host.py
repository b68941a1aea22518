"""CPU-only checks of the C-ABI library: it loads, exports what include/pl.h declares, and its host
logic (slot table, page accounting, version/flip rules, error codes) behaves as the Actor loop of
Alg. 2 requires.  A bookkeeping-only engine (device = PL_DEVICE_NONE) computes no token."""
import os
import re

import numpy as np
import pytest

import paper_2509_19128_amd as pl
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
M = synth.CONFIGS["tiny"]


def _engine(**kw):
    args = dict(max_batch=4, max_context=128, kv_pool_tokens=64 * 8, kv_page_tokens=64, device=pl.PL_DEVICE_NONE, seed=1)
    args.update(kw)
    return pl.Engine.from_model(M, **args)


def _loaded(**kw):
    e = _engine(**kw)
    e.load_weights(np.zeros(e.weight_nbytes() // 2, np.uint16))
    return e


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "pl.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(pl_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(pl.EXPORTS)
    L = pl.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_weight_layout_matches_documented_order_and_size():
    e = _engine()
    lay = e.weight_layout()
    names = [n for n, _, _ in lay]
    assert names[0] == "embed" and names[-2:] == ["gf", "lm_head"]
    assert names[1:7] == ["l0.g1", "l0.w_qkv", "l0.w_o", "l0.g2", "l0.w_gu", "l0.w_d"]
    off = 0
    for _, o, (r, c) in lay:
        assert o == off
        off += r * c
    assert off * 2 == e.weight_nbytes() == 2 * (M.streamed_params() + M.vocab * M.d_model)
    # gate/up interleave and q|k|v row order are pure layout: packing then reading back is a permutation
    W = synth.make_weights(M, 3)
    blob = e.pack_weights(W, synth.f32_to_bf16_bits)
    d = dict((n, (o, s)) for n, o, s in lay)
    def rows(name):      # undo the operand ordering with the element formula of include/pl.h
        o, (r, c) = d[name]
        flat = synth.bf16_bits_to_f32(blob[o:o + r * c])
        rr, cc = np.meshgrid(np.arange(r), np.arange(c), indexing="ij")
        idx = ((cc // 64) * (r // 32) + rr // 32) * 2048 + ((cc % 32) // 8) * 512 + ((cc % 64) // 32) * 256 + (rr % 32) * 8 + cc % 8
        return flat[idx]
    gu = rows("l1.w_gu")
    assert np.array_equal(gu[64:96], synth.bf16_round(W["l1.wg"][32:64]))
    assert np.array_equal(gu[96:128], synth.bf16_round(W["l1.wu"][32:64]))
    qkv = rows("l0.w_qkv")
    assert np.array_equal(qkv[M.q_dim:M.q_dim + M.kv_dim], synth.bf16_round(W["l0.wk"]))
    o, (r, c) = d["embed"]
    assert np.array_equal(synth.bf16_bits_to_f32(blob[o:o + r * c]).reshape(r, c), synth.bf16_round(W["embed"]))


def test_unpack_is_the_inverse_of_pack():
    e = _engine()
    W = synth.make_weights(M, 5)
    U = e.unpack_weights(e.pack_weights(W, synth.f32_to_bf16_bits), synth.bf16_bits_to_f32)
    assert set(U) == set(W)
    for k in W:
        assert np.array_equal(U[k], synth.bf16_round(W[k])), k
    one = e.unpack_weights(e.pack_weights(W, synth.f32_to_bf16_bits), synth.bf16_bits_to_f32, names={"l1.w_gu"})
    assert set(one) == {"l1.wg", "l1.wu"}


@pytest.mark.parametrize("bad", [dict(head_dim=48), dict(n_q_heads=7), dict(d_model=320), dict(vocab=100),
                                 dict(n_kv_heads=0)])
def test_create_rejects_unsupported_shapes(bad):
    m = synth.ModelCfg(**{**M.__dict__, **bad})
    with pytest.raises(pl.PlError) as ex:
        pl.Engine.from_model(m, max_batch=2, max_context=64, kv_pool_tokens=128, device=pl.PL_DEVICE_NONE)
    assert ex.value.code == pl.PL_E_INVAL


def test_error_codes():
    e = _engine()
    with pytest.raises(pl.PlError) as ex:
        e.decode_step()
    assert ex.value.code == pl.PL_E_STATE                      # step before weights
    with pytest.raises(pl.PlError) as ex:
        e.swap_weights(np.zeros(e.weight_nbytes() // 2, np.uint16))
    assert ex.value.code == pl.PL_E_STATE                      # swap before weights
    with pytest.raises(pl.PlError) as ex:
        e.load_weights(np.zeros(10, np.uint16))
    assert ex.value.code == pl.PL_E_INVAL                      # wrong blob size
    e = _loaded()
    assert e.decode_step()["n"] == 0                           # no active slot: an empty step
    for bad in (dict(temperature=0.0), dict(max_new=0), dict(prompt=[]), dict(prompt=[M.vocab])):
        a = dict(seq_id=1, prompt=[1, 2], max_new=4, temperature=1.0)
        a.update(bad)
        with pytest.raises(pl.PlError) as ex:
            e.add_sequence(**a)
        assert ex.value.code == pl.PL_E_INVAL
    with pytest.raises(pl.PlError) as ex:
        e.add_sequence(1, [1] * 100, 30)
    assert ex.value.code == pl.PL_E_CTX                        # 100 + 30 - 1 > 128
    with pytest.raises(pl.PlError) as ex:
        e.retire_sequence(2)
    assert ex.value.code == pl.PL_E_STATE                      # idle slot
    for i in range(4):
        assert e.add_sequence(i, [1, 2, 3], 4) == i
    with pytest.raises(pl.PlError) as ex:
        e.add_sequence(9, [1], 1)
    assert ex.value.code == pl.PL_E_NOSLOT
    e.swap_weights(np.zeros(e.weight_nbytes() // 2, np.uint16), flags=pl.PL_SWAP_ASYNC)
    with pytest.raises(pl.PlError) as ex:
        e.swap_weights(np.zeros(e.weight_nbytes() // 2, np.uint16))
    assert ex.value.code == pl.PL_E_BUSY                       # previous update not active yet
    with pytest.raises(pl.PlError) as ex:
        e.swap_weights(np.zeros(3, np.uint16))
    assert ex.value.code == pl.PL_E_INVAL


def test_kv_pool_exhaustion_leaves_engine_unchanged():
    e = _loaded(kv_pool_tokens=64 * 3, max_context=128)
    e.add_sequence(1, [1] * 60, 60)
    e.add_sequence(2, [1] * 100, 5)                              # two pages
    with pytest.raises(pl.PlError) as ex:
        e.add_sequence(3, [1] * 10, 5)                           # pool is full
    assert ex.value.code == pl.PL_E_NOKV and e.num_active() == 2
    assert e.stats()["kv_pages_free"] == 0
    for _ in range(64):
        e.decode_step()
    with pytest.raises(pl.PlError) as ex:                        # sequence 1 needs a second page now
        e.decode_step()
    assert ex.value.code == pl.PL_E_NOKV
    st = e.stats()
    assert st["steps"] == 64 and e.num_active() == 2
    e.retire_sequence(1)                                         # sequence 2 (slot 1): frees two pages
    assert e.stats()["kv_pages_free"] == 2
    assert e.decode_step()["n"] == 1


def test_life_cycle_refill_and_versions():
    e = _loaded()
    lens = {0: 3, 1: 5, 2: 2, 3: 4, 4: 3, 5: 2}
    nxt, done = 0, {}
    emitted = {}
    for step in range(30):
        while e.num_active() < 4 and nxt < len(lens):
            e.add_sequence(nxt, [1, 2, 3], lens[nxt])
            nxt += 1
        if e.num_active() == 0:
            break
        if nxt < len(lens):
            assert e.num_active() == 4                           # refilled to H before every step
        if step == 4:
            v = e.swap_weights(np.zeros(e.weight_nbytes() // 2, np.uint16), flags=pl.PL_SWAP_WAIT)
            assert v == 1
        r = e.decode_step()
        assert len(set(r["weight_version"].tolist())) == 1       # one version per step
        assert r["weight_version"][0] == (0 if step < 4 else 1)
        for i in range(r["n"]):
            sid = int(r["seq_id"][i])
            assert bool(r["emitted"][i]) == (r["position"][i] >= 2)
            emitted[sid] = emitted.get(sid, 0) + int(r["emitted"][i])
            if r["finished"][i]:
                done[sid] = int(r["position"][i]) + 1
                e.retire_sequence(int(r["slot"][i]))
    assert emitted == lens
    assert done == {k: 3 + v - 1 for k, v in lens.items()}       # n_prompt + max_new - 1 cached positions
    st = e.stats()
    assert st["tokens_emitted"] == sum(lens.values()) and st["swaps"] == 1 and st["active_version"] == 1
    assert st["kv_pages_free"] == st["kv_pages_total"]


def test_forced_tokens_are_reported_and_async_swap_flips_at_a_step_boundary():
    e = _loaded()
    e.add_sequence(1, [5, 6], 3)
    f = np.full(4, -1, np.int32)
    f[0] = 77
    assert e.decode_step(f)["token"][0] == 77
    e.swap_weights(np.zeros(e.weight_nbytes() // 2, np.uint16), flags=pl.PL_SWAP_ASYNC)
    assert e.swap_poll() == (True, 0)                            # staged, not active until a step runs
    assert e.decode_step()["weight_version"][0] == 1
    assert e.swap_poll() == (False, 1)


def test_mid_flight_admission_hook():
    e = _loaded()
    s = e.debug_add_sequence_at(9, None, 16, 64, 1.0, context_len=70, n_emitted=55, last_token=3)
    st = e.stats()
    assert st["kv_pages_total"] - st["kv_pages_free"] == 2       # 70 positions: two 64-token pages
    r = e.decode_step()
    assert r["position"][0] == 70 and r["emitted"][0] == 1
    with pytest.raises(pl.PlError):
        e.debug_add_sequence_at(10, None, 16, 64, 1.0, context_len=5, n_emitted=0, last_token=3)  # prompt needed


def test_batched_prefill_bookkeeping():
    """pl_prefill reads all prompt positions but the last; the next step reads that one and emits."""
    e = _loaded()
    s0 = e.add_sequence(1, [5, 6, 7, 8, 9, 10, 11], 10)
    s1 = e.add_sequence(2, [4], 10)
    assert e.prefill(s0) == 6 and e.prefill(s0) == 0             # nothing left the second time
    assert e.prefill(s1) == 0                                    # a one-token prompt has nothing to prefill
    st = e.stats()
    assert st["prefill_positions"] == 6 and st["prefill_passes"] == 1   # passes hold up to 256 rows
    assert st["steps"] == 0 and st["tokens_emitted"] == 0
    r = e.decode_step()
    assert r["n"] == 2 and r["position"].tolist() == [6, 0] and r["emitted"].tolist() == [1, 1]
    with pytest.raises(pl.PlError) as ex:
        e.prefill(3)                                             # idle slot
    assert ex.value.code == pl.PL_E_STATE
    # a partly read prompt: two steps one token at a time, then the rest in one go
    s2 = e.add_sequence(3, list(range(10, 20)), 2)
    e.decode_step(); e.decode_step()
    assert e.prefill(s2) == 7
    r = e.decode_step()
    i = r["slot"].tolist().index(s2)
    assert r["position"][i] == 9 and r["emitted"][i] == 1


def test_cache_recomputation_bookkeeping():
    e = _loaded()
    s0 = e.add_sequence(1, [5, 6, 7], 10)
    for _ in range(4):
        e.decode_step()
    blob = np.zeros(e.weight_nbytes() // 2, np.uint16)
    e.swap_weights(blob, flags=pl.PL_SWAP_ASYNC | pl.PL_SWAP_RECOMPUTE_KV)
    assert e.stats()["recompute_positions"] == 0                 # nothing happens before the step boundary
    r = e.decode_step()
    assert r["weight_version"][0] == 1 and e.stats()["recompute_positions"] == 4
    s1 = e.debug_add_sequence_at(9, None, 16, 64, 1.0, context_len=20, n_emitted=5, last_token=3)
    with pytest.raises(pl.PlError) as ex:                        # no history for the slot admitted mid-life
        e.swap_weights(blob, flags=pl.PL_SWAP_WAIT | pl.PL_SWAP_RECOMPUTE_KV)
    assert ex.value.code == pl.PL_E_STATE
    with pytest.raises(pl.PlError):
        e.debug_set_history(s1, np.arange(19))                   # must cover exactly the 20 positions read
    e.debug_set_history(s1, np.arange(20))
    e.swap_weights(blob, flags=pl.PL_SWAP_WAIT | pl.PL_SWAP_RECOMPUTE_KV)
    e.decode_step()
    assert e.stats()["recompute_positions"] == 4 + 5 + 20
    with pytest.raises(pl.PlError) as ex:
        e.swap_weights(blob, flags=8)
    assert ex.value.code == pl.PL_E_INVAL


def test_c_helper_packs_the_same_blob_as_the_numpy_permutation():
    """pl_pack_weights (what a C caller uses) against the layout formula of include/pl.h, written out
    independently in Engine.pack_weights and checked element by element in the layout test above."""
    e = _engine()
    W = synth.make_weights(M, 11)
    assert np.array_equal(e.pack_weights_c(W), e.pack_weights(W, synth.f32_to_bf16_bits))
    blob = np.zeros(e.weight_nbytes() // 2, np.uint16)
    bits = synth.f32_to_bf16_bits(W["l1.wd"]).reshape(W["l1.wd"].shape)    # bf16 bit patterns as the source
    L = pl.lib()
    assert L.pl_pack_weights(e._h, b"l1.wd", bits.ctypes.data, 0, blob.ctypes.data) == 0
    d = dict((n, (o, s)) for n, o, s in e.weight_layout())
    o, (r, c) = d["l1.w_d"]
    assert np.array_equal(blob[o:o + r * c], pl.operand_order(bits))
    assert L.pl_pack_weights(e._h, b"l9.wq", bits.ctypes.data, 0, blob.ctypes.data) == pl.PL_E_INVAL
    assert L.pl_pack_weights(e._h, b"l0.wx", bits.ctypes.data, 0, blob.ctypes.data) == pl.PL_E_INVAL


def test_kv_pool_sized_automatically_and_bad_pool_sizes():
    e = _engine(kv_pool_tokens=0, kv_page_tokens=64)              # bookkeeping engine: the most the slots can use
    assert e.stats()["kv_pages_total"] == 4 * 2
    with pytest.raises(pl.PlError) as ex:
        _engine(kv_pool_tokens=-5)
    assert ex.value.code == pl.PL_E_INVAL
    with pytest.raises(pl.PlError) as ex:
        _engine(kv_pool_tokens=10, kv_page_tokens=64)             # less than one page
    assert ex.value.code == pl.PL_E_INVAL


def test_create_rejects_a_weight_matrix_the_gemm_cannot_address():
    """vocab x d_model x 2 bytes >= 2 GiB would wrap the GEMM's 32-bit buffer addressing."""
    big = synth.ModelCfg(1, 8192, 64, 8, 128, 8192, 131072 + 32)
    with pytest.raises(pl.PlError) as ex:
        pl.Engine.from_model(big, max_batch=2, max_context=64, kv_pool_tokens=128, device=pl.PL_DEVICE_NONE)
    assert ex.value.code == pl.PL_E_INVAL and "2 GiB" in str(ex.value)
    ok = synth.ModelCfg(1, 8192, 64, 8, 128, 8192, 131072 - 32)
    pl.Engine.from_model(ok, max_batch=2, max_context=64, kv_pool_tokens=128, device=pl.PL_DEVICE_NONE).close()


def test_odd_batch_sizes_keep_the_step_metadata_aligned():
    """Every per-row array of the step metadata must be aligned for its type at any max_batch."""
    for B in (1, 3, 257, 511):
        e = _loaded(max_batch=B, kv_pool_tokens=64 * B)
        ids = [(1 << 40) + 7 * i for i in range(B)]
        for i in range(B):
            e.add_sequence(ids[i], [1, 2], 2)
        r = e.decode_step()
        assert r["n"] == B and r["seq_id"].tolist() == ids
        e.close()


def test_recomputation_is_refused_at_the_flip_if_a_slot_lost_its_history_meanwhile():
    e = _loaded()
    e.add_sequence(1, [5, 6, 7], 10)
    e.decode_step()
    blob = np.zeros(e.weight_nbytes() // 2, np.uint16)
    e.swap_weights(blob, flags=pl.PL_SWAP_ASYNC | pl.PL_SWAP_RECOMPUTE_KV)
    s1 = e.debug_add_sequence_at(9, None, 16, 64, 1.0, context_len=20, n_emitted=5, last_token=3)   # after the request
    with pytest.raises(pl.PlError) as ex:
        e.decode_step()
    assert ex.value.code == pl.PL_E_STATE
    assert e.swap_poll() == (True, 0) and e.stats()["steps"] == 1    # nothing changed: still staged, old version
    e.debug_set_history(s1, np.arange(20))
    r = e.decode_step()
    assert r["weight_version"].tolist() == [1, 1] and e.stats()["recompute_positions"] == 1 + 20


def test_background_prompt_reading_bookkeeping():
    e = _loaded()
    s0 = e.add_sequence(1, [5, 6, 7, 8, 9, 10, 11], 10)
    s1 = e.add_sequence(2, [4, 5], 3)
    assert e.prefill_async(s0) == 6
    with pytest.raises(pl.PlError) as ex:
        e.prefill_async(s0)
    assert ex.value.code == pl.PL_E_BUSY
    assert e.stats()["prefill_positions"] == 6 and e.stats()["steps"] == 0
    r = e.decode_step()                       # a bookkeeping engine finishes the reading at once
    assert r["n"] == 2 and r["position"].tolist() == [6, 0] and r["emitted"].tolist() == [1, 0]
    s2 = e.add_sequence(3, list(range(10, 30)), 2)
    assert e.prefill_async(s2) == 19
    e.retire_sequence(s2)                     # retiring a slot that is still reading is allowed
    assert e.num_active() == 2
    assert e.prefill_async(s1) == 0           # nothing left to read
    s3 = e.add_sequence(4, list(range(30, 40)), 2)
    assert e.prefill_async(s3) == 9 and e.prefill(s3) == 0      # the blocking call waits for the reading under way
    r = e.decode_step()
    assert s3 in r["slot"].tolist()


def test_fp32_test_build_blob_is_row_major_fp32():
    e = _engine(dtype=pl.PL_F32)
    W = synth.make_weights(M, 13)
    assert e.weight_nbytes() == 4 * (M.streamed_params() + M.vocab * M.d_model)
    blob = e.pack_weights(W, None)
    assert blob.dtype == np.float32
    d = dict((n, (o, s)) for n, o, s in e.weight_layout())
    o, (r, c) = d["l1.w_qkv"]
    assert np.array_equal(blob[o:o + r * c].reshape(r, c), np.concatenate([W["l1.wq"], W["l1.wk"], W["l1.wv"]]))
    o, (r, c) = d["l0.w_gu"]
    assert np.array_equal(blob[o:o + r * c].reshape(r, c), np.concatenate([W["l0.wg"], W["l0.wu"]]))
    o, (r, c) = d["l1.g2"]
    assert np.array_equal(blob[o:o + r], W["l1.g2"])
    e.load_weights(blob)
    e.add_sequence(1, [1, 2, 3], 2)
    assert e.decode_step()["n"] == 1
    with pytest.raises(pl.PlError) as ex:
        _engine(dtype=7)
    assert ex.value.code == pl.PL_E_INVAL


def test_tied_embeddings_blob_has_no_lm_head():
    e = _engine(tie_embeddings=1)
    names = [n for n, _, _ in e.weight_layout()]
    assert names[0] == "embed" and names[-1] == "gf" and "lm_head" not in names
    assert e.weight_nbytes() == 2 * M.streamed_params()          # embedding table in, LM head out: same count
    W = synth.make_weights(M, 17)
    blob = e.pack_weights(W, synth.f32_to_bf16_bits)
    assert blob.size * 2 == e.weight_nbytes()
    assert np.array_equal(e.pack_weights_c(W), blob)
    L = pl.lib()
    assert L.pl_pack_weights(e._h, b"lm_head", blob.ctypes.data, 0, blob.ctypes.data) == pl.PL_E_INVAL
    e.load_weights(blob)
    e.add_sequence(1, [1, 2], 2)
    assert e.decode_step()["n"] == 1


def test_gemm_plan_is_a_function_of_the_largest_row_count_only():
    """The K split an engine fixes for its products (host logic only).  Every slice must be non-empty in units
    of 4 k-steps of 64; the SwiGLU product is split only where the 7B shape leaves 40 of 296 tiles over, and
    then into as many slices as give each of the 256 compute units one."""
    def slices_ok(K, s):
        units = K // 256
        return 1 <= s <= units and (s - 1) * -(-units // s) < units
    # SwiGLU products: 7B at 256 slots, the same at 128 slots, 1.5B, 32B
    assert pl.pl_debug_gemm_plan(256, 2 * 18944, 3584, 1) == (1, 32768, 5, 5 * 256 * (2 * 18944 - 32768))
    assert pl.pl_debug_gemm_plan(200, 2 * 18944, 3584, 1)[:3] == (1, 32768, 5)
    assert pl.pl_debug_gemm_plan(128, 2 * 18944, 3584, 1) == (1, 2 * 18944, 1, 0)
    assert pl.pl_debug_gemm_plan(64, 2 * 8960, 1536, 1) == (1, 2 * 8960, 1, 0)
    assert pl.pl_debug_gemm_plan(256, 2 * 8960, 1536, 1) == (1, 2 * 8960, 1, 0)       # narrower than 128 x 256 tiles
    assert pl.pl_debug_gemm_plan(256, 2 * 16384, 3584, 1) == (1, 2 * 16384, 1, 0)      # exactly one round of tiles
    # plain products: one split count for all columns, never an empty slice
    for M_max in (1, 32, 64, 128, 256, 512):
        for N, K in [(4608, 3584), (3584, 3584), (3584, 18944), (2048, 1536), (1536, 8960), (7168, 5120), (5120, 27648),
                     (152064, 3584)]:
            s, n_main, rs, ws = pl.pl_debug_gemm_plan(M_max, N, K, 0)
            assert n_main == N and rs == 1 and ws == 0 and slices_ok(K, s), (M_max, N, K, s)
    for bad in [(0, 4608, 3584, 0), (513, 4608, 3584, 0), (256, 4608, 3584, 2), (256, 16, 3584, 0)]:
        with pytest.raises(pl.PlError):
            pl.pl_debug_gemm_plan(*bad)
