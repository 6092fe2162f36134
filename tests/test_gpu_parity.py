"""GPU parity: every entry point of the C-ABI library against the CPU oracle on the same seeded inputs.
Indexing results must match bit for bit; products within the stated relative error
(1e-4 fp32, 1e-2 bf16 inputs with fp32 accumulation), Frobenius-norm and max-norm."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import parse_oracle as po

pytestmark = pytest.mark.gpu

pa = pytest.importorskip("paper_2605_08568_amd")
from helpers import (check_guards, decode_multi_guarded, forward_guarded, guarded_bytes, i32, mfma16_u, mfma16_v, oracle_factors,  # noqa: E402
                     prefill_multi_guarded, upload_layer, upload_tokens)

TOL_F32, TOL_BF16 = 1e-4, 1e-2
DEV = "cuda"


def say(msg):
    print(msg, flush=True)


def assert_close(Y, Yref, tol, what):
    fro, mx = po.rel_errors(Y, Yref)
    say(f"    {what}: fro {fro:.2e} max {mx:.2e} (tol {tol:g})")
    assert fro <= tol and mx <= tol, (what, fro, mx)


# ------------------------------------------------------------------ a1 + a2 route
@pytest.mark.parametrize("dtype,lengths,d,G,k", [
    ("f32", [64, 64, 64, 64], 1024, 8, 4),
    ("bf16", [1, 7, 300, 33, 2], 512, 16, 8),
    ("f32", [1] * 9, 264, 20, 10),
    ("bf16", [513, 40], 4096, 64, 1),
    ("f32", [5, 90, 2], 16384, 12, 4),          # the largest model width the router accepts (more than 64 KiB of LDS)
])
def test_route_matches_oracle(dtype, lengths, d, G, k):
    say(f"route dtype={dtype} lengths={lengths} d={d} G={G} k={k}")
    rng = np.random.default_rng(101)
    off = si.offsets_from_lengths(lengths)
    X = si.make_tokens(rng, int(off[-1]), d, dtype)
    Wr = si.make_router(rng, 1, G, d)[0]
    Xv = si.bf16_bits_to_f32(X).astype(np.float64) if dtype == "bf16" else X.astype(np.float64)
    E = po.pool(Xv, off)
    ref, margin = po.route(E, Wr, k)
    S = po.route_scores(E, Wr)
    assert np.all(margin > 1e-4 * np.abs(S).max()), "re-seed: a top-k decision is within rounding"
    P = len(lengths)
    scores = torch.empty((P, G), dtype=torch.float32, device=DEV)
    emb = torch.empty((P, d), dtype=torch.float32, device=DEV)
    sub = pa.route(upload_tokens(X, dtype), i32(off), torch.from_numpy(Wr).to(DEV), k, scores_out=scores, emb_out=emb)
    torch.cuda.synchronize()
    assert np.array_equal(sub.cpu().numpy(), ref)
    assert np.allclose(emb.cpu().numpy(), E, rtol=1e-5, atol=1e-6)
    assert np.allclose(scores.cpu().numpy(), S, rtol=1e-4, atol=1e-5)
    # the embedding-only call: same bits as the router call's embedding, output between guard bands
    whole, mid = guarded_bytes(P * d * 4)
    emb2 = pa.pool(upload_tokens(X, dtype), i32(off), emb_out=mid[:P * d * 4].view(torch.float32).view(P, d))
    check_guards(whole, "pool")
    assert torch.equal(emb2, emb) and bool(torch.all(mid[P * d * 4:] == 0xA5))


def test_route_strided_output_and_determinism():
    say("route strided output / repeatability")
    rng = np.random.default_rng(102)
    off = si.offsets_from_lengths([50, 3, 120])
    X = si.make_tokens(rng, int(off[-1]), 256, "bf16")
    Wr = si.make_router(rng, 1, 12, 256)[0]
    ref, _ = po.route(po.pool(si.bf16_bits_to_f32(X).astype(np.float64), off), Wr, 5)
    out = torch.full((3, 3, 5), -7, dtype=torch.int32, device=DEV)
    Xd, offd, Wd = upload_tokens(X, "bf16"), i32(off), torch.from_numpy(Wr).to(DEV)
    pa.route(Xd, offd, Wd, 5, subset_out=out[:, 1, :], subset_stride=15)
    e1 = torch.empty((3, 256), dtype=torch.float32, device=DEV); e2 = torch.empty_like(e1)
    pa.route(Xd, offd, Wd, 5, emb_out=e1); pa.route(Xd, offd, Wd, 5, emb_out=e2)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.array_equal(o[:, 1, :], ref) and np.all(o[:, 0, :] == -7) and np.all(o[:, 2, :] == -7)
    assert torch.equal(e1, e2)


# ------------------------------------------------------------------ a3 cache
def _cache_inputs(P, d, L, G, nclus, seed):
    rng = np.random.default_rng(seed)
    E, cid = si.clustered_embeddings(rng, P, d, nclus, 0.1)
    Wr = si.make_router(rng, L, G, d)
    return E, cid, Wr


def _check_cache_batch(cache, oc, E, tau, Wr):
    e_ref, h_ref, s_ref, sims_ref, rmargin = oc.lookup_or_route(E, tau, Wr, return_detail=True)
    # decisions must not sit within rounding of the threshold or of a router tie
    finite = np.isfinite(sims_ref)
    assert np.all(np.abs(sims_ref[finite] - tau) > 1e-3), "re-seed: similarity within rounding of tau"
    assert np.all(rmargin > 1e-5), "re-seed: router near-tie"
    entry, hit, sim, subs = cache.lookup_or_route(torch.from_numpy(E).to(DEV), tau, torch.from_numpy(Wr).to(DEV))
    torch.cuda.synchronize()
    assert np.array_equal(entry.cpu().numpy(), e_ref)
    assert np.array_equal(hit.cpu().numpy(), h_ref)
    assert np.array_equal(subs.cpu().numpy(), s_ref)
    assert np.allclose(sim.cpu().numpy()[finite], sims_ref[finite], atol=2e-5)
    assert cache.count() == oc.count


def test_cache_sequential_batches_match_oracle():
    say("cache lookup_or_route, three batches, clustered embeddings")
    P, d, L, G, k = 48, 512, 3, 20, 10
    E, cid, Wr = _cache_inputs(3 * P, d, L, G, 7, 201)
    cache = pa.Cache(64, d, L, k, P)
    oc = po.PatternCache(64, d, L, k)
    for b in range(3):
        _check_cache_batch(cache, oc, E[b * P:(b + 1) * P], 0.9, Wr)
    assert cache.count() == len(set(cid.tolist()))
    # pure lookup afterwards: same answers as the oracle's, nothing inserted
    q = np.concatenate([E[:5], -E[5:7]]).astype(np.float32)
    ent_ref, sim_ref = oc.lookup(q, 0.9)
    ent, sim, subs = cache.lookup(torch.from_numpy(q).to(DEV), 0.9)
    torch.cuda.synchronize()
    assert np.array_equal(ent.cpu().numpy(), ent_ref) and np.allclose(sim.cpu().numpy(), sim_ref, atol=2e-5)
    for p in range(len(q)):
        if ent_ref[p] >= 0:
            assert np.array_equal(subs[p].cpu().numpy(), oc.values[ent_ref[p]])
        else:
            assert np.all(subs[p].cpu().numpy() == -1)          # untouched on a miss
    assert cache.count() == oc.count
    cache.close()


def test_cache_at_the_largest_model_width():
    say("cache lookup_or_route at d=16384: small-batch (one launch) and large-batch (two launches) paths")
    d, L, G, k = 16384, 2, 8, 3
    for P, seed in ((6, 211), (70, 212)):        # 70 > the small-batch limit of 64
        E, cid, Wr = _cache_inputs(2 * P, d, L, G, 9, seed)
        cache = pa.Cache(16, d, L, k, P)
        oc = po.PatternCache(16, d, L, k)
        for b in range(2):
            _check_cache_batch(cache, oc, E[b * P:(b + 1) * P], 0.9, Wr)
        cache.close()


def test_cache_empty_full_and_insert():
    say("cache: empty lookup, explicit insert, capacity overflow")
    d, L, G, k = 256, 2, 8, 3
    E, cid, Wr = _cache_inputs(12, d, L, G, 12, 202)     # 12 distinct clusters -> all miss
    cache = pa.Cache(4, d, L, k, 16)
    oc = po.PatternCache(4, d, L, k)
    ent, sim, _ = cache.lookup(torch.from_numpy(E[:3]).to(DEV), 0.9)
    torch.cuda.synchronize()
    assert ent.cpu().tolist() == [-1, -1, -1] and np.all(np.isneginf(sim.cpu().numpy()))
    # explicit insert of entry 0, then a batch that overflows the capacity of 4
    s0 = np.stack([po.route(E[0:1].astype(np.float64), Wr[l], k)[0][0] for l in range(L)])
    cache.insert(torch.from_numpy(E[0]).to(DEV), i32(s0)); oc.insert(E[0], s0)
    assert cache.count() == 1
    _check_cache_batch(cache, oc, E, 0.9, Wr)
    assert cache.count() == 4
    # a full cache drops an explicit insert on the device and counts it; the host call only enqueues
    for extra in (5, 6):
        cache.insert(torch.from_numpy(E[extra]).to(DEV), i32(s0))
    assert cache.count() == 4 and cache.dropped() == 2
    _check_cache_batch(cache, oc, E[:4], 0.9, Wr)          # the four entries are untouched: same hits as the oracle's
    cache.clear()
    assert cache.count() == 0 and cache.dropped() == 0
    cache.insert(torch.from_numpy(E[0]).to(DEV), i32(s0))
    assert cache.count() == 1 and cache.dropped() == 0
    cache.close()


def test_cache_clustered_workload_hit_rate():
    say("cache: 256 prompts, 16 clusters, d=4096, tau=0.9 -> 93.75 % hits")
    E, cid, off, Wr = si.config4_embeddings()
    cache = pa.Cache(1024, 4096, 3, 10, 256)
    oc = po.PatternCache(1024, 4096, 3, 10)
    _check_cache_batch(cache, oc, E, 0.9, Wr)
    entry, hit, sim, subs = cache.lookup_or_route(torch.from_numpy(E).to(DEV), 0.9, torch.from_numpy(Wr).to(DEV))
    torch.cuda.synchronize()
    assert cache.count() == 16 and int(hit.sum().item()) == 256          # second pass: everything hits
    cache.close()


def test_config4_grouped_execution_full_size_sampled():
    """The pattern-cache / grouped-execution workload at full size: 256 prompts from 16 clusters, lengths 32..2048
    (about 270 K tokens), gate / up / down at the MLP shapes, cache probe -> aggregation of the 16 new entries per layer
    -> prefill plan -> planned prefill.  Indexing against the oracle bit for bit; outputs of 8 sampled prompts (the
    shortest, the longest, the first, the last and four more, several of them sharing a pattern) against the oracle's
    forward on sampled rows."""
    say("config 4 at full size: cache -> pack -> plan -> planned prefill of gate/up/down, 8 sampled prompts vs the oracle")
    E, cid, off_h, Wr_h = si.config4_embeddings()
    P, d, G, k, R, hidden, inter, L = E.shape[0], E.shape[1], 20, 10, 2560, 4096, 11008, 3
    gs, rS, rows, n_slots = R // G, k * (R // G), int(off_h[-1]), 32
    shapes = [("gate", hidden, inter), ("up", hidden, inter), ("down", inter, hidden)]
    gen = torch.Generator(device=DEV); gen.manual_seed(85684)
    layers_rm, layers = [], []
    for nm, n, m in shapes:
        Vt = (torch.randn((R, n), device=DEV, generator=gen) * 0.02).to(torch.bfloat16)
        Ut = (torch.randn((R, m), device=DEV, generator=gen) * 0.02).to(torch.bfloat16)
        rm = pa.Layer(Vt, Ut, n, m, R, G, pa.PARSE_ROWMAJOR)
        layers_rm.append(rm); layers.append(pa.layer_to_mfma16(rm))
    Xh = torch.randn((rows, hidden), device=DEV, generator=gen).to(torch.bfloat16)
    Xi = torch.randn((rows, inter), device=DEV, generator=gen).to(torch.bfloat16)
    Ed, off, Wr = torch.from_numpy(E).to(DEV), i32(off_h), torch.from_numpy(Wr_h).to(DEV)
    cache = pa.Cache(n_slots, d, L, k, P)
    entry, hit, sim, subs = cache.lookup_or_route(Ed, 0.9, Wr)
    oc = po.PatternCache(n_slots, d, L, k)
    e_ref, h_ref, s_ref = oc.lookup_or_route(E, 0.9, Wr_h)
    torch.cuda.synchronize()
    assert np.array_equal(entry.cpu().numpy(), e_ref) and np.array_equal(hit.cpu().numpy(), h_ref)
    assert np.array_equal(subs.cpu().numpy(), s_ref) and int(h_ref.sum()) == 240 and cache.count() == 16
    plan = pa.prefill_plan(off, entry, rows, n_slots)
    words = plan.view(torch.int32).cpu().numpy()
    rowmap_ref, tpat_ref = po.plan_rows(off_h, e_ref, n_slots, 256)
    cap = int(words[3]); rm0 = 16 + (cap + 15) // 16 * 16
    assert int(words[0]) == len(tpat_ref) and np.array_equal(words[16:16 + len(tpat_ref)], tpat_ref)
    assert np.array_equal(words[rm0:rm0 + len(rowmap_ref)], rowmap_ref)
    lens = np.diff(off_h)
    sample = sorted({int(np.argmin(lens)), int(np.argmax(lens)), 0, P - 1, 7, 100, 101, 200})
    rng = np.random.default_rng(9)
    ws = None
    for l, (nm, n, m) in enumerate(shapes):
        Vs = torch.empty((n_slots, rS, n), dtype=torch.bfloat16, device=DEV)
        Us = torch.empty((n_slots, rS, m), dtype=torch.bfloat16, device=DEV)
        pa.pack_new_entries(layers[l], subs.view(P, L * k)[:, l * k:], L * k, k, entry, hit, Vs, Us)
        X = Xh if n == hidden else Xi
        Y = pa.lowrank_prefill_planned(layers[l], pa.Patterns(k, n_slots, Vs, Us), X, off, entry, plan)
        torch.cuda.synchronize()
        Vt64 = layers_rm[l].Vt.float().cpu().numpy().astype(np.float64)
        U64 = layers_rm[l].Ut.float().cpu().numpy().astype(np.float64).T.copy()
        Wcache = {}
        for p in sample:
            a, b = int(off_h[p]), int(off_h[p + 1])
            ts = np.unique(np.concatenate([[a, b - 1], rng.integers(a, b, size=6)]))
            key = tuple(s_ref[p, l].tolist())
            if key not in Wcache:
                Wcache[key] = po.reconstruct(U64, np.ones(R), Vt64, s_ref[p, l], gs)
            tsd = torch.from_numpy(ts).to(DEV)
            Yref = X[tsd].float().cpu().numpy().astype(np.float64) @ Wcache[key].T
            # the oracle's forward is this same product with the reconstruction done inside; checked equal on one prompt
            if p == sample[0]:
                Yf = po.forward(U64, np.ones(R), Vt64, gs, X[tsd].float().cpu().numpy().astype(np.float64), [0, len(ts)], s_ref[p:p + 1, l])
                assert np.allclose(Yf, Yref, rtol=0, atol=1e-12)
            assert_close(Y[tsd].float().cpu().numpy(), Yref, TOL_BF16, f"{nm} prompt {p} ({b - a} tokens, entry {e_ref[p]})")
        del Vs, Us, Y
    cache.close()


# ------------------------------------------------------------------ a5 bucket
@pytest.mark.parametrize("P,k,npat,stride", [(32, 10, 4, 10), (256, 10, 16, 30), (1, 3, 1, 3), (1024, 2, 700, 2)])
def test_bucket_matches_oracle(P, k, npat, stride):
    say(f"bucket P={P} k={k} patterns<={npat} stride={stride}")
    rng = np.random.default_rng(301)
    pats = np.stack([np.sort(rng.choice(24, size=k, replace=False)) for _ in range(npat)]).astype(np.int32)
    which = rng.integers(0, npat, size=P)
    full = rng.integers(0, 24, size=(P, stride)).astype(np.int32)
    full[:, :k] = pats[which]
    pid_r, perm_r, off_r, n_r, rep_r = po.bucket(full[:, :k])
    pid, perm, off, n, rep = pa.bucket_patterns(i32(full), k, stride)
    torch.cuda.synchronize()
    assert int(n.item()) == n_r
    assert np.array_equal(pid.cpu().numpy(), pid_r) and np.array_equal(perm.cpu().numpy(), perm_r)
    assert np.array_equal(off.cpu().numpy()[:n_r + 1], off_r) and np.all(off.cpu().numpy()[n_r + 1:] == P)
    assert np.array_equal(rep.cpu().numpy()[:n_r], rep_r) and np.all(rep.cpu().numpy()[n_r:] == -1)


@pytest.mark.parametrize("P,k,npat,stride,n_slots", [(8, 8, 3, 8, 32), (37, 5, 6, 9, 4), (256, 10, 16, 30, 64), (300, 4, 20, 4, 16), (1, 3, 1, 3, 1)])
def test_bucket_and_plan_in_one_launch_equal_the_separate_calls(P, k, npat, stride, n_slots):
    """The launch that buckets the prompts and builds the prefill plan: every output against the oracle and, bit for
    bit, against the two separate calls (P = 300 takes the two-launch path behind the same entry point); outputs sit
    between guard bands."""
    say(f"bucket + plan in one call P={P} k={k} patterns<={npat} stride={stride} slots={n_slots}")
    rng = np.random.default_rng(311 + P)
    pats = np.stack([np.sort(rng.choice(24, size=k, replace=False)) for _ in range(npat)]).astype(np.int32)
    which = rng.integers(0, npat, size=P)
    full = rng.integers(0, 24, size=(P, stride)).astype(np.int32)
    full[:, :k] = pats[which]
    lengths = rng.integers(0, 700, size=P)
    lengths[rng.integers(0, P)] = 257
    off = si.offsets_from_lengths([int(v) for v in lengths])
    rows = int(off[-1])
    entry = rng.integers(-1, n_slots + 1, size=P).astype(np.int32)        # some ids out of range: zero rows
    subd, offd, entd = i32(full), i32(off), i32(entry)
    ref_b = pa.bucket_patterns(subd, k, stride)
    ref_plan = pa.prefill_plan(offd, entd, rows, n_slots)
    bufs = []
    for t in list(ref_b) + [ref_plan]:
        nbytes = t.numel() * t.element_size()
        whole, mid = guarded_bytes(nbytes)
        bufs.append((whole, mid, mid[:nbytes].view(t.dtype), nbytes))
    out, plan = pa.bucket_and_plan(subd, k, stride, offd, entd, rows, n_slots, out=tuple(b[2] for b in bufs[:5]), plan=bufs[5][2])
    torch.cuda.synchronize()
    for whole, mid, _, nbytes in bufs:
        check_guards(whole, "bucket + plan")
        assert bool(torch.all(mid[nbytes:] == 0xA5)), "bucket + plan: stores beyond an output"
    pid_r, perm_r, off_r, n_r, rep_r = po.bucket(full[:, :k])
    assert int(out[3].item()) == n_r
    assert np.array_equal(out[0].cpu().numpy(), pid_r) and np.array_equal(out[1].cpu().numpy(), perm_r)
    for a, b in zip(out, ref_b):
        assert torch.equal(a, b)
    words, ref_words = plan.view(torch.int32).cpu().numpy(), ref_plan.view(torch.int32).cpu().numpy()
    rowmap_ref, tpat_ref = po.plan_rows(off, entry, n_slots, 256)
    nt, cap = int(words[0]), int(words[3])
    rm0 = 16 + (cap + 15) // 16 * 16
    assert nt == len(tpat_ref) and np.array_equal(words[16:16 + nt], tpat_ref)
    assert np.array_equal(words[rm0:rm0 + nt * 256], rowmap_ref)
    assert np.array_equal(words[:16 + nt], ref_words[:16 + nt]) and np.array_equal(words[rm0:rm0 + nt * 256], ref_words[rm0:rm0 + nt * 256])


# ------------------------------------------------------------------ a4 pack (+ offline reorder)
@pytest.mark.parametrize("dtype,n,m,R,G,subset", [
    ("f32", 1024, 1024, 256, 8, [1, 2, 5, 7]),
    ("bf16", 512, 768, 256, 8, [0, 3, 4]),
    ("bf16", 1032, 520, 96, 3, [2]),
])
def test_pack_rowmajor_bytes(dtype, n, m, R, G, subset):
    say(f"pack row-major dtype={dtype} n={n} m={m} R={R} G={G} S={subset}")
    lay = si.small_layer(401, n, m, R, G, dtype)
    Vr, Ur = po.pack(lay.Vt_store, lay.Ut_store, subset, lay.gs)
    Vs, Us = pa.pack_experts(upload_layer(lay), i32(subset))
    torch.cuda.synchronize()
    get = pa.bf16_to_bits if dtype == "bf16" else (lambda t: t.cpu().numpy())
    assert get(Vs).tobytes() == Vr.tobytes() and get(Us).tobytes() == Ur.tobytes()


def test_reorder_and_pack_in_operand_order():
    say("offline reorder to operand order + pack of patterns, byte-exact through the documented index map")
    lay = si.small_layer(402, 512, 768, 256, 8, "bf16")
    dl = pa.layer_to_mfma16(upload_layer(lay))
    torch.cuda.synchronize()
    assert pa.bf16_to_bits(dl.Vt).tobytes() == mfma16_v(lay.Vt_store).tobytes()
    assert pa.bf16_to_bits(dl.Ut).tobytes() == mfma16_u(lay.Ut_store).tobytes()
    # patterns of a batch, packed without a host round trip: rows 0,1,3 are the representatives
    subs = np.array([[0, 2, 7], [1, 2, 3], [0, 2, 7], [4, 5, 6]], np.int32)
    pid, perm, off, npat, rep = pa.bucket_patterns(i32(subs), 3)
    Vs, Us = pa.pack_patterns(dl, i32(subs), 3, 3, rep, npat, 4)
    torch.cuda.synchronize()
    for j, row in enumerate([0, 1, 3]):
        Vr, Ur = po.pack(lay.Vt_store, lay.Ut_store, subs[row], lay.gs)
        assert pa.bf16_to_bits(Vs[j]).tobytes() == mfma16_v(Vr).tobytes()
        assert pa.bf16_to_bits(Us[j]).tobytes() == mfma16_u(Ur).tobytes()


def test_pack_new_cache_entries_only():
    say("pack keyed by cache entry: only this batch's new entries are packed, into their entry's slot")
    lay = si.small_layer(404, 256, 512, 256, 8, "bf16")
    dl = pa.layer_to_mfma16(upload_layer(lay))
    d, L, k, P = 256, 1, 3, 10
    rng = np.random.default_rng(405)
    E, cid = si.clustered_embeddings(rng, P, d, 4, 0.05)
    Wr = si.make_router(rng, L, 8, d)
    oc = po.PatternCache(16, d, L, k)
    e_ref, h_ref, s_ref = oc.lookup_or_route(E, 0.9, Wr)
    cache = pa.Cache(16, d, L, k, P)
    entry, hit, sim, subs = cache.lookup_or_route(torch.from_numpy(E).to(DEV), 0.9, torch.from_numpy(Wr).to(DEV))
    Vs = torch.zeros((6, k * lay.gs, lay.n), dtype=torch.bfloat16, device=DEV)
    Us = torch.zeros((6, k * lay.gs, lay.m), dtype=torch.bfloat16, device=DEV)
    pa.pack_new_entries(dl, subs, L * k, k, entry, hit, Vs, Us)
    torch.cuda.synchronize()
    assert np.array_equal(entry.cpu().numpy(), e_ref) and np.array_equal(hit.cpu().numpy(), h_ref)
    n_new = int((h_ref == 0).sum())
    assert n_new == 4
    for p in range(P):
        if h_ref[p] == 0:
            Vr, Ur = po.pack(lay.Vt_store, lay.Ut_store, s_ref[p, 0], lay.gs)
            assert pa.bf16_to_bits(Vs[e_ref[p]]).tobytes() == mfma16_v(Vr).tobytes()
            assert pa.bf16_to_bits(Us[e_ref[p]]).tobytes() == mfma16_u(Ur).tobytes()
    assert torch.all(Vs[n_new:] == 0) and torch.all(Us[n_new:] == 0)     # slots of no new entry stay untouched
    # a second batch of the same prompts hits everywhere: nothing is packed
    Vs.zero_()
    entry, hit, sim, subs = cache.lookup_or_route(torch.from_numpy(E).to(DEV), 0.9, torch.from_numpy(Wr).to(DEV))
    pa.pack_new_entries(dl, subs, L * k, k, entry, hit, Vs, Us)
    torch.cuda.synchronize()
    assert int(hit.sum().item()) == P and torch.all(Vs == 0)
    cache.close()


def test_pack_many_patterns_spread_over_a_large_batch():
    """Work lists longer than one wavefront: 300 prompts of which every third-or-so is a new cache entry (misses
    spread over the whole batch), and a pack_patterns call over 200 patterns.  Every workgroup must walk the same
    list, else some slabs are copied twice and others never: byte equality with the oracle's pack per slot, and
    canary slots stay untouched."""
    say("pack: 300-prompt batch with scattered new entries; 200 patterns in one call")
    lay = si.small_layer(406, 256, 288, 256, 8, "bf16")
    dl = pa.layer_to_mfma16(upload_layer(lay))
    k, P, n_slots = 3, 300, 160
    rng = np.random.default_rng(407)
    subs = np.stack([np.sort(rng.choice(lay.G, size=k, replace=False)) for _ in range(P)]).astype(np.int32)
    hit = (rng.random(P) < 0.6).astype(np.uint8)
    entry = np.full(P, -1, np.int32)
    miss = np.flatnonzero(hit == 0)
    assert len(miss) > 64 and miss[-1] > 256
    slots = rng.permutation(n_slots)[:len(miss)].astype(np.int32)      # new entries land in scattered slots
    entry[miss] = slots
    entry[np.flatnonzero(hit == 1)] = rng.integers(0, n_slots, size=int(hit.sum()))
    canary = 0x3F80                                                    # bf16 1.0
    Vs = torch.full((n_slots, k * lay.gs, lay.n), 1.0, dtype=torch.bfloat16, device=DEV)
    Us = torch.full((n_slots, k * lay.gs, lay.m), 1.0, dtype=torch.bfloat16, device=DEV)
    pa.pack_new_entries(dl, i32(subs), k, k, i32(entry), torch.from_numpy(hit).to(DEV), Vs, Us)
    torch.cuda.synchronize()
    Vb, Ub = pa.bf16_to_bits(Vs), pa.bf16_to_bits(Us)
    written = set()
    for p in miss:
        Vr, Ur = po.pack(lay.Vt_store, lay.Ut_store, subs[p], lay.gs)
        assert Vb[entry[p]].tobytes() == mfma16_v(Vr).tobytes(), f"prompt {p} slot {entry[p]} (right factor)"
        assert Ub[entry[p]].tobytes() == mfma16_u(Ur).tobytes(), f"prompt {p} slot {entry[p]} (left factor)"
        written.add(int(entry[p]))
    for sl in range(n_slots):
        if sl not in written:
            assert np.all(Vb[sl] == canary) and np.all(Ub[sl] == canary), f"slot {sl} was written"
    # pack_patterns over 200 patterns taken from scattered representative prompts
    npat = 200
    rep = rng.permutation(P)[:npat].astype(np.int32)
    Vp = torch.full((npat + 2, k * lay.gs, lay.n), 1.0, dtype=torch.bfloat16, device=DEV)
    Up = torch.full((npat + 2, k * lay.gs, lay.m), 1.0, dtype=torch.bfloat16, device=DEV)
    pa.pack_patterns(dl, i32(subs), k, k, i32(rep), i32([npat]), npat + 2, Vp, Up)
    torch.cuda.synchronize()
    Vb, Ub = pa.bf16_to_bits(Vp), pa.bf16_to_bits(Up)
    for j in range(npat):
        Vr, Ur = po.pack(lay.Vt_store, lay.Ut_store, subs[rep[j]], lay.gs)
        assert Vb[j].tobytes() == mfma16_v(Vr).tobytes() and Ub[j].tobytes() == mfma16_u(Ur).tobytes(), f"pattern {j}"
    assert np.all(Vb[npat:] == canary) and np.all(Ub[npat:] == canary)


def test_pack_skips_invalid_group_ids():
    say("pack: an id outside [0, G) leaves its slab untouched")
    lay = si.small_layer(403, 256, 256, 64, 4, "f32")
    dl = upload_layer(lay)
    Vs = torch.full((32, 256), 9.0, device=DEV); Us = torch.full((32, 256), 9.0, device=DEV)
    pa.pack_experts(dl, i32([1, 77]), Vs, Us)
    torch.cuda.synchronize()
    assert np.array_equal(Vs[:16].cpu().numpy(), lay.Vt_store[16:32]) and torch.all(Vs[16:] == 9.0)


# ------------------------------------------------------------------ a6 prefill forward
def _run_prefill(lay, lengths, subsets_per_prompt, seed, dtype, schedule=0):
    rng = np.random.default_rng(seed)
    off = si.offsets_from_lengths(lengths)
    X = si.make_tokens(rng, int(off[-1]), lay.n, dtype)
    Xv = si.bf16_bits_to_f32(X).astype(np.float64) if dtype == "bf16" else X.astype(np.float64)
    U0, sg, V = oracle_factors(lay)
    Yref = po.forward(U0, sg, V, lay.gs, Xv, off, subsets_per_prompt)
    subs = np.asarray(subsets_per_prompt, np.int32)
    k = subs.shape[1]
    dl = upload_layer(lay)
    if dtype == "bf16":
        dl = pa.layer_to_mfma16(dl)
    sd = i32(subs)
    pid, perm, boff, npat, rep = pa.bucket_patterns(sd, k)
    Vs, Us = pa.pack_patterns(dl, sd, k, k, rep, npat, len(lengths))
    Y = forward_guarded(pa.PARSE_PREFILL, dl, pa.Patterns(k, len(lengths), Vs, Us, schedule=schedule),
                           upload_tokens(X, dtype), i32(off), pid, no_workspace=(schedule == 1))
    torch.cuda.synchronize()
    Yg = Y.float().cpu().numpy().astype(np.float64)
    return Yg, Yref, off


def test_prefill_config0_fp32():
    say("prefill config 0 (fp32, n=m=1024, R=256, 8 groups, top-4, 4 x 64 tokens), routed subsets")
    w = si.config0()
    lay = w.layers[0]
    subs, margin = po.route(po.pool(w.X_values(), w.tok_offsets), w.Wr[0], w.k)
    dl = upload_layer(lay)
    sd = i32(subs)
    pid, perm, boff, npat, rep = pa.bucket_patterns(sd, w.k)
    Vs, Us = pa.pack_patterns(dl, sd, w.k, w.k, rep, npat, w.P)
    Y = forward_guarded(pa.PARSE_PREFILL, dl, pa.Patterns(w.k, w.P, Vs, Us), upload_tokens(w.X, "f32"),
                           i32(w.tok_offsets), pid)
    torch.cuda.synchronize()
    Yref = po.forward(lay.U0, lay.sigma, lay.V, lay.gs, w.X_values(), w.tok_offsets, subs)
    for p in range(w.P):
        a, b = w.tok_offsets[p], w.tok_offsets[p + 1]
        assert_close(Y[a:b].cpu().numpy(), Yref[a:b], TOL_F32, f"prompt {p}")


@pytest.mark.parametrize("n,m,R,G,k,lengths,schedule", [
    (512, 768, 256, 8, 4, [70, 1, 33, 129, 64], 1),       # r_S = 128: one rank block per wave, ragged tiles
    (512, 768, 256, 8, 4, [70, 1, 33, 129, 64], 2),
    (1024, 1024, 512, 4, 3, [64, 200], 1),                # r_S = 384: uneven rank blocks per wave
    (1024, 1024, 512, 4, 3, [64, 200], 2),
    (528, 544, 160, 5, 2, [5, 90], 0),                    # n not a multiple of the staged tile, r_S = 64
    (512, 512, 2560, 20, 10, [40, 100], 1),               # r_S = 1280: 32-token workgroups
    (512, 800, 2560, 20, 10, [40, 300], 2),               # two launches, output blocks not a multiple of a chunk
    (1024, 4096, 1024, 8, 4, [512, 512, 37], 0),          # default choice at a size with whole 128-row tiles
    (256, 256, 1024, 8, 8, [9000, 7400], 2),              # many token tiles: 128-token tiles in both launches
    (512, 768, 256, 8, 4, [70, 1, 33, 129, 64], 3),       # planned schedule: every prompt its own pattern, ragged
    (1024, 1024, 512, 4, 3, [64, 200], 3),                # planned, r_S = 384: a partial column tile in the first product
    (512, 800, 2560, 20, 10, [40, 300], 3),               # planned, r_S = 1280, 25 output blocks (partial tile)
    (256, 1024, 1024, 8, 8, [9000, 7400], 3),             # planned, 256-row tiles in both launches, short reduction
    (256, 1024, 1024, 8, 8, [9000, 7400], 0),             # the default choice at that size
    (64, 64, 64, 2, 1, [300], 3),                         # planned, the smallest shapes: one reduction slice
])
def test_prefill_bf16_small(n, m, R, G, k, lengths, schedule):
    say(f"prefill bf16 n={n} m={m} R={R} G={G} k={k} lengths={lengths} schedule={schedule}")
    if R > min(n, m):
        lay = si.make_layer(np.random.default_rng(501), n, m, min(n, m), 1, "bf16")
        # stored rank above min(n, m) cannot be orthonormal: tile independent blocks instead (values only matter
        # through the stored arrays, which the oracle reads back)
        reps = R // min(n, m)
        lays = [si.make_layer(np.random.default_rng(510 + i), n, m, min(n, m), 1, "bf16") for i in range(reps)]
        lay = si.Layer(n, m, R, G, "bf16", None, None, None,
                       np.concatenate([l.Vt_store for l in lays]), np.concatenate([l.Ut_store for l in lays]))
    else:
        lay = si.small_layer(502, n, m, R, G, "bf16")
    rng = np.random.default_rng(503)
    subs = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in lengths]).astype(np.int32)
    Yg, Yref, off = _run_prefill(lay, lengths, subs, 504, "bf16", schedule)
    for p in range(len(lengths)):
        assert_close(Yg[off[p]:off[p + 1]], Yref[off[p]:off[p + 1]], TOL_BF16, f"prompt {p}")


@pytest.mark.parametrize("n,m,R,G,k,lengths", [
    (2048, 512, 256, 8, 3, [200]),              # one short prompt: 4 token tiles x 1 rank tile -> 4 slices of the reduction
    (4096, 512, 512, 8, 4, [70, 1, 130]),       # three short prompts with different subsets, 8 slices (ragged last tile)
    (1024, 256, 128, 4, 2, [33, 500]),          # 2 slices of 8 staged steps each
])
def test_prefill_of_short_prompts_splits_the_first_reduction(n, m, R, G, k, lengths):
    """A batch too short to fill the chip with tiles of the first product: its reduction range is cut in slices whose fp32
    partial sums a second small launch adds and rounds.  Planned schedule through parse_lowrank_forward (guards around Y
    and the workspace of exactly the queried size), over a ready plan, and two layers in one call -- every prompt against
    the oracle, and the three entry points bit-identical."""
    say(f"prefill of short prompts (split first product) n={n} m={m} R={R} G={G} k={k} lengths={lengths}")
    lay = si.make_layer(np.random.default_rng(661), n, m, R, G, "bf16", fast=True)
    rng = np.random.default_rng(662)
    subs = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in lengths]).astype(np.int32)
    Yg, Yref, off = _run_prefill(lay, lengths, subs, 663, "bf16", 3)
    for p in range(len(lengths)):
        assert_close(Yg[off[p]:off[p + 1]], Yref[off[p]:off[p + 1]], TOL_BF16, f"prompt {p}")
    # the same call over a ready plan, and as a two-layer call (the second layer is the same factors)
    X = si.make_tokens(np.random.default_rng(663), int(off[-1]), n, "bf16")
    dl = pa.layer_to_mfma16(upload_layer(lay))
    sd = i32(subs)
    pid, perm, boff, npat, rep = pa.bucket_patterns(sd, k)
    Vs, Us = pa.pack_patterns(dl, sd, k, k, rep, npat, len(lengths))
    pt = pa.Patterns(k, len(lengths), Vs, Us, schedule=3)
    Xd, offd = upload_tokens(X, "bf16"), i32(off)
    rows = int(off[-1])
    plan = pa.prefill_plan(offd, pid, rows, len(lengths))
    need = pa.lowrank_prefill_planned_workspace_bytes(dl, rows, len(lengths), k, len(lengths))
    whole, mid = guarded_bytes(need)
    Y1 = pa.lowrank_prefill_planned(dl, pt, Xd, offd, pid, plan, workspace=mid[:need])
    check_guards(whole, "planned prefill over a ready plan: workspace")
    assert np.array_equal(Y1.float().cpu().numpy().astype(np.float64), Yg)
    Ys = prefill_multi_guarded([dl, dl], [pt, pt], Xd, offd, pid)
    torch.cuda.synchronize()
    assert torch.equal(Ys[0].view(torch.int16), Y1.view(torch.int16)) and torch.equal(Ys[1].view(torch.int16), Y1.view(torch.int16))


def test_prefill_plan_matches_the_row_grouping_and_serves_shared_patterns():
    """The prefill plan against the oracle's row grouping (bit-exact), then the planned product with prompts that share
    patterns in interleaved arrival order, one prompt with an invalid pattern id (zero rows), and guard rows around Y."""
    say("prefill plan: row map, tile patterns; planned product with shared patterns and an invalid id")
    n, m, R, G, k = 512, 640, 256, 8, 3
    lay = si.small_layer(521, n, m, R, G, "bf16")
    lengths = [300, 17, 256, 90, 1, 513, 64, 40]
    pid_h = np.array([2, 0, 2, 5, 0, 1, 9, 1], np.int32)          # 9 is out of range for 6 slots
    n_slots = 6
    rng = np.random.default_rng(522)
    slot_subs = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(n_slots)]).astype(np.int32)
    off = si.offsets_from_lengths(lengths)
    rows = int(off[-1])
    X = si.make_tokens(rng, rows, n, "bf16")
    Xv = si.bf16_bits_to_f32(X).astype(np.float64)
    dl = pa.layer_to_mfma16(upload_layer(lay))
    Vs, Us = pa.pack_patterns(dl, i32(slot_subs), k, k, None, None, n_slots)
    offd, pidd, Xd = i32(off), i32(pid_h), upload_tokens(X, "bf16")
    plan = pa.prefill_plan(offd, pidd, rows, n_slots)
    torch.cuda.synchronize()
    words = plan.view(torch.int32).cpu().numpy()
    rowmap_ref, tpat_ref = po.plan_rows(off, pid_h, n_slots, 256)
    nt, cap = int(words[0]), int(words[3])
    assert nt == len(tpat_ref) and int(words[1]) == nt * 256 and int(words[2]) == 256
    assert np.array_equal(words[16:16 + nt], tpat_ref)
    rm0 = 16 + (cap + 15) // 16 * 16
    assert np.array_equal(words[rm0:rm0 + nt * 256], rowmap_ref)
    # planned product, output between guard rows
    guard = 4
    Ybuf = torch.full((rows + 2 * guard, m), 7.0, dtype=torch.bfloat16, device=DEV)
    Y = Ybuf[guard:guard + rows]
    pt = pa.Patterns(k, n_slots, Vs, Us)
    pa.lowrank_prefill_planned(dl, pt, Xd, offd, pidd, plan, Y=Y)
    Y2 = forward_guarded(pa.PARSE_PREFILL, dl, pt.with_schedule(pa.PARSE_SCHED_PLANNED), Xd, offd, pidd)
    torch.cuda.synchronize()
    assert torch.all(Ybuf[:guard] == 7.0) and torch.all(Ybuf[guard + rows:] == 7.0), "stores outside Y"
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16)), "ready plan vs plan built inside the call"
    U0, sg, V = oracle_factors(lay)
    Yn = Y.float().cpu().numpy().astype(np.float64)
    for p, L_ in enumerate(lengths):
        a, b = off[p], off[p + 1]
        if pid_h[p] >= n_slots:
            assert np.all(Yn[a:b] == 0), "prompt with an invalid pattern id must give zero rows"
            continue
        Yref = po.forward(U0, sg, V, lay.gs, Xv[a:b], [0, b - a], slot_subs[pid_h[p]][None, :])
        assert_close(Yn[a:b], Yref, TOL_BF16, f"prompt {p} (pattern {pid_h[p]})")


def test_prefill_invalid_pattern_gives_zero_rows_and_is_repeatable():
    say("prefill bf16: out-of-range pattern id -> zero rows; two runs give the same bits")
    lay = si.small_layer(505, 256, 256, 128, 4, "bf16")
    dl = pa.layer_to_mfma16(upload_layer(lay))
    subs = i32([[0, 1], [2, 3]])
    Vs, Us = pa.pack_patterns(dl, subs, 2, 2, None, None, 2)
    X = upload_tokens(si.make_tokens(np.random.default_rng(1), 100, 256, "bf16"), "bf16")
    off = i32([0, 30, 70, 100]); pid = i32([1, 5, 0])
    pt = pa.Patterns(2, 2, Vs, Us)
    Y1 = forward_guarded(pa.PARSE_PREFILL, dl, pt, X, off, pid)
    Y2 = forward_guarded(pa.PARSE_PREFILL, dl, pt, X, off, pid)
    torch.cuda.synchronize()
    assert torch.equal(Y1.view(torch.int16), Y2.view(torch.int16))
    assert torch.all(Y1[30:70] == 0) and torch.any(Y1[:30] != 0) and torch.any(Y1[70:] != 0)


def test_prefill_config1_full_size_sampled():
    say("prefill config 1 (bf16 4096x4096, R=2048, 16 groups, top-8, 8 x 512 tokens): sampled rows vs oracle")
    w = si.config1()
    lay = w.layers[0]
    Xv = w.X_values()
    subs, margin = po.route(po.pool(Xv, w.tok_offsets), w.Wr[0], w.k)
    dl = pa.layer_to_mfma16(upload_layer(lay))
    Xd, offd = upload_tokens(w.X, "bf16"), i32(w.tok_offsets)
    sub_d = pa.route(Xd, offd, torch.from_numpy(w.Wr[0]).to(DEV), w.k)
    pid, perm, boff, npat, rep = pa.bucket_patterns(sub_d, w.k)
    Vs, Us = pa.pack_patterns(dl, sub_d, w.k, w.k, rep, npat, w.P)
    Ys = {}
    for schedule in (1, 2, 3):
        Ys[schedule] = forward_guarded(pa.PARSE_PREFILL, dl, pa.Patterns(w.k, w.P, Vs, Us, schedule=schedule), Xd, offd, pid)
        torch.cuda.synchronize()
    assert np.all(margin > 1e-4) and np.array_equal(sub_d.cpu().numpy(), subs)
    # the launch configuration the benchmark times: a ready plan, then the planned call
    rows = int(w.tok_offsets[-1])
    plan = pa.prefill_plan(offd, pid, rows, w.P)
    Ys["ready plan"] = pa.lowrank_prefill_planned(dl, pa.Patterns(w.k, w.P, Vs, Us), Xd, offd, pid, plan)
    torch.cuda.synchronize()
    assert torch.equal(Ys["ready plan"].view(torch.int16), Ys[3].view(torch.int16))
    U0, sg, V = oracle_factors(lay)
    rng = np.random.default_rng(7)
    for p in range(w.P):
        ts = w.tok_offsets[p] + np.concatenate([[0, 63, 64, 511], rng.integers(0, 512, size=4)])
        # the oracle's own forward (dense reconstruction of W_S, then apply) on the sampled rows as one prompt
        Yref = po.forward(U0, sg, V, lay.gs, Xv[ts], [0, len(ts)], subs[p:p + 1])
        for schedule, Y in Ys.items():
            assert_close(Y[torch.from_numpy(ts).to(DEV)].float().cpu().numpy(), Yref, TOL_BF16,
                         f"prompt {p} schedule {schedule}")


# ------------------------------------------------------------------ a7 decode
@pytest.mark.parametrize("n,m,R,G,k,B,npat,schedule", [
    (1024, 1536, 640, 20, 10, 32, 4, 0),
    (512, 256, 256, 8, 3, 5, 2, 0),
    (2752, 1024, 640, 20, 10, 32, 4, 0),   # n/16 not divisible by the slice count
    (4096, 11008, 2560, 20, 10, 32, 4, 0), # the decode workload's gate/up shape (two column blocks per workgroup)
    (11008, 4096, 2560, 20, 10, 32, 4, 0), # the decode workload's down shape
    (512, 16384, 96, 3, 2, 32, 3, 0),      # three rank blocks (a partial quad), many column blocks
    (512, 32768, 96, 3, 2, 9, 3, 0),       # four column blocks per workgroup
    (2048, 2048, 2048, 64, 20, 32, 4, 0),  # the most groups a layer may have (64 of 32 ranks): quads span four groups
    (8192, 512, 256, 8, 3, 32, 4, 0),      # a long reduction over few rank blocks: 16 slices, two stagings of x each
    (4096, 4096, 1536, 16, 8, 1, 1, 0),    # one sequence: eight ranks per workgroup on the vector units
    (11008, 4096, 2048, 16, 8, 1, 1, 0),   # ... a reduction whose step count is no multiple of four (688 steps, 3 batches of loads)
    (1040, 512, 256, 8, 3, 2, 2, 0),       # two sequences, 65 reduction steps (a ragged last instruction)
    (2752, 1024, 640, 20, 10, 3, 2, 0),    # three sequences (computed as four)
    (512, 256, 256, 8, 3, 4, 4, 0),        # four sequences, four patterns
    (32, 64, 32, 1, 1, 1, 1, 0),           # a tiny layer: two reduction steps, one instruction, three idle wavefronts
    (16384, 256, 64, 2, 1, 4, 2, 0),       # four sequences whose x rows do not fit the small-batch staging: the matrix path
])
def test_decode_matches_oracle_and_prefill(n, m, R, G, k, B, npat, schedule):
    say(f"decode n={n} m={m} R={R} G={G} k={k} B={B} patterns={npat} schedule={schedule}")
    _decode_case(n, m, R, G, k, B, npat)


def test_decode_plan_contents_and_planned_step():
    """The decode plan (group masks, ascending list of used groups) against a plain restatement from the subsets, and the
    planned two-launch step: bit-identical to the ordinary calls (which build the same plan inside), on two layers that
    share x, with guard bytes around the outputs and the intermediate workspace."""
    say("decode plan: masks / used list; planned step = ordinary step bit for bit")
    n, B, npat = 1024, 29, 5
    shapes = [(1536, 640, 20, 10), (512, 256, 8, 3)]
    rng = np.random.default_rng(611)
    seq_pat = rng.integers(0, npat, size=B).astype(np.int32)
    seq_pat[3] = 77                                            # an invalid pattern id: that sequence gets zeros
    x = si.make_tokens(rng, B, n, "bf16")
    xd, pid = upload_tokens(x, "bf16"), i32(seq_pat)
    layers, pats, subs_h = [], [], []
    for i, (m, R, G, k) in enumerate(shapes):
        lay = si.make_layer(np.random.default_rng(612 + i), n, m, R, G, "bf16")
        sub = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(npat)]).astype(np.int32)
        layers.append(pa.layer_to_mfma16(upload_layer(lay))); subs_h.append((lay, sub, G, k))
        pats.append(pa.Patterns(k, npat, subsets=i32(sub)))
    plan = pa.decode_plan(layers, pats, pid)
    torch.cuda.synchronize()
    PLAN_WORDS = 704      # per layer: count, 64 used ids, 64 masks, padding to 192, then 512 arrival counters
    assert plan.numel() >= len(shapes) * PLAN_WORDS * 4
    words = plan.view(torch.int32).cpu().numpy()
    for li, (lay, sub, G, k) in enumerate(subs_h):
        w = words[li * PLAN_WORDS:(li + 1) * PLAN_WORDS]
        assert np.all(w[192:] == 0), "arrival counters start at zero"
        used, mlist = po.decode_groups(sub, seq_pat, G)
        masks = np.zeros(64, np.uint32)
        masks[:G] = np.array(mlist, dtype=np.uint64).astype(np.uint32)
        assert int(w[0]) == len(used) and w[1:1 + len(used)].tolist() == used and np.all(w[1 + len(used):65] == -1)
        assert np.array_equal(w[65:129].view(np.uint32), masks)
    # planned step between guards
    def guarded(rows, cols):
        buf = torch.full((rows + 2, cols), 5.0, dtype=torch.bfloat16, device=DEV)
        return buf, buf[1:1 + rows]
    bufs = [guarded(B, m) for (m, R, G, k) in shapes]
    need = pa.lowrank_decode_planned_workspace_bytes(layers)
    wsbuf = torch.full((need + 512,), 0x5A, dtype=torch.uint8, device=DEV)
    pa.lowrank_decode_planned(layers, xd, plan, [v for _, v in bufs], wsbuf[256:256 + need])
    ys_multi = decode_multi_guarded(layers, pats, xd, pid)
    torch.cuda.synchronize()
    assert torch.all(wsbuf[:256] == 0x5A) and torch.all(wsbuf[256 + need:] == 0x5A), "stores outside the workspace"
    after = plan.view(torch.int32).cpu().numpy()
    assert np.array_equal(after, words), "a decode call leaves the plan as it found it (arrival counters back at zero)"
    for li, (lay, sub, G, k) in enumerate(subs_h):
        buf, view = bufs[li]
        assert torch.all(buf[0] == 5.0) and torch.all(buf[-1] == 5.0), "stores outside Y"
        y_single = forward_guarded(pa.PARSE_DECODE, layers[li], pats[li], xd, None, pid)
        torch.cuda.synchronize()
        assert torch.equal(view.view(torch.int16), ys_multi[li].view(torch.int16))
        assert torch.equal(view.view(torch.int16), y_single.view(torch.int16))
        U0, sg, V = oracle_factors(lay)
        ok = np.flatnonzero((seq_pat >= 0) & (seq_pat < npat))
        Yo = po.decode_step(U0, sg, V, lay.gs, si.bf16_bits_to_f32(x[ok]).astype(np.float64), sub[seq_pat[ok]])
        yn = view.float().cpu().numpy().astype(np.float64)
        assert_close(yn[ok], Yo, TOL_BF16, f"layer {li}")
        assert np.all(yn[3] == 0), "a sequence with an invalid pattern id must get zeros"


def _decode_case(n, m, R, G, k, B, npat):
    lay = si.make_layer(np.random.default_rng(601), n, m, R, G, "bf16", fast=(R > 1024))
    rng = np.random.default_rng(602)
    pats = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(npat)]).astype(np.int32)
    seq_pat = (np.arange(B) % npat).astype(np.int32)
    x = si.make_tokens(rng, B, n, "bf16")
    U0, sg, V = oracle_factors(lay)
    # at the full workload shape the dense oracle is run on a sample of the sequences (one per pattern, two here)
    rows = np.arange(B) if (R <= 1024 or B <= 2) else np.array([1, B - 2])
    Yref = po.decode_step(U0, sg, V, lay.gs, si.bf16_bits_to_f32(x[rows]).astype(np.float64), pats[seq_pat[rows]])
    dl = pa.layer_to_mfma16(upload_layer(lay))
    xd = upload_tokens(x, "bf16")
    pt = pa.Patterns(k, npat, subsets=i32(pats))
    y1 = forward_guarded(pa.PARSE_DECODE, dl, pt, xd, None, i32(seq_pat))
    y2 = forward_guarded(pa.PARSE_DECODE, dl, pt, xd, None, i32(seq_pat))
    torch.cuda.synchronize()
    assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))
    y1n = y1.float().cpu().numpy()
    for i, b in enumerate(rows):
        assert_close(y1n[b:b + 1], Yref[i:i + 1], TOL_BF16, f"sequence {b}")
    # cross-kernel check: the prefill kernel on the same single rows and subsets
    Vs, Us = pa.pack_patterns(dl, i32(pats), k, k, None, None, npat)
    yp = forward_guarded(pa.PARSE_PREFILL, dl, pa.Patterns(k, npat, Vs, Us), xd, i32(np.arange(B + 1)), i32(seq_pat))
    torch.cuda.synchronize()
    assert_close(y1n, yp.float().cpu().numpy(), TOL_BF16, "decode vs prefill kernel")


def test_decode_more_than_32_sequences_in_panels():
    """70 sequences = panels of 32, 32 and 6: every panel has its own masks; single-layer and fused calls, all rows
    against the oracle."""
    say("decode B=70 (three panels), single call and two layers in one call")
    n, B, npat = 1024, 70, 5
    shapes = [(768, 256, 8, 3), (512, 384, 12, 5)]
    rng = np.random.default_rng(621)
    seq_pat = rng.integers(0, npat, size=B).astype(np.int32)
    x = si.make_tokens(rng, B, n, "bf16")
    xd, pid = upload_tokens(x, "bf16"), i32(seq_pat)
    layers, pats, host = [], [], []
    for i, (m, R, G, k) in enumerate(shapes):
        lay = si.make_layer(np.random.default_rng(622 + i), n, m, R, G, "bf16")
        sub = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(npat)]).astype(np.int32)
        layers.append(pa.layer_to_mfma16(upload_layer(lay))); host.append((lay, sub))
        pats.append(pa.Patterns(k, npat, subsets=i32(sub)))
    ys = decode_multi_guarded(layers, pats, xd, pid)
    torch.cuda.synchronize()
    xv = si.bf16_bits_to_f32(x).astype(np.float64)
    for li, (lay, sub) in enumerate(host):
        y1 = forward_guarded(pa.PARSE_DECODE, layers[li], pats[li], xd, None, pid)
        torch.cuda.synchronize()
        U0, sg, V = oracle_factors(lay)
        Yo = po.decode_step(U0, sg, V, lay.gs, xv, sub[seq_pat])
        for y in (y1, ys[li]):
            assert y.shape == (B, lay.m)
            yn = y.float().cpu().numpy().astype(np.float64)
            for b in range(B):
                assert_close(yn[b:b + 1], Yo[b:b + 1], TOL_BF16, f"layer {li} sequence {b}")


def test_decode_of_a_few_sequences_masks_and_panels():
    """The small-batch kernels (one to four sequences): sequences with DIFFERENT patterns share a group's stream and are
    masked per sequence; an invalid pattern id gives a zero row; the planned step equals the ordinary one bit for bit and
    stays inside its buffers; and a batch of 33 ends in a panel of one sequence, which takes the same kernels."""
    say("decode of 2-4 sequences with different patterns, an invalid id, and a 33-sequence batch (last panel of one)")
    n, m, R, G, k, npat = 1024, 640, 512, 16, 5, 6
    lay = si.make_layer(np.random.default_rng(641), n, m, R, G, "bf16")
    rng = np.random.default_rng(642)
    sub = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(npat)]).astype(np.int32)
    dl = pa.layer_to_mfma16(upload_layer(lay))
    pt = pa.Patterns(k, npat, subsets=i32(sub))
    U0, sg, V = oracle_factors(lay)
    for B, seq_pat in ((2, [3, 0]), (3, [5, 99, 1]), (4, [2, 2, 4, -1]), (33, list(rng.integers(0, npat, size=33)))):
        seq_pat = np.array(seq_pat, np.int32)
        x = si.make_tokens(rng, B, n, "bf16")
        xd, pid = upload_tokens(x, "bf16"), i32(seq_pat)
        y = forward_guarded(pa.PARSE_DECODE, dl, pt, xd, None, pid)
        torch.cuda.synchronize()
        yn = y.float().cpu().numpy().astype(np.float64)
        ok = np.flatnonzero((seq_pat >= 0) & (seq_pat < npat))
        Yo = po.decode_step(U0, sg, V, lay.gs, si.bf16_bits_to_f32(x[ok]).astype(np.float64), sub[seq_pat[ok]])
        for i, b in enumerate(ok):
            assert_close(yn[b:b + 1], Yo[i:i + 1], TOL_BF16, f"B={B} sequence {b}")
        for b in np.setdiff1d(np.arange(B), ok):
            assert np.all(yn[b] == 0), "a sequence with an invalid pattern id must get zeros"
        if B <= 32:
            plan = pa.decode_plan([dl], [pt], pid)
            nbytes = B * m * 2
            whole, mid = guarded_bytes(nbytes)
            wsb = pa.lowrank_decode_planned_workspace_bytes([dl])
            wwhole, wmid = guarded_bytes(wsb)
            yv = mid[:nbytes].view(torch.bfloat16).view(B, m)
            pa.lowrank_decode_planned([dl], xd, plan, [yv], wmid[:wsb])
            check_guards(whole, "planned small-batch decode: Y"); check_guards(wwhole, "planned small-batch decode: workspace")
            assert bool(torch.all(mid[nbytes:] == 0xA5))
            assert torch.equal(yv.view(torch.int16), y.view(torch.int16))


def test_steps_replayed_from_a_graph_equal_the_eager_steps():
    """Every call of the path only enqueues kernels, so whole steps can be recorded into a HIP graph.  Three graphs -- a
    decode step with a split reduction (arrival counters drawn and reset inside every replay), a decode step of four
    sequences whose kernels need more than 64 KiB of LDS (the limit is raised inside the capture), and two consecutive
    prefill steps over the pattern cache (its probe alternates between two device counters) -- are each replayed
    three times with eager work of the same kind in between; every replay must reproduce the eager result bit for bit."""
    say("graph capture: decode (split reduction), small-batch decode (88 KiB LDS), two prefill steps with the cache")
    rng = np.random.default_rng(651)
    side = torch.cuda.Stream()

    def capture(fn):
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):           # warm-up outside the capture, as torch asks
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g

    # --- decode: n = 8192 over few rank blocks -> 16 slices with tickets; then 4 sequences at n = 11008
    for (n, m, R, G, k, B, npat) in ((8192, 512, 256, 8, 3, 32, 4), (11008, 512, 256, 8, 3, 4, 2)):
        lay = si.make_layer(np.random.default_rng(652), n, m, R, G, "bf16", fast=True)
        sub = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(npat)]).astype(np.int32)
        dl = pa.layer_to_mfma16(upload_layer(lay))
        pt = pa.Patterns(k, npat, subsets=i32(sub))
        pid = i32((np.arange(B) % npat).astype(np.int32))
        xs = [upload_tokens(si.make_tokens(rng, B, n, "bf16"), "bf16") for _ in range(2)]
        x = xs[0].clone()
        y = torch.empty((B, m), dtype=torch.bfloat16, device=DEV)
        ws = torch.empty(pa.lowrank_decode_planned_workspace_bytes([dl]), dtype=torch.uint8, device=DEV)
        plan = pa.decode_plan([dl], [pt], pid)
        g = capture(lambda: pa.lowrank_decode_planned([dl], x, plan, [y], ws))
        for rep in range(3):
            x.copy_(xs[rep % 2])
            pa.lowrank_decode_planned([dl], x, plan, [y], ws)          # eager
            torch.cuda.synchronize()
            ref = y.clone(); y.zero_()
            g.replay(); torch.cuda.synchronize()
            assert torch.equal(y.view(torch.int16), ref.view(torch.int16)), f"decode n={n} B={B}: replay {rep} differs"

    # --- prefill: pool -> probe (route on miss) -> buckets + plan -> aggregation of new entries -> planned product
    n, m, R, G, k, P, n_slots = 512, 384, 256, 8, 3, 6, 16         # room for the patterns of both token sets
    lay = si.small_layer(653, n, m, R, G, "bf16")
    dl = pa.layer_to_mfma16(upload_layer(lay))
    lengths = [70, 300, 5, 129, 64, 256]
    off = si.offsets_from_lengths(lengths); rows = int(off[-1])
    offd = i32(off)
    Wr = torch.from_numpy(si.make_router(rng, 1, G, n)).to(DEV)
    Xs = [upload_tokens(si.make_tokens(rng, rows, n, "bf16"), "bf16") for _ in range(2)]
    X = Xs[0].clone()
    cache = pa.Cache(n_slots, n, 1, k, P)
    emb = torch.empty((P, n), dtype=torch.float32, device=DEV)
    ws_pool = torch.empty(max(pa.route_workspace_bytes(rows, P, n), 256), dtype=torch.uint8, device=DEV)
    entry = torch.empty(P, dtype=torch.int32, device=DEV); hit = torch.empty(P, dtype=torch.uint8, device=DEV)
    sim = torch.empty(P, dtype=torch.float32, device=DEV); sub = torch.empty((P, 1, k), dtype=torch.int32, device=DEV)
    bout = (torch.empty(P, dtype=torch.int32, device=DEV), torch.empty(P, dtype=torch.int32, device=DEV),
            torch.empty(P + 1, dtype=torch.int32, device=DEV), torch.empty(1, dtype=torch.int32, device=DEV),
            torch.empty(P, dtype=torch.int32, device=DEV))
    Vs = torch.zeros((n_slots, k * lay.gs, n), dtype=torch.bfloat16, device=DEV)
    Us = torch.zeros((n_slots, k * lay.gs, m), dtype=torch.bfloat16, device=DEV)
    pt = pa.Patterns(k, n_slots, Vs, Us)
    plan = torch.empty(pa.prefill_plan_bytes(rows, P, n_slots), dtype=torch.uint8, device=DEV)
    Y = torch.empty((rows, m), dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(max(pa.lowrank_prefill_planned_workspace_bytes(dl, rows, P, k, n_slots), 256), dtype=torch.uint8, device=DEV)

    def step():
        pa.pool(X, offd, emb, ws_pool)
        cache.lookup_or_route(emb, 0.9, Wr, entry, hit, sim, sub)
        pa.bucket_and_plan(sub, k, k, offd, entry, rows, n_slots, bout, plan)
        pa.pack_new_entries(dl, sub, k, k, entry, hit, Vs, Us)
        pa.lowrank_prefill_planned(dl, pt, X, offd, entry, plan, Y, ws)

    for _ in range(4):                                 # an even number of probes; the host-side bound of the entry count
        step()                                         # has reached the capacity, so the recorded probe covers every entry
    torch.cuda.synchronize()
    g = capture(lambda: (step(), step()))
    for rep in range(3):
        X.copy_(Xs[rep % 2])
        step(); step(); torch.cuda.synchronize()
        ref, eref, href = Y.clone(), entry.clone(), hit.clone()
        Y.zero_(); entry.fill_(-5)
        g.replay(); torch.cuda.synchronize()
        assert torch.equal(Y.view(torch.int16), ref.view(torch.int16)) and torch.equal(entry, eref) and torch.equal(hit, href), \
            f"prefill: replay {rep} differs"
    cache.close()


def test_decode_with_a_shared_head_streams_it_once():
    """Shared experts (Sec. 4.4): every pattern starts with the same two groups.  Decode reads the layer's own store by
    group id, so the shared groups are simply groups that every sequence selected: streamed once, applied to all."""
    say("decode: patterns with a shared head of two groups")
    n, m, R, G, k, B, npat, ns = 1024, 768, 384, 12, 5, 19, 4, 2
    lay = si.make_layer(np.random.default_rng(631), n, m, R, G, "bf16")
    rng = np.random.default_rng(632)
    shared = np.array([0, 1], np.int32)                        # the two largest-sigma groups
    sub = np.stack([np.concatenate([shared, np.sort(rng.choice(np.arange(ns, G), size=k - ns, replace=False))])
                    for _ in range(npat)]).astype(np.int32)
    seq_pat = rng.integers(0, npat, size=B).astype(np.int32)
    x = si.make_tokens(rng, B, n, "bf16")
    dl = pa.layer_to_mfma16(upload_layer(lay))
    pt = pa.Patterns(k, npat, subsets=i32(sub))
    plan = pa.decode_plan([dl], [pt], i32(seq_pat))
    y = forward_guarded(pa.PARSE_DECODE, dl, pt, upload_tokens(x, "bf16"), None, i32(seq_pat))
    torch.cuda.synchronize()
    words = plan.view(torch.int32).cpu().numpy()
    present = np.uint32(0)
    for b in range(B):
        present |= np.uint32(1 << b)
    assert np.uint32(words[65 + 0]) == present and np.uint32(words[65 + 1]) == present   # every sequence holds the shared groups
    U0, sg, V = oracle_factors(lay)
    Yo = po.decode_step(U0, sg, V, lay.gs, si.bf16_bits_to_f32(x).astype(np.float64), sub[seq_pat])
    yn = y.float().cpu().numpy().astype(np.float64)
    for b in range(B):
        assert_close(yn[b:b + 1], Yo[b:b + 1], TOL_BF16, f"sequence {b}")


def test_rank_granular_decode_over_packed_blocks():
    """Rank-granular patterns (one expert per rank) have no groups to mask on: a decode step is the product over each
    sequence's own aggregated block, one row per sequence -- the prefill kernels with unit-length prompts.  All three
    schedules, every sequence against the oracle."""
    say("rank-granular decode: one token per sequence over the aggregated rank blocks")
    n, m, R, K, B = 512, 768, 512, 128, 11
    lay = si.small_layer(911, n, m, R, R, "bf16")
    rng = np.random.default_rng(912)
    subs = np.stack([np.sort(rng.choice(R, size=K, replace=False)) for _ in range(B)]).astype(np.int32)
    x = si.make_tokens(rng, B, n, "bf16")
    dl = upload_layer(lay)
    Vs, Us = pa.pack_ranks(dl, i32(subs), K, B)
    desc = pa.Layer(dl.Vt, dl.Ut, n, m, R, R // 32, pa.PARSE_MFMA16)
    off = np.arange(B + 1, dtype=np.int32)
    U0, sg, V = oracle_factors(lay)
    Yo = po.forward(U0, sg, V, 1, si.bf16_bits_to_f32(x).astype(np.float64), off, subs)
    for schedule in (1, 2, 3):
        y = forward_guarded(pa.PARSE_PREFILL, desc, pa.Patterns(K // 32, B, Vs, Us, schedule=schedule),
                               upload_tokens(x, "bf16"), i32(off), i32(np.arange(B, dtype=np.int32)),
                               no_workspace=(schedule == 1))
        torch.cuda.synchronize()
        yn = y.float().cpu().numpy().astype(np.float64)
        for b in range(B):
            assert_close(yn[b:b + 1], Yo[b:b + 1], TOL_BF16, f"schedule {schedule} sequence {b}")


def test_decode_unselected_groups_are_not_needed():
    say("decode: factors of groups nobody selected may hold anything (they are never read into the result)")
    lay = si.small_layer(603, 512, 512, 256, 8, "bf16")
    pats = np.array([[0, 3], [3, 6]], np.int32)
    seq_pat = np.array([0, 1, 1, 0, 5], np.int32)             # sequence 4: invalid pattern -> zero row
    x = si.make_tokens(np.random.default_rng(2), 5, 512, "bf16")
    poisoned = si.Layer(lay.n, lay.m, lay.R, lay.G, "bf16", None, None, None, lay.Vt_store.copy(), lay.Ut_store.copy())
    for g in (1, 2, 4, 5, 7):
        poisoned.Vt_store[g * 32:(g + 1) * 32] = 0x7FC0        # NaN bit pattern
        poisoned.Ut_store[g * 32:(g + 1) * 32] = 0x7FC0
    outs = []
    for l in (lay, poisoned):
        dl = pa.layer_to_mfma16(upload_layer(l))
        outs.append(forward_guarded(pa.PARSE_DECODE, dl, pa.Patterns(2, 2, subsets=i32(pats)),
                                       upload_tokens(x, "bf16"), None, i32(seq_pat)))
    torch.cuda.synchronize()
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
    assert torch.all(outs[0][4] == 0) and torch.any(outs[0][0] != 0)


@pytest.mark.parametrize("shapes,n,B", [
    ([(1536, 640, 20, 10), (1536, 640, 20, 10)], 1024, 32),                      # gate/up-like pair
    ([(512, 256, 8, 3), (256, 128, 4, 2), (768, 256, 8, 4)], 512, 7),           # Q/K/V-like, different m, R, G, k
    ([(11008, 2560, 20, 10), (11008, 2560, 20, 10)], 4096, 32),                  # the decode workload's gate + up
    ([(4096, 1536, 16, 8), (4096, 1536, 16, 8), (4096, 1536, 16, 8)], 4096, 1),   # q/k/v of one sequence (small-batch kernel)
    ([(1536, 640, 20, 10), (768, 256, 8, 4)], 1024, 3),                           # three sequences, two different layers
])
def test_decode_multi_matches_oracle_and_single_calls(shapes, n, B):
    """Horizontal fusion (Sec. 4.4, Eq. 11-12): layers sharing x in one decode step = the separate steps."""
    say(f"decode_multi n={n} B={B} layers={shapes}")
    rng = np.random.default_rng(611)
    x = si.make_tokens(rng, B, n, "bf16")
    xd = upload_tokens(x, "bf16")
    npat = 4 if B >= 4 else 1
    seq_pat = (np.arange(B) % npat).astype(np.int32)
    layers, patterns, refs, rows_of = [], [], [], []
    for li, (m, R, G, k) in enumerate(shapes):
        lay = si.make_layer(np.random.default_rng(620 + li), n, m, R, G, "bf16", fast=(R > 1024))
        pats = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(npat)]).astype(np.int32)
        U0, sg, V = oracle_factors(lay)
        rows = np.arange(B) if R <= 1024 else np.array([0, B - 1])
        refs.append(po.decode_step(U0, sg, V, lay.gs, si.bf16_bits_to_f32(x[rows]).astype(np.float64), pats[seq_pat[rows]]))
        rows_of.append(rows)
        layers.append(pa.layer_to_mfma16(upload_layer(lay)))
        patterns.append(pa.Patterns(k, npat, subsets=i32(pats)))
    pid = i32(seq_pat)
    ys = decode_multi_guarded(layers, patterns, xd, pid)
    ys2 = decode_multi_guarded(layers, patterns, xd, pid)
    torch.cuda.synchronize()
    for li in range(len(shapes)):
        assert torch.equal(ys[li].view(torch.int16), ys2[li].view(torch.int16))
        yn = ys[li].float().cpu().numpy()
        for i, b in enumerate(rows_of[li]):
            assert_close(yn[b:b + 1], refs[li][i:i + 1], TOL_BF16, f"layer {li} sequence {b}")
        single = forward_guarded(pa.PARSE_DECODE, layers[li], patterns[li], xd, None, pid)
        torch.cuda.synchronize()
        assert_close(yn, single.float().cpu().numpy(), TOL_BF16, f"layer {li}: fused vs separate call")


@pytest.mark.parametrize("shapes,n,lengths", [
    ([(768, 256, 8, 4), (512, 256, 4, 2), (1024, 512, 4, 3)], 512, [70, 1, 33, 129, 64]),   # Q/K/V-like, ragged
    ([(1024, 1024, 8, 4), (1024, 1024, 8, 4)], 1024, [512, 300]),                            # gate/up-like
])
def test_prefill_multi_matches_oracle_and_single_calls(shapes, n, lengths):
    """Horizontal fusion (Sec. 4.4, Eq. 11-12): layers sharing X in two launches = the separate two-launch calls."""
    say(f"prefill_multi n={n} lengths={lengths} layers={shapes}")
    rng = np.random.default_rng(711)
    off = si.offsets_from_lengths(lengths)
    X = si.make_tokens(rng, int(off[-1]), n, "bf16")
    Xv = si.bf16_bits_to_f32(X).astype(np.float64)
    Xd, offd = upload_tokens(X, "bf16"), i32(off)
    P = len(lengths)
    pid = i32(np.arange(P, dtype=np.int32))
    layers, patterns, refs = [], [], []
    for li, (m, R, G, k) in enumerate(shapes):
        lay = si.small_layer(720 + li, n, m, R, G, "bf16")
        subs = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in lengths]).astype(np.int32)
        U0, sg, V = oracle_factors(lay)
        refs.append(po.forward(U0, sg, V, lay.gs, Xv, off, subs))
        dl = pa.layer_to_mfma16(upload_layer(lay))
        Vs, Us = pa.pack_patterns(dl, i32(subs), k, k, None, None, P)
        layers.append(dl)
        patterns.append(pa.Patterns(k, P, Vs, Us))
    # the fused call under each schedule it takes (default = planned when the queried workspace is given): against the
    # oracle, and bit for bit against the separate calls under the same schedule
    for schedule in (pa.PARSE_SCHED_AUTO, pa.PARSE_SCHED_PLANNED, pa.PARSE_SCHED_TILES):
        pats = [pt.with_schedule(schedule) for pt in patterns]
        ys = prefill_multi_guarded(layers, pats, Xd, offd, pid)
        torch.cuda.synchronize()
        same_as = pa.PARSE_SCHED_TILES if schedule == pa.PARSE_SCHED_TILES else pa.PARSE_SCHED_PLANNED
        for li in range(len(shapes)):
            yn = ys[li].float().cpu().numpy().astype(np.float64)
            for p in range(P):
                assert_close(yn[off[p]:off[p + 1]], refs[li][off[p]:off[p + 1]], TOL_BF16, f"schedule {schedule} layer {li} prompt {p}")
            single = forward_guarded(pa.PARSE_PREFILL, layers[li], patterns[li].with_schedule(same_as), Xd, offd, pid)
            torch.cuda.synchronize()
            assert torch.equal(single.view(torch.int16), ys[li].view(torch.int16)), f"schedule {schedule} layer {li}: fused vs separate call"


def test_shared_head_route_cache_pack_and_prefill():
    """Shared experts at the head of memory (Sec. 4.4): groups 0..n_shared-1 in every subset, stored once; the
    per-pattern blocks hold the rest.  Route and cache give the oracle's subsets; the product equals the oracle
    and is bit-identical to the same subsets packed whole."""
    say("shared head: route, cache route-on-miss, two-block pack, prefill")
    n, m, R, G, k, ns = 512, 768, 512, 8, 4, 2
    lengths = [70, 1, 200, 129]
    lay = si.small_layer(801, n, m, R, G, "bf16")
    rng = np.random.default_rng(802)
    off = si.offsets_from_lengths(lengths)
    X = si.make_tokens(rng, int(off[-1]), n, "bf16")
    Xv = si.bf16_bits_to_f32(X).astype(np.float64)
    Wr = (rng.standard_normal((1, G, n)) / np.sqrt(n)).astype(np.float32)
    E = po.pool(Xv, off)
    subs_ref, margin = po.route(E, Wr[0], k, n_shared=ns)
    assert np.all(margin > 1e-4 * np.abs(E @ Wr[0].T.astype(np.float64)).max())
    assert np.all(subs_ref[:, :ns] == np.arange(ns))
    Xd, offd, Wrd = upload_tokens(X, "bf16"), i32(off), torch.from_numpy(Wr).to(DEV)
    P = len(lengths)
    emb = torch.empty((P, n), dtype=torch.float32, device=DEV)
    subs = pa.route(Xd, offd, Wrd[0], k, emb_out=emb, n_shared=ns)
    torch.cuda.synchronize()
    assert np.array_equal(subs.cpu().numpy(), subs_ref)
    # the cache routes its misses the same way
    cache = pa.Cache(16, n, 1, k, P)
    cache.set_shared(ns)
    oc = po.PatternCache(16, n, 1, k, n_shared=ns)
    ent_ref, hit_ref, sub_ref = oc.lookup_or_route(E, 0.9, Wr.astype(np.float64))
    ent = torch.empty(P, dtype=torch.int32, device=DEV); hit = torch.empty(P, dtype=torch.uint8, device=DEV)
    sim = torch.empty(P, dtype=torch.float32, device=DEV); sub = torch.empty((P, 1, k), dtype=torch.int32, device=DEV)
    cache.lookup_or_route(emb, 0.9, Wrd, ent, hit, sim, sub)
    torch.cuda.synchronize()
    assert np.array_equal(ent.cpu().numpy(), ent_ref) and np.array_equal(hit.cpu().numpy(), hit_ref)
    assert np.array_equal(sub.cpu().numpy(), sub_ref)
    cache.close()
    # two-block pack: shared block once, per-pattern blocks with the other k - ns groups
    dl = pa.layer_to_mfma16(upload_layer(lay))
    sd = i32(subs_ref)
    Vsh, Ush = pa.pack_experts(dl, i32(np.arange(ns, dtype=np.int32)))
    Vp, Up = pa.pack_patterns(dl, sd[:, ns:], k, k - ns, None, None, P)
    Vw, Uw = pa.pack_patterns(dl, sd, k, k, None, None, P)
    torch.cuda.synchronize()
    gs = lay.gs
    for p in range(P):   # whole block = shared block followed by the pattern's own block (slabs stay contiguous)
        assert torch.equal(Vw[p, :ns * gs].view(torch.int16), Vsh.view(torch.int16))
        assert torch.equal(Vw[p, ns * gs:].view(torch.int16), Vp[p].view(torch.int16))
        assert torch.equal(Uw[p, ns * gs:].view(torch.int16), Up[p].view(torch.int16))
    pid = i32(np.arange(P, dtype=np.int32))
    y_sh = forward_guarded(pa.PARSE_PREFILL, dl, pa.Patterns(k, P, Vp, Up, Vt_shared=Vsh, Ut_shared=Ush, n_shared=ns,
                                                                 schedule=pa.PARSE_SCHED_TILES), Xd, offd, pid)
    y_whole = forward_guarded(pa.PARSE_PREFILL, dl, pa.Patterns(k, P, Vw, Uw, schedule=pa.PARSE_SCHED_TILES), Xd, offd, pid)
    torch.cuda.synchronize()
    assert torch.equal(y_sh.view(torch.int16), y_whole.view(torch.int16))
    U0, sg, V = oracle_factors(lay)
    Yref = po.forward(U0, sg, V, lay.gs, Xv, off, subs_ref)
    yn = y_sh.float().cpu().numpy().astype(np.float64)
    for p in range(P):
        assert_close(yn[off[p]:off[p + 1]], Yref[off[p]:off[p + 1]], TOL_BF16, f"prompt {p}")
    # the planned schedule reads the shared head the same way: bit-identical to the whole blocks under that schedule,
    # through the all-in-one call (fixed and automatic choice) and through the call that takes a ready plan
    pt_sh = pa.Patterns(k, P, Vp, Up, Vt_shared=Vsh, Ut_shared=Ush, n_shared=ns)
    y_pw = forward_guarded(pa.PARSE_PREFILL, dl, pa.Patterns(k, P, Vw, Uw, schedule=pa.PARSE_SCHED_PLANNED), Xd, offd, pid)
    y_ps = forward_guarded(pa.PARSE_PREFILL, dl, pt_sh.with_schedule(pa.PARSE_SCHED_PLANNED), Xd, offd, pid)
    y_auto = forward_guarded(pa.PARSE_PREFILL, dl, pt_sh, Xd, offd, pid)
    plan = pa.prefill_plan(offd, pid, int(off[-1]), P)
    y_plan = pa.lowrank_prefill_planned(dl, pt_sh, Xd, offd, pid, plan)
    torch.cuda.synchronize()
    for nm, y in (("planned", y_ps), ("auto", y_auto), ("ready plan", y_plan)):
        assert torch.equal(y.view(torch.int16), y_pw.view(torch.int16)), nm
    ypn = y_ps.float().cpu().numpy().astype(np.float64)
    for p in range(P):
        assert_close(ypn[off[p]:off[p + 1]], Yref[off[p]:off[p + 1]], TOL_BF16, f"planned, prompt {p}")
    # the fused kernel reads one block per pattern: a shared head is refused there, not silently ignored
    with pytest.raises(pa.ParseError):
        forward_guarded(pa.PARSE_PREFILL, dl, pt_sh, Xd, offd, pid, no_workspace=True)
    with pytest.raises(pa.ParseError):
        forward_guarded(pa.PARSE_PREFILL, dl, pt_sh.with_schedule(pa.PARSE_SCHED_FUSED), Xd, offd, pid)


def test_shared_head_planned_on_the_large_tile_path():
    """A batch long enough for the 256 x 256 tiles of both products (24576 rows), one shared group of 128 ranks at
    the head of every pattern: bit-identical to the same subsets packed whole, sampled rows against the oracle."""
    say("shared head, planned schedule, 6 x 4096 tokens (large tiles in both products)")
    n, m, R, G, k, ns, P, T = 1024, 1024, 1024, 8, 4, 1, 6, 4096
    lay = si.make_layer(np.random.default_rng(811), n, m, R, G, "bf16", fast=True)
    rng = np.random.default_rng(812)
    off = si.offsets_from_lengths([T] * P)
    X = si.make_tokens(rng, P * T, n, "bf16")
    subs = np.stack([np.concatenate([[0], np.sort(rng.choice(np.arange(1, G), size=k - 1, replace=False))])
                     for _ in range(P)]).astype(np.int32)
    dl = pa.layer_to_mfma16(upload_layer(lay))
    sd = i32(subs)
    Vsh, Ush = pa.pack_experts(dl, i32(np.arange(ns, dtype=np.int32)))
    Vp, Up = pa.pack_patterns(dl, sd[:, ns:], k, k - ns, None, None, P)
    Vw, Uw = pa.pack_patterns(dl, sd, k, k, None, None, P)
    Xd, offd, pid = upload_tokens(X, "bf16"), i32(off), i32(np.arange(P, dtype=np.int32))
    y_sh = forward_guarded(pa.PARSE_PREFILL, dl, pa.Patterns(k, P, Vp, Up, Vt_shared=Vsh, Ut_shared=Ush, n_shared=ns,
                                                                 schedule=pa.PARSE_SCHED_PLANNED), Xd, offd, pid)
    y_w = forward_guarded(pa.PARSE_PREFILL, dl, pa.Patterns(k, P, Vw, Uw, schedule=pa.PARSE_SCHED_PLANNED), Xd, offd, pid)
    torch.cuda.synchronize()
    assert torch.equal(y_sh.view(torch.int16), y_w.view(torch.int16))
    U0, sg, V = oracle_factors(lay)
    yn = y_sh.float().cpu().numpy().astype(np.float64)
    for p in range(P):
        rows = np.sort(rng.choice(T, size=6, replace=False)) + p * T
        rows[0], rows[-1] = p * T, (p + 1) * T - 1              # first and last row of the prompt
        Yo = po.forward(U0, sg, V, lay.gs, si.bf16_bits_to_f32(X[rows]).astype(np.float64),
                        np.array([0, len(rows)], np.int32), subs[p:p + 1])
        assert_close(yn[rows], Yo, TOL_BF16, f"prompt {p}")


def test_rank_granular_route_pack_and_prefill():
    """The paper's own formulation (Sec. 4.1, Eq. 4-5): one expert per rank, router R^d -> R^R, top-K ranks;
    the K scattered rank rows are aggregated into one block (Sec. 4.4) and the prefill kernels run on it."""
    say("rank-granular: route_ranks (with exact ties), pack_ranks, prefill")
    n, m, R, K = 512, 768, 512, 256
    lengths = [70, 1, 200, 129, 33]
    lay = si.small_layer(901, n, m, R, R, "bf16")              # G = R: groups of one rank
    rng = np.random.default_rng(902)
    off = si.offsets_from_lengths(lengths)
    X = si.make_tokens(rng, int(off[-1]), n, "bf16")
    Xv = si.bf16_bits_to_f32(X).astype(np.float64)
    Wr = (rng.standard_normal((R, n)) / np.sqrt(n)).astype(np.float32)
    Wr[7] = Wr[300]; Wr[8] = Wr[300]; Wr[511] = Wr[0]          # exact ties: the lower rank id must win
    E = po.pool(Xv, off)
    S = E @ Wr.T.astype(np.float64)
    subs_ref = np.stack([po.topk_ascending(S[p], K)[0] for p in range(len(lengths))])
    # the decision margin of the fixed seed, apart from the planted ties (which fp32 reproduces exactly)
    for p in range(len(lengths)):
        srt = np.sort(S[p])[::-1]
        assert srt[K - 1] - srt[K] > 1e-6 or srt[K - 1] == srt[K]
    Xd, offd, Wrd = upload_tokens(X, "bf16"), i32(off), torch.from_numpy(Wr).to(DEV)
    P = len(lengths)
    scores = torch.empty((P, R), dtype=torch.float32, device=DEV)
    subs = pa.route_ranks(Xd, offd, Wrd, K, scores_out=scores)
    subs2 = pa.route_ranks(Xd, offd, Wrd, K)
    torch.cuda.synchronize()
    assert np.allclose(scores.cpu().numpy(), S, atol=2e-4 * np.abs(S).max())
    sg = subs.cpu().numpy()
    assert np.array_equal(sg, subs2.cpu().numpy())
    mism = [p for p in range(P) if not np.array_equal(sg[p], subs_ref[p])]
    for p in mism:   # a near-tie at the cut may flip under fp32 scoring: accept only swaps within 1e-5 of the cut
        a, b = set(sg[p]) - set(subs_ref[p]), set(subs_ref[p]) - set(sg[p])
        cut = np.sort(S[p])[::-1][K - 1]
        assert len(a) == len(b) and all(abs(S[p][g] - cut) < 1e-5 * np.abs(S).max() for g in a | b), f"prompt {p}"
    assert all(list(r) == sorted(set(r)) for r in sg)
    # gather + reorder against the oracle's row gather pushed through the documented layout map
    dl = upload_layer(lay)                                     # row-major bf16
    sd = i32(sg)
    Vs, Us = pa.pack_ranks(dl, sd, K, P)
    torch.cuda.synchronize()
    for p in range(P):
        Vref, Uref = po.pack(lay.Vt_store, lay.Ut_store, sg[p], 1)
        assert np.array_equal(Vs[p].view(torch.int16).cpu().numpy().view(np.uint16), mfma16_v(Vref))
        assert np.array_equal(Us[p].view(torch.int16).cpu().numpy().view(np.uint16), mfma16_u(Uref))
    # prefill on the aggregated blocks: the layer is described in 32-rank units
    desc = pa.Layer(dl.Vt, dl.Ut, n, m, R, R // 32, pa.PARSE_MFMA16)
    pid = i32(np.arange(P, dtype=np.int32))
    U0, sgm, V = oracle_factors(lay)
    Yref = po.forward(U0, sgm, V, 1, Xv, off, sg)
    for schedule in (1, 2, 3):
        y = forward_guarded(pa.PARSE_PREFILL, desc, pa.Patterns(K // 32, P, Vs, Us, schedule=schedule), Xd, offd, pid,
                               no_workspace=(schedule == 1))
        torch.cuda.synchronize()
        yn = y.float().cpu().numpy().astype(np.float64)
        for p in range(P):
            assert_close(yn[off[p]:off[p + 1]], Yref[off[p]:off[p + 1]], TOL_BF16, f"schedule {schedule} prompt {p}")


def test_config3_layer_projections_with_padded_groups():
    """One layer of the full-stack workload at its real shapes: q/k/v (4096x4096, 16 groups of 80 ranks padded to
    96), gate/up (4096->11008, groups of 112 padded to 128) and down, top-8 of 16; q/k/v and gate/up go through
    the horizontally fused calls.  Prefill on one 192-token prompt and one decode token, oracle on sampled rows."""
    say("config3 layer: q,k,v fused; gate,up fused; down; prefill (192 tokens) + decode (1 sequence)")
    hidden, inter, G, k, T = 4096, 11008, 16, 8, 192
    rng = np.random.default_rng(931)
    shapes = {"q": (hidden, hidden), "k": (hidden, hidden), "v": (hidden, hidden),
              "gate": (hidden, inter), "up": (hidden, inter), "down": (inter, hidden)}
    lays, dls, pats, subsets = {}, {}, {}, {}
    for i, (nm, (n, m)) in enumerate(shapes.items()):
        R, gs = si.config3_ranks(n, m, G)
        lay = si.pad_groups(si.make_layer(np.random.default_rng(940 + i), n, m, R, G, "bf16", fast=True), 32)
        assert lay.gs % 32 == 0
        sub = np.sort(rng.choice(G, size=k, replace=False)).astype(np.int32)[None, :]
        lays[nm], subsets[nm] = lay, sub
        dls[nm] = pa.layer_to_mfma16(upload_layer(lay))
        Vs, Us = pa.pack_patterns(dls[nm], i32(sub), k, k, None, None, 1)
        pats[nm] = pa.Patterns(k, 1, Vs, Us, subsets=i32(sub))
    off = np.array([0, T], np.int32)
    pid = i32(np.zeros(1, np.int32))
    sample = np.array([0, 77, T - 1])

    def check(nm, y, Xbits, rows, what):
        U0, sg, V = oracle_factors(lays[nm])
        Xv = si.bf16_bits_to_f32(Xbits[rows]).astype(np.float64)
        ref = po.forward(U0, sg, V, lays[nm].gs, Xv, np.array([0, len(rows)], np.int32), subsets[nm])
        assert_close(y.float().cpu().numpy()[rows].astype(np.float64), ref, TOL_BF16, f"{what} {nm}")

    Xh = si.make_tokens(rng, T, hidden, "bf16"); Xi = si.make_tokens(rng, T, inter, "bf16")
    Xhd, Xid, offd = upload_tokens(Xh, "bf16"), upload_tokens(Xi, "bf16"), i32(off)
    for group, Xb, Xd in ((["q", "k", "v"], Xh, Xhd), (["gate", "up"], Xh, Xhd)):
        ys = prefill_multi_guarded([dls[g] for g in group], [pats[g] for g in group], Xd, offd, pid)
        torch.cuda.synchronize()
        for g, y in zip(group, ys):
            check(g, y, Xb, sample, "prefill")
    y = forward_guarded(pa.PARSE_PREFILL, dls["down"], pats["down"], Xid, offd, pid)
    torch.cuda.synchronize()
    check("down", y, Xi, sample, "prefill")
    # decode: one sequence, one token
    one = np.array([0])
    for group, Xb, Xd in ((["q", "k", "v"], Xh, Xhd), (["gate", "up"], Xh, Xhd)):
        ys = decode_multi_guarded([dls[g] for g in group], [pats[g] for g in group], Xd[:1].contiguous(), pid)
        torch.cuda.synchronize()
        for g, yv in zip(group, ys):
            check(g, yv, Xb, one, "decode")
    yv = forward_guarded(pa.PARSE_DECODE, dls["down"], pats["down"], Xid[:1].contiguous(), None, pid)
    torch.cuda.synchronize()
    check("down", yv, Xi, one, "decode")


def test_router_training_step_matches_oracle():
    """Sec. 4.2: loss and straight-through gradient of the router matrix for one batch, against the oracle on the
    same rounded inputs (bf16 factors, tokens and dense targets)."""
    say("router training step: loss and gradient of Wr")
    n, m, R, G, k, tau, eps = 512, 384, 256, 8, 3, 0.5, 1e-6
    lengths = [70, 1, 130]
    lay = si.small_layer(951, n, m, R, G, "bf16")
    rng = np.random.default_rng(952)
    off = si.offsets_from_lengths(lengths)
    X = si.make_tokens(rng, int(off[-1]), n, "bf16")
    Xv = si.bf16_bits_to_f32(X).astype(np.float64)
    Wd = rng.standard_normal((m, n)) / np.sqrt(n)
    Yd_bits = si.f32_to_bf16_bits((Xv @ Wd.T).astype(np.float32))
    Yd = si.bf16_bits_to_f32(Yd_bits).astype(np.float64)
    Wr = (rng.standard_normal((G, n)) / np.sqrt(n) * 4.0).astype(np.float32)
    U0, sg, V = oracle_factors(lay)
    loss_ref, grad_ref, dm_ref = po.router_grad(U0, sg, V, lay.gs, Xv, off, Yd, Wr.astype(np.float64), k, tau, eps)
    # GPU: route (embedding, scores, hard subset), routed output, then the training step
    P = len(lengths)
    dl_rm = upload_layer(lay)
    dl = pa.layer_to_mfma16(dl_rm)
    Xd, offd, Wrd = upload_tokens(X, "bf16"), i32(off), torch.from_numpy(Wr).to(DEV)
    emb = torch.empty((P, n), dtype=torch.float32, device=DEV)
    scores = torch.empty((P, G), dtype=torch.float32, device=DEV)
    subs = pa.route(Xd, offd, Wrd, k, scores_out=scores, emb_out=emb)
    Vs, Us = pa.pack_patterns(dl, subs, k, k, None, None, P)
    yhat = forward_guarded(pa.PARSE_PREFILL, dl, pa.Patterns(k, P, Vs, Us), Xd, offd, i32(np.arange(P, dtype=np.int32)))
    ydd = upload_tokens(Yd_bits, "bf16")
    loss, grad = pa.router_grad(dl, pa.rankmajor_left_factor(dl_rm), Xd, offd, yhat, ydd, emb, scores, k, tau, eps)
    loss2, grad2 = pa.router_grad(dl, pa.rankmajor_left_factor(dl_rm), Xd, offd, yhat, ydd, emb, scores, k, tau, eps)
    torch.cuda.synchronize()
    assert torch.equal(grad, grad2) and torch.equal(loss, loss2)
    assert np.allclose(loss.cpu().numpy(), loss_ref, rtol=1e-2)
    gg = grad.cpu().numpy().astype(np.float64)
    err = np.linalg.norm(gg - grad_ref) / np.linalg.norm(grad_ref)
    say(f"    gradient: fro {err:.3e} max {np.abs(gg - grad_ref).max() / np.abs(grad_ref).max():.3e}; "
        f"loss rel {np.abs(loss.cpu().numpy() - loss_ref).max() / np.abs(loss_ref).max():.3e}")
    assert err <= TOL_BF16, f"gradient relative error {err:.3e}"          # measured 2.7e-4 / 2.3e-4
    assert np.abs(gg - grad_ref).max() <= TOL_BF16 * np.abs(grad_ref).max()


def test_multi_calls_with_four_layers_and_a_shared_head():
    """Four layers in one decode call (different widths, one needing several column blocks per workgroup) and
    four layers in one prefill call of which one uses a shared head."""
    say("decode_multi x4 and prefill_multi x4 (one layer with a shared head)")
    n, B = 512, 32
    rng = np.random.default_rng(961)
    shapes = [(256, 128, 4, 2), (16384, 96, 3, 2), (768, 256, 8, 3), (512, 512, 4, 4)]     # (m, R, G, k)
    x = si.make_tokens(rng, B, n, "bf16")
    xd = upload_tokens(x, "bf16")
    seq_pat = (np.arange(B) % 3).astype(np.int32)
    layers, pats, refs = [], [], []
    for li, (m, R, G, k) in enumerate(shapes):
        lay = si.small_layer(970 + li, n, m, R, G, "bf16")
        sub = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(3)]).astype(np.int32)
        U0, sg, V = oracle_factors(lay)
        refs.append(po.decode_step(U0, sg, V, lay.gs, si.bf16_bits_to_f32(x).astype(np.float64), sub[seq_pat]))
        layers.append(pa.layer_to_mfma16(upload_layer(lay)))
        pats.append(pa.Patterns(k, 3, subsets=i32(sub)))
    ys = decode_multi_guarded(layers, pats, xd, i32(seq_pat))
    torch.cuda.synchronize()
    for li in range(4):
        assert_close(ys[li].float().cpu().numpy().astype(np.float64), refs[li], TOL_BF16, f"decode layer {li}")
    # prefill: four layers sharing X, layer 2 with a shared head of one group
    lengths = [130, 64, 7]
    off = si.offsets_from_lengths(lengths)
    X = si.make_tokens(rng, int(off[-1]), n, "bf16")
    Xv = si.bf16_bits_to_f32(X).astype(np.float64)
    Xd, offd = upload_tokens(X, "bf16"), i32(off)
    P = len(lengths)
    pshapes = [(256, 256, 2, 1), (768, 512, 4, 2), (512, 512, 4, 3), (1024, 256, 2, 2)]     # k*gs multiples of 128
    layers, pats, refs = [], [], []
    for li, (m, R, G, k) in enumerate(pshapes):
        lay = si.small_layer(980 + li, n, m, R, G, "bf16")
        ns = 1 if li == 2 else 0
        sub = np.stack([np.concatenate([np.arange(ns), ns + np.sort(rng.choice(G - ns, size=k - ns, replace=False))])
                        for _ in lengths]).astype(np.int32)
        U0, sg, V = oracle_factors(lay)
        refs.append(po.forward(U0, sg, V, lay.gs, Xv, off, sub))
        dl = pa.layer_to_mfma16(upload_layer(lay))
        sd = i32(sub)
        if ns:
            Vsh, Ush = pa.pack_experts(dl, i32(np.arange(ns, dtype=np.int32)))
            Vp, Up = pa.pack_patterns(dl, sd[:, ns:], k, k - ns, None, None, P)
            pats.append(pa.Patterns(k, P, Vp, Up, Vt_shared=Vsh, Ut_shared=Ush, n_shared=ns))
        else:
            Vp, Up = pa.pack_patterns(dl, sd, k, k, None, None, P)
            pats.append(pa.Patterns(k, P, Vp, Up))
        layers.append(dl)
    for schedule in (pa.PARSE_SCHED_AUTO, pa.PARSE_SCHED_TILES):       # planned (the default here) and two-launch
        ys = prefill_multi_guarded(layers, [pt.with_schedule(schedule) for pt in pats], Xd, offd, i32(np.arange(P, dtype=np.int32)))
        torch.cuda.synchronize()
        for li in range(4):
            yn = ys[li].float().cpu().numpy().astype(np.float64)
            for p in range(P):
                assert_close(yn[off[p]:off[p + 1]], refs[li][off[p]:off[p + 1]], TOL_BF16,
                             f"prefill schedule {schedule} layer {li} prompt {p}")


def test_rank_router_at_its_limits():
    """8192 ranks (the selection kernel's limit), 40 prompts (five scoring blocks), K = 32."""
    say("route_ranks: G=8192, P=40, K=32")
    d, G, K, P = 256, 8192, 32, 40
    rng = np.random.default_rng(991)
    E = rng.standard_normal((P, d)).astype(np.float32)
    Wr = (rng.standard_normal((G, d)) / np.sqrt(d)).astype(np.float32)
    S = E.astype(np.float64) @ Wr.T.astype(np.float64)
    ref = np.stack([po.topk_ascending(S[p], K)[0] for p in range(P)])
    off = i32(np.arange(P + 1, dtype=np.int32))            # ready-made embeddings: prompts of length 1
    subs = pa.route_ranks(torch.from_numpy(E).to(DEV), off, torch.from_numpy(Wr).to(DEV), K)
    torch.cuda.synchronize()
    sg = subs.cpu().numpy()
    for p in range(P):
        if not np.array_equal(sg[p], ref[p]):             # only a swap at a near-tie of the cut is acceptable
            a, b = set(sg[p]) - set(ref[p]), set(ref[p]) - set(sg[p])
            cut = np.sort(S[p])[::-1][K - 1]
            assert len(a) == len(b) and all(abs(S[p][g] - cut) < 1e-5 * np.abs(S).max() for g in a | b), f"prompt {p}"
        assert list(sg[p]) == sorted(set(sg[p]))
