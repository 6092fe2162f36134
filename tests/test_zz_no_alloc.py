"""The decode entry point that allocates nothing (parse_lowrank_decode_static) against the ordinary decode call
(parse_lowrank_forward, PARSE_DECODE, caller's workspace): same kernels, so the outputs must be bit-identical, on
two calls in a row of which the second is smaller (the fixed scratch array keeps the first call's contents), and
against the CPU oracle within the bf16 tolerance."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import parse_oracle as po

pytestmark = pytest.mark.gpu

pa = pytest.importorskip("paper_2605_08568_amd")
from helpers import i32, oracle_factors, upload_layer, upload_tokens  # noqa: E402

DEV = "cuda"


def _case(n, m, R, G, k, B, npat, seed):
    lay = si.make_layer(np.random.default_rng(seed), n, m, R, G, "bf16", fast=(R > 1024))
    rng = np.random.default_rng(seed + 1)
    pats = np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(npat)]).astype(np.int32)
    seq_pat = (np.arange(B) % npat).astype(np.int32)
    x = si.make_tokens(rng, B, n, "bf16")
    dl = pa.layer_to_mfma16(upload_layer(lay))
    return lay, pats, seq_pat, x, dl


def test_decode_static_matches_decode_with_workspace_twice_in_a_row():
    print("decode without allocation: large call, then a smaller call on the same scratch array", flush=True)
    cases = [(1024, 1536, 640, 20, 10, 32, 4, 9101), (512, 256, 256, 8, 3, 5, 2, 9103)]
    for n, m, R, G, k, B, npat, seed in cases:
        print(f"  n={n} m={m} R={R} G={G} k={k} B={B}", flush=True)
        lay, pats, seq_pat, x, dl = _case(n, m, R, G, k, B, npat, seed)
        xd, pid, subs = upload_tokens(x, "bf16"), i32(seq_pat), i32(pats)
        pt = pa.Patterns(k, npat, subsets=subs)
        y_ref = pa.lowrank_forward(pa.PARSE_DECODE, dl, pt, xd, None, pid)
        y = torch.full((B, m), 7.0, dtype=torch.bfloat16, device=DEV)      # caller-owned output
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        pa.lowrank_decode_static(dl, pt, xd, pid, y)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), "differs from the call with a workspace"
        U0, sg, V = oracle_factors(lay)
        Yo = po.decode_step(U0, sg, V, lay.gs, si.bf16_bits_to_f32(x).astype(np.float64), pats[seq_pat])
        fro, mx = po.rel_errors(y.float().cpu().numpy(), Yo)
        print(f"    vs oracle: fro {fro:.2e} max {mx:.2e}", flush=True)
        assert fro <= 1e-2 and mx <= 1e-2


def test_decode_static_rejects_a_layer_beyond_its_capacity():
    cap = int(pa.lib().parse_lowrank_decode_static_capacity())
    assert cap == 4 << 20
    # 64 bytes of scratch per stored rank, 128 more per stored rank and slice of the reduction (two slices at n = 8192),
    # and the plan: 5 MiB, beyond the fixed array
    R, G, n = 16384, 64, 8192
    Vt = torch.zeros((R, n), dtype=torch.bfloat16, device=DEV); Ut = torch.zeros((R, 256), dtype=torch.bfloat16, device=DEV)
    big = pa.Layer(Vt, Ut, n, 256, R, G, pa.PARSE_MFMA16)
    assert pa.lowrank_workspace_bytes(pa.PARSE_DECODE, big, 4, 2) > cap
    pt = pa.Patterns(2, 1, subsets=i32(np.array([[0, 1]], np.int32)))
    x = torch.zeros((4, n), dtype=torch.bfloat16, device=DEV); y = torch.full((4, 256), 3.0, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(pa.ParseError) as ei:
        pa.lowrank_decode_static(big, pt, x, i32(np.zeros(4, np.int32)), y)
    assert ei.value.status == -5
    torch.cuda.synchronize()
    assert torch.all(y == 3.0)     # nothing was launched
