"""sv_attn_decode_static (split-KV scratch in a fixed device array inside the library, no allocation) against
sv_attn_decode (scratch in the caller's arena): two calls in a row through the C ABI, the second on a smaller
input, so that whatever the first call left in the shared array must not leak into the second."""
import numpy as np
import pytest
import torch

import paper_2510_09608_amd as sv
import sv_inputs as si
from oracle import sv_oracle as orc
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
HQ, HKV, D = 28, 4, 128


def _bf(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV).to(torch.bfloat16)


def test_static_scratch_decode_matches_arena_decode_twice():
    lens = [9000, 777, 4100, 33, 2600, 5392, 1, 6111]
    S = len(lens)
    print(f"static-scratch decode: {S} streams, lengths {lens}", flush=True)
    cache = sv.Cache(1, HQ, HKV, D, sv.SV_DTYPE_BF16, sv.SV_ROPE_NONE, 1e6, (0, 0, 0), S, max(lens) + 8, 16)
    ks, vs = [], []
    for s_, n in enumerate(lens):
        gids = np.arange(n)
        k = si.normal(40 + s_, si.TENSOR_K, 0, gids, HKV, D, True)
        v = si.normal(40 + s_, si.TENSOR_V, 0, gids, HKV, D, True)
        cache.append(s_, 0, np.zeros(n, dtype=np.uint8), None, _bf(k), _bf(v))
        ks.append(k), vs.append(v)
    q = si.normal(39, si.TENSOR_Q, 0, np.arange(S), HQ, D, True)
    qd = _bf(q)

    def both(ids):
        sel = qd[ids].contiguous()
        o_arena, o_static = torch.empty_like(sel), torch.full_like(sel, float("nan"))
        cache.attn_decode(0, ids, sel, o_arena)
        cache.attn_decode_static(0, ids, sel, o_static)
        torch.cuda.synchronize()
        a, b = gu.host(o_arena), gu.host(o_static)
        assert np.isfinite(b).all()
        assert gu.max_err(b, a) <= gu.TOL["bf16"]
        for j, s_ in enumerate(ids):                       # and against the oracle itself
            n = lens[s_]
            ref = orc.gqa_attention(q[s_:s_ + 1].astype(np.float64), ks[s_].astype(np.float64),
                                    vs[s_].astype(np.float64), np.array([n - 1]), True)
            assert gu.max_err(b[j:j + 1], ref) <= gu.TOL["bf16"], (s_, n)
        return float(np.abs(a - b).max())

    d1 = both(list(range(S)))            # 8 rows, up to 9000 keys: many key ranges per row
    d2 = both([3, 6, 1])                 # 3 short rows right after: fewer ranges, most of the array untouched
    d3 = both([0])                       # one row: the instantiation that merges its key ranges inside the launch
    d4 = both([4])                       # and a shorter one right after it
    print(f"  largest difference to the arena-scratch call: {d1:.3e}, {d2:.3e}, {d3:.3e}, {d4:.3e}", flush=True)

    # limits: too many rows for the array is an error, not a silent clamp
    ids = np.zeros(65, dtype=np.int32)
    big = torch.zeros(65, HQ, D, device=DEV, dtype=torch.bfloat16)
    with pytest.raises(sv.SvError) as e:
        cache.attn_decode_static(0, ids, big, torch.empty_like(big))
    assert e.value.status == -2
    # the generic-kernel configuration has no static-scratch variant
    c2 = sv.Cache(1, 2, 1, 64, sv.SV_DTYPE_F32, sv.SV_ROPE_NONE, 1e4, (0, 0, 0), 1, 16, 16)
    z = torch.zeros(4, 1, 64, device=DEV)
    c2.append(0, 0, np.zeros(4, dtype=np.uint8), None, z, z)
    with pytest.raises(sv.SvError) as e:
        c2.attn_decode_static(0, [0], torch.zeros(1, 2, 64, device=DEV), torch.zeros(1, 2, 64, device=DEV))
    assert e.value.status == -5


def test_static_scratch_decode_replayed_from_a_graph():
    """What the static-scratch call is for: captured once into a graph (nothing in it allocates), replayed several
    times with eager work of the library and synchronisations between the replays; every replay must give the eager
    call's result bit for bit (one row, whose key ranges meet inside the launch through words that the launch itself
    sets back to zero; and a batch of rows with its merge launch)."""
    lens = [6000, 1300, 2500]
    S = len(lens)
    cache = sv.Cache(1, HQ, HKV, D, sv.SV_DTYPE_BF16, sv.SV_ROPE_NONE, 1e6, (0, 0, 0), S, max(lens) + 8, 16)
    for s_, n in enumerate(lens):
        gids = np.arange(n)
        cache.append(s_, 0, np.zeros(n, dtype=np.uint8), None, _bf(si.normal(70 + s_, si.TENSOR_K, 0, gids, HKV, D, True)),
                     _bf(si.normal(70 + s_, si.TENSOR_V, 0, gids, HKV, D, True)))
    qd = _bf(si.normal(69, si.TENSOR_Q, 0, np.arange(S), HQ, D, True))
    for ids in ([0], [0, 1, 2]):
        print(f"static-scratch decode under graph replay: rows {ids}", flush=True)
        sel = qd[ids].contiguous()
        o_eager = torch.empty_like(sel)
        cache.attn_decode_static(0, ids, sel, o_eager)
        torch.cuda.synchronize()
        o_graph = torch.full_like(sel, float("nan"))
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            cache.attn_decode_static(0, ids, sel, o_graph)
        torch.cuda.synchronize()
        other = torch.empty_like(qd)
        for replay in range(4):
            o_graph.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(o_graph, o_eager), (ids, replay)
            # eager work of the library between the replays: other rows through both scratch regions
            cache.attn_decode_static(0, [1], qd[1:2].contiguous(), other[1:2])
            cache.attn_decode(0, list(range(S)), qd, other)
            torch.cuda.synchronize()
    cache.close()
