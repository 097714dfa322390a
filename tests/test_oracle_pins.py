"""Pins for the CPU oracle: hand-worked fixtures, closed forms, brute force, invariants.

None of these call the HIP library.  Each check is written against what the
paper's rule or plain mathematics fixes, not against the oracle's own code;
`test_planted_mistakes_are_caught` then breaks the oracle in ten plausible ways
and requires that some pin notices each one.
"""
import cmath
import math

import numpy as np
import pytest

import sv_inputs as si
from oracle import sv_oracle as orc
from oracle import sv_step
from tests import golden_io as gio

TEXT, VISION = orc.TEXT, orc.VISION


# ----------------------------------------------------------------------------
# helpers that do not use the oracle
# ----------------------------------------------------------------------------

def brute_attention(q, k, v, q_slots, group, causal=True):
    """Softmax attention in pure Python loops (math.exp), one scalar at a time."""
    n, Hq, d = len(q), len(q[0]), len(q[0][0])
    N = len(k)
    out = [[[0.0] * d for _ in range(Hq)] for _ in range(n)]
    for a in range(n):
        for h in range(Hq):
            kv = h // group
            vis = [j for j in range(N) if (not causal) or j <= q_slots[a]]
            sc = []
            for j in vis:
                dot = 0.0
                for i in range(d):
                    dot += q[a][h][i] * k[j][kv][i]
                sc.append(dot / math.sqrt(d))
            m = max(sc)
            w = [math.exp(s - m) for s in sc]
            z = sum(w)
            for jj, j in enumerate(vis):
                for i in range(d):
                    out[a][h][i] += w[jj] / z * v[j][kv][i]
    return np.array(out)


def complex_rope_1d(x, p, theta):
    """1-D rotary embedding as complex multiplication: (x_i + j x_{i+d/2}) e^{j p theta^(-2i/d)}."""
    d = len(x)
    half = d // 2
    out = [0.0] * d
    for i in range(half):
        z = complex(x[i], x[i + half]) * cmath.exp(1j * p * theta ** (-2.0 * i / d))
        out[i], out[i + half] = z.real, z.imag
    return out


def rng_normal(seed, *shape):
    return np.random.Generator(np.random.Philox(seed)).standard_normal(shape)


def run_stream_meta(stream_ops, rope_mode=orc.ROPE_1D, d=8, sections=(0, 0, 0)):
    st = orc.OracleStream(1, 1, 1, d, rope_mode, 10000.0, sections)
    for op in stream_ops:
        ty = TEXT if op[0] == "text" else VISION
        n = int(op[1])
        grid = tuple(int(x) for x in op[2:5]) if len(op) >= 5 else None
        st.append_meta([ty] * n, grid)
        st.append_kv(0, np.zeros((n, 1, d)), np.zeros((n, 1, d)))
    return st


# ----------------------------------------------------------------------------
# eviction and positions against hand-worked fixtures
# ----------------------------------------------------------------------------

def check_golden_tiny_stream():
    g = gio.read_keyed("evict_tiny_stream.txt")
    w = si.workload_tiny()
    st = sv_step.new_stream(w, [0])
    lens = {int(r[0]): [int(x) for x in r[1:]] for r in g["len"]}
    for c in range(w.n_chunks):
        before = len(st)
        r = sv_step.step_chunk(st, w, c, [0], want_outputs=False)
        after_v = r["n_retained"] + w.vision_per_chunk
        assert [before, r["n_retained"], after_v, len(st)] == lens[c], c
        if c == 9:
            assert r["gids_after_evict"] == gio.expand_ranges(g["retained_at_chunk"][0][1:])
    st.evict(w.n_sink, w.vision_window, w.text_window)
    assert st.gid == gio.expand_ranges(g["retained_final"][0])
    assert st.positions()[:, 0].tolist() == list(range(56))


def check_golden_fig3_budgets():
    g = gio.read_keyed("evict_fig3_budgets.txt")
    ns, vw, tw = (int(x) for x in g["budgets"][0])
    for key_pairs, key_ret in (("pairs", "retained"), ("pairs_under_budget", "retained_under_budget")):
        st = orc.OracleStream(1, 1, 1, 4)
        for _ in range(int(g[key_pairs][0][0])):
            for ty in (VISION, TEXT):
                st.append_meta([ty])
                st.append_kv(0, np.zeros((1, 1, 4)), np.zeros((1, 1, 4)))
        st.evict(ns, vw, tw)
        assert st.gid == [int(x) for x in g[key_ret][0]]
        if key_ret == "retained":
            assert st.positions()[:, 0].tolist() == [int(x) for x in g["positions"][0]]


def check_golden_mrope_positions():
    g = gio.read_keyed("mrope_positions.txt")
    st = run_stream_meta(g["append"], orc.ROPE_3D, 8, (2, 1, 1))
    before = st.positions()
    assert [tuple(r) for r in before.tolist()] == gio.triples(g["pos_before"][0])
    assert st.next_position() == int(g["next_before"][0][0])
    old_gid = list(st.gid)
    ns, vw, tw = (int(x) for x in g["evict"][0])
    st.evict(ns, vw, tw)
    assert st.gid == [int(x) for x in g["retained_gids"][0]]
    after = st.positions()
    assert [tuple(r) for r in after.tolist()] == gio.triples(g["pos_after"][0])
    assert st.next_position() == int(g["next_after"][0][0])
    # the shift is one scalar per token: identical for t, h and w
    delta = [int(x) for x in g["delta"][0]]
    for j, gid in enumerate(st.gid):
        i = old_gid.index(gid)
        assert (before[i] - after[j]).tolist() == [delta[j]] * 3


def test_golden_tiny_stream():
    check_golden_tiny_stream()


def test_golden_fig3_budgets():
    check_golden_fig3_budgets()


def test_golden_mrope_positions():
    check_golden_mrope_positions()


# ----------------------------------------------------------------------------
# eviction invariants
# ----------------------------------------------------------------------------

def _random_stream(seed, n_ops=30):
    rng = np.random.Generator(np.random.Philox(seed))
    ops = []
    for _ in range(n_ops):
        if rng.random() < 0.5:
            ops.append(("text", int(rng.integers(1, 6))))
        else:
            T, H, W = (int(x) for x in rng.integers(1, 4, size=3))
            ops.append(("vision", T * H * W, T, H, W))
    return ops


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_incremental_equals_one_shot_and_idempotent(seed):
    ops = _random_stream(seed)
    budgets = (3, 11, 5)
    inc = orc.OracleStream(1, 1, 1, 8, orc.ROPE_3D, 1e4, (2, 1, 1))
    one = orc.OracleStream(1, 1, 1, 8, orc.ROPE_3D, 1e4, (2, 1, 1))
    seen = set()
    for op in ops:
        ty = TEXT if op[0] == "text" else VISION
        grid = tuple(op[2:5]) if len(op) == 5 else None
        prev = set(inc.gid)
        inc.evict(*budgets)
        assert set(inc.gid) <= prev                      # nothing evicted comes back
        seen |= prev - set(inc.gid)
        for s in (inc, one):
            s.append_meta([ty] * op[1], grid)
            s.append_kv(0, np.zeros((op[1], 1, 8)), np.zeros((op[1], 1, 8)))
        assert not (seen & set(inc.gid))
    inc.evict(*budgets)
    one.evict(*budgets)
    assert inc.gid == one.gid
    assert (inc.positions() == one.positions()).all()
    again = list(inc.gid)
    inc.evict(*budgets)
    assert inc.gid == again
    # counts: sink u window over text, window over vision (set arithmetic, not the keep loop)
    n_t = sum(1 for t in one.type if t == TEXT)
    n_v = len(one.gid) - n_t
    assert n_t == min(one.n_text, len(set(range(3)) | set(range(max(0, one.n_text - 5), one.n_text))))
    assert n_v == min(one.n_vis, 11)


def test_zero_and_infinite_budgets():
    ops = _random_stream(7)
    st = run_stream_meta(ops, orc.ROPE_3D, 8, (2, 1, 1))
    n_all, n_text = len(st), st.n_text
    st.evict(0, orc.INF, orc.INF)
    assert len(st) == n_all
    st.evict(0, 0, orc.INF)
    assert len(st) == n_text and all(t == TEXT for t in st.type)
    assert st.positions()[:, 0].tolist() == list(range(n_text))    # text only: contiguous scalars
    st.evict(2, 0, 0)
    assert st.rank == [0, 1]
    st.evict(0, 0, 0)
    assert len(st) == 0 and st.next_position() == 0


def test_positions_bounded_in_steady_state():
    """Positions stop growing once the stream is longer than the budgets (Sec. 2.1, Contiguous RoPE)."""
    w = si.workload_qwen_layer(n_chunks=70)
    st = orc.OracleStream(1, 1, 1, 2, orc.ROPE_3D, 1e6, (1, 0, 0))
    z = lambda n: np.zeros((n, 1, 2))
    st.append_meta([TEXT] * w.preamble_text)
    st.append_kv(0, z(w.preamble_text), z(w.preamble_text))
    maxima = []
    for c in range(w.n_chunks):
        st.evict(w.n_sink, w.vision_window, w.text_window)
        st.append_meta([VISION] * 256, (1, 16, 16))
        st.append_kv(0, z(256), z(256))
        st.append_meta([TEXT] * 16)
        st.append_kv(0, z(16), z(16))
        maxima.append(int(st.positions().max()))
        # scalar position sequence has no gaps: text tokens and block bases step by 1 / extent
    # 512 sink + 256 text whose vision is gone + 16 x (16 + 16) + (16 + 16) new = 1312 positions
    assert maxima[32:] == [1311] * (w.n_chunks - 32)
    assert len(st) == 512 + 512 + 4096 + 272


# ----------------------------------------------------------------------------
# RoPE
# ----------------------------------------------------------------------------

def check_rope_closed_forms():
    # d = 2: one pair, frequency theta^0 = 1 -> plane rotation by p radians
    for p in (0, 1, 5, 77):
        y = orc.rope(np.array([[[1.0, 0.0]]]), np.array([[p, p, p]]), orc.ROPE_1D, 1e4, (0, 0, 0))
        assert np.allclose(y[0, 0], [math.cos(p), math.sin(p)], atol=1e-14)
    # d = 4: pairs (0,2) and (1,3); second pair turns at theta^(-1/2)
    y = orc.rope(np.array([[[0.0, 1.0, 0.0, 0.0]]]), np.array([[3, 3, 3]]), orc.ROPE_1D, 100.0, (0, 0, 0))
    assert np.allclose(y[0, 0], [0.0, math.cos(0.3), 0.0, math.sin(0.3)], atol=1e-14)
    # general d against complex multiplication
    x = rng_normal(11, 5, 2, 16)
    pos = np.array([[p] * 3 for p in (0, 1, 7, 300, 1311)])
    y = orc.rope(x, pos, orc.ROPE_1D, 1e6, (0, 0, 0))
    for a in range(5):
        for h in range(2):
            assert np.allclose(y[a, h], complex_rope_1d(list(x[a, h]), int(pos[a, 0]), 1e6), atol=1e-12)
    assert np.array_equal(y[0], x[0])                                   # position 0 is the identity
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-12)


def check_rope_sections():
    d, sec = 16, (2, 3, 3)
    x = rng_normal(12, 1, 1, d)
    base = orc.rope(x, np.array([[4, 4, 4]]), orc.ROPE_3D, 1e4, sec)
    one_d = orc.rope(x, np.array([[4, 4, 4]]), orc.ROPE_1D, 1e4, (0, 0, 0))
    assert np.allclose(base, one_d, atol=1e-14)          # t = h = w reduces to 1-D RoPE
    half = d // 2
    spans = {0: range(0, 2), 1: range(2, 5), 2: range(5, 8)}
    for axis in range(3):
        p = np.array([[4, 4, 4]])
        p[0, axis] = 9
        y = orc.rope(x, p, orc.ROPE_3D, 1e4, sec)
        changed = {i for i in range(half) if not np.allclose(y[0, 0, [i, i + half]], base[0, 0, [i, i + half]])}
        assert changed == set(spans[axis]), (axis, changed)
        # and those pairs are turned exactly as 1-D RoPE at position 9 would turn them
        ref = orc.rope(x, np.array([[9, 9, 9]]), orc.ROPE_1D, 1e4, (0, 0, 0))
        for i in spans[axis]:
            assert np.allclose(y[0, 0, [i, i + half]], ref[0, 0, [i, i + half]], atol=1e-14)


def check_rope_relative_invariance():
    d, sec = 16, (2, 3, 3)
    q = rng_normal(13, 1, 1, d)
    k = rng_normal(14, 1, 1, d)
    pq, pk = np.array([[40, 37, 45]]), np.array([[12, 20, 3]])
    for mode in (orc.ROPE_1D, orc.ROPE_3D):
        s0 = (orc.rope(q, pq, mode, 1e6, sec) * orc.rope(k, pk, mode, 1e6, sec)).sum()
        for shift in (1, 17, 1000):
            s1 = (orc.rope(q, pq + shift, mode, 1e6, sec) * orc.rope(k, pk + shift, mode, 1e6, sec)).sum()
            assert abs(s0 - s1) < 1e-10
    # group law: turning by a then by b is turning by a + b
    x = rng_normal(15, 3, 2, d)
    pa, pb = np.array([[5, 6, 7]] * 3), np.array([[11, 2, 30]] * 3)
    two = orc.rope(orc.rope(x, pa, orc.ROPE_3D, 1e6, sec), pb, orc.ROPE_3D, 1e6, sec)
    assert np.allclose(two, orc.rope(x, pa + pb, orc.ROPE_3D, 1e6, sec), atol=1e-12)


def test_rope_closed_forms():
    check_rope_closed_forms()


def test_rope_sections():
    check_rope_sections()


def test_rope_relative_invariance():
    check_rope_relative_invariance()


# ----------------------------------------------------------------------------
# attention
# ----------------------------------------------------------------------------

def check_attention_brute_force():
    n, N, Hq, Hkv, d = 3, 9, 4, 2, 6
    q, k, v = rng_normal(21, n, Hq, d), rng_normal(22, N, Hkv, d), rng_normal(23, N, Hkv, d)
    slots = [4, 6, 8]
    for causal in (True, False):
        got = orc.gqa_attention(q, k, v, np.array(slots), causal)
        ref = brute_attention(q.tolist(), k.tolist(), v.tolist(), slots, Hq // Hkv, causal)
        assert np.allclose(got, ref, atol=1e-13), causal
    # grouped heads == plain multi-head attention on K, V repeated per group
    k_rep, v_rep = np.repeat(k, Hq // Hkv, axis=1), np.repeat(v, Hq // Hkv, axis=1)
    mha = orc.gqa_attention(q, k_rep, v_rep, np.array(slots), True)
    assert np.allclose(mha, orc.gqa_attention(q, k, v, np.array(slots), True), atol=1e-14)


def check_attention_closed_forms():
    n, N, Hq, Hkv, d = 2, 7, 2, 1, 4
    q = rng_normal(31, n, Hq, d)
    k = rng_normal(32, N, Hkv, d)
    slots = np.array([3, 6])
    v0 = rng_normal(33, 1, Hkv, d)
    out = orc.gqa_attention(q, k, np.repeat(v0, N, axis=0), slots, True)
    assert np.allclose(out, np.broadcast_to(v0[0, 0], out.shape), atol=1e-14)      # constant V
    v = rng_normal(34, N, Hkv, d)
    out = orc.gqa_attention(q, np.repeat(k[:1], N, axis=0), v, slots, True)          # equal keys -> mean of visible V
    assert np.allclose(out[0, 0], v[:4, 0].mean(axis=0), atol=1e-14)
    assert np.allclose(out[1, 1], v[:7, 0].mean(axis=0), atol=1e-14)
    out = orc.gqa_attention(q, k, v, np.array([0, 0]), True)                         # one visible key
    assert np.allclose(out, np.broadcast_to(v[0, 0], out.shape), atol=1e-14)
    kk = k.copy()
    kk[2, 0] = 200.0 * q[0, 0] / np.linalg.norm(q[0, 0])                             # one dominant key
    out = orc.gqa_attention(q[:1, :1], kk, v, np.array([6]), True)
    assert np.allclose(out[0, 0], v[2, 0], atol=1e-9)


def check_under_budget_is_full_causal_attention():
    """While nothing is evicted the stream step is plain causal attention over everything so far."""
    w = si.workload_tiny(n_chunks=3)
    st = sv_step.new_stream(w, [0])
    outs, gids = [], []
    for c in range(3):
        r = sv_step.step_chunk(st, w, c, [0])
        assert r["n_retained"] == 20 * c
        outs.append(r["prefill"][0])
        outs.extend(o[0] for o in r["decode"])
    got = np.concatenate(outs)                                    # [60, Hq, d] in arrival order
    q, k, v = w.qkv(0, np.arange(60))
    theta, d = w.rope_theta, w.head_dim
    qr = [[complex_rope_1d(list(map(float, q[t, h])), t, theta) for h in range(w.n_q_heads)] for t in range(60)]
    kr = [[complex_rope_1d(list(map(float, k[t, h])), t, theta) for h in range(w.n_kv_heads)] for t in range(60)]
    ref = brute_attention(qr, kr, v.astype(np.float64).tolist(), list(range(60)), w.n_q_heads // w.n_kv_heads)
    assert np.allclose(got, ref, atol=1e-12)


def check_position_shift_leaves_attention_unchanged():
    """After eviction only position differences matter: re-basing every position changes nothing."""
    w = si.workload_tiny(n_chunks=6)
    st = sv_step.new_stream(w, [0])
    for c in range(5):
        sv_step.step_chunk(st, w, c, [0], want_outputs=False)
    r = sv_step.step_chunk(st, w, 5, [0])
    n = len(st)
    K, V = np.stack(st.k[0]), np.stack(st.v[0])
    pos = st.positions() + 1234
    ch = w.chunk(5)
    q, _, _ = w.qkv(0, np.arange(ch.vision.gid0, ch.vision.gid0 + 16))
    slots = np.arange(n - 20, n - 4)
    qr = orc.rope(q, pos[slots], w.rope_mode, w.rope_theta, w.mrope_sections)
    kr = orc.rope(K, pos, w.rope_mode, w.rope_theta, w.mrope_sections)
    # decode tokens of this chunk sit after the vision chunk and are masked out for its queries
    out = orc.gqa_attention(qr, kr, V, slots, True)
    assert np.allclose(out, r["prefill"][0], atol=1e-11)


def test_attention_brute_force():
    check_attention_brute_force()


def test_attention_closed_forms():
    check_attention_closed_forms()


def test_under_budget_is_full_causal_attention():
    check_under_budget_is_full_causal_attention()


def test_position_shift_leaves_attention_unchanged():
    check_position_shift_leaves_attention_unchanged()


# ----------------------------------------------------------------------------
# planted mistakes: every mutant must trip at least one pin
# ----------------------------------------------------------------------------

ALL_CHECKS = [check_golden_tiny_stream, check_golden_fig3_budgets, check_golden_mrope_positions,
              check_rope_closed_forms, check_rope_sections, check_rope_relative_invariance,
              check_attention_brute_force, check_attention_closed_forms,
              check_under_budget_is_full_causal_attention]


def _mutants():
    real_rope, real_attn, real_angles, real_inv = orc.rope, orc.gqa_attention, orc.rope_angles, orc.inv_freq
    S = orc.OracleStream

    def rope_wrong_sign(x, pos, mode, theta, sec):
        return real_rope(x, -np.asarray(pos), mode, theta, sec)

    def rope_interleaved(x, pos, mode, theta, sec):
        x = np.asarray(x, dtype=np.float64)
        d = x.shape[-1]
        perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])
        inv = np.argsort(perm)
        return real_rope(x[..., perm], pos, mode, theta, sec)[..., inv]

    def inv_freq_half_exponent(d, theta):
        return np.float64(theta) ** (-1.0 * np.arange(d // 2) / d)

    def angles_sections_reversed(pos, d, mode, theta, sec):
        return real_angles(np.asarray(pos)[..., ::-1], d, mode, theta, tuple(sec)[::-1]) if mode == orc.ROPE_3D \
            else real_angles(pos, d, mode, theta, sec)

    def attn_no_scale(q, k, v, slots, causal=True):
        return real_attn(np.asarray(q) * math.sqrt(q.shape[-1]), k, v, slots, causal)

    def attn_strict_mask(q, k, v, slots, causal=True):
        return real_attn(q, k, v, np.maximum(np.asarray(slots) - 1, 0), causal)

    def attn_head_mod(q, k, v, slots, causal=True):
        Hq, Hkv = q.shape[1], k.shape[1]
        order = [(h % Hkv) * (Hq // Hkv) + h // Hkv for h in range(Hq)]
        out = real_attn(q[:, np.argsort(order)], k, v, slots, causal)
        return out[:, order]

    def keep_sink_any_type(self, ns, vw, tw):
        windows_only = S._real_keep(self, 0, vw, tw)
        return [f or g < ns for f, g in zip(windows_only, self.gid)]

    def keep_window_off_by_one(self, ns, vw, tw):
        return S._real_keep(self, ns, vw, tw if tw <= 0 else tw - 1)

    def positions_no_extent(self):
        saved = self.extent
        self.extent = [1] * len(saved)
        try:
            return S._real_positions(self)
        finally:
            self.extent = saved

    return [
        ("rope", rope_wrong_sign), ("rope", rope_interleaved), ("inv_freq", inv_freq_half_exponent),
        ("rope_angles", angles_sections_reversed), ("gqa_attention", attn_no_scale),
        ("gqa_attention", attn_strict_mask), ("gqa_attention", attn_head_mod),
        ("OracleStream.keep_flags", keep_sink_any_type), ("OracleStream.keep_flags", keep_window_off_by_one),
        ("OracleStream.positions", positions_no_extent),
    ]


def test_planted_mistakes_are_caught(monkeypatch):
    orc.OracleStream._real_keep = orc.OracleStream.keep_flags
    orc.OracleStream._real_positions = orc.OracleStream.positions
    try:
        for target, fn in _mutants():
            with monkeypatch.context() as m:
                if target.startswith("OracleStream."):
                    m.setattr(orc.OracleStream, target.split(".")[1], fn)
                else:
                    m.setattr(orc, target, fn)
                caught = False
                for chk in ALL_CHECKS:
                    try:
                        chk()
                    except AssertionError:
                        caught = True
                        break
                assert caught, f"no pin notices the planted mistake {fn.__name__}"
        for chk in ALL_CHECKS:       # and the real oracle passes them all again
            chk()
    finally:
        del orc.OracleStream._real_keep
        del orc.OracleStream._real_positions
