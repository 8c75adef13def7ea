"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without a GPU.

Each test is chosen so that a plausible mistake in the oracle (a dropped term,
a wrong sign or index, a transposed operand, an off-by-one in positions or in
the mask) makes at least one of them fail.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle.toy import ToyModel
from helpers import rope_complex, sdpa_causal, sdpa_masked

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(path):
    with open(os.path.join(GOLDEN, path)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- layout (Sec. 3.3, 3.2.3)
def test_layout_printed_example():
    for row in _rows("layout_example.txt"):
        arrow = row.index("->")
        sizes = [int(x) for x in row[:arrow]]
        expect = int(row[arrow + 1])
        starts, span = oracle.layout(sizes + [7])
        assert starts[-1] == expect
        assert span == expect + 7
        assert starts[0] == 0 and starts[1] == sizes[0]


def test_layout_union_shares_start_and_spans_largest_child():
    # module(5), union{7, 3, 9}, module(4)
    starts, span = oracle.layout([5, 7, 3, 9, 4], [-1, 0, 0, 0, -1])
    assert starts == [5 * 0, 5, 5, 5, 5 + 9]
    assert span == 5 + 9 + 4
    # two unions back to back are distinct
    starts, span = oracle.layout([2, 6, 4, 1], [0, 0, 1, 1])
    assert starts == [0, 0, 6, 6] and span == 10


def test_layout_rejects_split_union_and_negative_size():
    with pytest.raises(ValueError):
        oracle.layout([1, 2, 3], [0, -1, 0])
    with pytest.raises(ValueError):
        oracle.layout([1, -2], [-1, -1])


def test_layout_brute_force_random_schemas():
    """Against a direct restatement: start = number of position IDs consumed by earlier entries."""
    rng = np.random.default_rng(7)
    for _ in range(50):
        n_groups = int(rng.integers(1, 8))
        sizes, uids, expect, cursor = [], [], [], 0
        for g in range(n_groups):
            if rng.random() < 0.5:
                s = int(rng.integers(0, 40))
                sizes.append(s); uids.append(-1); expect.append(cursor); cursor += s
            else:
                kids = [int(x) for x in rng.integers(0, 40, size=int(rng.integers(1, 4)))]
                for s in kids:
                    sizes.append(s); uids.append(g); expect.append(cursor)
                cursor += max(kids)
        starts, span = oracle.layout(sizes, uids)
        assert starts == expect and span == cursor


def test_text_positions_continue_after_preceding_module():
    # Sec. 3.4: text between A and B starts at A's concluding position
    a_start, a_len = 110, 40
    pos = oracle.text_positions(a_start, a_len, 5)
    assert pos.tolist() == [150, 151, 152, 153, 154]
    assert oracle.text_positions(0, 0, 3).tolist() == [0, 1, 2]


# ---------------------------------------------------------------- memory per token (Table 2)
def test_bytes_per_token_matches_table2():
    for name, layers, hidden, printed in _rows("table2_mb_per_token.txt"):
        b = oracle.bytes_per_token(int(layers), 1, int(hidden), 2)
        assert b == 2 * int(layers) * int(hidden) * 2
        mib = b / 2 ** 20
        decimals = len(printed.split(".")[1])
        cut = math.floor(mib * 10 ** decimals) / 10 ** decimals
        assert abs(cut - float(printed)) < 1e-9, (name, mib, printed)
    # Llama-7B-shaped attention (32 kv heads x 128) is exactly half a MiB per token
    assert oracle.bytes_per_token(32, 32, 128, 2) == 512 * 1024


# ---------------------------------------------------------------- RoPE (Sec. 3.3, 4.2)
def test_rope_closed_forms_fix_direction_pairing_and_frequency():
    # d = 2: theta_0 = 1.  (1, 0) at position 1 -> (cos 1, sin 1): counter-clockwise.
    y = oracle.rope(np.array([[[1.0, 0.0]]]), [1])
    assert np.allclose(y[0, 0], [math.cos(1.0), math.sin(1.0)], atol=1e-15)
    # d = 4, base 10000: theta_1 = 10000^(-2/4) = 0.01; element 1 pairs with element 3.
    y = oracle.rope(np.array([[[0.0, 1.0, 0.0, 0.0]]]), [100])
    assert np.allclose(y[0, 0], [0.0, math.cos(1.0), 0.0, math.sin(1.0)], atol=1e-13)
    # element 2 (upper half of pair 0) at position 2: (x0, x2) = (0, 1) -> (-sin 2, cos 2)
    y = oracle.rope(np.array([[[0.0, 0.0, 1.0, 0.0]]]), [2])
    assert np.allclose(y[0, 0], [-math.sin(2.0), 0.0, math.cos(2.0), 0.0], atol=1e-15)
    # another base
    y = oracle.rope(np.array([[[0.0, 1.0, 0.0, 0.0]]]), [3], base=100.0)
    assert np.allclose(y[0, 0], [0.0, math.cos(0.3), 0.0, math.sin(0.3)], atol=1e-13)


def test_rope_matches_complex_formulation_at_discontinuous_positions():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((9, 3, 64))
    pos = np.array([0, 1, 5, 110, 111, 4095, 8192, 16383, 7], dtype=np.int32)
    # theta_i computed two ways differs by ~1 ulp; times position 16383 that is ~2e-12 of angle
    assert np.allclose(oracle.rope(x, pos), rope_complex(x, pos), atol=1e-11, rtol=0)


def test_rope_identity_norm_and_additivity():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((6, 2, 32))
    assert np.array_equal(oracle.rope(x, np.zeros(6, dtype=np.int32)), x)
    p1 = np.array([3, 50, 0, 9, 1000, 77], dtype=np.int32)
    p2 = np.array([4, 60, 5, 0, 1234, 1], dtype=np.int32)
    y = oracle.rope(x, p1)
    half = 16
    assert np.allclose(y[..., :half] ** 2 + y[..., half:] ** 2, x[..., :half] ** 2 + x[..., half:] ** 2, atol=1e-12)
    assert np.allclose(oracle.rope(y, p2), oracle.rope(x, p1 + p2), atol=1e-11)


def test_rope_inner_product_depends_on_relative_position_only():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 1, 64)); k = rng.standard_normal((1, 1, 64))
    ref = float((oracle.rope(q, [300]) * oracle.rope(k, [120])).sum())
    for shift in (1, 77, 5000):
        got = float((oracle.rope(q, [300 + shift]) * oracle.rope(k, [120 + shift])).sum())
        assert abs(got - ref) < 1e-10


# ---------------------------------------------------------------- assembly (Sec. 3.4)
def test_assemble_is_packed_concat_with_schema_positions():
    rng = np.random.default_rng(3)
    sizes = [5, 3, 4]
    starts, _ = oracle.layout(sizes)
    K = [rng.integers(0, 2 ** 16, size=(n, 2, 4), dtype=np.uint16) for n in sizes]
    V = [rng.integers(0, 2 ** 16, size=(n, 2, 4), dtype=np.uint16) for n in sizes]
    # import modules 2 and 0 (1 omitted), listed in that order
    oK, oV, pos = oracle.assemble([K[2], K[0]], [V[2], V[0]], [starts[2], starts[0]])
    assert np.array_equal(oK, np.concatenate([K[2], K[0]]))
    assert np.array_equal(oV, np.concatenate([V[2], V[0]]))
    assert pos.tolist() == [8, 9, 10, 11, 0, 1, 2, 3, 4]
    assert oK.nbytes == (4 + 5) * 2 * 4 * 2


def test_omitting_a_module_leaves_other_positions_unchanged():
    sizes = [6, 10, 8]
    starts, _ = oracle.layout(sizes)
    z = [np.zeros((n, 1, 2), dtype=np.float32) for n in sizes]
    _, _, pos_all = oracle.assemble(z, z, starts)
    _, _, pos_02 = oracle.assemble([z[0], z[2]], [z[0], z[2]], [starts[0], starts[2]])
    assert pos_all.tolist() == list(range(24))
    # module 2 keeps 16..23 although module 1 is absent: a gap in the IDs, none in the buffer
    assert pos_02.tolist() == list(range(0, 6)) + list(range(16, 24))


def test_assemble_keeps_every_bit_pattern():
    words = np.arange(65536, dtype=np.uint16).reshape(64, 8, 128)   # includes NaNs, -0, denormals as bf16
    flipped = np.ascontiguousarray(~words)
    oK, oV, _ = oracle.assemble([words[:40], words[40:]], [flipped[:40], flipped[40:]], [0, 40])
    assert np.array_equal(oK.view(np.uint16), words)
    assert np.array_equal(oV.view(np.uint16), flipped)


# ---------------------------------------------------------------- attention (Sec. 3.4)
def _rand(rng, *shape):
    return rng.standard_normal(shape)


def test_attn_contiguous_positions_is_textbook_causal_attention():
    """All tokens 'uncached' at positions 0..n-1: must equal library causal attention."""
    rng = np.random.default_rng(10)
    n, H, d = 37, 3, 16
    Q, K, V = _rand(rng, n, H, d), _rand(rng, n, H, d), _rand(rng, n, H, d)
    pos = np.arange(n, dtype=np.int32)
    out = oracle.attn(Q, pos, oracle.rope(K, pos), V, pos)
    ref = sdpa_causal(rope_complex(Q, pos), rope_complex(K, pos), V)
    assert np.allclose(out, ref, atol=1e-12, rtol=0)


def test_attn_mask_is_on_positions_not_buffer_order_and_sees_gaps():
    """Shuffled buffer, discontinuous IDs, a query inside a gap: against library attention with an explicit mask."""
    rng = np.random.default_rng(11)
    H, d = 2, 32
    k_pos = np.concatenate([np.arange(0, 20), np.arange(100, 130), np.arange(50, 60)]).astype(np.int32)
    perm = rng.permutation(len(k_pos))
    k_pos = k_pos[perm]
    q_pos = np.array([25, 55, 129, 130, 4000, 0], dtype=np.int32)
    Q, K, V = _rand(rng, len(q_pos), H, d), _rand(rng, len(k_pos), H, d), _rand(rng, len(k_pos), H, d)
    out = oracle.attn(Q, q_pos, rope_complex(K, k_pos), V, k_pos)
    allow = k_pos[None, :] <= q_pos[:, None]
    ref = sdpa_masked(rope_complex(Q, q_pos), rope_complex(K, k_pos), V, allow)
    assert np.allclose(out, ref, atol=1e-12, rtol=0)


def test_attn_single_visible_key_returns_its_value():
    rng = np.random.default_rng(12)
    K, V = _rand(rng, 5, 1, 8), _rand(rng, 5, 1, 8)
    k_pos = np.array([9, 3, 7, 8, 10], dtype=np.int32)
    out = oracle.attn(_rand(rng, 1, 1, 8), [3], K, V, k_pos)
    assert np.allclose(out[0, 0], V[1, 0], atol=1e-15)


def test_attn_query_without_visible_key_is_zero():
    rng = np.random.default_rng(13)
    out = oracle.attn(_rand(rng, 2, 2, 8), [0, 5], _rand(rng, 3, 2, 8), _rand(rng, 3, 2, 8), [6, 7, 8])
    assert np.array_equal(out, np.zeros_like(out))
    out = oracle.attn(_rand(rng, 2, 2, 8), [0, 5], np.zeros((0, 2, 8)), np.zeros((0, 2, 8)), np.zeros(0, dtype=np.int32))
    assert np.array_equal(out, np.zeros_like(out))


def test_attn_identical_keys_average_the_visible_values():
    rng = np.random.default_rng(14)
    n = 12
    K = np.repeat(_rand(rng, 1, 2, 16), n, axis=0)
    V = _rand(rng, n, 2, 16)
    k_pos = np.arange(n, dtype=np.int32) * 3
    q_pos = np.array([0, 10, 33, 100], dtype=np.int32)
    out = oracle.attn(_rand(rng, 4, 4, 16), q_pos, K, V, k_pos)
    for i, qp in enumerate(q_pos):
        vis = k_pos <= qp
        for h in range(4):
            assert np.allclose(out[i, h], V[vis, h // 2].mean(axis=0), atol=1e-13)


def test_attn_scale_is_one_over_sqrt_d():
    """Two keys, hand-computed softmax: q=k0=(2,0,0,0) at position 0, k1=0 -> weights from s0 = 4/sqrt(4) = 2."""
    Q = np.array([[[2.0, 0, 0, 0]]]); K = np.array([[[2.0, 0, 0, 0]], [[0.0, 0, 0, 0]]])
    V = np.array([[[1.0, 0, 0, 0]], [[0.0, 1.0, 0, 0]]])
    out = oracle.attn(Q, [0], K, V, [0, 0])
    w0 = math.exp(2.0) / (math.exp(2.0) + 1.0)
    assert np.allclose(out[0, 0], [w0, 1 - w0, 0, 0], atol=1e-15)


def test_attn_rotates_queries_with_the_same_convention_as_keys():
    """q.k after rotation is cos((p_q - p_k) theta): d=2, unit vectors."""
    Q = np.array([[[1.0, 0.0]]]); Kraw = np.array([[[1.0, 0.0]], [[1.0, 0.0]]])
    k_pos = np.array([2, 5], dtype=np.int32)
    V = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    out = oracle.attn(Q, [6], oracle.rope(Kraw, k_pos), V, k_pos)
    s = np.array([math.cos(4.0), math.cos(1.0)]) / math.sqrt(2.0)
    w = np.exp(s) / np.exp(s).sum()
    assert np.allclose(out[0, 0], w, atol=1e-14)


def test_attn_permutation_of_modules_does_not_change_output():
    # Sec. 3.4: order of concatenation does not matter
    rng = np.random.default_rng(15)
    sizes = [7, 11, 5]
    starts, span = oracle.layout(sizes)
    K = [oracle.rope(_rand(rng, n, 2, 16), np.arange(s, s + n)) for n, s in zip(sizes, starts)]
    V = [_rand(rng, n, 2, 16) for n in sizes]
    Q = _rand(rng, 4, 4, 16); q_pos = np.arange(span, span + 4, dtype=np.int32)
    outs = []
    for order in ([0, 1, 2], [2, 0, 1], [1, 2, 0]):
        aK, aV, aP = oracle.assemble([K[i] for i in order], [V[i] for i in order], [starts[i] for i in order])
        outs.append(oracle.attn(Q, q_pos, aK, aV, aP))
    assert np.allclose(outs[0], outs[1], atol=1e-13) and np.allclose(outs[0], outs[2], atol=1e-13)


def test_attn_gqa_equals_mha_with_repeated_kv_heads():
    rng = np.random.default_rng(16)
    nq, nk, Hq, Hkv, d = 5, 23, 6, 2, 16
    Q, K, V = _rand(rng, nq, Hq, d), _rand(rng, nk, Hkv, d), _rand(rng, nk, Hkv, d)
    k_pos = np.arange(nk, dtype=np.int32); q_pos = np.arange(nk, nk + nq, dtype=np.int32)
    g = oracle.attn(Q, q_pos, K, V, k_pos)
    m = oracle.attn(Q, q_pos, np.repeat(K, Hq // Hkv, axis=1), np.repeat(V, Hq // Hkv, axis=1), k_pos)
    assert np.allclose(g, m, atol=1e-14)
    # and a head really reads kv head h // group: make kv head 1 special
    V2 = V.copy(); V2[:, 1] += 100.0
    g2 = oracle.attn(Q, q_pos, K, V2, k_pos)
    assert np.allclose(g2[:, :3], g[:, :3], atol=1e-12) and np.allclose(g2[:, 3:], g[:, 3:] + 100.0, atol=1e-10)


def test_attn_masked_slots_cannot_leak():
    rng = np.random.default_rng(17)
    nk = 20
    K, V = _rand(rng, nk, 1, 8), _rand(rng, nk, 1, 8)
    k_pos = np.arange(nk, dtype=np.int32) * 2
    Q = _rand(rng, 3, 1, 8); q_pos = np.array([7, 20, 39], dtype=np.int32)
    ref = oracle.attn(Q, q_pos, K, V, k_pos)
    Kp, Vp = K.copy(), V.copy()
    Vp[k_pos > 39] = 1e4; Kp[k_pos > 39] = np.nan
    got = oracle.attn(Q, q_pos, Kp, Vp, k_pos)
    assert np.allclose(got, ref, atol=1e-14)
    Vp = V.copy(); Vp[k_pos > 20] = 1e4
    got = oracle.attn(Q, q_pos, K, Vp, k_pos)
    assert np.allclose(got[:2], ref[:2], atol=1e-14) and not np.allclose(got[2], ref[2])


def test_attn_shift_of_all_positions_is_invisible():
    # Sec. 3.1: only relative positions matter
    rng = np.random.default_rng(18)
    Kraw, V, Q = _rand(rng, 30, 2, 32), _rand(rng, 30, 2, 32), _rand(rng, 4, 2, 32)
    k_pos = np.concatenate([np.arange(0, 10), np.arange(40, 60)]).astype(np.int32)
    q_pos = np.array([60, 61, 62, 63], dtype=np.int32)
    a = oracle.attn(Q, q_pos, oracle.rope(Kraw, k_pos), V, k_pos)
    b = oracle.attn(Q, q_pos + 777, oracle.rope(Kraw, k_pos + 777), V, k_pos + 777)
    assert np.allclose(a, b, atol=1e-10)


# ---------------------------------------------------------------- equivalence (Sec. 3.1, 3.3, 3.4)
def test_full_masked_reduces_to_causal_attention_for_one_module():
    rng = np.random.default_rng(20)
    n, H, d = 19, 2, 16
    Q, K, V = _rand(rng, n, H, d), _rand(rng, n, H, d), _rand(rng, n, H, d)
    pos = np.arange(5, 5 + n, dtype=np.int32)
    out, K_enc = oracle.full_masked(Q, K, V, pos, np.zeros(n, dtype=np.int32))
    assert np.allclose(K_enc, rope_complex(K, pos), atol=1e-12)
    assert np.allclose(out, sdpa_causal(rope_complex(Q, pos), rope_complex(K, pos), V), atol=1e-12)


def test_cached_attention_equals_full_recompute_under_module_local_mask():
    """Brute force on a tiny prompt: 3 modules (one omitted), uncached text after them."""
    rng = np.random.default_rng(21)
    Hq, Hkv, d = 4, 2, 16
    sizes = [6, 9, 7]
    starts, span = oracle.layout(sizes)
    imported = [2, 0]                      # module 1 omitted; listed out of position order
    Kraw = {m: _rand(rng, sizes[m], Hkv, d) for m in imported}
    V = {m: _rand(rng, sizes[m], Hkv, d) for m in imported}
    Qm = {m: _rand(rng, sizes[m], Hq, d) for m in imported}
    n_new = 5
    q_pos = oracle.text_positions(starts[2], sizes[2], n_new)
    Qn, Kn, Vn = _rand(rng, n_new, Hq, d), _rand(rng, n_new, Hkv, d), _rand(rng, n_new, Hkv, d)
    # full sequence
    pos = np.concatenate([np.arange(starts[m], starts[m] + sizes[m]) for m in imported] + [q_pos]).astype(np.int32)
    mod = np.concatenate([np.full(sizes[m], m) for m in imported] + [np.full(n_new, -1)]).astype(np.int32)
    full_out, K_enc = oracle.full_masked(np.concatenate([Qm[m] for m in imported] + [Qn]),
                                         np.concatenate([Kraw[m] for m in imported] + [Kn]),
                                         np.concatenate([V[m] for m in imported] + [Vn]), pos, mod)
    # a reused module's K equals that module's K computed alone at its schema positions
    off = 0
    enc = {}
    for m in imported:
        enc[m] = oracle.rope(Kraw[m], np.arange(starts[m], starts[m] + sizes[m]))
        assert np.allclose(K_enc[off:off + sizes[m]], enc[m], atol=1e-13)
        off += sizes[m]
    # cached path
    aK, aV, aP = oracle.assemble([enc[m] for m in imported], [V[m] for m in imported], [starts[m] for m in imported])
    K_all = np.concatenate([aK, oracle.rope(Kn, q_pos)]); V_all = np.concatenate([aV, Vn])
    cached = oracle.attn(Qn, q_pos, K_all, V_all, np.concatenate([aP, q_pos]))
    assert np.allclose(cached, full_out[-n_new:], atol=1e-12)
    # module rows of the full pass equal the module attended alone
    alone, _ = oracle.full_masked(Qm[2], Kraw[2], V[2], np.arange(starts[2], starts[2] + sizes[2]), np.zeros(sizes[2], dtype=np.int32))
    assert np.allclose(full_out[:sizes[2]], alone, atol=1e-12)


@pytest.mark.parametrize("case", ["all", "omit_middle", "text_in_gap", "union_sibling"])
def test_toy_transformer_cached_equals_masked_full_pass(case):
    model = ToyModel(seed=5)
    rng = np.random.default_rng(30)
    if case == "union_sibling":
        sizes, uids = [6, 5, 9, 4], [-1, 0, 0, -1]
        imported = [0, 2, 3]
    else:
        sizes, uids = [6, 8, 5], [-1, -1, -1]
        imported = {"all": [0, 1, 2], "omit_middle": [2, 0], "text_in_gap": [0, 2]}[case]
    starts, span = oracle.layout(sizes, uids)
    toks = {m: rng.integers(0, 97, size=sizes[m]) for m in imported}
    last = max(imported, key=lambda m: starts[m] + sizes[m])
    new_pos = oracle.text_positions(starts[last], sizes[last], 4)
    if case == "text_in_gap":
        # three tokens right after module 0, inside the hole module 1 left
        new_pos = np.concatenate([oracle.text_positions(starts[0], sizes[0], 3), new_pos]).astype(np.int32)
    new_toks = rng.integers(0, 97, size=len(new_pos))
    # path A
    tokens = np.concatenate([toks[m] for m in imported] + [new_toks])
    pos = np.concatenate([np.arange(starts[m], starts[m] + sizes[m]) for m in imported] + [new_pos]).astype(np.int32)
    mod = np.concatenate([np.full(sizes[m], m) for m in imported] + [np.full(len(new_pos), -1)]).astype(np.int32)
    hA = model.forward_full_masked(tokens, pos, mod)[-len(new_pos):]
    # path B
    states = [model.encode_module(toks[m], starts[m]) for m in imported]
    hB = model.forward_cached(states, [starts[m] for m in imported], new_toks, new_pos)
    assert np.abs(hA - hB).max() < 1e-11
    assert np.abs(hA).max() > 0.1


def test_toy_transformer_detects_wrong_positions():
    """The pin has teeth: encoding a module at the wrong start breaks the equivalence."""
    model = ToyModel(seed=5)
    rng = np.random.default_rng(31)
    sizes = [6, 8]
    starts, _ = oracle.layout(sizes)
    toks = [rng.integers(0, 97, size=n) for n in sizes]
    new_pos = oracle.text_positions(starts[1], sizes[1], 3)
    new_toks = rng.integers(0, 97, size=3)
    tokens = np.concatenate(toks + [new_toks])
    pos = np.concatenate([np.arange(0, 6), np.arange(6, 14), new_pos]).astype(np.int32)
    mod = np.array([0] * 6 + [1] * 8 + [-1] * 3, dtype=np.int32)
    hA = model.forward_full_masked(tokens, pos, mod)[-3:]
    good = model.forward_cached([model.encode_module(toks[0], 0), model.encode_module(toks[1], 6)], [0, 6], new_toks, new_pos)
    bad = model.forward_cached([model.encode_module(toks[0], 0), model.encode_module(toks[1], 7)], [0, 6], new_toks, new_pos)
    assert np.abs(hA - good).max() < 1e-11
    assert np.abs(hA - bad).max() > 1e-4


# ---------------------------------------------------------------- cost model (Sec. 2.2, 5.4)
# ------------------------------------------------------------------ parameterised modules (Sec. 3.2.2, Sec. 3.3)
def _param_case(rng, n_arg, H=2, d=8, start=110, n_mod=12, off=5, plen=4, n_new=3):
    Kmod = rope_complex(rng.standard_normal((n_mod, H, d)), np.arange(start, start + n_mod))
    Vmod = rng.standard_normal((n_mod, H, d))
    K, V, P = oracle.assemble([Kmod], [Vmod], [start])
    Ka, Va = rng.standard_normal((n_arg, H, d)), rng.standard_normal((n_arg, H, d))
    Q = rng.standard_normal((n_new, H, d))
    q_pos = np.arange(start + n_mod, start + n_mod + n_new, dtype=np.int32)
    return K, V, P, Ka, Va, Q, q_pos, off, plen


def test_param_positions_follow_the_logged_placeholders():
    rng = np.random.default_rng(40)
    for line in open(os.path.join(GOLDEN, "param_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        lhs, rhs = line.split("->")
        start, off, plen, n_arg = (int(t) for t in lhs.split())
        want_pos = [int(t) for t in rhs.split("|")[0].split()]
        want_none = int(rhs.split("|")[1])
        K, V, P, Ka, Va, *_ = _param_case(rng, n_arg, start=start, off=off, plen=plen)
        K2, V2, P2 = oracle.fill_param(K, V, P, off, plen, Ka, Va)
        assert P2[off:off + n_arg].tolist() == want_pos
        assert int(np.sum(P2 == oracle.POS_NONE)) == want_none
        assert np.array_equal(np.delete(P2, np.s_[off + n_arg:off + plen]), np.delete(P, np.s_[off + n_arg:off + plen]))


def test_param_full_length_argument_equals_module_encoded_with_the_argument_in_place():
    rng = np.random.default_rng(41)
    K, V, P, Ka, Va, Q, q_pos, off, plen = _param_case(rng, 4)
    K2, V2, P2 = oracle.fill_param(K, V, P, off, plen, Ka, Va)
    # the module as it would have been encoded had the argument's tokens stood where the placeholders are
    K_ref, V_ref = K.copy(), V.copy()
    K_ref[off:off + plen] = rope_complex(Ka, P[off:off + plen])
    V_ref[off:off + plen] = Va
    assert np.allclose(K2, K_ref, rtol=0, atol=1e-12) and np.array_equal(V2, V_ref) and np.array_equal(P2, P)
    # rows outside the parameter are untouched, bit for bit
    keep = np.r_[0:off, off + plen:len(P)]
    assert np.array_equal(K2[keep], K[keep]) and np.array_equal(V2[keep], V[keep])


@pytest.mark.parametrize("n_arg", [0, 1, 3])
def test_param_shorter_argument_trailing_placeholders_stop_being_tokens(n_arg):
    """Attention over the filled buffer equals attention over the buffer with the unused placeholder rows cut out."""
    rng = np.random.default_rng(42 + n_arg)
    K, V, P, Ka, Va, Q, q_pos, off, plen = _param_case(rng, n_arg)
    K2, V2, P2 = oracle.fill_param(K, V, P, off, plen, Ka, Va)
    got = oracle.attn(Q, q_pos, K2, V2, P2)
    cut = np.s_[off + n_arg:off + plen]
    Kc, Vc, Pc = np.delete(K2, cut, axis=0), np.delete(V2, cut, axis=0), np.delete(P2, cut)
    assert not np.any(Pc == oracle.POS_NONE)
    # library attention on the shortened buffer (every remaining key precedes every query here)
    ref = sdpa_masked(rope_complex(Q, q_pos), Kc, Vc, np.ones((len(q_pos), len(Pc)), dtype=bool))
    assert np.allclose(got, ref, rtol=0, atol=1e-12)
    # and the placeholder states that were left behind cannot leak, whatever they hold
    V3 = V2.copy()
    V3[cut] = 1e6
    assert np.array_equal(oracle.attn(Q, q_pos, K2, V3, P2), got)


def test_param_argument_longer_than_parameter_is_rejected():
    rng = np.random.default_rng(46)
    K, V, P, Ka, Va, *_rest, off, plen = _param_case(rng, 5)
    with pytest.raises(ValueError):
        oracle.fill_param(K, V, P, off, plen, Ka, Va)


# ------------------------------------------------------------------ ALiBi at arbitrary position IDs (Sec. 4.2)
def test_alibi_slopes_match_the_published_sequence():
    for line in open(os.path.join(GOLDEN, "alibi_slopes.txt")).read().splitlines():
        if not line.strip() or line.startswith("#"):
            continue
        n, vals = line.split(":")
        want = [2.0 ** float(t[2:]) for t in vals.split()]
        got = oracle.alibi_slopes(int(n))
        assert got.shape == (int(n),)
        assert np.allclose(got, want, rtol=1e-15, atol=0)


def test_alibi_zero_queries_give_the_geometric_closed_form():
    """Q = 0 leaves only the bias: over positions 0..n-1 the last token's weights are r^(n-1-j) (1-r)/(1-r^n),
    r = exp(-slope); V = identity rows exposes the weights themselves."""
    n, H = 24, 4
    slopes = oracle.alibi_slopes(H)
    Q = np.zeros((1, H, n))
    K = np.random.default_rng(50).standard_normal((n, H, n))
    V = np.broadcast_to(np.eye(n)[:, None, :], (n, H, n)).copy()
    pos = np.arange(n, dtype=np.int32)
    out = oracle.attn_alibi(Q, pos[-1:], K, V, pos, slopes)
    for h in range(H):
        r = math.exp(-slopes[h])
        want = np.array([r ** (n - 1 - j) for j in range(n)]) * (1 - r) / (1 - r ** n)
        assert np.allclose(out[0, h], want, rtol=1e-12, atol=1e-15)


def test_alibi_distance_is_measured_in_position_ids_not_buffer_rows():
    """A module left out of the prompt (positions 3..9 missing) keeps its distance: weights follow 11 - pos."""
    H, slopes = 2, np.array([0.3, 0.05])
    k_pos = np.array([10, 11, 0, 1, 2], dtype=np.int32)          # buffer order differs from position order
    n = len(k_pos)
    V = np.broadcast_to(np.eye(n)[:, None, :], (n, H, n)).copy()
    out = oracle.attn_alibi(np.zeros((1, H, n)), np.array([11], dtype=np.int32), np.ones((n, H, n)), V, k_pos, slopes)
    for h in range(H):
        w = np.exp(-slopes[h] * (11 - k_pos))
        assert np.allclose(out[0, h], w / w.sum(), rtol=1e-12)
    # a key whose position lies after the query's is hidden
    out2 = oracle.attn_alibi(np.zeros((1, H, n)), np.array([10], dtype=np.int32), np.ones((n, H, n)), V, k_pos, slopes)
    assert np.all(out2[0, :, 1] == 0.0) and np.allclose(out2[0].sum(axis=-1), 1.0)


def test_alibi_matches_library_attention_with_an_additive_mask():
    """torch's scaled_dot_product_attention with a float mask -slope*(p_q - p_k) (and -inf where hidden), GQA
    expanded by hand, keys in shuffled buffer order, position IDs with gaps."""
    rng = np.random.default_rng(51)
    Hq, Hkv, d, nk, nq = 6, 2, 16, 40, 7
    slopes = oracle.alibi_slopes(Hq)
    k_pos = rng.permutation(np.r_[0:15, 30:45, 60:70]).astype(np.int32)
    q_pos = np.array([70, 71, 72, 20, 44, 5, 69], dtype=np.int32)
    Q, K, V = rng.standard_normal((nq, Hq, d)), rng.standard_normal((nk, Hkv, d)), rng.standard_normal((nk, Hkv, d))
    got = oracle.attn_alibi(Q, q_pos, K, V, k_pos, slopes)
    g = Hq // Hkv
    Kx, Vx = np.repeat(K, g, axis=1), np.repeat(V, g, axis=1)
    dist = (q_pos[:, None] - k_pos[None, :]).astype(np.float64)
    bias = np.where(dist >= 0, -slopes[:, None, None] * dist[None], -np.inf)          # [Hq, nq, nk]
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    ref = torch.nn.functional.scaled_dot_product_attention(t(Q).permute(1, 0, 2)[None], t(Kx).permute(1, 0, 2)[None],
                                                           t(Vx).permute(1, 0, 2)[None], attn_mask=t(bias)[None])
    ref = ref[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, ref, rtol=0, atol=1e-12)


def test_alibi_depends_on_position_differences_only_and_reduces_to_plain_attention():
    rng = np.random.default_rng(52)
    Hq, Hkv, d, nk, nq = 4, 4, 8, 12, 3
    Q, K, V = rng.standard_normal((nq, Hq, d)), rng.standard_normal((nk, Hkv, d)), rng.standard_normal((nk, Hkv, d))
    k_pos = np.arange(nk, dtype=np.int32) * 2
    q_pos = np.array([23, 24, 11], dtype=np.int32)
    slopes = oracle.alibi_slopes(Hq)
    a = oracle.attn_alibi(Q, q_pos, K, V, k_pos, slopes)
    b = oracle.attn_alibi(Q, q_pos + 1000, K, V, k_pos + 1000, slopes)
    assert np.allclose(a, b, rtol=0, atol=1e-13)
    # slope 0 at position 0 everywhere: no bias, nothing hidden, and the rotary path's rotation is the identity
    z = np.zeros(nk, dtype=np.int32)
    assert np.allclose(oracle.attn_alibi(Q, z[:nq], K, V, z, np.zeros(Hq)), oracle.attn(Q, z[:nq], K, V, z), rtol=0, atol=1e-13)
    # a steeper slope moves weight towards the nearest visible key (V = key index makes that measurable)
    Vi = np.broadcast_to(k_pos[:, None, None].astype(np.float64), (nk, Hkv, d)).copy()
    flat = oracle.attn_alibi(np.zeros((1, Hq, d)), q_pos[:1], K, Vi, k_pos, np.full(Hq, 0.01))
    steep = oracle.attn_alibi(np.zeros((1, Hq, d)), q_pos[:1], K, Vi, k_pos, np.full(Hq, 2.0))
    assert np.all(steep > flat) and np.all(steep <= 22.0)


# ------------------------------------------------------------------ scaffolding (Sec. 3.3)
def _parse_scaffolds(text):
    out = []
    for part in text.split("/"):
        m, o = part.strip().split(">")
        out.append(([int(t) for t in m.split(",")], [int(t) for t in o.split(",")]))
    return out


def test_scaffold_resolution_follows_the_worked_examples():
    for line in open(os.path.join(GOLDEN, "scaffold_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        imports, scaffolds, want = line.rstrip("\n").split(";")
        got = oracle.resolve_scaffolds([int(t) for t in imports.split()], _parse_scaffolds(scaffolds))
        assert got == [int(t) for t in want.split()], line


@pytest.mark.parametrize("case", ["adjacent", "module_between", "not_all_imported"])
def test_toy_transformer_scaffold_equals_pass_with_a_shared_span(case):
    """Serving with a scaffold's jointly encoded states equals ONE pass over the prompt in which the scaffold's
    members see each other (and every other module still sees only itself).  If a member is missing from the
    prompt, nothing is overridden and the ordinary module-local equivalence holds."""
    model = ToyModel(seed=6)
    rng = np.random.default_rng(60)
    sizes = [6, 7, 5, 4]
    starts, _ = oracle.layout(sizes)
    scaffold_members = {"adjacent": [0, 1], "module_between": [0, 2], "not_all_imported": [0, 3]}[case]
    imported = [0, 1, 2]
    toks = {m: rng.integers(0, 97, size=sizes[m]) for m in range(4)}
    own = {m: model.encode_module(toks[m], starts[m]) for m in range(4)}
    joint = model.encode_scaffold([(toks[m], starts[m]) for m in scaffold_members])
    store = dict(own)
    for m, st in zip(scaffold_members, joint):
        store[100 + m] = st
    resolved = oracle.resolve_scaffolds(imported, [(scaffold_members, [100 + m for m in scaffold_members])])
    assert (resolved != imported) == (case != "not_all_imported")
    new_pos = oracle.text_positions(starts[2], sizes[2], 4)
    new_toks = rng.integers(0, 97, size=4)
    start_of = lambda i: starts[i - 100] if i >= 100 else starts[i]
    hB = model.forward_cached([store[i] for i in resolved], [start_of(i) for i in resolved], new_toks, new_pos)
    # one pass: members of a complete scaffold share a span id
    span = {m: m for m in imported}
    if case != "not_all_imported":
        for m in scaffold_members:
            span[m] = 50
    tokens = np.concatenate([toks[m] for m in imported] + [new_toks])
    pos = np.concatenate([np.arange(starts[m], starts[m] + sizes[m]) for m in imported] + [new_pos]).astype(np.int32)
    mod = np.concatenate([np.full(sizes[m], span[m]) for m in imported] + [np.full(4, -1)]).astype(np.int32)
    hA = model.forward_full_masked(tokens, pos, mod)[-4:]
    assert np.abs(hA - hB).max() < 1e-11
    if case != "not_all_imported":   # and the override matters: the members' own states give something else
        hC = model.forward_cached([own[i] for i in imported], [starts[i] for i in imported], new_toks, new_pos)
        assert np.abs(hA - hC).max() > 1e-4
