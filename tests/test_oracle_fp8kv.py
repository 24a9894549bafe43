"""Pins for the 8-bit (E4M3) K/V storage variant of the attention oracle (CPU only).

The paper leaves the K/V precision open, so this variant is the same definition on dequantised
values: a stored element stands for its kv head's scale times the value of its code.  The code
table is pinned to the format's published special values and to a library's conversion; the
attention on codes is pinned to the (separately pinned) attention on plain arrays and to an
independent sequential statement in numpy.
"""
import numpy as np
import pytest
import torch

import oracle
import ygg_workloads as wl


def test_code_table_special_values():
    d = oracle.fp8_e4m3_decode(np.arange(256, dtype=np.uint8))
    # format definition: bias 7, three mantissa bits, subnormals below 2^-6, largest finite 448, one NaN per sign
    assert d[0x00] == 0.0 and d[0x80] == 0.0 and np.signbit(d[0x80])
    assert d[0x01] == 2.0 ** -9 and d[0x07] == 7 * 2.0 ** -9 and d[0x08] == 2.0 ** -6
    assert d[0x38] == 1.0 and d[0x3C] == 1.5 and d[0x40] == 2.0 and d[0xB8] == -1.0
    assert d[0x7E] == 448.0 and d[0xFE] == -448.0
    assert np.isnan(d[0x7F]) and np.isnan(d[0xFF]) and np.isfinite(np.delete(d, [0x7F, 0xFF])).all()
    # strictly increasing over the positive finite codes, antisymmetric in the sign bit
    assert (np.diff(d[:0x7F]) > 0).all()
    assert np.array_equal(d[0x80:0xFF], -d[:0x7F])


def test_code_table_matches_library_conversion():
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    d = oracle.fp8_e4m3_decode(codes)
    fin = np.isfinite(lib)
    assert np.array_equal(np.isfinite(d), fin)
    assert np.array_equal(d[fin], lib[fin])


def test_input_quantiser_matches_library_conversion_and_round_trips():
    r = np.random.default_rng(5)
    for sigma in (0.01, 1.0, 60.0):
        x = np.clip(r.standard_normal(100_000) * sigma, -448, 448)
        lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(wl.f64_to_fp8_e4m3_bits(x), lib)
    codes = np.delete(np.arange(256, dtype=np.uint8), [0x7F, 0xFF])
    assert np.array_equal(wl.f64_to_fp8_e4m3_bits(oracle.fp8_e4m3_decode(codes)), codes)
    # ties go to the even mantissa; magnitudes beyond the largest finite value saturate
    assert list(wl.f64_to_fp8_e4m3_bits(np.array([1.0625, 1.1875, 1e9, -1e9, 2.0 ** -10, 3 * 2.0 ** -10]))) == \
        [0x38, 0x3A, 0x7E, 0xFE, 0x00, 0x02]


def _case(seed, B=2, N=9, Hq=4, Hkv=2, Dh=8, L=(5, 11), qdtype="f32", pow2=False, scale=0.37):
    cap = max(L) + 3
    r = np.random.default_rng(seed)
    parent = np.stack([wl.random_topological_tree(seed, N, sub=b) for b in range(B)])
    c = dict(q=wl.normal(seed, 2, (B, N, Hq, Dh), qdtype), seq_lens=np.array(L[:B], np.int32), parent_idx=parent,
             scale=scale)
    for name, shape in (("k_cache", (B, cap, Hkv, Dh)), ("v_cache", (B, cap, Hkv, Dh)),
                        ("k_tree", (B, N, Hkv, Dh)), ("v_tree", (B, N, Hkv, Dh))):
        codes = r.integers(0, 256, size=shape, dtype=np.uint8)
        codes[(codes & 0x7F) == 0x7F] = 0x3A          # no NaN codes
        c[name] = codes
    if pow2:
        c["k_scale"] = (2.0 ** r.integers(-9, -3, size=Hkv)).astype(np.float32)
        c["v_scale"] = (2.0 ** r.integers(-8, -2, size=Hkv)).astype(np.float32)
    else:
        c["k_scale"] = r.uniform(0.002, 0.02, size=Hkv).astype(np.float32)
        c["v_scale"] = r.uniform(0.01, 0.05, size=Hkv).astype(np.float32)
    return c


def _run(c):
    return oracle.tree_attention_fp8kv(c["q"], c["k_cache"], c["v_cache"], c["seq_lens"], c["k_tree"], c["v_tree"],
                                       c["k_scale"], c["v_scale"], c["parent_idx"], c["scale"])


def _dequant(codes, scale):
    return oracle.fp8_e4m3_decode(codes) * scale.astype(np.float64)[None, None, :, None]


@pytest.mark.parametrize("seed", [1, 2])
def test_power_of_two_scales_equal_plain_attention_bit_for_bit(seed):
    """With power-of-two scales the dequantised K/V are exact fp32 numbers, so the code path and the
    plain fp32 path see the same operands and must return the same doubles."""
    c = _case(seed, pow2=True)
    out, lse = _run(c)
    f32 = {n: _dequant(c[n], c[n[0] + "_scale"]).astype(np.float32) for n in ("k_cache", "v_cache", "k_tree", "v_tree")}
    for n in f32:
        assert np.array_equal(f32[n].astype(np.float64), _dequant(c[n], c[n[0] + "_scale"]))
    ref, ref_lse = oracle.tree_attention(c["q"], f32["k_cache"], f32["v_cache"], c["seq_lens"], f32["k_tree"],
                                         f32["v_tree"], c["parent_idx"], c["scale"])
    assert np.array_equal(out, ref) and np.array_equal(lse, ref_lse)


@pytest.mark.parametrize("qdtype", ["f32", "bf16"])
def test_general_scales_against_sequential_path_attention(qdtype):
    """Independent statement: dequantise in numpy, lay prefix + root path out as one sequence, plain
    softmax attention for its last token.  Distinct scales per kv head and per tensor kind, so a
    scale taken from the wrong head or the wrong tensor fails."""
    c = _case(7, Hq=6, Hkv=3, qdtype=qdtype)
    out, lse = _run(c)
    K = {n: _dequant(c[n], c[n[0] + "_scale"]) for n in ("k_cache", "v_cache", "k_tree", "v_tree")}
    q = wl.storage_to_f64(c["q"])
    B, N, Hq, Dh = q.shape
    G = Hq // c["k_tree"].shape[2]
    for b in range(B):
        L = int(c["seq_lens"][b])
        for i in range(N):
            path, a = [], i
            while a != -1:
                path.append(a)
                a = int(c["parent_idx"][b, a])
            path = path[::-1]
            for h in range(Hq):
                kv = h // G
                Ks = np.concatenate([K["k_cache"][b, :L, kv], K["k_tree"][b, path, kv]])
                Vs = np.concatenate([K["v_cache"][b, :L, kv], K["v_tree"][b, path, kv]])
                s = (Ks @ q[b, i, h]) * c["scale"]
                w = np.exp(s - s.max())
                np.testing.assert_allclose(out[b, i, h], (w / w.sum()) @ Vs, rtol=1e-12, atol=1e-13)
                np.testing.assert_allclose(lse[b, i, h], s.max() + np.log(w.sum()), rtol=1e-12, atol=1e-13)
    row, row_lse = oracle.attention_row_fp8kv(c["q"], c["k_cache"], c["v_cache"], c["seq_lens"], c["k_tree"],
                                              c["v_tree"], c["k_scale"], c["v_scale"], c["parent_idx"], c["scale"],
                                              1, N - 1, Hq - 1)
    assert np.array_equal(row, out[1, N - 1, Hq - 1]) and row_lse == lse[1, N - 1, Hq - 1]


def test_workload_generator_codes_cover_the_range_and_dequantise_close():
    cfg = wl.scaled(wl.CONFIGS[2], n_q_heads=4, n_kv_heads=2, prefix_len=64)
    d = wl.attention_inputs_fp8kv(cfg)
    bf = wl.attention_inputs(cfg)
    for n in ("k", "v"):
        codes = np.concatenate([d[n + "_cache"].reshape(-1, 2, 128), d[n + "_tree"].reshape(-1, 2, 128)])
        assert ((codes & 0x7F) != 0x7F).all()
        assert ((codes & 0x7F).max(axis=(0, 2)) == 0x7E).all()      # each head's largest magnitude sits at 448
        deq = oracle.fp8_e4m3_decode(d[n + "_cache"]) * d[n + "_scale"].astype(np.float64)[None, None, :, None]
        ref = wl.storage_to_f64(bf[n + "_cache"])                   # same draws, rounded to bf16 instead
        # the format keeps 4 significant bits (relative step 2^-3): error below 2^-4 of the magnitude plus
        # half a subnormal step, plus the bf16 rounding of the comparison value
        assert (np.abs(deq - ref) <= np.abs(ref) * (2.0 ** -4 + 2.0 ** -8) + d[n + "_scale"].max() * 2.0 ** -10).all()
