"""Pins for the 4-bit expert format (section 3.2: experts are kept in INT4): the oracle's dequantisation against
hand-typed values, the size of a block, the input recipe's rounding bound, and the library's host-side packer
against the layout written out independently here."""
import numpy as np
import pytest

import oracle
from workload import MoEConfig, Workload, bf16_bits_to_f32, f32_to_bf16_bits, quantize_int4


def bits(x):
    return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_dequant_hand_values():
    codes = np.full((2, 64), 8, dtype=np.uint8)
    codes[0, 0], codes[0, 31], codes[0, 32], codes[1, 63] = 15, 0, 9, 3
    scale = bits([[0.5, 2.0], [0.25, -3.0]])
    w = oracle.dequant_int4(codes, scale)
    assert w.shape == (2, 64) and w.dtype == np.float32
    assert w[0, 0] == 3.5 and w[0, 31] == -4.0            # 0.5 * (15 - 8), 0.5 * (0 - 8)
    assert w[0, 32] == 2.0                                 # second group of the row: 2.0 * (9 - 8)
    assert w[1, 63] == 15.0                                # -3.0 * (3 - 8)
    w[0, 0] = w[0, 31] = w[0, 32] = w[1, 63] = 0.0
    assert not w.any()                                     # code 8 is zero


def test_dequant_group_indexing_by_brute_force():
    r = np.random.default_rng(0)
    codes = r.integers(0, 16, size=(5, 96), dtype=np.uint8)
    sb = bits(r.uniform(0.01, 1.0, size=(5, 3)))
    w = oracle.dequant_int4(codes, sb)
    s32 = bf16_bits_to_f32(sb)
    for i in range(5):
        for j in range(96):
            assert w[i, j] == np.float32(s32[i, j // 32]) * np.float32(int(codes[i, j]) - 8)


def test_block_size_is_four_and_a_half_bits_per_weight():
    assert oracle.expert_bytes_int4(4096, 14336) * 8 == int(4.5 * 3 * 4096 * 14336)
    assert oracle.expert_bytes_int4(2048, 1024) == 3_538_944
    assert oracle.expert_bytes(2048, 1024, 2) / oracle.expert_bytes_int4(2048, 1024) == pytest.approx(16 / 4.5)


def test_input_recipe_rounds_to_the_nearest_code():
    cfg = MoEConfig(name="q", cfg_id=77, dtype="bf16", n_layers=1, d_model=128, d_ff=64, n_experts=2, n_shared=0,
                    top_k=1, capacity=1, n_seqs=1, n_steps=1, prefill_len=0, beta=0.0, pref_lo=1, pref_hi=1, delta=0.0)
    wg = Workload(cfg).expert(0, 1)[0]
    codes, sb = quantize_int4(wg)
    assert codes.dtype == np.uint8 and codes.max() <= 15 and codes.shape == wg.shape and sb.shape == (64, 4)
    w = bf16_bits_to_f32(wg).astype(np.float64)
    deq = oracle.dequant_int4(codes, sb).astype(np.float64)
    s = np.repeat(bf16_bits_to_f32(sb).astype(np.float64), 32, axis=1)
    # half a step, plus the clipping that the bf16 rounding of the scale can cause at the group's extreme value
    assert (np.abs(w - deq) <= 0.5 * s + np.abs(w) * 2.0 ** -7).all()
    assert np.abs(w - deq).max() > 0.1 * s.min()           # it is a real quantisation, not a copy
    zero = np.zeros((1, 32), dtype=np.uint16)
    cz, sz = quantize_int4(zero)
    assert (cz == 8).all() and not oracle.dequant_int4(cz, sz).any()


def test_quantised_expert_stays_close_to_the_original():
    cfg = MoEConfig(name="q", cfg_id=78, dtype="bf16", n_layers=1, d_model=256, d_ff=64, n_experts=1, n_shared=0,
                    top_k=1, capacity=1, n_seqs=1, n_steps=1, prefill_len=0, beta=0.0, pref_lo=1, pref_hi=1, delta=0.0)
    wl = Workload(cfg)
    full = [bf16_bits_to_f32(m) for m in wl.expert(0, 0)]
    q4 = [oracle.dequant_int4(c, s) for c, s in wl.expert_int4(0, 0)]
    x = np.random.default_rng(1).standard_normal(256)
    a, b = oracle.expert_swiglu(x, *full), oracle.expert_swiglu(x, *q4)
    assert 0.01 < np.abs(a - b).max() / np.abs(a).max() < 0.5


# ------------------------------------------------------------------ host-side packer of the library
def element_location(d, f, m, row, col):
    """Byte offset and nibble of code (matrix m, row, col) in an INT4 tiled block, from the layout's definition."""
    gate_up_total = (f // 16) * (d // 128) * 2304
    if m < 2:
        rt, r = divmod(row, 16)
        sb, k = divmod(col, 128)
        j, kk = divmod(k, 32)
        q, e = divmod(kk, 8)
        lane = q * 16 + r
        byte0 = (rt * (d // 128) + sb) * 2304 + m * 1024 + lane * 16 + j * 4
    else:
        dq, rr = divmod(row, 64)
        n, j = divmod(rr, 4)
        c, kk = divmod(col, 32)
        q, e = divmod(kk, 8)
        lane = q * 16 + n
        byte0 = gate_up_total + (c * (d // 64) + dq) * 1152 + lane * 16 + j * 4
    nib = (e & 1) * 4 + (e >> 1)
    return byte0 + nib // 2, nib % 2


def scale_location(d, f, m, row, g):
    gate_up_total = (f // 16) * (d // 128) * 2304
    if m < 2:
        rt, r = divmod(row, 16)
        sb, j = divmod(g, 4)
        return (rt * (d // 128) + sb) * 2304 + 2048 + r * 16 + m * 8 + j * 2
    dq, rr = divmod(row, 64)
    n, j = divmod(rr, 4)
    return gate_up_total + (g * (d // 64) + dq) * 1152 + 1024 + n * 8 + j * 2


def test_library_packer_places_every_code_and_scale():
    from paper_2602_11192_amd import binding as B
    d, f = 256, 64
    r = np.random.default_rng(5)
    codes = r.integers(0, 16, size=3 * d * f, dtype=np.uint8)
    scales = r.integers(1, 2 ** 15, size=3 * d * f // 32, dtype=np.uint16)
    nbytes = B.moe_expert_block_bytes(d, f, B.MOE_DTYPE_BF16, B.MOE_LAYOUT_TILED_INT4)
    assert nbytes == oracle.expert_bytes_int4(d, f)
    blk = np.zeros(nbytes, dtype=np.uint8)
    B.moe_pack_expert_int4(codes, scales, blk, d, f)
    shapes = [(f, d), (f, d), (d, f)]
    off_c, off_s = 0, 0
    seen = np.zeros(nbytes * 2, dtype=bool)
    for m, (rows, cols) in enumerate(shapes):
        cm = codes[off_c:off_c + rows * cols].reshape(rows, cols)
        sm = scales[off_s:off_s + rows * cols // 32].reshape(rows, cols // 32)
        for row in range(rows):
            for col in range(cols):
                byte, hi = element_location(d, f, m, row, col)
                assert (blk[byte] >> (4 * hi)) & 15 == cm[row, col], (m, row, col)
                assert not seen[2 * byte + hi]
                seen[2 * byte + hi] = True
            for g in range(cols // 32):
                o = scale_location(d, f, m, row, g)
                assert int(blk[o]) | (int(blk[o + 1]) << 8) == sm[row, g], (m, row, g)
                assert not seen[2 * o] and not seen[2 * o + 2]
                seen[2 * o:2 * o + 4] = True
        off_c += rows * cols
        off_s += rows * cols // 32
    assert seen.all()                                      # every nibble of the block is accounted for
    bad = codes.copy()
    bad[7] = 16
    with pytest.raises(B.MoeError):
        B.moe_pack_expert_int4(bad, scales, blk, d, f)
    assert B.moe_expert_block_bytes(100, 64, B.MOE_DTYPE_BF16, B.MOE_LAYOUT_TILED_INT4) == 0
