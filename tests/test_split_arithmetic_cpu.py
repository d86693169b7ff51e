"""CPU checks of the arithmetic behind the NF_CONTRACT_BF16X6 / NF_CONTRACT_BF16X9 modes (no GPU, no library code):
the three-way split of an fp32 number into bfloat16 pieces as the kernels do it (truncation to the
top 16 bits, remainders in fp32), written out in numpy.

* every piece is a bfloat16 (low 16 bits zero) and the pieces sum to the number exactly;
* each of the nine piece products is exact in fp32;
* the pieces fall off by at least 2^-7 and 2^-15 of |x|, so the three products the kernels leave out
  (m*l, l*m, l*l) are together below 2^-21 of |x*w| in the worst case (about 2^-24 in the root mean square);
* all nine piece products together ARE the product x*w, exactly (the nine-product mode);
* a dot product from the six kept products, with the fp32 accumulator rounded once per MFMA (16
  reduction indices), is as close to the fp64 result as the same dot product with the accumulator
  rounded once per fp32 MFMA (2 reduction indices).
"""
import numpy as np


def split3(x):
    x = np.asarray(x, dtype=np.float32)
    top = np.uint32(0xFFFF0000)
    h = (x.view(np.uint32) & top).view(np.float32)
    r1 = (x - h).astype(np.float32)
    m = (r1.view(np.uint32) & top).view(np.float32)
    r2 = (r1 - m).astype(np.float32)
    return h, m, r2


def samples(rng, n):
    x = rng.standard_normal(n).astype(np.float32)
    scale = np.exp2(rng.integers(-20, 20, n)).astype(np.float32)
    return np.concatenate([x * scale, np.float32([0.0, 1.0, -1.0, 1.0 + 2.0**-23, 3.4e38, -1.2e-30, 2.0**-120])])


def test_pieces_are_bf16_and_sum_exactly():
    rng = np.random.default_rng(0)
    x = samples(rng, 200000)
    h, m, l = split3(x)
    for p in (h, m, l):
        assert np.all((p.view(np.uint32) & np.uint32(0xFFFF)) == 0)
    assert np.array_equal(h.astype(np.float64) + m.astype(np.float64) + l.astype(np.float64), x.astype(np.float64))
    # the remainders the kernels compute in fp32 are exact
    assert np.array_equal((x.astype(np.float64) - h.astype(np.float64)), (x - h).astype(np.float64))
    # magnitudes: each piece at most 2^-8 of the previous one's scale
    nz = x != 0
    assert np.all(np.abs(m[nz]) <= np.abs(x[nz]) * 2.0**-7)
    assert np.all(np.abs(l[nz]) <= np.abs(x[nz]) * 2.0**-15)


def test_piece_products_are_exact_and_the_dropped_ones_are_tiny():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(100000) * 3).astype(np.float32)
    w = (rng.standard_normal(100000) * 0.05).astype(np.float32)
    xs, ws = split3(x), split3(w)
    for a in xs:
        for b in ws:
            p64 = a.astype(np.float64) * b.astype(np.float64)
            assert np.array_equal((a * b).astype(np.float64), p64)  # 8 x 8 significant bits fit in 24
    kept = sum(xs[i].astype(np.float64) * ws[j].astype(np.float64) for i, j in ((0, 0), (0, 1), (1, 0), (1, 1), (0, 2), (2, 0)))
    exact = x.astype(np.float64) * w.astype(np.float64)
    nz = exact != 0
    rel = np.abs(kept[nz] - exact[nz]) / np.abs(exact[nz])
    assert np.max(rel) < 2.0**-21
    assert np.sqrt(np.mean(rel**2)) < 2.0**-23  # measured: 2^-24


def test_six_product_dot_is_as_close_as_fp32():
    rng = np.random.default_rng(2)
    K = 4608
    errs6, errs32 = [], []
    for _ in range(64):
        x = np.maximum(rng.standard_normal(K), 0).astype(np.float32)   # post-ReLU activations
        w = (rng.standard_normal(K) * 0.05).astype(np.float32)
        ref = float(np.dot(x.astype(np.float64), w.astype(np.float64)))
        xs, ws = split3(x), split3(w)
        acc6 = np.float32(0)
        acc32 = np.float32(0)
        # 16 reduction indices per MFMA, six MFMAs per slab, fp32 accumulator between them
        for k0 in range(0, K, 16):
            sl = slice(k0, k0 + 16)
            for i, j in ((0, 0), (0, 1), (1, 0), (1, 1), (0, 2), (2, 0)):
                acc6 = np.float32(acc6 + np.float32(np.sum(xs[i][sl].astype(np.float64) * ws[j][sl].astype(np.float64))))
            for k in range(k0, k0 + 16, 2):  # v_mfma_f32_32x32x2_f32: two reduction indices per instruction
                acc32 = np.float32(acc32 + np.float32(float(x[k]) * float(w[k]) + float(x[k + 1]) * float(w[k + 1])))
        errs6.append(abs(float(acc6) - ref))
        errs32.append(abs(float(acc32) - ref))
    rms6, rms32 = np.sqrt(np.mean(np.square(errs6))), np.sqrt(np.mean(np.square(errs32)))
    assert rms6 <= 2.0 * rms32 + 1e-9, (rms6, rms32)


def test_nine_piece_products_are_the_product():
    """NF_CONTRACT_BF16X9: nothing is left out, so what enters the fp32 accumulation for one
    multiply-add is x*w itself (each piece product is exact, and they sum to it exactly in fp64)."""
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(100000) * np.exp2(rng.integers(-12, 12, 100000))).astype(np.float32)
    w = (rng.standard_normal(100000) * 0.05).astype(np.float32)
    xs, ws = split3(x), split3(w)
    total = np.zeros(x.shape, dtype=np.float64)
    for a in xs:
        for b in ws:
            total += a.astype(np.float64) * b.astype(np.float64)
    # fp64 holds every partial sum exactly here: all terms are multiples of the smallest product's
    # unit and the sum spans fewer than 53 bits
    assert np.array_equal(total, x.astype(np.float64) * w.astype(np.float64))
