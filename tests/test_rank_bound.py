"""CPU checks of the arithmetic behind probe selection's ranking values (no GPU, no library call):
the bf16 split of fp32 operands and the error bound that the kernels attach to a = |c|^2 - 2 q.c.
The kernels short-list with a() and decide with exact distances; these tests pin the claim that the
short list cannot miss a cluster, i.e. that the bound really bounds the error of the emulated arithmetic."""
import numpy as np
import pytest


def bf16_round(x):
    """fp32 -> nearest bf16 (ties to even), returned as fp32 with the low 16 bits clear."""
    b = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32)


def split(x):
    hi = bf16_round(x)
    rest = (x - hi).astype(np.float32)
    assert np.array_equal(rest.astype(np.float64), x.astype(np.float64) - hi.astype(np.float64))   # exact in fp32
    return hi, bf16_round(rest)


def rank_error_bound(d, qn, cmax):
    return ((3 * d + 8) * 2.0 ** -22 + 5.0e-5) * (qn + cmax)


def _cases():
    rng = np.random.default_rng(20230117)
    yield "integer grid", rng.integers(0, 256, size=(40, 128)).astype(np.float32), rng.integers(0, 256, size=(300, 128)).astype(np.float32)
    u = rng.standard_normal((40, 96)); v = rng.standard_normal((300, 96))
    yield "unit norm", (u / np.linalg.norm(u, axis=1, keepdims=True)).astype(np.float32), (v / np.linalg.norm(v, axis=1, keepdims=True)).astype(np.float32)
    yield "mixed scales", (rng.standard_normal((40, 64)) * 10.0 ** rng.integers(-6, 6, size=(1, 64))).astype(np.float32), \
        (rng.standard_normal((300, 64)) * 10.0 ** rng.integers(-6, 6, size=(1, 64))).astype(np.float32)
    yield "far from the origin", (1000.0 + rng.standard_normal((40, 32))).astype(np.float32), (1000.0 + rng.standard_normal((300, 32))).astype(np.float32)


@pytest.mark.parametrize("name,q,c", list(_cases()), ids=[n for n, _, _ in _cases()])
def test_split_remainder_is_within_its_bound(name, q, c):
    qh, ql = split(q)
    ch, cl = split(c)
    for x, h, l in ((q, qh, ql), (c, ch, cl)):
        assert np.all(np.abs(x.astype(np.float64) - h - l) <= 2.0 ** -16 * np.abs(x))
    f = np.float64
    exact = q.astype(f) @ c.astype(f).T
    kept = qh.astype(f) @ ch.astype(f).T + qh.astype(f) @ cl.astype(f).T + ql.astype(f) @ ch.astype(f).T
    mags = np.abs(q).astype(f) @ np.abs(c).astype(f).T
    assert np.all(np.abs(exact - kept) <= 3.02 * 2.0 ** -16 * mags)


@pytest.mark.parametrize("name,q,c", list(_cases()), ids=[n for n, _, _ in _cases()])
def test_emulated_ranking_value_stays_inside_the_bound(name, q, c):
    # fp32 accumulation of the 3 d exact products in a scrambled order, fp32 norm, fp32 multiply-add
    rng = np.random.default_rng(7)
    qh, ql = split(q)
    ch, cl = split(c)
    d = q.shape[1]
    cn = np.zeros(len(c), dtype=np.float32)
    for t in range(d):
        cn = (c[:, t] * c[:, t] + cn).astype(np.float32)
    cmax = float(cn.max())
    exact_a = (c.astype(np.float64) ** 2).sum(1)[None, :] - 2.0 * (q.astype(np.float64) @ c.astype(np.float64).T)
    terms = np.concatenate([qh[:, None, :] * ch[None, :, :], qh[:, None, :] * cl[None, :, :], ql[:, None, :] * ch[None, :, :]], axis=2)
    assert terms.dtype == np.float32        # bf16 x bf16 is exact in fp32
    order = rng.permutation(3 * d)
    acc = np.zeros(terms.shape[:2], dtype=np.float32)
    for t in order:
        acc = (acc + terms[:, :, t]).astype(np.float32)
    a = (np.float32(-2.0) * acc + cn[None, :]).astype(np.float32)
    qn = (q.astype(np.float64) ** 2).sum(1)
    delta = rank_error_bound(d, qn, cmax)[:, None]
    worst = np.max(np.abs(a.astype(np.float64) - exact_a) / delta)
    assert worst <= 0.5, f"{name}: error reaches {worst:.3f} of the bound"


def test_tagged_key_brackets_the_key():
    rng = np.random.default_rng(3)
    f = np.concatenate([rng.standard_normal(1000) * 1e3, -np.abs(rng.standard_normal(1000)), [0.0, -0.0]]).astype(np.float32)
    b = f.view(np.uint32)
    key = b ^ np.where(b >> 31, np.uint32(0xFFFFFFFF), np.uint32(0x80000000))
    order = np.argsort(key, kind="stable")
    assert np.all(np.diff(f[order]) >= 0)                          # the key map is monotone
    for col in (0, 17, 63):
        tagged = (key & np.uint32(0xFFFFFFC0)) | np.uint32(col)
        assert np.all((tagged & np.uint32(0xFFFFFFC0)) <= key) and np.all(key <= (tagged | np.uint32(63)))
        # what clearing six bits can lower a value by: 63 units in the last place, under 2^-17 of its magnitude
        # (or 63 denormal steps next to zero)
        lowered = (key & np.uint32(0xFFFFFFC0))
        back = lowered ^ np.where(lowered >> 31, np.uint32(0x80000000), np.uint32(0xFFFFFFFF))
        g = back.view(np.float32)
        ok = np.isfinite(g)
        assert np.all(g[ok] <= f[ok]) and np.all((f[ok].astype(np.float64) - g[ok]) <= 2.0 ** -17 * np.abs(f[ok]) + 64 * 2.0 ** -149)
