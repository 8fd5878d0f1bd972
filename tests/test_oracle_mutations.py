"""Do the oracle's pins bite?  Each case plants one plausible mistake in a temporary copy of
oracle.cpp (on the CPU, never in the product), rebuilds it, and requires that the pins --
hand-worked fixtures, brute force, closed forms, the literal transcription -- reject it.
The unmodified source must pass the same pins."""
import importlib.util
import os
import subprocess
import sys

import numpy as np
import pytest

from _util import csr_from_rows, csr_from_edges, random_csr, random_sym_csr, load_golden, f16, bf16, bf16_to_f64

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "oracle.cpp")

MUTATIONS = {
    "none": None,
    "bound drops the absolute values": ("bd[j] += std::fabs(a) * std::fabs(b);", "bd[j] += a * b;"),
    "B row taken from the row index": ("B + (int64_t)colidx[p] * N;", "B + (int64_t)(i % 3) * N;"),
    "fp16 subnormal scale": ("std::ldexp((double)f, -24)", "std::ldexp((double)f, -25)"),
    "fp16 exponent bias": ("std::ldexp((double)(f + 1024), e - 25)", "std::ldexp((double)(f + 1024), e - 24)"),
    "bf16 exponent bias": ("std::ldexp((double)(f + 128), e - 134)", "std::ldexp((double)(f + 128), e - 133)"),
    "bf16 subnormal scale": ("std::ldexp((double)f, -133)", "std::ldexp((double)f, -134)"),
    "bf16 read as fp16": ("return value_type == 1 ? bf2d(h) : h2d(h);", "return h2d(h);"),
    "sddmm takes the Y row from the row index": ("const uint16_t* y = Y + (int64_t)colidx[p] * N;", "const uint16_t* y = Y + (int64_t)(i % 3) * N;"),
    "sddmm bound drops the absolute values": ("mag += std::fabs(a) * std::fabs(b);\n            }\n            const double scale",
                                              "mag += a * b;\n            }\n            const double scale"),
    "padding repeats the first column": ("cols[std::min<int64_t>(t * TW + c, d - 1)]", "cols[(t * TW + c < d) ? t * TW + c : 0]"),
    "bit index transposed": ("int bit = (int)((r - r0) * TW + cc % TW);\n                    uint64_t& word",
                             "int bit = (int)((cc % TW) * WH + (r - r0));\n                    uint64_t& word"),
    "rank counts the bit itself": ("(((uint64_t)1 << (bit % 64)) - 1)", "(((uint64_t)2 << (bit % 64)) - 1)"),
    "columns not condensed per window": ("cols.erase(std::unique(cols.begin(), cols.end()), cols.end());", ""),
    "gain with the wrong sign": ("e.second * two_m - dsum[e.first] * dsum[v]", "e.second * two_m + dsum[e.first] * dsum[v]"),
    "gain ties go to the higher id": ("if (best < 0 || s > best_s) { best = e.first; best_s = s; }",
                                      "if (best < 0 || s >= best_s) { best = e.first; best_s = s; }"),
    "merge even without gain": ("if (best >= 0 && best_s > 0) {", "if (best >= 0) {"),
    "descending degree order": ("return adj[a].size() < adj[b].size();", "return adj[a].size() > adj[b].size();"),
    "chain ties go to the later leaf": ("count[q] > count[best]))", "count[q] >= count[best]))"),
    "chain needs two shared columns": ("count[q] >= 1 &&", "count[q] >= 2 &&"),
    "chain ignores segments": ("for (size_t s = tree_begin; s < seq.size(); s += seg_len)", "for (size_t s = tree_begin; s < seq.size(); s += 1 << 30)"),
    "imbalance divides by W-1": ("return s / (double)W;", "return s / (double)(W - 1);"),
}


def _load_variant(tmp_path, name):
    text = open(SRC).read()
    if MUTATIONS[name] is not None:
        old, new = MUTATIONS[name]
        assert text.count(old) == 1, f"mutation anchor for '{name}' not found exactly once"
        text = text.replace(old, new)
    d = tmp_path / "orc"
    d.mkdir()
    (d / "oracle.cpp").write_text(text)
    for f in ("__init__.py", "literal.py"):
        (d / f).write_text(open(os.path.join(ROOT, "oracle", f)).read())
    spec = importlib.util.spec_from_file_location(f"orc_variant_{abs(hash(name))}", str(d / "__init__.py"),
                                                  submodule_search_locations=[str(d)])
    mod = importlib.util.module_from_spec(spec)
    sys.modules[spec.name] = mod
    spec.loader.exec_module(mod)
    lit_spec = importlib.util.spec_from_file_location(spec.name + ".literal", str(d / "literal.py"))
    lit = importlib.util.module_from_spec(lit_spec)
    lit_spec.loader.exec_module(lit)
    return mod, lit


def _pins(orc, lit):
    """The pins, condensed; raises AssertionError on the first one that fails."""
    rng = np.random.default_rng(0)
    # fp16 decode against numpy
    bits = np.arange(0, 65536, 7, dtype=np.uint16)
    got = np.array([orc._load().orc_f16_to_f64(int(b)) for b in bits])
    np.testing.assert_array_equal(got, bits.view(np.float16).astype(np.float64))
    # SpMM against a dense matmul on an independently built dense A
    M, K, N = 9, 14, 5
    A = np.zeros((M, K), np.float16)
    mask = rng.random((M, K)) < 0.4
    A[mask] = rng.uniform(-2, 2, mask.sum()).astype(np.float16)
    rowptr, colidx, vals = csr_from_rows([np.nonzero(mask[i])[0].tolist() for i in range(M)], A[mask])
    Bf = rng.uniform(-1, 1, (K, N)).astype(np.float16)
    C, bound = orc.spmm(rowptr, colidx, vals, Bf.view(np.uint16))
    np.testing.assert_allclose(C, A.astype(np.float64) @ Bf.astype(np.float64), atol=1e-13)
    np.testing.assert_allclose(bound, np.abs(A).astype(np.float64) @ np.abs(Bf).astype(np.float64), atol=1e-13)
    # bfloat16: decode against the bits placed in the upper half of a binary32, SpMM against a dense matmul
    bits = np.arange(0, 65536, 5, dtype=np.uint16)
    got = np.array([orc._load().orc_bf16_to_f64(int(b)) for b in bits])
    np.testing.assert_array_equal(got, bf16_to_f64(bits))
    a_bits, b_bits = bf16(rng.uniform(-2, 2, mask.sum())), bf16(rng.uniform(-1, 1, (K, N)))
    Ad = np.zeros((M, K))
    Ad[mask] = bf16_to_f64(a_bits)
    C, _ = orc.spmm(rowptr, colidx, a_bits, b_bits, value_type="bf16")
    np.testing.assert_allclose(C, Ad @ bf16_to_f64(b_bits), atol=1e-13)
    # sampled dense-dense product against a masked dense matmul (X is M x N, Y is K x N)
    Xf = rng.uniform(-1, 1, (M, 6)).astype(np.float16)
    Yf = rng.uniform(-1, 1, (K, 6)).astype(np.float16)
    sd, sb = orc.sddmm(rowptr, colidx, Xf.view(np.uint16), Yf.view(np.uint16), vals)
    np.testing.assert_allclose(sd, (Xf.astype(np.float64) @ Yf.astype(np.float64).T)[mask] * A[mask].astype(np.float64), atol=1e-13)
    np.testing.assert_allclose(sb, (np.abs(Xf).astype(np.float64) @ np.abs(Yf).astype(np.float64).T)[mask]
                               * np.abs(A[mask]).astype(np.float64), atol=1e-13)
    # format: hand-worked example, closed form, literal transcription, round trip
    g = load_golden("format_8x8_toy.json")
    rowptr, colidx, vals = csr_from_rows(g["rows"])
    fmt = orc.encode(rowptr, colidx, vals, None, 8, 8)
    assert list(fmt["row_window_offset"]) == g["row_window_offset"] and list(fmt["tc_offset"]) == g["tc_offset"]
    assert list(fmt["sparse_a_to_b"]) == g["sparse_a_to_b"]
    assert [int(x) for x in fmt["tc_local_bit"]] == [sum(1 << b for b in bits) for bits in g["tile_bits"]]
    assert fmt["vals"].view(np.float16).astype(int).tolist() == g["packed_values"]
    assert sum(fmt[k].nbytes for k in ("row_window_offset", "tc_offset", "sparse_a_to_b", "tc_local_bit")) == 148
    rowptr, colidx, vals = random_csr(rng, 70, 90, 0.1)
    perm = rng.permutation(70).astype(np.int32)
    fmt = orc.encode(rowptr, colidx, vals, perm, 16, 16)
    rp, ci, va = orc.decode(fmt)
    for r in range(70):
        i = perm[r]
        assert ci[rp[r]:rp[r + 1]].tolist() == colidx[rowptr[i]:rowptr[i + 1]].tolist()
        assert va[rp[r]:rp[r + 1]].tolist() == vals[rowptr[i]:rowptr[i + 1]].tolist()
    # reordering: hand-worked graphs and the literal transcription
    g = load_golden("reorder_two_triangles.json")
    rowptr, colidx, _ = csr_from_edges(g["M"], g["edges"])
    parent, child = orc.dendrogram(rowptr, colidx)
    assert list(parent) == g["parent"]
    assert list(orc.ordering(rowptr, colidx, parent, child, 1024)[0]) == g["perm"]
    g = load_golden("ordering_chain.json")
    rowptr, colidx, _ = csr_from_rows(g["rows"])
    assert list(orc.ordering(rowptr, colidx, g["parent"], g["child_order"], 6)[0]) == g["perm_seg6"]
    assert list(orc.ordering(rowptr, colidx, g["parent"], g["child_order"], 3)[0]) == g["perm_seg3"]
    for seed in range(4):
        r2 = np.random.default_rng(seed)
        rowptr, colidx, _ = random_sym_csr(r2, 60, 4.0)
        parent, child = orc.dendrogram(rowptr, colidx)
        lparent, lchild = lit.dendrogram(rowptr, colidx)
        assert list(parent) == lparent and list(child) == lchild
        assert list(orc.ordering(rowptr, colidx, parent, child, 9)[0]) == lit.ordering(rowptr, colidx, lparent, lchild, 9)[0]
    star = csr_from_edges(12, [(0, i) for i in range(1, 12)])
    assert list(orc.dendrogram(star[0], star[1])[0]) == lit.dendrogram(star[0], star[1])[0]
    # imbalance degree: |0-10|*3 + |40-10| over 4 windows
    assert orc.ibd(np.array([0, 0, 0, 0, 40], np.int32)) == pytest.approx(15.0)


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_pins_reject_planted_mistakes(tmp_path, name):
    orc, lit = _load_variant(tmp_path, name)
    if name == "none":
        _pins(orc, lit)
    else:
        with pytest.raises((AssertionError, ValueError)):
            _pins(orc, lit)
