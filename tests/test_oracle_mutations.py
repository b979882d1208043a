"""The pins must be able to tell a wrong oracle from a right one.

Each case plants one plausible mistake in a copy of the oracle's source (CPU only), builds it,
swaps it in for the real library and expects at least one pin of tests/test_oracle_pins.py to fail.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "smfg_oracle.c")

MUTATIONS = [
    ("index drawn from [0, j) instead of [0, j]", "(uint64_t)(j + 1u)", "(uint64_t)(j)"),
    ("collision keeps t instead of taking j", "p[s] = taken ? j : t;", "p[s] = taken ? t : j;"),
    ("membership search skips the latest pick", "for (uint32_t q = 0; q < s; ++q)",
     "for (uint32_t q = 0; q + 1 < s; ++q)"),
    ("counter: node and hop swapped", "{v, h, s >> 2, 0u}", "{h, v, s >> 2, 0u}"),
    ("counter: draw index not advanced per block", "{v, h, s >> 2, 0u}", "{v, h, 0u, 0u}"),
    ("always word 0 of the block", "out[s & 3u]", "out[0]"),
    ("key halves swapped", "{(uint32_t)rng_key, (uint32_t)(rng_key >> 32)}",
     "{(uint32_t)(rng_key >> 32), (uint32_t)rng_key}"),
    ("Philox multiplier off by a bit", "0xD2511F53u", "0xD2511F51u"),
    ("Philox with 9 rounds", "r < 10", "r < 9"),
    ("key bumped before the first round", "if (r > 0) {", "if (r >= 0) {"),
    ("Philox output words permuted", "c[0] = n0; c[1] = lo1; c[2] = n2; c[3] = lo0;",
     "c[0] = n0; c[1] = lo0; c[2] = n2; c[3] = lo1;"),
    ("Philox round mixes the wrong high word", "uint32_t n0 = hi1 ^ c[1] ^ k[0];",
     "uint32_t n0 = hi0 ^ c[1] ^ k[0];"),
    ("nodes met in a hop are expanded in the same hop", "i < n_dst && status", "i < n && status"),
    ("block stores global instead of local ids", "bi[e++] = local_of[g];", "bi[e++] = g;"),
    # not listed: drawing when degree == fanout.  Floyd's rule with k = deg returns the identity
    # order whatever the words are, so that change alters no output.
    ("degree just above the fanout takes the whole row", "if (d == -1 || deg <= (uint32_t)d) {",
     "if (d == -1 || deg <= (uint32_t)d + 1u) {"),
    ("fanout -1 treated as fanout 1", "if (d == -1 || deg <= (uint32_t)d) {\n    for",
     "if (d == -1) d = 1;\n  if (deg <= (uint32_t)d) {\n    for"),
    ("positions ignored: first k neighbours", "indices[a + (int64_t)p[s]]", "indices[a + (int64_t)s]"),
    ("feature row taken by local id", "(int64_t)node_ids[j] * row_stride", "j * row_stride"),
    ("block indptr shifted by one", "bp[i + 1] = (int32_t)e;", "bp[i] = (int32_t)e;"),
    ("mean divides by k + 1", "mean[i * dim + c] = k > 0 ? s / k : 0.0;", "mean[i * dim + c] = k > 0 ? s / (k + 1) : 0.0;"),
    ("mean reads the destination's own row", "int64_t at = (int64_t)indices[e] * dim + c;",
     "int64_t at = (int64_t)i * dim + c;"),
    ("layer: weight halves swapped", "double w_own = wj[c], w_agg = wj[dim + c];",
     "double w_own = wj[dim + c], w_agg = wj[c];"),
    ("layer: weight read transposed", "const double *wj = w + (int64_t)j * 2 * dim;",
     "const double *wj = w + (int64_t)j;"),
    ("layer: bias dropped", "double s = bias ? bias[j] : 0.0;", "double s = 0.0;"),
    ("layer: ReLU never applied", "(relu && s < 0.0) ? 0.0 : s;", "s;"),
    ("layer: ReLU always applied", "(relu && s < 0.0) ? 0.0 : s;", "(s < 0.0) ? 0.0 : s;"),
    ("layer: own row taken from the mean", "s += w_own * own + w_agg * mean_tmp[at];",
     "s += w_own * mean_tmp[at] + w_agg * mean_tmp[at];"),
    ("half exponent bias off by one", "int e = ex - 15;", "int e = ex - 14;"),
    ("half subnormals scaled as normals", "v = (double)man / 1024.0 / 16384.0;", "v = (double)man / 1024.0 / 32768.0;"),
    ("label taken by position instead of node", "(const char *)labels + (int64_t)seeds[i] * elem_bytes",
     "(const char *)labels + (int64_t)i * elem_bytes"),
    ("only the new frontier is expanded in the next hop", "for (int64_t i = 0; i < n_dst",
     "for (int64_t i = (h == 0 ? 0 : counts[h - 1]); i < n_dst"),
]


def _pins():
    """The pins in cheap-to-expensive order, as argument-free callables."""
    drv = pins.philox_driver()
    yield lambda: pins.test_philox_matches_library_engine(drv)
    yield lambda: pins.test_draw_word_layout(drv)
    yield pins.test_index_from_word_is_floor_scaling
    for n, k in [(4, 2), (5, 3), (6, 4)]:
        yield lambda n=n, k=k: pins.test_floyd_exhaustive_uniform(n, k)
    for fan in [(3,), (4, 2), (2, 3, 2)]:
        yield lambda fan=fan: pins.test_invariants_small_graphs(1, fan)
    for L in (1, 2, 3):
        yield lambda L=L: pins.test_full_neighbourhood_equals_bfs(L)
    yield pins.test_fanout_all_equals_large_fanout_and_bfs
    yield pins.test_consumer_contract_prefix_and_last_block
    yield pins.test_keying_properties
    yield lambda: pins.test_label_slice_is_plain_indexing(np.int32)
    yield pins.test_half_decoding_matches_numpy_for_every_bit_pattern
    yield lambda: pins.test_mean_aggregate_equals_sparse_matrix_product(np.float16)
    yield lambda: pins.test_sage_layer_equals_dense_linear_algebra(np.float16, True, True)
    yield lambda: pins.test_sage_layer_equals_dense_linear_algebra(np.float32, False, True)
    yield lambda: pins.test_chi_square_uniform_subsets(8, 3)
    yield lambda: pins.test_chi_square_uniform_subsets(40, 15)


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(what, old, new, tmp_path, monkeypatch):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation anchor not unique: {old!r}"
    src, lib = tmp_path / "mut.c", tmp_path / "libmut.so"
    src.write_text(text.replace(old, new))
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-o", str(lib), str(src)])
    oracle._load()
    monkeypatch.setattr(oracle, "_lib", oracle._configure(ctypes.CDLL(str(lib))))
    caught = None
    for pin in _pins():
        try:
            pin()
        except BaseException as e:       # an assertion, or a crash turned into an exception
            if isinstance(e, (KeyboardInterrupt, pytest.skip.Exception)):
                raise
            caught = e
            break
    assert caught is not None, f"no pin noticed: {what}"


def test_unmutated_oracle_passes_the_same_pins():
    for pin in _pins():
        pin()
