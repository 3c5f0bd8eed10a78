"""Do the oracle's pins have teeth?  Each case plants one plausible mistake in a copy of the oracle's
C source (a dropped term, a wrong sign or index, a swapped rule), builds it beside the real one and
runs the pin tests named for it against that library in a fresh interpreter: they must fail.

Only the CPU oracle is touched; nothing here runs on a GPU.
"""
import os
import subprocess
import sys

import pytest

REPO = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(REPO, "oracle", "efanna_oracle.c")

DIST = ["tests/test_oracle_dist.py"]
TREES = ["tests/test_oracle_trees.py"]
GRAPH = ["tests/test_oracle_graph.py"]
CONQUER = ["tests/test_oracle_conquer.py"]
SEARCH = ["tests/test_oracle_search.py"]
PROJ = ["tests/test_oracle_projection.py"]

# (name, text in the oracle, what the mistake turns it into, pin files that must notice)
MUTANTS = [
    ("distance: partial sums added one after the other instead of in the tree",
     "    for (int s = 8; s >= 1; s >>= 1)\n        for (int l = 0; l < s; ++l) acc[l] = acc[l] + acc[l + s];",
     "    for (int l = 1; l < 16; ++l) acc[0] = acc[0] + acc[l];", DIST),
    ("distance: tree pairs neighbours first (l+1, l+2, l+4, l+8)",
     "    for (int s = 8; s >= 1; s >>= 1)\n        for (int l = 0; l < s; ++l) acc[l] = acc[l] + acc[l + s];",
     "    for (int s = 1; s < 16; s <<= 1)\n        for (int l = 0; l < 16; l += 2 * s) acc[l] = acc[l] + acc[l + s];",
     DIST),
    ("distance: multiply and add rounded separately",
     "acc[j & 15] = fmaf(diff, diff, acc[j & 15]);", "acc[j & 15] = acc[j & 15] + diff * diff;", DIST),
    ("distance: eight partial sums instead of sixteen",
     "acc[j & 15] = fmaf(diff, diff, acc[j & 15]);", "acc[j & 7] = fmaf(diff, diff, acc[j & 7]);", DIST),
    ("generator: second multiplier of the finaliser off by one digit",
     "0x94D049BB133111EBULL", "0x94D049BB133111E9ULL", DIST),
    ("trees: a value equal to the mean goes left",
     "< sum) c->perm[b + nl++] = id;", "<= sum) c->perm[b + nl++] = id;", TREES),
    ("trees: a node of exactly S points is split",
     "if (cnt <= c->S) {", "if (cnt < c->S) {", TREES),
    ("trees: split dimension drawn from the parent's number",
     "uint64_t draw = oracle_node_rand(c->seed, c->tree, heap_id);",
     "uint64_t draw = oracle_node_rand(c->seed, c->tree, heap_id >> 1);", TREES),
    ("trees: degenerate split puts the odd point on the left",
     "mid = b + cnt / 2; /* degenerate", "mid = b + (cnt + 1) / 2; /* degenerate", TREES),
    ("trees: coordinates rounded to 2^-19 instead of 2^-20",
     "rint((double)x * 1048576.0)", "rint((double)x * 524288.0)", TREES),
    ("trees: right part written back in reverse order (partition not stable)",
     "memcpy(c->perm + b + nl, c->tmp, (size_t)nr * sizeof(int32_t));",
     "for (int64_t r = 0; r < nr; ++r) c->perm[b + nl + r] = c->tmp[nr - 1 - r];", TREES),
    ("trees, variance rule: the square of the sum is not taken off",
     "__int128 v = (__int128)m * s2 - s * s;", "__int128 v = (__int128)m * s2;", TREES),
    ("trees, variance rule: the whole node is the sample",
     "int64_t m = e - b < 100 ? e - b : 100;", "int64_t m = e - b;", TREES),
    ("trees, variance rule: the smallest variances are kept",
     "while (pos > 0 && topv[pos - 1] < v) --pos;", "while (pos > 0 && topv[pos - 1] > v) --pos;", TREES),
    ("trees, variance rule: of equal variances the later dimension comes first",
     "while (pos > 0 && topv[pos - 1] < v) --pos;", "while (pos > 0 && topv[pos - 1] <= v) --pos;", TREES),
    ("trees, variance rule: squares added in 64 bits",
     "s2 += (__int128)q * q;", "s2 += (__int128)(int64_t)((uint64_t)q * (uint64_t)q);", TREES),
    ("trees, variance rule: four candidates instead of five",
     "return top[draw % (uint64_t)n_top];", "return top[draw % (uint64_t)(n_top > 4 ? 4 : n_top)];", TREES),
    ("trees, projections: the signs are ignored",
     "v += (z >> 63) ? -q : q;", "v += q;", PROJ),
    ("trees, projections: seven terms instead of eight",
     "for (int k = 0; k < RP_TERMS; ++k) {\n        uint64_t z = mix64((r << 8)",
     "for (int k = 0; k < RP_TERMS - 1; ++k) {\n        uint64_t z = mix64((r << 8)", PROJ),
    ("trees, projections: the code keeps the wrong bits of the draw",
     "((draw >> 34) & 0x3FFFFFFFULL)", "(draw & 0x3FFFFFFFULL)", PROJ),
    ("trees, projections: routing in a sibling subtree looks at one coordinate only",
     "int left = nd->dim == -1 || (int64_t)nd->cnt * node_value(xi, d, nd->dim) < nd->sum;",
     "int left = nd->dim < 0 || (int64_t)nd->cnt * quantise(xi[nd->dim]) < nd->sum;", PROJ),
    ("search, projections: a projection node sends every query left",
     "            if (nd->dim != -1) {\n                int64_t diff", "            if (nd->dim >= 0) {\n                int64_t diff", PROJ),
    ("lists: equal distances ordered by the larger id",
     "(da == db && ia < ib)", "(da == db && ia > ib)", GRAPH),
    ("lists: an id already present is entered again",
     "        if (pool[s].id == id) return 0;\n", "        if (pool[s].id == id && 0) return 0;\n", GRAPH),
    ("NN-descent: sampled entries keep their mark",
     "                    e->is_new = 0;\n", "", GRAPH),
    ("NN-descent: old entries beyond the last sampled new one are taken too",
     "for (int32_t s = 0; s < cnt[i] && a < L; ++s) {\n                entry *e = &pool[i * K + s];\n                if (e->is_new) {",
     "for (int32_t s = 0; s < cnt[i]; ++s) {\n                entry *e = &pool[i * K + s];\n                if (e->is_new && a >= L) continue;\n                if (e->is_new) {",
     GRAPH),
    ("NN-descent: reverse lists keep the largest hashes",
     "if (x->hash != y->hash) return (x->hash > y->hash) - (x->hash < y->hash);",
     "if (x->hash != y->hash) return (x->hash < y->hash) - (x->hash > y->hash);", GRAPH),
    ("NN-descent: reverse-old lists drawn from the reverse-new stream",
     "2 * (iter0 + it) + 1, rod, rod_c", "2 * (iter0 + it), rod, rod_c", GRAPH),
    ("NN-descent: new x old pairs dropped from the join",
     "int32_t b_hi = cross_old && pass == 0 ? n_new : n_new + n_old;", "int32_t b_hi = n_new;", GRAPH),
    ("NN-descent: pair offered to one end point only",
     "                        updates += pool_insert_marked(pool + (int64_t)v * K, &cnt[v], K, dist, u, mark);\n", "", GRAPH),
    ("NN-descent: inserted entries are not marked new",
     "    pool[s].is_new = is_new;\n", "    pool[s].is_new = 0;\n", GRAPH),
    ("NN-descent: members of U_new stay in U_old",
     "if (!bsearch(&uo[s], un, (size_t)n_new, sizeof(int32_t), cmp_i32))", "if (1)", GRAPH),
    ("conquer: a node without a split test sends points right",
     "int left = nd->dim == -1 || (int64_t)nd->cnt * node_value(xi, d, nd->dim) < nd->sum;",
     "int left = nd->dim != -1 && (int64_t)nd->cnt * node_value(xi, d, nd->dim) < nd->sum;", CONQUER),
    ("conquer: the point's own side is searched instead of the sibling's",
     "int32_t c = nodes[up >> 1].child[1 - (up & 1)];", "int32_t c = nodes[up >> 1].child[up & 1];", CONQUER),
    ("search: the branch put aside forgets the priority of the path so far",
     "other = fma(gap, gap, prio);", "other = gap * gap;", SEARCH),
    ("search: the far child is followed and the near one put aside",
     "heap[n_heap].link = nd->child[left ? 1 : 0];\n            ++n_heap;\n            link = nd->child[left ? 0 : 1];",
     "heap[n_heap].link = nd->child[left ? 0 : 1];\n            ++n_heap;\n            link = nd->child[left ? 1 : 0];",
     SEARCH),
    ("search: equal priorities resolved by the larger link",
     "heap[h].link < heap[best].link))", "heap[h].link > heap[best].link))", SEARCH),
    ("generator: trees numbered from 0 in the seed offset",
     "0x9E3779B97F4A7C15ULL * (uint64_t)(tree + 1));", "0x9E3779B97F4A7C15ULL * (uint64_t)(tree));", DIST),
    ("trees: coordinates truncated instead of rounded",
     "(int64_t)rint((double)x * 1048576.0)", "(int64_t)((double)x * 1048576.0)", TREES),
    ("trees: children numbered 2h+1, 2h+2",
     "uint64_t child = depth < 60 ? 2 * heap_id : heap_id;", "uint64_t child = depth < 60 ? 2 * heap_id + 1 : heap_id;",
     TREES),
    ("init graph: the last member of a leaf is left out",
     "for (int32_t p = off[l]; p < off[l + 1]; ++p) {\n                        int32_t j = perm[(int64_t)t * n + p];\n                        if (j != i) cand[nc++] = j;",
     "for (int32_t p = off[l]; p < off[l + 1] - 1; ++p) {\n                        int32_t j = perm[(int64_t)t * n + p];\n                        if (j != i) cand[nc++] = j;",
     GRAPH),
    ("init graph: the point itself is a candidate",
     "if (j != i) cand[nc++] = j;", "cand[nc++] = j;", GRAPH),
    ("lists: a full list turns away an entry equal to its last one only",
     "if (*cnt == K && !entry_less(dist, id, pool[K - 1].dist, pool[K - 1].id)) return 0;",
     "if (*cnt == K && dist > pool[K - 1].dist) return 0;", GRAPH),
    ("conquer: stops one level below the depth asked for",
     "if (up < 0 || nd[up >> 1].depth < dep) break;", "if (up < 0 || nd[up >> 1].depth <= dep) break;", CONQUER),
    ("conquer: every ancestor's sibling is searched from the point's leaf-level parent",
     "up = pj < 0 ? -1 : pj * 2 + (nd[pj].child[1] == j);", "up = pj < 0 ? -1 : pj * 2 + (nd[pj].child[0] == j);",
     CONQUER),
    ("NN-descent, literal marking: what a new and an old member insert is marked new after all",
     "uint8_t mark = !(cross_old && pass == 1);", "uint8_t mark = 1;", GRAPH),
    ("NN-descent, literal marking: pairs of a new and an old member are inserted first",
     "int32_t b_lo = cross_old && pass == 1 ? n_new : a + 1;\n                    int32_t b_hi = cross_old && pass == 0 ? n_new : n_new + n_old;\n                    uint8_t mark = !(cross_old && pass == 1);",
     "int32_t b_lo = cross_old && pass == 0 ? n_new : a + 1;\n                    int32_t b_hi = cross_old && pass == 1 ? n_new : n_new + n_old;\n                    uint8_t mark = !(cross_old && pass == 0);",
     GRAPH),
    ("NN-descent: reverse hash takes (source, target)",
     "c->hash = oracle_reverse_hash(seed, iter, v, (int32_t)u);", "c->hash = oracle_reverse_hash(seed, iter, (int32_t)u, v);",
     GRAPH),
    ("NN-descent: reverse lists hold one member fewer",
     "int32_t keep = m < L ? (int32_t)m : L;", "int32_t keep = m < L ? (int32_t)m : L - 1;", GRAPH),
    ("NN-descent: early termination compares with <=",
     "if ((double)fresh < delta * (double)n * (double)K) break;", "if ((double)fresh <= delta * (double)n * (double)K) break;",
     GRAPH),
    ("NN-descent: the iteration number does not enter the reverse hash",
     "reverse_lists(nw, nw_c, L, n, L, seed, 2 * (iter0 + it), rnw, rnw_c);",
     "reverse_lists(nw, nw_c, L, n, L, seed, 0, rnw, rnw_c);", GRAPH),
    ("search: one leaf fewer per tree",
     "const int32_t want = P / S / T + 1;", "const int32_t want = P / S / T > 0 ? P / S / T : 1;", SEARCH),
    ("search: the first pool is not cut to E",
     "int32_t cnt = 0, n_touched = 0, cap = E;", "int32_t cnt = 0, n_touched = 0, cap = P;", SEARCH),
    ("search: members already expanded are expanded, fresh ones are not",
     "                    if (pool[s].is_new) {\n                        pool[s].is_new = 0;\n                        expand[n_exp++]",
     "                    if (!pool[s].is_new) {\n                        pool[s].is_new = 0;\n                        expand[n_exp++]",
     SEARCH),
    ("search: a neighbour that was checked before is offered to the pool again",
     "                        if (j < 0 || checked[j]) continue;",
     "                        if (j < 0) continue;\n                        if (checked[j]) { pool_insert(pool, &cnt, cap, oracle_dist(q, X + (int64_t)j * d, d), j); continue; }",
     SEARCH),
    ("search: the gap to the split is not divided by the population",
     "double gap = (double)diff / ((double)nd->cnt * 1048576.0);", "double gap = (double)diff / 1048576.0;", SEARCH),
]


def _build_mutant(tmp_path, old, new):
    from oracle import binding
    src = open(SRC).read()
    assert src.count(old) == 1, "the text to replace must occur exactly once in the oracle"
    mutated = tmp_path / "efanna_oracle.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", *binding.CFLAGS, "-o", str(lib), str(mutated), "-lm"])
    return str(lib)


@pytest.mark.parametrize("name,old,new,files", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_notice(name, old, new, files, tmp_path):
    lib = _build_mutant(tmp_path, old, new)
    env = dict(os.environ, EFANNA_ORACLE_LIBRARY=lib)
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                          *files], cwd=REPO, env=env, capture_output=True, text=True, timeout=900)
    assert run.returncode == 1, f"no pin in {files} notices: {name}\n{run.stdout[-1500:]}"


def test_unchanged_copy_passes(tmp_path):
    """The harness itself: an unmodified copy, built and loaded the same way, passes a pin file."""
    lib = _build_mutant(tmp_path, "static uint64_t mix64(uint64_t z)", "static uint64_t mix64(uint64_t z)")
    env = dict(os.environ, EFANNA_ORACLE_LIBRARY=lib)
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                          *DIST, *TREES], cwd=REPO, env=env, capture_output=True, text=True, timeout=900)
    assert run.returncode == 0, run.stdout[-1500:]
