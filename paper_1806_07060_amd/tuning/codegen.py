"""Off-line phase, step 3: turn a trained model into the C++ that is compiled into the library.

Section 3 ('Model and code generation') and Section 4.2 of the paper: the
rules of the internal nodes and the configurations at the leaves are written
out as source code, which is then built into the library; the machine-learning
code itself is not shipped.  Also writes the constants of the traditional
"default" dispatch (Section 5): one tiled and one direct variant plus a size
threshold.

Two renderings of the same rules (`style`):
  "branches"  nested if-then-else, as the paper generates it (single trees only);
  "table"     the nodes as a constant array plus a short loop that walks it.  Same
              comparisons in the same order; a tree of thousands of leaves stays a
              few dozen KB of data instead of hundreds of KB of branches, which is
              what keeps a cold evaluation cheap (Section 3 asks for a selector of
              negligible cost).
A model is a single tree (nested dict), a forest (list of nested dicts whose
leaves carry cost lists), or a gated pair {"gate": G, "tree": ..., "forest": ...}:
the tree answers inputs whose work M*N*K is below G, the forest the others.
"""
import os

from .cart import FEATURES

HERE = os.path.dirname(os.path.abspath(__file__))
GENERATED_HEADER = os.path.join(os.path.dirname(HERE), "csrc", "mdg_select_generated.h")
INT64_MAX = (1 << 63) - 1
LEAF_FLAG = 0x80000000


def _emit(node, variant_names, indent, out):
    pad = "  " * indent
    if "leaf" in node:
        v = int(node["leaf"])
        out.append(f"{pad}return {v};  // {variant_names[v] if variant_names else ''}".rstrip())
        return
    out.append(f"{pad}if ({FEATURES[node['feature']]} <= {int(node['threshold'])}) {{")
    _emit(node["left"], variant_names, indent + 1, out)
    out.append(f"{pad}}} else {{")
    _emit(node["right"], variant_names, indent + 1, out)
    out.append(f"{pad}}}")


def flatten(tree, payload_of, base=0):
    """Nested tree -> list of (threshold, child, feature word) in breadth-first order, root first; the two
    children of an internal node sit next to each other (left at `child`, right at `child + 1`).  A leaf holds
    threshold INT64_MAX, its own index as child and LEAF_FLAG | payload << 4 as feature word, so that a walk that
    does not test for leaves simply stays on it (feature 0 is never greater than INT64_MAX).  `base` is the index
    the root will have in the array the rows are appended to."""
    rows, queue = [None], [(tree, 0)]
    while queue:
        nxt = []
        for node, at in queue:
            if "leaf" in node:
                p = int(payload_of(node))
                assert 0 <= p < (1 << 27)
                rows[at] = (INT64_MAX, base + at, LEAF_FLAG | (p << 4))
            else:
                child = len(rows)
                rows += [None, None]
                rows[at] = (int(node["threshold"]), base + child, int(node["feature"]))
                nxt += [(node["left"], child), (node["right"], child + 1)]
        queue = nxt
    return rows


def _height(tree):
    h, stack = 0, [(tree, 0)]
    while stack:
        n, d = stack.pop()
        if "leaf" in n:
            h = max(h, d)
        else:
            stack += [(n["left"], d + 1), (n["right"], d + 1)]
    return h


_NODE_DECL = [
    "// One node of a tree: go to `child` if x[feature] <= threshold, to `child + 1` otherwise.  A leaf has",
    "// threshold INT64_MAX, child = its own index and feature = 0x80000000 | payload << 4.",
    "struct mdg_generated_node { int64_t threshold; uint32_t child; uint32_t feature; };",
    "static inline uint32_t mdg_generated_walk(const mdg_generated_node* nodes, uint32_t i, const int64_t* x) {",
    "  for (;;) {",
    "    const mdg_generated_node n = nodes[i];",
    "    if (n.feature & 0x80000000u) return (n.feature >> 4) & 0x7ffffffu;",
    "    i = n.child + (uint32_t)(x[n.feature] > n.threshold);",
    "  }",
    "}",
    "",
]


def _node_rows(rows):
    return [f"  {{{f'{thr}LL' if thr < INT64_MAX else 'INT64_MAX'}, {child}u, {feat:#x}u}}," for thr, child, feat in rows]


def _tree_table(tree, name):
    rows = flatten(tree, lambda leaf: leaf["leaf"])
    return [f"static const mdg_generated_node {name}[] = {{"] + _node_rows(rows) + ["};", ""]


def _forest_tables(trees, n_variants, keep):
    """Leaf table, node table, roots and the summing evaluator of a forest."""
    assert 0 < n_variants <= 255
    leaves, rows, roots = [], [], []

    def payload(leaf):
        leaves.append(leaf)
        return len(leaves) - 1

    for tree in trees:
        roots.append(len(rows))
        rows += flatten(tree, payload, base=len(rows))
    height = max(_height(t) for t in trees)
    lines = [f"#define MDG_GENERATED_FOREST_TREES {len(trees)}",
             f"#define MDG_GENERATED_FOREST_HEIGHT {height}",
             "// per leaf: how many variants are listed, their ids and mean costs (cheapest first), and the cost that",
             "// stands in for every variant not listed",
             f"struct mdg_generated_leaf {{ int32_t rest; int32_t n; uint8_t id[{keep}]; int32_t cost[{keep}]; }};",
             "static const mdg_generated_leaf mdg_generated_leaves[] = {"]
    for leaf in leaves:
        ids, costs = list(leaf["ids"]), list(leaf["costs"])
        assert len(ids) == len(costs) <= keep and all(0 <= v < n_variants for v in ids)
        pad = [0] * (keep - len(ids))
        lines.append(f"  {{{int(leaf['rest'])}, {len(ids)}, {{{', '.join(map(str, ids + pad))}}}, "
                     f"{{{', '.join(map(str, costs + pad))}}}}},")
    lines += ["};", "", "static const mdg_generated_node mdg_generated_forest_nodes[] = {"] + _node_rows(rows) + ["};"]
    lines += [f"static const uint32_t mdg_generated_forest_roots[{len(trees)}] = {{{', '.join(f'{r}u' for r in roots)}}};",
              "",
              "// All trees are walked together, one level per pass (independent loads overlap); a walk that has reached",
              "// its leaf stays there.  Then the leaves' cost lists are summed per variant.",
              "static inline int mdg_generated_forest_select(const int64_t* x) {",
              "  uint32_t at[MDG_GENERATED_FOREST_TREES];",
              "  for (int t = 0; t < MDG_GENERATED_FOREST_TREES; ++t) at[t] = mdg_generated_forest_roots[t];",
              "  for (int level = 0; level < MDG_GENERATED_FOREST_HEIGHT; ++level) {",
              "    uint32_t inner = 0;",
              "    for (int t = 0; t < MDG_GENERATED_FOREST_TREES; ++t) {",
              "      const mdg_generated_node n = mdg_generated_forest_nodes[at[t]];",
              "      inner |= ~n.feature;",
              "      at[t] = n.child + (uint32_t)(x[n.feature & 15u] > n.threshold);",
              "    }",
              "    if (!(inner & 0x80000000u)) break;  // every walk stands on a leaf",
              "  }",
              f"  int64_t score[{n_variants}] = {{0}};  // summed cost minus the part common to all variants",
              "  for (int t = 0; t < MDG_GENERATED_FOREST_TREES; ++t) {",
              "    const mdg_generated_leaf& l = mdg_generated_leaves[(mdg_generated_forest_nodes[at[t]].feature >> 4) & 0x7ffffffu];",
              "    for (int e = 0; e < l.n; ++e) score[l.id[e]] += (int64_t)l.cost[e] - l.rest;",
              "  }",
              "  int best = 0;",
              f"  for (int v = 1; v < {n_variants}; ++v)",
              "    if (score[v] < score[best]) best = v;  // first minimum: ties go to the lowest id",
              "  return best;",
              "}",
              ""]
    return lines


def tree_to_cpp(model, selector_name, variant_names=None, default_tiled=0, default_direct=0,
                default_threshold=512.0 ** 3, provenance="", n_variants=None, keep=8, style="branches"):
    """C++ header text defining mdg_generated_select() for a single tree, a forest or a gated pair (see the module
    text).  `style` is the rendering of the single tree; a forest is always a table.  A forest needs n_variants or
    variant_names."""
    gated = isinstance(model, dict) and "gate" in model
    tree = model["tree"] if gated else (model if isinstance(model, dict) else None)
    forest = model["forest"] if gated else (list(model) if isinstance(model, (list, tuple)) else None)
    if forest is not None and n_variants is None:
        n_variants = len(variant_names)
    assert style in ("table", "branches")
    lines = [
        "// GENERATED by paper_1806_07060_amd/tuning/codegen.py -- do not edit.",
        "// The trained model over (M, N, K, tA, tB), the products M*N, M*N*K and the rows / columns a 32-, 64- or",
        "// 128-wide tile grid adds beyond M / N; leaves are variant ids of the library's variant table.",
    ]
    if provenance:
        lines += [f"// {l}" for l in provenance.splitlines()]
    lines += [
        "#pragma once",
        "#include <stdint.h>",
        "",
        f"#define MDG_GENERATED_SELECTOR_NAME \"{selector_name}\"",
        f"#define MDG_GENERATED_DEFAULT_THRESHOLD {float(default_threshold)!r} /* M*N*K at which the default dispatch "
        "switches to the tiled kernel */",
        f"#define MDG_GENERATED_DEFAULT_TILED {int(default_tiled)}",
        f"#define MDG_GENERATED_DEFAULT_DIRECT {int(default_direct)}",
        "",
    ]
    if forest is not None or style == "table":
        lines += _NODE_DECL
    if tree is not None:
        if style == "table":
            lines += _tree_table(tree, "mdg_generated_tree_nodes")
            lines += ["static inline int mdg_generated_tree_select(const int64_t* x) {",
                      "  return (int)mdg_generated_walk(mdg_generated_tree_nodes, 0, x);", "}", ""]
        else:
            lines += ["// the single tree as nested if-then-else (Section 3, 'Model and code generation')",
                      "static inline int mdg_generated_tree_select(const int64_t* x) {",
                      "  const int64_t " + ", ".join(f"{name} = x[{i}]" for i, name in enumerate(FEATURES)) + ";",
                      "  " + " ".join(f"(void){name};" for name in FEATURES)]
            body = []
            _emit(tree, variant_names, 1, body)
            lines += body
            if "leaf" not in tree:
                lines.append("  return 0;  // unreachable")
            lines += ["}", ""]
    if forest is not None:
        lines += _forest_tables(forest, n_variants, keep)
    lines += [
        "static inline int mdg_generated_select(int tA, int tB, int64_t M, int64_t N, int64_t K) {",
        "  // derived features: size of C and amount of work, saturating (M, N, K < 2^31, so M*N cannot overflow)",
        "  const int64_t MN = M * N;",
        "  const int64_t MNK = (K > 0 && MN > INT64_MAX / K) ? INT64_MAX : MN * K;",
        "  // tile fit: (t - X mod t) mod t for t = 32, 64, 128 (0 when X is an exact multiple; M, N >= 0)",
        "  const int64_t padM32 = (32 - (M & 31)) & 31, padM64 = (64 - (M & 63)) & 63, padM128 = (128 - (M & 127)) & 127;",
        "  const int64_t padN32 = (32 - (N & 31)) & 31, padN64 = (64 - (N & 63)) & 63, padN128 = (128 - (N & 127)) & 127;",
        "  const int64_t x[16] = {M, N, K, tA, tB, MN, MNK, padM32, padM64, padM128, padN32, padN64, padN128, 0, 0, 0};",
    ]
    if gated:
        lines += [f"  // the cheap model for small problems, the expensive one where its cost is negligible",
                  f"  if (MNK < {int(model['gate'])}LL) return mdg_generated_tree_select(x);",
                  "  return mdg_generated_forest_select(x);"]
    elif forest is not None:
        lines.append("  return mdg_generated_forest_select(x);")
    else:
        lines.append("  return mdg_generated_tree_select(x);")
    lines.append("}")
    return "\n".join(lines) + "\n"


def write_header(model, selector_name, path=GENERATED_HEADER, **kw):
    text = tree_to_cpp(model, selector_name, **kw)
    with open(path, "w") as f:
        f.write(text)
    return path


def internal_thresholds(model):
    """(feature, threshold) of every internal node (tests probe threshold - 1, threshold, threshold + 1)."""
    if isinstance(model, dict) and "gate" in model:
        stack = [model["tree"]] + list(model["forest"])
    else:
        stack = list(model) if isinstance(model, (list, tuple)) else [model]
    out = []
    while stack:
        n = stack.pop()
        if "leaf" not in n:
            out.append((n["feature"], n["threshold"]))
            stack += [n["left"], n["right"]]
    return out
