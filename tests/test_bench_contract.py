"""Host-side checks of the benchmark's contract and of the separation between the product path and
the oracle (no GPU needed)."""
import ast
import os
import subprocess
import sys

import workload

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_flop_count_of_the_headline_workload():
    """3 (24 T N_e^2 + 4 N_s^2 N_e N_b f) with f the fraction of sequence-tile pairs that hold a visible score:
    C2 has four sequence tiles, 10 of 16 pairs remain."""
    cfg = workload.CONFIGS[2]
    T = cfg.N_s * cfg.N_b
    dense = 3 * (24 * T * cfg.N_e ** 2 + 4 * cfg.N_s ** 2 * cfg.N_e * cfg.N_b)
    assert workload.model_flops(cfg, tile_skip=False) == dense
    kept = 3 * (24 * T * cfg.N_e ** 2 + 4 * cfg.N_s ** 2 * cfg.N_e * cfg.N_b * 10 / 16)
    assert workload.model_flops(cfg, tile_skip=True) == kept
    assert len(workload.causal_tile_pairs(cfg)) == 10
    # visible pairs only: N_s (N_s + 1) / 2 of N_s^2
    vis = 3 * (24 * T * cfg.N_e ** 2 + 4 * (cfg.N_s * (cfg.N_s + 1) // 2) * cfg.N_e * cfg.N_b)
    assert workload.model_flops(cfg, visible_only=True) == vis
    # ragged sequence tiles of C4: 400 + 400 + 224, pairs counted with their real extents
    c4 = workload.CONFIGS[4]
    ext = [400, 400, 224]
    pairs = sum(ext[k] * ext[q] for q in range(3) for k in range(3) if k <= q)
    T4 = c4.N_s * c4.N_b
    assert workload.model_flops(c4) == 3 * (2 * T4 * (4 * c4.N_e ** 2 + 2 * c4.N_e * c4.N_m) + 4 * pairs * c4.N_e * c4.N_b)


def _imports(path):
    tree = ast.parse(open(path).read())
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            for a in node.names:
                yield node, a.name
        elif isinstance(node, ast.ImportFrom):
            yield node, node.module or ""


def test_the_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_13236_amd")
    for name in sorted(os.listdir(pkg)):
        if name.endswith(".py"):
            for _, mod in _imports(os.path.join(pkg, name)):
                assert not mod.split(".")[0] == "oracle", name
    assert not any(mod.split(".")[0] == "oracle" for _, mod in _imports(os.path.join(ROOT, "workload.py")))
    # the benchmark may call the oracle in its cpu_baseline leg only
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())
    for fn in [n for n in tree.body if isinstance(n, ast.FunctionDef)]:
        uses = any((isinstance(n, ast.ImportFrom) and (n.module or "").split(".")[0] == "oracle") or
                   (isinstance(n, ast.Import) and any(a.name.split(".")[0] == "oracle" for a in n.names)) for n in ast.walk(fn))
        assert uses == (fn.name == "cpu_baseline"), fn.name
    # and the oracle imports neither the package nor the workload generator
    for name in sorted(os.listdir(os.path.join(ROOT, "oracle"))):
        if name.endswith(".py"):
            for _, mod in _imports(os.path.join(ROOT, "oracle", name)):
                assert mod.split(".")[0] not in ("paper_2504_13236_amd", "workload", "bench"), (name, mod)
