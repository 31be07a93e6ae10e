"""The pins must be able to fail: plant one plausible mistake at a time in a COPY of the oracle (CPU only, in a
temporary directory) and check that the pin suite run against that copy reports a failure."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = {
    "position S+n instead of S+depth": ('pos = S + tree["depth"].astype(np.int64)', 'pos = S + np.arange(T)', "verify"),
    "RoPE sign": ("a * c - b * s, b * c + a * s", "a * c + b * s, b * c - a * s", "verify"),
    "softmax scale dropped": ("scale = 1.0 / np.sqrt(float(head_dim))", "scale = 1.0", "verify"),
    "tree mask dropped": ("sc = np.where(visible, sc, -np.inf)", "sc = sc + 0.0", "verify"),
    "gate and up swapped": ("x = x + (silu(gate) * up)", "x = x + (silu(up) * gate)", "verify"),
    "transposed Wq": ('q = xn @ np.asarray(lw["wq"], dtype=F64).T', 'q = xn @ np.asarray(lw["wq"], dtype=F64)', "verify"),
    "head residual dropped": ("z = h + silu(pre)", "z = silu(pre)", "verify"),
    "head bias dropped": ("pre = pre + np.asarray(head[\"b1\"], dtype=F64)", "pre = pre + 0.0", "verify"),
    "final norm dropped": ('hidden = rmsnorm(x, model["g_final"], model["cfg"]["rms_eps"])', "hidden = np.asarray(x, dtype=F64)", "verify"),
    "final norm without its gain": ('hidden = rmsnorm(x, model["g_final"], model["cfg"]["rms_eps"])', 'hidden = rmsnorm(x, 1.0, model["cfg"]["rms_eps"])', "verify"),
    "LM head replaced by the embedding": ('logits = hidden @ np.asarray(model["lm_head"], dtype=F64).T', 'logits = hidden @ np.asarray(model["embed"], dtype=F64).T', "verify"),
    "norm eps dropped": ("return x / np.sqrt(ms + eps) * np.asarray(g, dtype=F64)", "return x / np.sqrt(ms) * np.asarray(g, dtype=F64)", "verify"),
    "norm gain dropped": ("return x / np.sqrt(ms + eps) * np.asarray(g, dtype=F64)", "return x / np.sqrt(ms + eps)", "verify"),
    "match against own node instead of parent": ("tree_tokens[n] != node_argmax[parent[n]]", "tree_tokens[n] != node_argmax[n]", "accept"),
    "compaction source": ("src[:A] = S + np.asarray(acc_nodes[:A])", "src[:A] = S + np.arange(A)", "accept or verify"),
    "tie to highest path": ("if n_ok > best_len:", "if n_ok >= best_len:", "accept"),
}


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_planted_mistake_is_caught(tmp_path, name):
    old, new, select = MUTATIONS[name]
    for d in ("oracle", "workload", "tests"):
        shutil.copytree(os.path.join(ROOT, d), tmp_path / d, ignore=shutil.ignore_patterns("__pycache__", "golden"))
    src = (tmp_path / "oracle" / "medusa.py").read_text()
    assert old in src, f"mutation target not found: {old}"
    (tmp_path / "oracle" / "medusa.py").write_text(src.replace(old, new))
    files = [str(tmp_path / "tests" / f) for f in ("test_oracle_verify.py", "test_oracle_accept.py")]
    env = dict(os.environ, PYTHONPATH=str(tmp_path))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-k", select, *files],
                       cwd=tmp_path, env=env, capture_output=True, text=True)
    assert r.returncode == 1, f"pins did not catch '{name}':\n{r.stdout[-800:]}"
    assert "failed" in r.stdout
