"""Do the pins have teeth?  Plant one plausible mistake at a time in a *copy* of the
oracle's C source (CPU only), compile it, and require that at least one pin fails."""
import os
import subprocess

import pytest

import oracle
from oracle_pins import ALL_PINS

SRC = os.path.join(os.path.dirname(oracle.__file__), "placeto_oracle.c")

MUTATIONS = [
    ("residual self term dropped",
     "s[(size_t)v * H + h] += upd[h];", "s[(size_t)v * H + h] = upd[h];"),
    ("weight matrix read transposed",
     "x[i] * W[(size_t)i * n_out + j]", "x[i] * W[((size_t)j * n_in + i) % ((size_t)n_in * n_out)]"),
    ("ReLU missing", "(relu && s < 0.0) ? 0.0 : s", "s"),
    ("bias dropped", "double s = b[j];", "double s = 0.0 * b[j];"),
    ("f and g swapped in the top-down sweep",
     "sweep(p_f_td, p_g_td, L, H, n, order, a.par_cnt, a.par, td,",
     "sweep(p_g_td, p_f_td, L, H, n, order, a.par_cnt, a.par, td,"),
    ("top-down and bottom-up parameters swapped",
     "sweep(p_f_bu, p_g_bu, L, H, n, rev,", "sweep(p_f_td, p_g_td, L, H, n, rev,"),
    ("top-down sweep walks children",
     "order, a.par_cnt, a.par, td,", "rev, a.chi_cnt, a.chi, td,"),
    ("messages are the raw states, f skipped",
     "const double *m = msg + (size_t)nbr[v][j] * H;", "const double *m = s + (size_t)nbr[v][j] * H;"),
    ("one-hot device index reversed",
     "(placement[v] == d) ? 1.0 : 0.0", "(placement[v] == D - 1 - d) ? 1.0 : 0.0"),
    ("is-current and is-visited swapped",
     "phi[2 + D] = (v == cur) ? 1.0 : 0.0;\n        phi[3 + D] = feats[(size_t)v * 3 + 2];",
     "phi[3 + D] = (v == cur) ? 1.0 : 0.0;\n        phi[2 + D] = feats[(size_t)v * 3 + 2];"),
    ("run time and output size swapped",
     "phi[0] = feats[(size_t)v * 3 + 0];\n        phi[1] = feats[(size_t)v * 3 + 1];",
     "phi[1] = feats[(size_t)v * 3 + 0];\n        phi[0] = feats[(size_t)v * 3 + 1];"),
    ("current node pooled into a set", "if (cls[u] == 0) continue;", "if (cls[u] == 0) cls[u] = 3;"),
    ("ancestors and descendants swapped",
     "else if (up[u]) cls[u] = 1;\n        else if (down[u]) cls[u] = 2;",
     "else if (up[u]) cls[u] = 2;\n        else if (down[u]) cls[u] = 1;"),
    ("pooling ignores the device",
     "int32_t d = c->group_by_device ? placement[u] : 0;", "int32_t d = 0;"),
    ("pooled vectors laid out device-major in the policy input",
     "z + (size_t)(2 + i * G + d) * H", "z + (size_t)(2 + d * 3 + i) * H"),
    ("policy reads node 0's embedding instead of the current node's",
     "memcpy(z, td + (size_t)cur * H,", "memcpy(z, td + (size_t)0 * H,"),
    ("l_i sees the top-down half twice",
     "memcpy(agg + H, bu + (size_t)u * H,", "memcpy(agg + H, td + (size_t)u * H,"),
    ("l of the parent set used for every set", "mlp(p_l[i], L,", "mlp(p_l[0], L,"),
    ("h of the parent set used for every set", "mlp(p_h[i], L,", "mlp(p_h[0], L,"),
    ("policy hidden layer linear", "layer(p_pol, Z, H, 1, z, upd)", "layer(p_pol, Z, H, 0, z, upd)"),
    ("policy output layer has a ReLU", "layer(p2, H, D, 0, upd, logits);", "layer(p2, H, D, 1, upd, logits);"),
    ("softmax not normalised", "probs[d] /= tot;", "probs[d] /= 1.0;"),
    ("level = max over parents without the +1",
     "int32_t cand = td_level[a.par[v][j]] + 1;", "int32_t cand = td_level[a.par[v][j]] + (j == 0);"),
    ("bottom-up level walks parents",
     "for (int32_t j = 0; j < a.chi_cnt[v]; ++j) {\n                int32_t cand = bu_level[a.chi[v][j]] + 1;",
     "for (int32_t j = 0; j < a.par_cnt[v]; ++j) {\n                int32_t cand = bu_level[a.par[v][j]] + 1;"),
    ("second layer of an MLP skipped",
     "for (int32_t l = 0; l < n_layers; ++l) {\n        double *out = (l == n_layers - 1) ? y",
     "for (int32_t l = 0; l < n_layers; l += 2) {\n        double *out = (l + 2 >= n_layers) ? y"),
    ("bottom-up embedding starts from zero instead of x",
     "memcpy(bu + (size_t)v * H, td + (size_t)v * H, sizeof(double) * (size_t)H);",
     "memset(bu + (size_t)v * H, 0, sizeof(double) * (size_t)H);"),
]


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(what, old, new, tmp_path):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation anchor not unique: {old!r}"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    out = str(tmp_path / "libmutant.so")
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", out,
                    str(src), "-lm"], check=True)
    lib = oracle.load(out)
    caught = []
    for pin in ALL_PINS:
        try:
            pin(lib)
        except (AssertionError, ValueError):
            caught.append(pin.__name__)
            break
    assert caught, f"no pin notices: {what}"
