"""Mutation check of the oracle pins (CPU only): each plausible mistake is planted in a COPY of
the oracle's C source, the copy is built, and tests/test_oracle_pins.py must fail on it.  The
real oracle and the GPU path are never touched."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

C = os.path.join("oracle", "selsync_oracle.c")
PY = os.path.join("oracle", "selsync_oracle.py")

# (name, text in the oracle source, replacement[, file: the C source unless said otherwise])
MUT = [
 ("norm float product", "acc += (double)gh * (double)gh;\n    }\n    return acc;\n}\n\ndouble selsync_oracle_norm_sq_accum_bf16", "acc += (double)(gh * gh);\n    }\n    return acc;\n}\n\ndouble selsync_oracle_norm_sq_accum_bf16"),
 ("norm ignores scale", "float gh = grad_scale * g[j];\n        acc +=", "float gh = g[j];\n        acc +="),
 ("sgd wd sign", "float d = gh + dec;\n        float mom;\n        if (first) {\n            mom = d;\n        } else {\n            float mm = mu * m[j];\n            mom = mm + d;\n        }\n        float stepv = lr * mom;\n        m[j] = mom;\n        w[j] = w[j] - stepv;", "float d = gh - dec;\n        float mom;\n        if (first) {\n            mom = d;\n        } else {\n            float mm = mu * m[j];\n            mom = mm + d;\n        }\n        float stepv = lr * mom;\n        m[j] = mom;\n        w[j] = w[j] - stepv;"),
 ("sgd plus step", "w[j] = w[j] - stepv;", "w[j] = w[j] + stepv;"),
 ("sgd first ignored", "if (first) {\n            mom = d;\n        } else {\n            float mm = mu * m[j];\n            mom = mm + d;\n        }\n        float stepv = lr * mom;\n        m[j] = mom;\n        w[j]", "{\n            float mm = mu * m[j];\n            mom = mm + d;\n        }\n        float stepv = lr * mom;\n        m[j] = mom;\n        w[j]"),
 ("sgd momentum on d", "mom = mm + d;\n        }\n        float stepv = lr * mom;\n        m[j] = mom;\n        w[j]", "mom = mu * (m[j] + d);\n        }\n        float stepv = lr * mom;\n        m[j] = mom;\n        w[j]"),
 ("tracker alpha^j", "pow(1.0 - t->alpha, (double)j)", "pow(t->alpha, (double)j)"),
 ("tracker oldest first", "t->hist[t->len - 1 - j]", "t->hist[j]"),
 ("tracker no fabs", "fabs(s - t->s_prev) / t->s_prev", "(s - t->s_prev) / t->s_prev"),
 ("tracker divide by s", "fabs(s - t->s_prev) / t->s_prev", "fabs(s - t->s_prev) / s"),
 ("tracker unnormalised", "double s = num / den;", "double s = num;"),
 ("avg drops last", "for (int k = 0; k < K; ++k)\n            s += (double)replicas[k][j];", "for (int k = 0; k < K - 1; ++k)\n            s += (double)replicas[k][j];"),
 ("avg float accumulate", "double s = 0.0;\n        for (int k = 0; k < K; ++k)\n            s += (double)replicas[k][j];\n        float mean = (float)(s / (double)K);", "float s = 0.0f;\n        for (int k = 0; k < K; ++k)\n            s += replicas[k][j];\n        float mean = s / (float)K;"),
 ("avg no writeback", "for (int k = 0; k < K; ++k)\n            replicas[k][j] = mean;", "for (int k = 1; k < K; ++k)\n            replicas[k][j] = mean;"),
 ("flag strict", "return delta_g >= threshold ? 1 : 0;", "return delta_g > threshold ? 1 : 0;"),
 ("bf16 truncates", "u += 0x7fffu + lsb;", "u += 0;"),
 ("bf16 ties away", "u += 0x7fffu + lsb;", "u += 0x8000u;"),
 ("plain sgd ignores decay", "float d = gh + dec;\n        float stepv = lr * d;\n        w[j] = w[j] - stepv;", "float d = gh;\n        float stepv = lr * d;\n        w[j] = w[j] - stepv;"),
 ("plain sgd plus step", "float stepv = lr * d;\n        w[j] = w[j] - stepv;", "float stepv = lr * d;\n        w[j] = w[j] + stepv;"),
 ("nesterov looks at old buffer", "float look = mu * mom;\n        float dir = d + look;\n        float stepv = lr * dir;\n        m[j] = mom;\n        w[j]", "float look = mu * m[j];\n        float dir = d + look;\n        float stepv = lr * dir;\n        m[j] = mom;\n        w[j]"),
 ("nesterov drops gradient term", "float dir = d + look;\n        float stepv = lr * dir;\n        m[j] = mom;\n        w[j]", "float dir = look;\n        float stepv = lr * dir;\n        m[j] = mom;\n        w[j]"),
 ("nesterov stores direction", "float stepv = lr * dir;\n        m[j] = mom;\n        w[j]", "float stepv = lr * dir;\n        m[j] = dir;\n        w[j]"),
 ("grad mean drops last worker", "for (int k = 0; k < K; ++k) {\n            float gh = grad_scale * grads[k][j];", "for (int k = 0; k < K - 1; ++k) {\n            float gh = grad_scale * grads[k][j];"),
 ("grad mean scaled after the sum", "float gh = grad_scale * grads[k][j];\n            s += (double)gh;\n        }\n        gbar[j] = (float)(s / (double)K);", "float gh = grads[k][j];\n            s += (double)gh;\n        }\n        gbar[j] = grad_scale * (float)(s / (double)K);"),
 # mistakes in the composition of the gradient-aggregation variants (oracle/selsync_oracle.py)
 ("ga sync applies own gradient", "sgd_update(params[k], mom(k), gbar, lr, momentum, weight_decay, 1.0, first, nesterov=nesterov)", "sgd_update(params[k], mom(k), grads[k], lr, momentum, weight_decay, grad_scale, first, nesterov=nesterov)", PY),
 ("ga scales the mean again", "sgd_update(params[k], mom(k), gbar, lr, momentum, weight_decay, 1.0, first, nesterov=nesterov)", "sgd_update(params[k], mom(k), gbar, lr, momentum, weight_decay, grad_scale, first, nesterov=nesterov)", PY),
 ("ga leaves stale bf16 copies", "copies[k][t][...] = f32_to_bf16(params[k][t])\n\n\ndef ga_update_adam", "pass\n\n\ndef ga_update_adam", PY),
 ("ga adam applies own gradient", "adam_update(params[k], m[k], v[k], gbar, lr, beta1, beta2, eps, weight_decay, step, 1.0)", "adam_update(params[k], m[k], v[k], grads[k], lr, beta1, beta2, eps, weight_decay, step, grad_scale)", PY),
 ("ga adam scales the mean again", "adam_update(params[k], m[k], v[k], gbar, lr, beta1, beta2, eps, weight_decay, step, 1.0)", "adam_update(params[k], m[k], v[k], gbar, lr, beta1, beta2, eps, weight_decay, step, grad_scale)", PY),
 # mixed precision (C source)
 ("bf16 widening shifts by 15", "uint32_t u = ((uint32_t)h) << 16;", "uint32_t u = ((uint32_t)h) << 15;"),
 ("mixed sgd copy taken before the step", "master[j] = master[j] - stepv;\n        copy[j] = selsync_oracle_f32_to_bf16(master[j]);\n    }\n}\n\n/*\n * Momentum-free", "copy[j] = selsync_oracle_f32_to_bf16(master[j]);\n        master[j] = master[j] - stepv;\n    }\n}\n\n/*\n * Momentum-free"),
 ("mixed sgd steps the rounded copy", "float dec = wd * master[j];\n        float d = gh + dec;\n        float mom;\n        if (first) {\n            mom = d;\n        } else {\n            float mm = mu * m[j];\n            mom = mm + d;\n        }\n        float stepv = lr * mom;\n        m[j] = mom;\n        master[j] = master[j] - stepv;", "float dec = wd * master[j];\n        float d = gh + dec;\n        float mom;\n        if (first) {\n            mom = d;\n        } else {\n            float mm = mu * m[j];\n            mom = mm + d;\n        }\n        float stepv = lr * mom;\n        m[j] = mom;\n        master[j] = selsync_oracle_bf16_to_f32(copy[j]) - stepv;"),
 ("mixed norm of the unscaled gradient", "float gh = grad_scale * selsync_oracle_bf16_to_f32(g[j]);\n        acc +=", "float gh = selsync_oracle_bf16_to_f32(g[j]);\n        acc +="),
 ("mixed average leaves worker copies stale", "masters[k][j] = mean;\n            copies[k][j] = h;", "masters[k][j] = mean;"),
 ("mixed average rounds the masters too", "global_master[j] = mean;\n        global_copy[j] = h;", "mean = selsync_oracle_bf16_to_f32(h);\n        global_master[j] = mean;\n        global_copy[j] = h;"),
 # Adam as the local update (C source)
 ("adam second moment not squared", "float t5 = t4 * gd;\n        float vn = t3 + t5;\n        float mh = mn / bc1;\n        float vh = vn / bc2;\n        float num = lr * mh;\n        float den = sqrtf(vh) + eps;\n        float q = num / den;\n        m[j] = mn;\n        v[j] = vn;\n        w[j] = w[j] - q;\n    }\n}\n\nvoid selsync_oracle_adam_bf16", "float t5 = t4;\n        float vn = t3 + t5;\n        float mh = mn / bc1;\n        float vh = vn / bc2;\n        float num = lr * mh;\n        float den = sqrtf(vh) + eps;\n        float q = num / den;\n        m[j] = mn;\n        v[j] = vn;\n        w[j] = w[j] - q;\n    }\n}\n\nvoid selsync_oracle_adam_bf16"),
 ("adam no bias correction of v", "float vh = vn / bc2;\n        float num = lr * mh;\n        float den = sqrtf(vh) + eps;\n        float q = num / den;\n        m[j] = mn;\n        v[j] = vn;\n        w[j] = w[j] - q;\n    }\n}\n\nvoid selsync_oracle_adam_bf16", "float vh = vn;\n        float num = lr * mh;\n        float den = sqrtf(vh) + eps;\n        float q = num / den;\n        m[j] = mn;\n        v[j] = vn;\n        w[j] = w[j] - q;\n    }\n}\n\nvoid selsync_oracle_adam_bf16"),
 ("adam eps under the root", "float den = sqrtf(vh) + eps;\n        float q = num / den;\n        m[j] = mn;\n        v[j] = vn;\n        w[j] = w[j] - q;\n    }\n}\n\nvoid selsync_oracle_adam_bf16", "float den = sqrtf(vh + eps);\n        float q = num / den;\n        m[j] = mn;\n        v[j] = vn;\n        w[j] = w[j] - q;\n    }\n}\n\nvoid selsync_oracle_adam_bf16"),
 ("adam first step keeps stale buffers", "float mo = first ? 0.0f : m[j];\n        float vo = first ? 0.0f : v[j];\n        float t1 = b1 * mo;\n        float t2 = omb1 * gd;\n        float mn = t1 + t2;\n        float t3 = b2 * vo;\n        float t4 = omb2 * gd;\n        float t5 = t4 * gd;\n        float vn = t3 + t5;\n        float mh = mn / bc1;\n        float vh = vn / bc2;\n        float num = lr * mh;\n        float den = sqrtf(vh) + eps;\n        float q = num / den;\n        m[j] = mn;\n        v[j] = vn;\n        w[j] = w[j] - q;\n    }\n}\n\nvoid selsync_oracle_adam_bf16", "float mo = m[j];\n        float vo = v[j];\n        float t1 = b1 * mo;\n        float t2 = omb1 * gd;\n        float mn = t1 + t2;\n        float t3 = b2 * vo;\n        float t4 = omb2 * gd;\n        float t5 = t4 * gd;\n        float vn = t3 + t5;\n        float mh = mn / bc1;\n        float vh = vn / bc2;\n        float num = lr * mh;\n        float den = sqrtf(vh) + eps;\n        float q = num / den;\n        m[j] = mn;\n        v[j] = vn;\n        w[j] = w[j] - q;\n    }\n}\n\nvoid selsync_oracle_adam_bf16"),
 # tracker window and conventions (C source)
 ("tracker keeps one value too many", "if (t->len == t->window) {\n        memmove(t->hist, t->hist + 1, (size_t)(t->window - 1) * sizeof(double));\n        t->len -= 1;\n    }\n    t->hist[t->len++] = x;", "t->hist[t->len < t->window ? t->len++ : t->window - 1] = x;"),
 ("tracker first step compares with zero", "if (!t->has_prev) {\n        delta = 0.0;\n    } else if", "if (0) {\n        delta = 0.0;\n    } else if"),
 # partitioner and counters (oracle/selsync_oracle.py)
 ("seldp rotates the other way", "order.extend(chunks[(worker + j) % num_workers])", "order.extend(chunks[(worker - j) % num_workers])", PY),
 ("seldp does not rotate", "order.extend(chunks[(worker + j) % num_workers])", "order.extend(chunks[j % num_workers])", PY),
 ("chunks give the extra sample to the last workers", "size = base + (1 if c < rem else 0)", "size = base + (1 if c >= num_workers - rem else 0)", PY),
 ("lssr counts synchronising steps", "return self.steps_local / tot if tot else float(\"nan\")", "return self.steps_sync / tot if tot else float(\"nan\")", PY),
 ("all workers must agree to synchronise", "sync = int(any(fs))", "sync = int(all(fs))", PY),
 ("ga local step averages anyway", "    if not sync:\n        for k in range(K):\n            sgd_update(", "    if False:\n        for k in range(K):\n            sgd_update(", PY),
]


@pytest.fixture(scope="module")
def tree(tmp_path_factory):
    base = str(tmp_path_factory.mktemp("mutants"))
    for d in ("oracle", "tests", "paper_2307_07950_amd"):
        shutil.copytree(os.path.join(ROOT, d), os.path.join(base, d),
                        ignore=shutil.ignore_patterns("*.so", "__pycache__", "csrc", "*.tmp.*"))
    return base


def run_pins(base):
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-q", "-x",
                        "-p", "no:cacheprovider"], cwd=base, capture_output=True, text=True, timeout=300)
    return r.returncode, r.stdout[-2000:]


def test_unmutated_copy_passes(tree):
    rc, out = run_pins(tree)
    assert rc == 0, out


@pytest.mark.parametrize("mut", MUT, ids=[m[0].replace(" ", "_") for m in MUT])
def test_pins_catch_planted_mistake(tree, mut):
    name, old, new = mut[:3]
    rel = mut[3] if len(mut) > 3 else C
    path = os.path.join(tree, rel)
    good = open(os.path.join(ROOT, rel)).read()
    assert good.count(old) >= 1, "mutation site not found: %s" % name
    try:
        open(path, "w").write(good.replace(old, new, 1))
        os.utime(path, None)
        rc, out = run_pins(tree)
        assert rc != 0, "the pins did not notice: %s" % name
    finally:
        open(path, "w").write(good)
        os.utime(path, None)
