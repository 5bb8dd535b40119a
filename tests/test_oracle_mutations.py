"""How sharp the oracle's pins are: single mistakes are planted in a private copy of the oracle
(on the CPU), and for every one of them at least one pin of test_oracle_pins.py must fail.
A mistake that no pin notices would mean the oracle could be wrong in that way unnoticed."""
import importlib.util
import itertools
import os
import shutil
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
C_FILE, PY_FILE = "xq_oracle.c", "xq_oracle.py"

# (file, original text, planted text)
MUTANTS = [
    (C_FILE, "if (v < mn) mn = v;", "if (v > mn) mn = v;"),                              # min becomes max
    (C_FILE, "if (v > mx) mx = v;", "if (v >= mx) mx = mn;"),                            # max lost
    (C_FILE, "range / (float)n;", "range / (float)(n + 1);"),                            # 2^B levels instead of 2^B - 1
    (C_FILE, "float r = rintf(t);", "float r = floorf(t + 0.5f);"),                      # ties away from even
    (C_FILE, "float r = rintf(t);", "float r = floorf(t);"),                             # truncation
    (C_FILE, "volatile float c1 = eta * (float)n;", "volatile float c1 = eta;"),         # Alg. 2's form of the shift
    (C_FILE, "volatile float two_eta = 2.0f * eta;", "volatile float two_eta = eta;"),   # scale shrunk by eta, not 2 eta
    (C_FILE, "volatile float zc = mn + shift;", "volatile float zc = mn - shift;"),      # sign of the shift
    (C_FILE, "volatile float zc = mn + shift;", "volatile float zc = mn;"),              # zero-point not calibrated
    (C_FILE, "volatile float sc = c2 * s;", "volatile float sc = s;"),                   # scale not calibrated
    (C_FILE, "xqo_quantize_group(k + (long)G * g * D + d, D, g,", "xqo_quantize_group(k + (long)G * g * D + d, 1, g,"),      # keys grouped along channels
    (C_FILE, "xqo_quantize_group(v + (long)t * D + j * g, 1, g,", "xqo_quantize_group(v + (long)t * D + j, D / g, g,"),      # value groups interleaved
    (C_FILE, "long m = (long)(t / g) * D + d;", "long m = (long)(t / g) * D + (D - 1 - d);"),                                # key metadata of the wrong channel
    (C_FILE, "long m = (long)t * J + d / g;", "long m = (long)t * J + d % J;"),                                              # value metadata of the wrong group
    (C_FILE, "return g * ((over + g - 1) / g);", "return g * (over / g);"),              # packed length rounded down
    (C_FILE, "u[t] = sigma * acc;", "u[t] = acc;"),                                      # softmax scale dropped
    (C_FILE, "u[t] = exp(u[t] - m); denom += u[t];", "u[t] = exp(u[t] - m); denom += 1.0;"),   # wrong normaliser
    (C_FILE, "acc += u[t] * Vh[(long)t * D + d];", "acc += u[t] * Vh[(long)t * D + (D - 1 - d)];"),  # output channels mirrored
    (C_FILE, "acc += (double)xqo_half_to_float(q[d]) * Kh[(long)t * D + d];",
     "acc += (double)xqo_half_to_float(q[d]) * Kh[(long)t * D + (d ^ 1)];"),            # q . K with channels swapped in pairs
    (C_FILE, "int n = t + 1;", "int n = t;"),                                           # a prompt token does not see itself
    (C_FILE, "u[j] = sigma * acc;", "u[j] = acc;"),                                      # prefill softmax scale dropped
    (C_FILE, "acc += u[j] * (double)xqo_half_to_float(V[(long)j * D + d]);",
     "acc += u[j] * (double)xqo_half_to_float(V[(long)j * D + (D - 1 - d)]);"),          # prefill output channels mirrored
    (C_FILE, "int wi = d / per, bit = B * (d % per);", "int wi = d / per, bit = B * (per - 1 - d % per);"),  # MSB-first key words
    (C_FILE, "int slot = d / CPL, e = (t % 32) * CPL + d % CPL;", "int slot = d / CPL, e = (d % CPL) * 32 + (t % 32);"),  # value order inside a slot
    (C_FILE, "if (l < m || l % 2 == 0) bits +=", "if (l < m || l % 2 == 1) bits +="),    # second layer of a pair charged
    (C_FILE, "(l < q) ? 2.0 : 1.0;", "(l <= q) ? 2.0 : 1.0;"),                           # bit-width threshold off by one
    (C_FILE, "+ (1.0 - (double)gamma0) * e1[i] + 0.5);", "+ (1.0 - (double)gamma0) * e1[i]);"),  # merged codes floored
    (C_FILE, "else if (mode == 3) x = ceil(", "else if (mode == 3) x = floor("),         # ceiling mode floors
    (C_FILE, "if (lead < -14) lead = -14;", "if (lead < -15) lead = -15;"),              # fp16 subnormal quantum
    (PY_FILE, "return 2 if l < (self.vq if is_v else self.kq) else 1", "return 2 if l <= (self.vq if is_v else self.kq) else 1"),
    (PY_FILE, "return self.eta2 if B == 2 else self.eta1", "return self.eta1 if B == 2 else self.eta2"),       # eta of the other bit width
    (PY_FILE, "if l < (self.vm if is_v else self.km):", "if l < (self.km if is_v else self.vm):"),             # km and vm swapped
    (PY_FILE, "cl = self.share_group * (l // self.share_group) + self.share_dominant", "cl = self.share_group * (l // self.share_group)"),
    (PY_FILE, "return cl if cl < self.n_layers else l", "return cl"),                    # trailing group reads a layer that does not exist
    (PY_FILE, 'kc = state[sch.code_layer(l, False)]["k_codes"]',
     'kc = state[l]["k_codes"] if state[l]["k_codes"] is not None else state[l - 1]["k_codes"]'),            # always the layer below
    (PY_FILE, 'Kh = np.concatenate([dequant_k(kc, st["k_scale"], st["k_zero"], g)',
     'Kh = np.concatenate([dequant_k(kc, state[sch.code_layer(l, False)]["k_scale"], state[sch.code_layer(l, False)]["k_zero"], g)'),  # scale/zero of the code layer
    (PY_FILE, 'Vh = np.concatenate([dequant_v(vc, st["v_scale"], st["v_zero"], g)',
     'Vh = np.concatenate([dequant_v(vc, state[sch.code_layer(l, True)]["v_scale"], state[sch.code_layer(l, True)]["v_zero"], g)'),
    (PY_FILE, "k_res=K[l, Tq:].copy(), v_res=V[l, Tq:].copy()", "k_res=K[l, Tq:].copy(), v_res=K[l, Tq:].copy()"),   # keys in the value window
    (PY_FILE, "k1 = quantize_k(K[l + 1], g, R, bk, sch.eta(bk), True)[0]", "k1 = quantize_k(K[l], g, R, bk, sch.eta(bk), True)[0]"),  # merged with itself
    (PY_FILE, "kc = merge_codes(kc, k1, bk, sch.merge_mode, sch.gamma0)", "kc = merge_codes(k1, kc, bk, sch.merge_mode, sch.gamma0)"),  # merge weights swapped
]


def _pins():
    """Every pin of test_oracle_pins.py as (name, callable(oracle)), parametrised ones expanded."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import test_oracle_pins as pins
    out = []
    for name in sorted(dir(pins)):
        fn = getattr(pins, name)
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        axes = []
        for m in marks:
            names = [n.strip() for n in m.args[0].split(",")]
            axes.append([dict(zip(names, v if isinstance(v, (tuple, list)) else (v,))) for v in m.args[1]])
        for combo in itertools.product(*axes) if axes else [()]:
            kw = {}
            for d in combo:
                kw.update(d)
            out.append((name, (lambda o, fn=fn, kw=kw: fn(o, **kw))))
    return out


def _load_mutant(tmp, idx, fname, old, new):
    d = os.path.join(tmp, f"oracle_mut_{idx}")
    os.makedirs(d)
    for f in (C_FILE, PY_FILE, "build.py", "__init__.py"):
        shutil.copy(os.path.join(ROOT, "oracle", f), d)
    path = os.path.join(d, fname)
    src = open(path).read()
    assert src.count(old) >= 1, f"mutation target not found in {fname}: {old}"
    open(path, "w").write(src.replace(old, new, 1))
    pkg = f"oracle_mut_{idx}"
    spec = importlib.util.spec_from_file_location(pkg, os.path.join(d, "__init__.py"), submodule_search_locations=[d])
    mod = importlib.util.module_from_spec(spec)
    sys.modules[pkg] = mod
    spec.loader.exec_module(mod)
    sub = importlib.import_module(pkg + ".xq_oracle")
    sub.lib()
    return sub


@pytest.mark.parametrize("idx", range(len(MUTANTS)))
def test_planted_mistake_is_caught(idx, tmp_path):
    fname, old, new = MUTANTS[idx]
    mutant = _load_mutant(str(tmp_path), idx, fname, old, new)
    caught = None
    for name, run in _pins():
        try:
            run(mutant)
        except AssertionError:
            caught = name
            break
        except Exception as e:      # a crash of the planted code is a catch as well
            caught = f"{name} ({type(e).__name__})"
            break
    assert caught is not None, f"no pin notices: {old!r} -> {new!r}"


def test_the_unchanged_copy_passes(tmp_path):
    """The harness itself: a private copy without a planted mistake passes every pin."""
    clean = _load_mutant(str(tmp_path), "clean", C_FILE, "u[t] = sigma * acc;", "u[t] = sigma * acc;")
    for name, run in _pins():
        run(clean)
