"""Do the oracle's pins bite?  Every case plants ONE plausible mistake - a dropped term, a wrong sign or coefficient,
a misplaced epsilon, a wrong rounding rule, a missing check - in a copy of the oracle's C source (on the CPU, in a
temporary directory; oracle/ itself is never touched), builds the copy, lets the oracle's Python front load it, and
runs the pin tests of tests/test_oracle_*.py against it.  At least one pin must fail for every planted mistake: a
mistake that all pins let through would mean that the GPU path is being compared with an oracle nobody has checked
at that spot."""
import importlib
import inspect
import os
import subprocess

import pytest

import oracle as orc

PIN_MODULES = ["test_oracle_adamw", "test_oracle_norm_step", "test_oracle_convert", "test_oracle_accumulate",
               "test_oracle_fp16"]

# (what is planted, text in mlpo_oracle.c, its replacement, which occurrence of the text)
MISTAKES = [
    ("momentum takes beta1 of the gradient instead of 1 - beta1", "float t2 = c.omb1 * gi;", "float t2 = c.beta1 * gi;", 0),
    ("momentum subtracts the gradient term", "float mi = t1 + t2;", "float mi = t1 - t2;", 0),
    ("variance takes the gradient, not its square", "float gg = gi * gi;", "float gg = gi;", 0),
    ("variance takes 1 - beta1 of the square", "float t4 = c.omb2 * gg;", "float t4 = c.omb1 * gg;", 0),
    ("bias correction of v multiplies", "float q = r / c.sqbc2;", "float q = r * c.sqbc2;", 0),
    ("epsilon dropped", "float d = q + c.eps;", "float d = q;", 0),
    ("epsilon added before the bias correction of v", "float r = sqrtf(vi);", "float r = sqrtf(vi) + c.eps;", 0),
    ("epsilon added under the root", "float r = sqrtf(vi);", "float r = sqrtf(vi + c.eps);", 0),
    ("the update is added", "float pi = pd - upd;", "float pi = pd + upd;", 0),
    ("weight decay dropped", "float pd = p[i] * c.decay;", "float pd = p[i];", 0),
    ("the gradient multiplier is not applied", "float gi = orc_half_to_f32(g[i], half) * gmul;",
     "float gi = orc_half_to_f32(g[i], half);", 0),
    ("p16 is the downcast of the decayed old parameter", "p16[i] = orc_f32_to_half_rne(pi, half);",
     "p16[i] = orc_f32_to_half_rne(pd, half);", 0),
    ("new momentum not stored", "        m[i] = mi;\n", "", 0),
    ("step size multiplied by the bias correction", "c->step_size = (float)((double)hp->lr / bc1);",
     "c->step_size = (float)((double)hp->lr * bc1);", 0),
    ("bias correction of v without the root", "c->sqbc2 = (float)sqrt(bc2);", "c->sqbc2 = (float)bc2;", 0),
    ("decay factor without the learning rate", "c->decay = (float)(1.0 - (double)hp->lr * (double)hp->weight_decay);",
     "c->decay = (float)(1.0 - (double)hp->weight_decay);", 0),
    ("bias correction one step late", "bc1 = 1.0 - pow(b1, (double)step);", "bc1 = 1.0 - pow(b1, (double)(step + 1));", 0),
    ("bias correction of v with beta1", "bc2 = 1.0 - pow(b2, (double)step);", "bc2 = 1.0 - pow(b1, (double)step);", 0),
    ("l2 mode adds the decay coefficient, not decay times p", "float t0 = c.l2 * p[i];", "float t0 = c.l2;", 0),
    ("bf16 widening shifted by 15", "uint32_t w = (uint32_t)h << 16;", "uint32_t w = (uint32_t)h << 15;", 0),
    ("bf16 rounding: ties away from zero", "if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))",
     "if (lower >= 0x8000u)", 0),
    ("bf16 rounding: truncation", "        upper += 1u;\n", "        upper += 0u;\n", 0),
    ("bf16 rounding: a NaN becomes infinity", "return (uint16_t)(((w >> 16) & 0x8000u) | 0x7FC0u);",
     "return (uint16_t)(((w >> 16) & 0x8000u) | 0x7F80u);", 0),
    ("fp16 widening: exponent rebias off by one", "w = sign | ((e + 112u) << 23) | (frac << 13); /* rebias 15 -> 127 */",
     "w = sign | ((e + 113u) << 23) | (frac << 13);", 0),
    ("fp16 rounding: values from 65504 up become infinity", "if (mag >= 0x477FF000u)", "if (mag >= 0x477FE000u)", 0),
    ("fp16 rounding: subnormals keep one bit too few", "drop = (uint32_t)(13 + (-14 - e));", "drop = (uint32_t)(14 + (-14 - e));", 0),
    ("fp16 rounding: ties away from zero", "if (rest > half || (rest == half && (kept & 1u))) kept += 1u;",
     "if (rest >= half) kept += 1u;", 0),
    ("statistics of the scaled gradients", "float u = orc_half_to_f32(g[i], half) * inv_scale;",
     "float u = orc_half_to_f32(g[i], half);", 0),
    ("sum of the gradients, not of their squares", "s += (double)u * (double)u;", "s += (double)u;", 0),
    ("squares summed in fp32", "s += (double)u * (double)u;", "s += (double)(u * u);", 0),
    ("non-finite test also catches the largest finite values", "uint16_t mask = half == ORC_FP16 ? 0x7C00u : 0x7F80u;",
     "uint16_t mask = half == ORC_FP16 ? 0x7800u : 0x7F00u;", 0),
    ("non-finite test misses NaN payloads", "return (h & mask) == mask;", "return (h & 0x7FFFu) == mask;", 0),
    ("clip coefficient without the 1e-6", "coef = max_norm / (nrm + 1e-6f);", "coef = max_norm / nrm;", 0),
    ("clipping also when the norm is below the bound", "if (max_norm > 0.0f && nrm > max_norm)", "if (max_norm > 0.0f)", 0),
    ("gradient multiplier without the unscale factor", "*gmul = inv_scale * coef;", "*gmul = coef;", 0),
    ("norm without the root", "float nrm = (float)sqrt(sumsq);", "float nrm = (float)sumsq;", 0),
    ("a norm beyond fp32 does not skip the step", "if (!(norm <= FLT_MAX)) bad = 1u;", "if (0) bad = 1u;", 0),
    ("a flagged step is applied all the same", "    if (bad) return 0;\n", "    if (0) return 0;\n", 0),
    ("the step counter is not advanced", "steps_applied + 1, gmul, half);", "steps_applied + (steps_applied == 0), gmul, half);", 0),
    ("the processing order is ignored and a subgroup is visited twice",
     "const orc_subgroup* s = &sg[order ? order[k] : k];", "const orc_subgroup* s = &sg[order ? order[0] : k];", 0),
    ("accumulation subtracts", "float sum = orc_half_to_f32(acc[i], half) + orc_half_to_f32(g[i], half);",
     "float sum = orc_half_to_f32(acc[i], half) - orc_half_to_f32(g[i], half);", 0),
    ("the first micro-batch is added to what the buffer held", "            acc[i] = g[i];\n            continue;\n", "", 0),
    ("a NaN sum keeps whatever payload the addition produced", "acc[i] = (sum != sum) ? nan : orc_f32_to_half_rne(sum, half);",
     "acc[i] = orc_f32_to_half_rne(sum, half) | ((sum != sum) ? 1u : 0u);", 0),
]


def _pins():
    """The pin tests that take the oracle (and nothing else but parameters they are marked with), expanded."""
    out = []
    for name in PIN_MODULES:
        mod = importlib.import_module(name)
        for fname, fn in sorted(vars(mod).items()):
            if not fname.startswith("test_") or not callable(fn):
                continue
            params = list(inspect.signature(fn).parameters)
            if "oracle" not in params:
                continue
            others = [p for p in params if p != "oracle"]
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            if not others:
                out.append((f"{name}.{fname}", fn, {}))
            elif len(others) == 1 and len(marks) == 1 and marks[0].args[0] == others[0]:
                for v in marks[0].args[1]:
                    out.append((f"{name}.{fname}[{v}]", fn, {others[0]: v}))
    return out


def _build_mutant(tmp_path, old, new, nth):
    src = open(os.path.join(os.path.dirname(orc.__file__), "mlpo_oracle.c")).read()
    assert src.count(old) > nth, f"the text to replace is not in the oracle's source: {old!r}"
    at = -1
    for _ in range(nth + 1):
        at = src.index(old, at + 1)
    c_file = tmp_path / "mutant.c"
    c_file.write_text(src[:at] + new + src[at + len(old):])
    so = str(tmp_path / "libmutant.so")
    flags = [f for f in orc.CFLAGS if f not in ("-Wall", "-Wextra")]
    subprocess.run(["gcc", *flags, "-o", so, str(c_file), "-lm"], check=True)
    return so


def test_the_unchanged_oracle_passes_the_battery(oracle):
    """The battery itself: with the real oracle no pin may fail (otherwise a failure below would prove nothing)."""
    pins = _pins()
    assert len(pins) >= 45
    for label, fn, kw in pins:
        fn(oracle, **kw)


@pytest.mark.parametrize("case", range(len(MISTAKES)), ids=[m[0] for m in MISTAKES])
def test_a_planted_mistake_fails_a_pin(oracle, tmp_path, monkeypatch, case):
    what, old, new, nth = MISTAKES[case]
    so = _build_mutant(tmp_path, old, new, nth)
    monkeypatch.setattr(orc, "build", lambda force=False: so)
    monkeypatch.setattr(orc, "_lib", None)          # the front loads the library again: now the mutant
    caught = None
    for label, fn, kw in _pins():
        try:
            fn(orc, **kw)
        except (AssertionError, ArithmeticError, pytest.fail.Exception):
            caught = label
            break
    assert caught is not None, f"no pin noticed the planted mistake: {what}"
    print(f"{what}: caught by {caught}")


# ---- the allocation oracle (Eq. 1, Section 3.3): the same for its Python source ----------------------------------

TIER_MISTAKES = [
    ("floor instead of Eq. 1's ceiling", "t = {i: ceil(Fraction(m) * bw[i] / total) for i in tiers}",
     "t = {i: int(Fraction(m) * bw[i] / total) for i in tiers}"),
    ("the surplus is taken from the tier that finishes first", "worst = max(cand,", "worst = min(cand,"),
    ("the surplus is taken from the slowest tier whatever it holds", "key=lambda i: (Fraction(t[i]) / bw[i], -bw[i], i))",
     "key=lambda i: (-bw[i], i))"),
    ("shares relative to all tiers, not to those still open", "total = sum(bw[i] for i in tiers)", "total = sum(bw)"),
    ("capacities ignored", "trial[i] > capacity[i]]", "trial[i] > capacity[i] and False]"),
    ("a full tier keeps its share, not its capacity", "count[i] = capacity[i]\n", "count[i] = trial[i]\n"),
    ("the faster tier takes the lower ids", "key=lambda i: (bw[i], -i))", "key=lambda i: (-bw[i], i))"),
    ("observed bandwidth is time over bytes", "return [bm / s if", "return [s / bm if"),
    ("an idle tier loses its estimate", "else b for b, bm, s in", "else 0.0 for b, bm, s in"),
]


def _tier_pins():
    import test_tier_alloc as T
    return T, [T.test_paper_two_to_one_split, T.test_oracle_minimises_the_finishing_time_brute_force,
               T.test_oracle_special_cases, T.test_bandwidth_update_follows_the_observations]


@pytest.mark.parametrize("case", range(len(TIER_MISTAKES)), ids=[m[0] for m in TIER_MISTAKES])
def test_a_mistake_planted_in_the_allocation_oracle_fails_a_pin(monkeypatch, case):
    import types
    from oracle import tier_alloc
    what, old, new = TIER_MISTAKES[case]
    src = open(tier_alloc.__file__).read()
    assert src.count(old) == 1, f"the text to replace is not (or not once) in the oracle's source: {old!r}"
    mutant = types.ModuleType("tier_alloc_mutant")
    exec(compile(src.replace(old, new), "tier_alloc_mutant.py", "exec"), mutant.__dict__)
    T, pins = _tier_pins()
    for fn in pins:                                   # the battery itself: green with the real oracle
        fn()
    monkeypatch.setattr(T, "O", mutant)
    caught = None
    for fn in pins:
        try:
            fn()
        except (AssertionError, ArithmeticError, MemoryError, IndexError, KeyError):
            caught = fn.__name__
            break
    assert caught is not None, f"no pin noticed the planted mistake: {what}"
    print(f"{what}: caught by {caught}")
