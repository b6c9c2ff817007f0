"""Plants one mistake at a time in a copy of the oracle's C source (on the CPU) and checks
that the pins in test_oracle_pins.py notice: a pin set that lets a dropped term, a flipped
comparison or a wrong index through would not be pinning anything."""
import importlib.util
import shutil
from pathlib import Path

import pytest

import test_oracle_pins as pins

ORACLE_DIR = Path(__file__).resolve().parent.parent / "oracle"

MUTANTS = [
    ("tie goes to the higher index", "return (x->j > y->j) - (x->j < y->j);",
     "return (x->j < y->j) - (x->j > y->j);"),
    ("smallest scores kept", "return x->score > y->score ? -1 : 1;", "return x->score < y->score ? -1 : 1;"),
    ("magnitude instead of signed score", "out[j] = group_sum;", "out[j] = group_sum < 0 ? -group_sum : group_sum;"),
    ("transposed score operands", "s += (int64_t)q[c] * (int64_t)Kh[j * k + c];",
     "s += (int64_t)Qt[(n * L + j) * k + c] * (int64_t)Kh[(g * vec + r) * k + c];"),
    ("group sum keeps only the last row", "group_sum += s;", "group_sum = s;"),
    ("scale dropped", "S[t * keep + a] = scale * acc;", "S[t * keep + a] = acc;"),
    ("key row taken by list position", "const float *kr = K + (n * L + list[a]) * (int64_t)d;",
     "const float *kr = K + (n * L + a) * (int64_t)d;"),
    ("softmax not normalised", "p[a] = p[a] / z;", "p[a] = p[a];"),
    ("softmax of the negated score", "p[a] = exp(s[a] - m);", "p[a] = exp(m - s[a]);"),
    ("value row from the wrong head", "const float *vr = V + (n * L + list[a]) * (int64_t)d;",
     "const float *vr = V + (list[a]) * (int64_t)d;"),
    ("row reads its neighbour unit's list", "int64_t n = r / L, i = r % L, g = i / vec;",
     "int64_t n = r / L, i = r % L, g = (i / vec + 1) % G;"),
    ("list not sorted ascending", "qsort(out, (size_t)keep, sizeof(int32_t), by_int32);", ";"),
    ("keep rounds down", "floor(ratio * (double)L + 0.5)", "floor(ratio * (double)L)"),
    ("codes truncated instead of rounded", "float v = rintf(Y[t] * s);", "float v = truncf(Y[t] * s);"),
    ("quantiser range 2^(bits-1)", "const float qmax = (float)((1 << (bits - 1)) - 1);",
     "const float qmax = (float)(1 << (bits - 1));"),
    ("precision ignored: always the int8 range", "const float qmax = (float)((1 << (bits - 1)) - 1);",
     "const float qmax = 127.0f;"),
    ("packed fields in the opposite order", "<< (bits * f);", "<< (bits * (per - 1 - f));"),
    ("unpacking without sign extension", "codes[j] = (int8_t)(((int32_t)field ^ sign) - sign);",
     "codes[j] = (int8_t)field; (void)sign;"),
    ("threshold is strict", "if (sc[j] >= theta) {", "if (sc[j] > theta) {"),
    ("empty unit keeps the highest index among equals", "if (sc[j] > sc[best]) best = j;", "if (sc[j] >= sc[best]) best = j;"),
    ("empty unit keeps nothing", "if (count == 0) {\n                if (col) col[row_ptr[u]] = best;\n                count = 1;",
     "if (count < 0) {\n                if (col) col[row_ptr[u]] = best;\n                count = 1;"),
    # (starts at the unit before: every read stays inside col, a planted mistake must not fault)
    ("CSR row reads the keys of the unit before", "const int32_t *list = col + row_ptr[u];",
     "const int32_t *list = col + row_ptr[u > 0 ? u - 1 : 0];"),
    ("CSR weights not normalised", "const double w = p[a] / z;", "const double w = p[a]; (void)z;"),
    ("ternary projection ignores the minus signs", "else if (sign < 0) y = y - X[r * d + c];", "else if (sign < 0) y = y + X[r * d + c];"),
    ("projection matrix transposed", "y = fmaf(X[r * d + c], R[(int64_t)c * k + j], y);",
     "y = fmaf(X[r * d + c], R[(int64_t)(j % d) * k + (c % k)], y);"),
]

PIN_TESTS = [name for name in dir(pins) if name.startswith("test_")]


def load_oracle_copy(tmp_path, old, new):
    src = (ORACLE_DIR / "dsa_oracle.c").read_text()
    assert src.count(old) >= 1, f"mutation site not found: {old!r}"
    (tmp_path / "dsa_oracle.c").write_text(src.replace(old, new))
    shutil.copy(ORACLE_DIR / "dsa_oracle.py", tmp_path / "dsa_oracle.py")
    spec = importlib.util.spec_from_file_location(f"oracle_mutant_{abs(hash(old))}", tmp_path / "dsa_oracle.py")
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)      # paths inside are relative to its own (copied) file
    return mod


def run_pins(mod, workload):
    import inspect
    failures = []
    for name in PIN_TESTS:
        fn = getattr(pins, name)
        params = inspect.signature(fn).parameters
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        cases = [{}]
        for m in marks:
            names = [s.strip() for s in m.args[0].split(",")]
            cases = [dict(c, **dict(zip(names, v if isinstance(v, (tuple, list)) and len(names) > 1 else [v])))
                     for c in cases for v in m.args[1]]
        for case in cases:
            kwargs = dict(case)
            if "oracle" in params:
                kwargs["oracle"] = mod
            if "workload" in params:
                kwargs["workload"] = workload
            try:
                fn(**kwargs)
            except (AssertionError, ValueError):
                failures.append(name)
                break
    return failures


def test_unmutated_copy_passes(tmp_path, workload):
    mod = load_oracle_copy(tmp_path, "group_sum += s;", "group_sum += s;")
    assert run_pins(mod, workload) == []


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch(tmp_path, workload, what, old, new):
    mod = load_oracle_copy(tmp_path, old, new)
    assert run_pins(mod, workload), f"no pin noticed: {what}"
