"""The oracle and the HIP path are independent: neither imports, includes or links the other, and
only tests, the smoke check and the CPU-baseline leg of the bench script use the oracle."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sources(*dirs, ext=(".py", ".c", ".h", ".cpp", ".hip")):
    for d in dirs:
        for base, _, files in os.walk(os.path.join(ROOT, d)):
            if "__pycache__" in base:
                continue
            for f in files:
                if f.endswith(ext):
                    yield os.path.join(base, f)


def test_the_package_never_touches_the_oracle():
    for path in _sources("paper_2104_14129_amd", "include"):
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), path
        assert "actq_oracle" not in text and "orc_" not in text, path


def test_the_oracle_never_touches_the_package():
    for path in _sources("oracle"):
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+paper_2104_14129_amd\b", text, re.M), path
        assert not re.search(r'#include\s+[<"](actq|hip)', text), path
        assert "libactq.so" not in text and "hipcc" not in text, path


def test_the_bench_script_uses_the_oracle_only_for_its_cpu_baseline():
    text = open(os.path.join(ROOT, "bench.py")).read()
    for m in re.finditer(r"^(\s*)import oracle\b", text, re.M):
        before = text[:m.start()]
        guard = before.rstrip().splitlines()[-1]
        assert "no_cpu_baseline" in guard or "import" in guard or guard.strip().startswith("sys.path"), guard
    assert "from oracle" not in text.replace("_SINGLE_THREAD_LEG", "")


def test_the_shared_input_generators_hold_no_method_arithmetic():
    """synth.py draws inputs; it calls nothing of the method (no noise generator, no rounding, no
    packing, no statistics of groups) and imports neither side."""
    text = open(os.path.join(ROOT, "paper_2104_14129_amd", "synth.py")).read()
    code = re.sub(r'""".*?"""', "", text, flags=re.S)          # docstrings may name what the module is not
    code = re.sub(r"#.*", "", code)
    assert not re.search(r"^\s*(import|from)\s+(oracle|\.binding|\.layers|paper_2104_14129_amd)", code, re.M)
    for word in ("philox4x32", "packbits", "unpackbits", "np.floor", "quantize", "dequantize", "group_stats", "ctypes"):
        assert word not in code, word
