"""The CPU checker, the product and the input generators stay apart: the checker
imports nothing of the product, the product nothing of the checker, and the
generators neither."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sources(folder, exts=(".py", ".hip", ".hpp", ".cpp", ".h", ".c")):
    for base, _, names in os.walk(os.path.join(ROOT, folder)):
        for n in names:
            if n.endswith(exts):
                yield os.path.join(base, n)


def test_no_source_of_one_side_names_the_other():
    product = re.compile(r"paper_2605_22416_amd|libavmp|include/avmp")
    checker = re.compile(r"\boracle\b")
    for f in _sources("oracle"):
        assert not product.search(open(f).read()), f
    for f in list(_sources("paper_2605_22416_amd")) + list(_sources("include")):
        assert not checker.search(open(f).read()), f
    for f in _sources("gen"):
        text = open(f).read()
        assert not product.search(text) and not checker.search(text), f


def test_importing_the_checker_and_the_generators_loads_no_product_module():
    code = ("import sys; sys.path.insert(0, %r); import oracle.avmp_oracle, oracle.sampled, gen.inputs; "
            "bad = [m for m in sys.modules if m.startswith('paper_2605_22416_amd')]; "
            "assert not bad, bad" % ROOT)
    subprocess.run([sys.executable, "-c", code], check=True, cwd="/tmp")
