"""Formats the error log that the comparison bars of tests/util.py write (VER_PARITY_LOG=<file> while the GPU tests
run) as a markdown table: per bar and tensor, the largest elementwise and 2-norm relative error over all tests and
the test that produced it, then every tensor of the full-size `max` and `large` minibatches.

    VER_PARITY_LOG=/tmp/parity.log python -m pytest tests -m gpu
    python -m tests.parity_report /tmp/parity.log > profiles/parity_bf16.md
"""
import collections
import sys


def main(path):
    rows = [line.rstrip("\n").split("\t") for line in open(path) if line.strip()]
    agg = collections.OrderedDict()
    for test, bar, what, em, e2 in rows:
        what = what.replace(" (sampled pieces)", "")
        key = (bar, what.split(".")[-1] if what.startswith("layer") else what.split(" ")[0] if bar == "update" else what)
        a = agg.setdefault(key, [0.0, "", 0.0, "", 0])
        em, e2 = float(em), float(e2)
        if em >= a[0]:
            a[0], a[1] = em, test.split("::")[-1]
        if e2 >= a[2]:
            a[2], a[3] = e2, test.split("::")[-1]
        a[4] += 1
    out = ["# Measured parity errors of the GPU tests against the CPU oracle", "",
           "Written by `python -m tests.parity_report <log>` from the log of "
           "`VER_PARITY_LOG=<log> python -m pytest tests -m gpu` on one MI355X.  Elementwise = max |x - ref| / "
           "max(|ref|, rms(ref)) over the tensor; 2-norm = ||x - ref|| / ||ref||.  Bars (tests/util.py): `bf16` "
           "elementwise 2e-2 (the stated bar); `bf16-bptt` (d_x and the LSTM weight and bias gradients with bf16 "
           "operands) 2-norm 7e-3 and elementwise 7e-2; `update` (change of a weight tensor over a few optimiser "
           "steps, fp32 path) 2-norm 2e-4 and elementwise 2.5e-2.", "",
           "## Largest error per bar and tensor over all tests", "",
           "| bar | tensor | comparisons | max elementwise | in test | max 2-norm | in test |", "|---|---|---|---|---|---|---|"]
    for (bar, what), a in sorted(agg.items()):
        out.append(f"| {bar} | {what} | {a[4]} | {a[0]:.2e} | {a[1]} | {a[2]:.2e} | {a[3]} |")
    for name in ("max", "large"):
        sel = [r for r in rows if "test_full_size_minibatch[" + name in r[0]]
        if not sel:
            continue
        out += ["", f"## Full-size `{name}` minibatch (tests/test_gpu_full_size.py, launch configuration of bench.py)", "",
                "| tensor | bar | elementwise | 2-norm |", "|---|---|---|---|"]
        out += [f"| {r[2]} | {r[1]} | {float(r[3]):.2e} | {float(r[4]):.2e} |" for r in sel]
    print("\n".join(out))


if __name__ == "__main__":
    main(sys.argv[1])
