"""The pins must be able to tell a wrong oracle from a right one.  Each case below plants one
plausible mistake (a transposed or flipped kernel, a wrong sign, a dropped term, an off-by-one
extent, swapped axes, a forgotten stride ...) in a copy of oracle/conv_oracle.c, compiles it,
and runs the CPU pin files against that library in a child process: at least one pin has to
fail.  The unchanged copy has to pass, so a failure is the mistake's and not the harness's."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "conv_oracle.c")
PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_oracle_transpose_pins.py",
             "tests/test_oracle_compact_pins.py", "tests/test_oracle_channels_pins.py"]

# (name, function whose body is edited, text to find exactly once in it, replacement)
MISTAKES = [
    ("conv: kernel transposed", "oracle_conv", "K[a * k + b]", "K[b * k + a]"),
    ("conv: kernel flipped (a true convolution)", "oracle_conv", "K[a * k + b]", "K[(k - 1 - a) * k + (k - 1 - b)]"),
    ("conv: stride forgotten along lines", "oracle_conv", "(s * x + a) * W", "(x + a) * W"),
    ("conv: stride forgotten along columns", "oracle_conv", "(s * y + b)) * B", "(y + b)) * B"),
    ("conv: padded copy starts in the border column", "oracle_conv", "(i + p) * W + p", "(i + p) * W"),
    ("conv: padded copy one line too high", "oracle_conv", "((i + p) * W + p) * B", "((i + p - (p > 0)) * W + p) * B"),
    ("c(t): sign of the leading border term", "c_pad", "p - s * t", "s * t - p"),
    ("c(t): trailing border term dropped", "c_pad", " + imax64(0, s * t + k - extent - p)", ""),
    ("c(t): trailing border off by one", "c_pad", "s * t + k - extent - p)", "s * t + k - extent - p - 1)"),
    ("output extent without the + 1", "out_extent", "/ s + 1", "/ s + (extent + 2 * p == k)"),
    ("output extent pads one side only", "out_extent", "(extent + 2 * p - k) / s", "(extent + p - k) / s"),
    ("csr row: kernel transposed", "oracle_csr_row", "K[a * k + b]", "K[b * k + a]"),
    ("csr row: column index with the axes swapped", "oracle_csr_row", "(ip - p) * n + (jp - p)", "(jp - p) * m + (ip - p)"),
    ("csr row: last input line counted as border", "oracle_csr_row", "ip >= p + m", "ip >= p + m - 1"),
    ("csr row: first border column counted as input", "oracle_csr_row", "jp < p ||", "jp < p - 1 ||"),
    ("csr row: stride forgotten", "oracle_csr_row", "jp = s * y + b", "jp = y + b"),
    ("brute-force count: stride forgotten", "oracle_nnz_brute", "(s * y + b)", "(y + b)"),
    ("closed form: sum of the two factors", "oracle_nnz_closed",
     "imax64(0, k - c_pad(x, m, k, s, p)) * imax64", "imax64(0, k - c_pad(x, m, k, s, p)) + imax64"),
    ("closed form: c2 taken with m", "oracle_nnz_closed", "c_pad(y, n, k, s, p)", "c_pad(y, m, k, s, p)"),
    ("csc: rows of a column in descending order", "oracle_csc", "int64_t at = next[cbuf[e]]++;",
     "int64_t at = col_ptr[cbuf[e] + 1] - 1 - (next[cbuf[e]]++ - col_ptr[cbuf[e]]);"),
    ("T^T u: kernel transposed", "oracle_conv_t", "K[a * k + b]", "K[b * k + a]"),
    ("T^T u: border not cropped", "oracle_conv_t", "(float)plane[(i + p) * W + (j + p)]", "(float)plane[i * W + j]"),
    ("T^T u: stride forgotten", "oracle_conv_t", "plane[(s * x + a) * W + (s * y + b)] +=", "plane[(x + a) * W + (s * y + b)] +="),
    ("compact rows: base column without the padding shift", "oracle_compact_rows",
     "(s * x + a_lo - p) * n + (s * y + b_lo - p)", "(s * x + a_lo) * n + (s * y + b_lo)"),
    ("compact rows: r1 and r2 swapped in the word", "oracle_compact_rows",
     "(uint32_t)r1 << 8 | (uint32_t)b_lo << 16 | (uint32_t)r2 << 24", "(uint32_t)r2 << 8 | (uint32_t)b_lo << 16 | (uint32_t)r1 << 24"),
    ("compact decode: table read transposed", "oracle_compact_decode",
     "ktab[(a_lo + da) * k + (b_lo + db)]", "ktab[(b_lo + db) * k + (a_lo + da)]"),
    ("compact decode: line pitch of the output", "oracle_compact_decode", "da * n + db", "da * k + db"),
    ("channels: every channel uses the first kernel", "oracle_conv_channels", "K[(ch * k + a) * k + b]", "K[a * k + b]"),
    ("channels: last channel dropped", "oracle_conv_channels", "for (int64_t ch = 0; ch < C; ++ch)\n                    for",
     "for (int64_t ch = 0; ch < C - (C > 1); ++ch)\n                    for"),
    ("channels: planes of A one line apart", "oracle_conv_channels", "A + (ch * m + i) * n * B", "A + (ch + i) * n * B"),
]


def _function_span(src, name):
    """[start, end) of the body of function `name` (from its definition line to the closing brace in column 0)."""
    at = src.index(name + "(")
    while src[src.rindex("\n", 0, at) + 1] in " \t/*":       # a call or a comment, not the definition
        at = src.index(name + "(", at + 1)
    return at, src.index("\n}\n", at) + 3


def _plant(src, func, old, new):
    lo, hi = _function_span(src, func)
    body = src[lo:hi]
    assert body.count(old) == 1, "%r occurs %d times in %s" % (old, body.count(old), func)
    return src[:lo] + body.replace(old, new) + src[hi:]


def _build(src_text, path):
    c_file = path + ".c"
    with open(c_file, "w") as fh:
        fh.write(src_text)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", path, c_file, "-lm"], check=True)
    return path


# the pin file that covers a function of the oracle comes first in the child's run (it stops at the
# first failure), the others follow
FIRST = {"oracle_csc": 1, "oracle_conv_t": 1, "oracle_compact_rows": 2, "oracle_compact_decode": 2,
         "oracle_conv_channels": 3}


def _pins_pass(lib, func=None):
    env = dict(os.environ, CONV_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    first = FIRST.get(func, 0)
    files = [PIN_FILES[first]] + [f for i, f in enumerate(PIN_FILES) if i != first]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return r.returncode == 0, r.stdout[-2000:]


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """Every mutant (and the unchanged copy, under the key None) built and run against the pins, a
    few children at a time: {name: (pins passed, tail of the child's output)}."""
    from concurrent.futures import ThreadPoolExecutor
    root = tmp_path_factory.mktemp("mutants")
    src = open(SRC).read()
    jobs = [(None, None, src)] + [(name, func, _plant(src, func, old, new)) for name, func, old, new in MISTAKES]

    def run(job):
        idx, (name, func, text) = job
        return name, _pins_pass(_build(text, str(root / ("lib%d.so" % idx))), func)

    workers = max(1, min(6, len(os.sched_getaffinity(0))))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        return dict(pool.map(run, enumerate(jobs)))


def test_the_unchanged_copy_passes_every_pin(outcomes):
    ok, out = outcomes[None]
    assert ok, out


@pytest.mark.parametrize("name", [m[0] for m in MISTAKES])
def test_a_planted_mistake_fails_a_pin(outcomes, name):
    ok, out = outcomes[name]
    assert not ok, "no pin noticed: " + name
    assert "Error" in out or "assert" in out or "failed" in out, out      # a failing test, not a crash of the run
