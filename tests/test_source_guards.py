"""Source-level guards (CPU): properties of the HIP sources that a later edit could
silently break and that only show as rare wrong results on the GPU."""
import glob
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1606_04884_amd", "csrc")


def _call_args(text, start):
    """Arguments of the call whose opening parenthesis is at text[start]."""
    depth, args, cur = 0, [], []
    for ch in text[start:]:
        if ch in "([{":
            depth += 1
            if depth == 1:
                continue
        elif ch in ")]}":
            depth -= 1
            if depth == 0:
                args.append("".join(cur).strip())
                return args
        if ch == "," and depth == 1:
            args.append("".join(cur).strip())
            cur = []
        else:
            cur.append(ch)
    raise AssertionError("unbalanced call")


def test_wide_buffer_stores_pass_no_scalar_offset():
    """Buffer stores of more than 8 bytes must pass the literal 0 as their scalar offset (the
    row / channel part goes into the lane offset): with a scalar-register offset the compiler
    keeps no distance between such a store and a following vector instruction that overwrites
    its data registers, and on gfx950 some lanes then stored the new value (sporadic wrong
    pixels in the 16-byte-store epilogue of the streaming kernel)."""
    found = 0
    for path in sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.h"))):
        text = open(path).read()
        for m in re.finditer(r"__builtin_amdgcn_raw_buffer_store_b(96|128)\s*\(", text):
            args = _call_args(text, m.end() - 1)
            # (data, resource, lane offset, scalar offset, aux)
            assert len(args) == 5, (path, args)
            assert args[3] == "0", "%s: %s-bit buffer store with scalar offset %r" % (
                os.path.basename(path), m.group(1), args[3])
            found += 1
    assert found >= 1          # the guard must see the store it was written for


def test_no_source_names_build_documents_or_reference_paths():
    """Comments cite the paper by section only."""
    pat = re.compile(r"SURVEY|DESIGN\.md|VERDICT|ADVICE|BASELINE\.md|PAPER\.md|SPEC\.md|gpurun|/root/reference")
    files = (glob.glob(os.path.join(CSRC, "*")) + glob.glob(os.path.join(ROOT, "include", "*.h")) +
             glob.glob(os.path.join(ROOT, "paper_1606_04884_amd", "*.py")) + glob.glob(os.path.join(ROOT, "oracle", "*")))
    for path in files:
        if os.path.isfile(path) and not path.endswith(".so"):
            for i, line in enumerate(open(path, errors="ignore"), 1):
                assert not pat.search(line), "%s:%d: %s" % (path, i, line.strip())
