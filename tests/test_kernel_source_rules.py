"""Source-level rules of the kernels that count their own vector-memory requests (csrc/vmem.hpp).

The compiler knows nothing of a load issued through the inline-assembly wrappers: nothing stops a
wave from ending, or a function from returning into code that reuses the registers or the LDS
rows, while such a load is still in flight.  The rules checked here, on the text of the sources:

  1. every function that issues such loads reaches `wait_vm<0>()` after its last request, and no
     `return` between the first request and the end comes without one;
  2. those sources never read a layer operand through a plain dereference (`p.m[c]`, `*p.bias`):
     a load the compiler does see makes it wait for everything outstanding, and a hand count that
     was right becomes a stall (or, with its registers reassigned, wrong data).
"""
import os
import re

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "..", "paper_2103_16827_amd", "csrc")

LOADS = r"\b(?:direct_load16_scope\s*<[^>]*>|direct_load16_dev|direct_load16|direct_load4|gload16|gload4|gload_i8|bload16)\s*\("
WAIT0 = r"\bwait_vm\s*<\s*0\s*>\s*\(\s*\)"
OPERANDS = r"(?:bias|m|s|w|x|res|act_lut)"


def strip_comments(text):
    text = re.sub(r"/\*.*?\*/", lambda m: " " * len(m.group(0)), text, flags=re.S)
    return re.sub(r"//[^\n]*", lambda m: " " * len(m.group(0)), text)


def sources():
    out = {}
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".hpp")) and name != "vmem.hpp":
            out[name] = strip_comments(open(os.path.join(CSRC, name)).read())
    return out


def functions(text):
    """(name, body) of every __global__ / __device__ function definition in `text`."""
    found = []
    for m in re.finditer(r"__(?:global|device)__", text):
        i = text.find("(", m.end())
        # the parameter list: the first parenthesis that is not part of an attribute or launch bound
        while i >= 0:
            head = text[m.end():i]
            if re.search(r"(?:__launch_bounds__|__attribute__\s*\(?)\s*$", head):
                depth, j = 0, i
                while True:
                    depth += text[j] == "("
                    depth -= text[j] == ")"
                    j += 1
                    if depth == 0:
                        break
                i = text.find("(", j)
                continue
            break
        if i < 0:
            continue
        name = re.findall(r"(\w+)\s*$", text[m.end():i])
        depth, j = 0, i
        while True:
            depth += text[j] == "("
            depth -= text[j] == ")"
            j += 1
            if depth == 0:
                break
        k = j
        while k < len(text) and text[k] in " \n\t":
            k += 1
        if k >= len(text) or text[k] != "{":
            continue                      # a declaration
        depth, e = 0, k
        while True:
            depth += text[e] == "{"
            depth -= text[e] == "}"
            e += 1
            if depth == 0:
                break
        found.append((name[0] if name else "?", text[k:e]))
    return found


def lambda_spans(body):
    """Character ranges of the lambda bodies inside a function body (a `return` there leaves the
    lambda, not the function)."""
    spans = []
    for m in re.finditer(r"\[[&=]?\]\s*\(", body):
        depth, j = 0, m.end() - 1
        while True:
            depth += body[j] == "("
            depth -= body[j] == ")"
            j += 1
            if depth == 0:
                break
        k = body.find("{", j)
        if k < 0 or ";" in body[j:k]:
            continue
        depth, e = 0, k
        while True:
            depth += body[e] == "{"
            depth -= body[e] == "}"
            e += 1
            if depth == 0:
                break
        spans.append((k, e))
    return spans


def function_returns(body):
    spans = lambda_spans(body)
    return [r.start() for r in re.finditer(r"\breturn\b", body) if not any(a <= r.start() < b for a, b in spans)]


def test_the_splitter_sees_the_kernels():
    src = sources()
    names = {n for t in src.values() for n, _ in functions(t)}
    for want in ("pw_pipe_kernel", "pw_pipe_tile", "dw_pipe_kernel", "pw_tile_kernel", "team_kernel", "conv_pipe_kernel"):
        assert want in names, (want, sorted(names))


def test_every_function_with_hand_counted_loads_drains_them_before_it_ends():
    checked = []
    for fname, text in sources().items():
        for name, body in functions(text):
            loads = [m.start() for m in re.finditer(LOADS, body)]
            if not loads:
                continue
            waits = [m.start() for m in re.finditer(WAIT0, body)]
            assert waits and waits[-1] > loads[-1], f"{fname}:{name}: no wait_vm<0>() after its last request"
            for r in function_returns(body):
                if r < loads[0]:
                    continue              # leaves before anything was requested
                before = [q for q in loads if q < r]
                assert any(before[-1] < w < r for w in waits), \
                    f"{fname}:{name}: a return after a request without wait_vm<0>() in between"
            checked.append(f"{fname}:{name}")
    # the kernels known to use the wrappers are all among the checked ones
    for want in ("pw_pipe_tile", "dw_pipe_kernel", "pw_tile_kernel"):
        assert any(c.endswith(":" + want) for c in checked), checked


def test_the_checker_catches_a_missing_drain():
    bad = """
    __global__ void k(const int* p) {
      v4i a = gload16(p);
      wait_vm<0>();
      v4i b = gload16(p + 4);
      if (threadIdx.x == 0) return;
    }
    """
    (name, body), = functions(bad)
    loads = [m.start() for m in re.finditer(LOADS, body)]
    waits = [m.start() for m in re.finditer(WAIT0, body)]
    assert name == "k" and len(loads) == 2 and len(waits) == 1
    assert not waits[-1] > loads[-1]
    assert len(function_returns(body)) == 1
    with_lambda = "__device__ void f() { auto g = [&](int i) __attribute__((always_inline)) { return i; }; gload4(0); wait_vm<0>(); }"
    (_, body2), = functions(with_lambda)
    assert function_returns(body2) == []


def test_no_plain_dereference_of_layer_operands_where_loads_are_hand_counted():
    for fname, text in sources().items():
        if not re.search(LOADS, text):
            continue
        # (the layer's parameter block is called p in every kernel, v in the team kernel's layer view)
        for pat in (rf"\b[pv](?:\.|->){OPERANDS}\s*\[", rf"\*\s*\(?\s*[pv](?:\.|->){OPERANDS}\b(?!\s*[?!=])"):
            for m in re.finditer(pat, text):
                line = text.count("\n", 0, m.start()) + 1
                raise AssertionError(f"{fname}:{line}: operand read outside the vmem.hpp wrappers: "
                                     f"{text[m.start():m.end() + 20]!r}")
    assert re.search(rf"\b[pv](?:\.|->){OPERANDS}\s*\[", "x = p.m[co];") and re.search(
        rf"\*\s*\(?\s*[pv](?:\.|->){OPERANDS}\b(?!\s*[?!=])", "int b = *p.bias;")
