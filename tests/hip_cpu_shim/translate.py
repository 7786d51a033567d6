"""Rewrite HIP sources so that a host C++ compiler accepts them (test infrastructure only).

Three constructs have no host spelling: the triple-chevron launch and the two LDS
declarations.  `K<<<grid, block, lds, stream>>>(args);` becomes
`shim::launch(grid, block, lds, [&] { K(args); });`,
`extern __shared__ ... name[];` becomes `unsigned char *name = shim::dyn_smem;` and
`__shared__ T name[N];` becomes a per-workgroup heap block, `T *name = ...block_static(...)`.
Everything else compiles as it stands against hip_cpu_shim/hip/hip_runtime.h."""
import re
import sys


def _match_back(text, end):
    """Start of the kernel expression that ends at `end`: an identifier (with ::) and an
    optional template argument list."""
    i = end
    if text[i - 1] == ">":
        depth = 0
        while i > 0:
            i -= 1
            if text[i] == ">":
                depth += 1
            elif text[i] == "<":
                depth -= 1
                if depth == 0:
                    break
    while i > 0 and (text[i - 1].isalnum() or text[i - 1] in "_:"):
        i -= 1
    return i


def _match_paren(text, start):
    assert text[start] == "("
    depth = 0
    for i in range(start, len(text)):
        if text[i] == "(":
            depth += 1
        elif text[i] == ")":
            depth -= 1
            if depth == 0:
                return i
    raise ValueError("unbalanced parentheses")


def _split_top(s):
    parts, depth, cur = [], 0, ""
    for ch in s:
        if ch in "([{":
            depth += 1
        elif ch in ")]}":
            depth -= 1
        if ch == "," and depth == 0:
            parts.append(cur.strip())
            cur = ""
        else:
            cur += ch
    parts.append(cur.strip())
    return parts


def translate(text):
    text = re.sub(r"extern\s+__shared__[^;]*?\b(\w+)\[\];", r"unsigned char *\1 = shim::dyn_smem;", text)
    text = re.sub(r"(?<!extern )__shared__\s+([\w:<>]+)\s+(\w+)\[([^\]]+)\];",
                  r"\1 *\2 = static_cast<\1 *>(shim::block_static(sizeof(\1) * (\3)));", text)
    out, pos = "", 0
    while True:
        i = text.find("<<<", pos)
        if i < 0:
            break
        k0 = _match_back(text, i)
        j = text.find(">>>", i)
        cfg = _split_top(text[i + 3:j])
        while len(cfg) < 3:
            cfg.append("0")
        a0 = j + 3
        while text[a0].isspace():
            a0 += 1
        a1 = _match_paren(text, a0)
        kernel = text[k0:i]
        out += text[pos:k0] + f"shim::launch({cfg[0]}, {cfg[1]}, {cfg[2]}, [&] {{ {kernel}{text[a0:a1 + 1]}; }})"
        pos = a1 + 1
    return out + text[pos:]


if __name__ == "__main__":
    src, dst = sys.argv[1:3]
    open(dst, "w").write(translate(open(src).read()))
