"""Loads that the compiler does not know to be in flight (inline assembly), waited for by hand: the one-token
mat-vec's activations, and the requests of the attention's merging workgroup.  Between the requests and the wait
nothing may read, copy, spill or overwrite the destination registers: this compiles the kernels to assembly and
checks exactly that."""
import os
import re
import shutil
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2504_08791_amd", "csrc")
KERNEL = "_ZN5prima26gemv_q4k_persistent_kernelILi1EEEvNS_9PGemvArgsE"


def _need_hipcc():
    # no skip: the library cannot be built without hipcc either, and a silently skipped check of hand-waited loads
    # is worse than a red one
    assert shutil.which("hipcc") is not None, "hipcc not found: the assembly of the hand-waited loads cannot be checked"


def test_registers_of_early_loads_are_untouched_until_the_wait(tmp_path):
    _need_hipcc()
    out = tmp_path / "k.s"
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(CSRC, "q4k_gemv_mfma.hip")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = out.read_text().split("\n")
    start = next(i for i, l in enumerate(lines) if l.startswith(KERNEL + ":"))
    end = next(i for i in range(start, len(lines)) if "s_endpgm" in lines[i])
    body = lines[start:end]
    loads = []
    for i, l in enumerate(body):
        m = re.search(r"global_load_dwordx4 v\[(\d+):(\d+)\], v\[\d+:\d+\], off\s*$", l)
        if m and i > 0 and "#ASMSTART" in body[i - 1]:
            loads.append((i, int(m.group(1)), int(m.group(2))))
    assert len(loads) >= 8, "the hand-waited loads are gone"
    loads = loads[:8]   # the stand-alone kernel requests them once, first of all
    wait = next(i for i in range(loads[-1][0], len(body)) if "s_waitcnt vmcnt(5)" in body[i])
    regs = set()
    for _, a, b in loads:
        regs.update(range(a, b + 1))
    assert len(regs) == 32, "two loads share a destination register"
    load_lines = {i for i, _, _ in loads}
    for i in range(loads[0][0] + 1, wait):
        if i in load_lines:
            continue
        code = body[i].split(";")[0]
        used = {int(m.group(1)) for m in re.finditer(r"\bv(\d+)\b", code)}
        for m in re.finditer(r"\bv\[(\d+):(\d+)\]", code):
            used.update(range(int(m.group(1)), int(m.group(2)) + 1))
        assert not (used & regs), (i, body[i].strip())


def _regs_of(code):
    used = {int(m.group(1)) for m in re.finditer(r"\bv(\d+)\b", code)}
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", code):
        used.update(range(int(m.group(1)), int(m.group(2)) + 1))
    return used


def test_registers_of_the_attention_merge_requests_are_untouched_until_the_wait(tmp_path):
    _need_hipcc()
    """Every instantiation of the attention kernel: the 17 requests of a merge pass (one 8-byte, sixteen 16-byte,
    device scope, scalar base + lane offset; 18 in the pass that serves two queries) are followed by the hand-written
    wait with nothing but requests and scalar arithmetic in between, write 66 (68) distinct registers, and nothing is
    spilled anywhere in the kernel."""
    out = tmp_path / "a.s"
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(CSRC, "attn_decode.hip")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = out.read_text().split("\n")
    starts = [i for i, l in enumerate(lines) if re.match(r"_ZN5prima18attn_decode_kernelILi\d+ELi\d+EEEvNS_8AttnArgsE:", l)]
    assert len(starts) == 4
    for start in starts:
        end = next(i for i in range(start, len(lines)) if "s_endpgm" in lines[i])
        body = lines[start:end]
        assert not any("scratch_" in l.split(";")[0] for l in body), "the kernel spills registers"
        req = [(i, m) for i, l in enumerate(body)
               for m in [re.search(r"global_load_dwordx[24] v\[(\d+):(\d+)\], v\d+, s\[\d+:\d+\] sc1", l)] if m]
        assert len(req) >= 17, "the merge's requests are gone"
        # passes: runs of requests that end with the hand-written wait
        i = 0
        n_pass = 0
        while i < len(req):
            first = req[i][0]
            wait = next(k for k in range(first, len(body)) if "s_waitcnt vmcnt(0)" in body[k] and "#ASMSTART" in body[k - 1])
            group = [(k, m) for k, m in req if first <= k < wait]
            regs = set()
            for _, m in group:
                dst = set(range(int(m.group(1)), int(m.group(2)) + 1))
                assert not (dst & regs), "two requests share a destination register"
                regs |= dst
            # the first pass of a query also fetches (max, sum); a pass for two queries fetches both queries' (max, sum)
            assert len(regs) in (64, 66, 68), len(regs)
            lines_of_group = {k for k, _ in group}
            for k in range(first + 1, wait):
                if k in lines_of_group:
                    continue
                code = body[k].split(";")[0]
                assert not (_regs_of(code) & regs), (k, body[k].strip())
            n_pass += 1
            i += len(group)
        assert n_pass >= 2, "the pass for one query and the pass for two"
