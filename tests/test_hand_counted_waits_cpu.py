"""Static check of the loops that count outstanding vector-memory operations by hand.

Three kernels place `s_waitcnt vmcnt(n)` themselves in front of a bare `s_barrier`, because data that arrives by
LDS-direct loads (`buffer_load ... lds`) has to be complete for the other waves while the youngest n loads may stay
in flight: the GEMM (`linear_mfma_kernel`: n = 8, the register loads of the next W tile) and the two loader-wave
weight-gradient kernels (`wgrad_partial_ws_kernel`, `wgrad_partial_ws64_kernel`: n = the LDS-direct loads of one
chunk).  The counts are only right if the compiled loop holds exactly the vector-memory instructions the source
assumes, in the assumed order, and nothing else (a spill would add scratch traffic).  This test compiles the two
files to gfx950 assembly (no GPU needed) and counts.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2405_17991_amd import build as vbuild

VMEM = re.compile(r"^\s*(buffer|global|scratch|flat)_(load|store|atomic)\w*\s")
LABEL = re.compile(r"^(\.LBB\d+_\d+):")


def _device_asm(tmp_path_factory, src):
    if not (shutil.which("hipcc") or os.path.exists(vbuild.HIPCC)):
        pytest.skip("hipcc not available")
    out = tmp_path_factory.mktemp("asm") / (src + ".s")
    flags = [f for f in vbuild.FLAGS if f != "-fPIC"]
    cmd = [vbuild.HIPCC] + flags + ["--cuda-device-only", "-S", os.path.join(vbuild.CSRC, src), "-o", str(out),
                                    "-Rpass-analysis=kernel-resource-usage"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
    return out.read_text().splitlines(), r.stdout


@pytest.fixture(scope="module")
def linear_asm(tmp_path_factory):
    return _device_asm(tmp_path_factory, "linear.hip")


@pytest.fixture(scope="module")
def wgrad_asm(tmp_path_factory):
    return _device_asm(tmp_path_factory, "wgrad.hip")


def _kernels(lines, name):
    """{mangled name: body lines} of every kernel whose mangled name contains `name`."""
    out, cur = {}, None
    for l in lines:
        m = re.match(r"^(_Z\w+):", l)
        if m:
            cur = m.group(1) if name in m.group(1) else None
            if cur:
                out[cur] = []
        elif cur is not None:
            out[cur].append(l)
            if l.strip().startswith("s_endpgm"):
                cur = None
    return out


def _instr(l):
    return l.split(";")[0].strip()


def _hand_waits(body):
    """Indices of `s_waitcnt vmcnt(n)` whose next instruction is `s_barrier`, with n."""
    code = [(i, _instr(l)) for i, l in enumerate(body) if _instr(l) and not LABEL.match(l)]
    found = []
    for (i, a), (_, b) in zip(code, code[1:]):
        m = re.match(r"s_waitcnt vmcnt\((\d+)\)", a)
        if m and b == "s_barrier":
            found.append((i, int(m.group(1))))
    return found


BLOCK = re.compile(r"^(\.LBB\d+_\d+):|^; %bb\.\d+:")


def _loop_lines(body, idx):
    """Line indices of the innermost loop around line idx, from the compiler's own block annotations
    ("Loop Header" on the header's label, "in Loop: Header=BBn_m" on every other block of the loop; the
    blocks need not be contiguous, a rotated loop keeps its latch above its header).  Header lines first."""
    header = None
    for h in range(idx, -1, -1):
        m = LABEL.match(body[h])
        if m and ("Loop Header" in body[h] or "Loop Header" in body[h + 1]):
            header = m.group(1)
            break
    assert header, "no enclosing loop found"
    tag = "Header=" + header.lstrip(".L") + " "
    starts = [i for i, l in enumerate(body) if BLOCK.match(l)] + [len(body)]
    head, rest = [], []
    for a, b in zip(starts, starts[1:]):
        note = body[a] + " " + (body[a + 1] if a + 1 < len(body) and body[a + 1].lstrip().startswith(";") else "")
        if body[a].startswith(header + ":"):
            head = list(range(a, b))
        elif tag in note + " ":
            rest += list(range(a, b))
    assert head and idx in head + rest
    return head, rest


def _scratch_free(remarks, name):
    cur, seen = None, 0
    for line in remarks.splitlines():
        if "Function Name:" in line:
            cur = line.split("Function Name:")[1].split()[0]
        elif cur and name in cur:
            for key in ("VGPRs Spill:", "SGPRs Spill:", "ScratchSize [bytes/lane]:"):
                if key in line:
                    assert int(line.split(key)[1].split()[0]) == 0, (cur, line)
                    seen += 1
    assert seen >= 3, f"no resource remarks for {name}"


def test_gemm_loop_has_the_memory_instructions_its_wait_assumes(linear_asm):
    lines, remarks = linear_asm
    _scratch_free(remarks, "linear_mfma_kernel")
    kernels = _kernels(lines, "linear_mfma_kernel")
    assert len(kernels) == 3          # forward with S, forward without, grad_input
    for name, body in kernels.items():
        waits = [(i, n) for i, n in _hand_waits(body) if 0 < n < 63]      # 0: drain; 63: no vector-memory wait
        assert len(waits) == 1 and waits[0][1] == 8, (name, waits)
        w = waits[0][0]
        # the steady-state path of a k step: from the loop's header to the first branch back to it (side
        # blocks behind it belong to the last steps, which have no further tile to request)
        head, _ = _loop_lines(body, w)
        label = LABEL.match(body[head[0]]).group(1)
        back = next(i for i in range(w, len(body)) if re.match(r"s_c?branch\w*\s+" + re.escape(label) + r"$", _instr(body[i])))
        loop = list(range(head[0], back + 1))
        before = [_instr(body[i]) for i in loop if i < w and VMEM.match(body[i])]
        after = [_instr(body[i]) for i in loop if i > w and VMEM.match(body[i])]
        # in front of the wait: the eight register loads of the next W tile and nothing else, so that
        # everything older than them (the LDS-direct loads of the X tile) has landed when it returns
        assert len(before) == 8 and all(i.startswith("buffer_load_dwordx4 v[") and not i.endswith("lds") for i in before), (name, before)
        # behind the barrier: the eight LDS-direct loads of the X tile two steps ahead
        assert len(after) == 8 and all(i.startswith("buffer_load_dwordx4") and i.endswith("lds") for i in after), (name, after)
        mfma = [i for i in loop if "v_mfma_f32_16x16x32" in body[i]]
        assert len(mfma) in (128, 136), (name, len(mfma))       # 8 x 8 tiles x 2 halves (+ 8 for S)


@pytest.mark.parametrize("kernel,loads", [
    ("wgrad_partial_ws_kernelILi1E", 9), ("wgrad_partial_ws_kernelILi2E", 10), ("wgrad_partial_ws_kernelILi3E", 11),
    ("wgrad_partial_ws256_kernelILi1E", 9), ("wgrad_partial_ws256_kernelILi2E", 9), ("wgrad_partial_ws256_kernelILi3E", 10),
    ("wgrad_partial_ws256_kernelILi4E", 10), ("wgrad_partial_ws256_kernelILi5E", 11),
    ("wgrad_partial_ws64_kernelILi4E", 6), ("wgrad_partial_ws64_kernelILi5E", 7), ("wgrad_partial_ws64_kernelILi6E", 7),
])
def test_loader_wave_loop_waits_for_all_but_one_chunk(wgrad_asm, kernel, loads):
    lines, remarks = wgrad_asm
    _scratch_free(remarks, kernel)
    kernels = _kernels(lines, kernel)
    assert len(kernels) == 1
    body = next(iter(kernels.values()))
    waits = [(i, n) for i, n in _hand_waits(body) if 0 < n < 63]      # 0: drain; 63: no vector-memory wait
    assert len(waits) == 1 and waits[0][1] == loads, waits
    head, rest = _loop_lines(body, waits[0][0])
    vm = [_instr(body[i]) for i in head + rest if VMEM.match(body[i])]
    # one chunk's LDS-direct loads per trip and nothing else: "at most `loads` outstanding" then means
    # every chunk but the youngest has landed
    assert len(vm) == loads and all(i.endswith("lds") for i in vm), vm
    # a trip starts with the wait and the barrier; the loads come behind them (the slot they refill was
    # read by the computing waves before that barrier)
    assert not [i for i in head if i < waits[0][0] and VMEM.match(body[i])]
