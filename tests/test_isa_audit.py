"""Static check of the machine code of the kernels with hand-written LDS reads (attention and
the 16x16x32 GEMM ring loop).

Their LDS fragment reads are inline assembly with hand-written `s_waitcnt lgkmcnt(n)`: the
compiler does not know that the destination registers of such a read are filled later, so
nothing may touch them before a wait that covers the read, and no read may be in flight
across a label, a branch or a barrier (register copies at control-flow joins would move stale
values).  This test compiles the kernels to assembly and checks exactly that.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2510_10129_amd import build

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _regs(tok):
    """Vector registers named by an operand: (file, number) pairs, file = 'v' or 'a'."""
    m = re.match(r"([va])\[(\d+):(\d+)\]$", tok)
    if m:
        return {(m.group(1), r) for r in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = re.match(r"([va])(\d+)$", tok)
    return {(m.group(1), int(m.group(2)))} if m else set()


def audit(asm_text):
    """Returns (number of hand-written LDS reads seen, list of violations) for one kernel's
    assembly.  Hand-written = inside an inline-assembly block (;;#ASMSTART .. ;;#ASMEND); the
    compiler's own LDS operations only take part in the counting of lgkmcnt."""
    outstanding, seen, bad, in_asm = [], 0, [], False      # outstanding: (dest registers, line, by hand)
    for n, line in enumerate(asm_text.split("\n")):
        if "#ASMSTART" in line:
            in_asm = True
            continue
        if "#ASMEND" in line:
            in_asm = False
            continue
        t = line.split(";")[0].strip().split()
        if not t:
            continue
        op, args = t[0], [a.strip(",") for a in t[1:]]
        if op.startswith("ds_"):                     # LDS operations return in issue order
            dst = _regs(args[0]) if (op.startswith("ds_read") or op.startswith("ds_bpermute")) else set()
            used = set().union(*[_regs(a) for a in args[1:]]) if len(args) > 1 else set()
            for rs, ln, hand in outstanding:
                if hand and rs & (used | dst):
                    bad.append((n, line.strip(), "register of the LDS read at line %d" % ln))
            by_hand = in_asm and op.startswith("ds_read")
            seen += by_hand
            outstanding.append((dst, n, by_hand))
            continue
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", line)
            if m:
                k = int(m.group(1))
                outstanding = outstanding[len(outstanding) - k:] if k else []
            continue
        if op.endswith(":") or op.startswith("s_cbranch") or op in ("s_branch", "s_barrier", "s_endpgm"):
            if any(hand for _, _, hand in outstanding):
                bad.append((n, line.strip(), "hand-written LDS read in flight across control flow"))
            outstanding = [o for o in outstanding if not o[2]]
            continue
        if op.startswith("s_") or op.startswith("."):
            continue
        touched = set().union(*[_regs(a) for a in args]) if args else set()
        for rs, ln, hand in outstanding:
            if hand and rs & touched:
                bad.append((n, line.strip(), "register of the LDS read at line %d" % ln))
    return seen, bad


def test_audit_catches_a_planted_early_use():
    A, E = ";;#ASMSTART\n", ";;#ASMEND\n"
    ok = A + "ds_read_b128 v[4:7], v1\n" + E + "s_waitcnt lgkmcnt(0)\nv_mfma_f32_32x32x16_bf16 v[16:31], v[4:7], v[8:11], v[16:31]\n"
    assert audit(ok) == (1, [])
    early = A + "ds_read_b128 v[4:7], v1\n" + E + "v_mov_b32_e32 v9, v5\ns_waitcnt lgkmcnt(0)\n"
    assert len(audit(early)[1]) == 1
    two = (A + "ds_read_b128 v[4:7], v1\n" + E + A + "ds_read_b128 v[12:15], v1 offset:64\n" + E +
           "s_waitcnt lgkmcnt(1)\nv_mov_b32_e32 v9, v5\nv_mov_b32_e32 v9, v13\n")
    assert [b[0] for b in audit(two)[1]] == [8]          # the first has arrived, the second has not
    across = A + "ds_read_b128 v[4:7], v1\n" + E + "s_barrier\ns_waitcnt lgkmcnt(0)\n"
    assert len(audit(across)[1]) == 1
    own = "ds_bpermute_b32 v0, v1, v2\ns_cbranch_execz .L1\ns_waitcnt lgkmcnt(0)\nv_add_f32_e32 v0, v0, v3\n"
    assert audit(own) == (0, [])                         # the compiler's own operations are its business


@pytest.mark.skipif(shutil.which(HIPCC) is None, reason="hipcc not found")
def test_attention_kernel_reads_are_waited_for(tmp_path):
    out = tmp_path / "attention.s"
    cmd = [HIPCC, *build.FLAGS, "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(build.CSRC, "attention.hip")]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    text = out.read_text()
    kernels = re.findall(r"^(_ZN\S*sparse_attn_kernel\S*):[^\n]*\n(.*?)s_endpgm", text, flags=re.S | re.M)
    assert len(kernels) == 2, [k[0] for k in kernels]
    for name, body in kernels:
        seen, bad = audit(body)
        assert seen >= 40, (name, seen)
        assert not bad, (name, bad[:5])


@pytest.mark.skipif(shutil.which(HIPCC) is None, reason="hipcc not found")
def test_gemm_ring16_kernel_reads_are_waited_for(tmp_path):
    out = tmp_path / "gemm.s"
    cmd = [HIPCC, *build.FLAGS, "-S", "--cuda-device-only", "-o", str(out), os.path.join(build.CSRC, "gemm.hip")]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    text = out.read_text()
    kernels = re.findall(r"^(_ZN\S*gemm_ring16_kernel\S*):[^\n]*\n(.*?)s_endpgm", text, flags=re.S | re.M)
    assert len(kernels) >= 20, [k[0] for k in kernels]    # four tile shapes x four epilogues + 2 x two split-K instances
    for name, body in kernels:
        seen, bad = audit(body)
        assert seen >= 8 * 8, (name, seen)                # 8, 10 or 12 fragment reads per slice, 8 slice blocks
        assert not bad, (name, bad[:5])
