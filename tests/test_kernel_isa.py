"""Host-side check of what the compiler made of the attention kernel's streaming loops.

The decode kernel lives on counting its outstanding loads exactly: one `s_waitcnt vmcnt(0)`
inside a streaming loop drains the whole KV pipeline every step and costs several per cent
of bandwidth, without any test of results noticing.  Small source changes have flipped the
compiler into that mode before, so the generated code itself is checked: in the innermost
MFMA loops of k_attention there is no full wait on vector memory, no scratch traffic, and
the kernel keeps two waves per SIMD (at most 256 VGPRs)."""
import os
import re
import subprocess
import tempfile

from paper_2505_04021_amd import build as B


def device_assembly():
    out = os.path.join(tempfile.mkdtemp(prefix="pkv_isa_"), "attn.s")
    flags = [f for f in B.FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags + ["--cuda-device-only", "-S",
                                                                      os.path.join(B.CSRC, "attn_kernels.hip"), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return open(out).read()


def kernel_body(asm, mangled_part):
    lines = asm.split("\n")
    start = [i for i, l in enumerate(lines) if re.match(r"^_Z\w*" + mangled_part + r"\w*:", l)][0]
    end = [i for i, l in enumerate(lines) if ".end_amdhsa_kernel" in l and i > start][0]
    labels, insn = {}, []
    for l in lines[start:end]:
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if m:
            labels[m.group(1)] = len(insn)
            continue
        t = l.strip()
        if t and not t.startswith((";", ".", "//")):
            insn.append(t)
    meta = "\n".join(lines[end:end + 400])
    return insn, labels, meta


def innermost_mfma_loops(insn, labels, min_mfma=20):
    mf = [i for i, t in enumerate(insn) if t.startswith("v_mfma")]
    loops = []
    for i, t in enumerate(insn):
        m = re.match(r"s_c?branch\w*\s+(\.LBB\d+_\d+)", t)
        if m and m.group(1) in labels and labels[m.group(1)] < i:
            a = labels[m.group(1)]
            if sum(1 for x in mf if a <= x <= i) >= min_mfma:
                loops.append((a, i))
    return [l for l in loops if not any(o != l and o[0] >= l[0] and o[1] <= l[1] for o in loops)]


def test_streaming_loops_keep_exact_load_counts():
    asm = device_assembly()
    # both forms (two waves per SIMD / one wave per SIMD), each with bf16 / e4m3 x head dim 128 / 64
    for name, n_loops, max_vgpr in (("11k_attentionE", 4, 256), ("16k_attention_deepE", 4, 512)):
        insn, labels, _ = kernel_body(asm, name)
        loops = innermost_mfma_loops(insn, labels)
        assert len(loops) == n_loops, (name, loops)
        for a, b in loops:
            seg = insn[a:b]
            assert sum(t.startswith("buffer_load_dwordx4") for t in seg) >= 12
            full = [t for t in seg if t.startswith("s_waitcnt") and re.search(r"vmcnt\(0\)", t)]
            assert not full, f"{name} loop {a}..{b} drains vector memory: {full[:3]}"
            assert not any(t.startswith("scratch_") for t in seg), f"{name} loop {a}..{b} spills to scratch"
        vg = [int(x) for x in re.findall(r"\.name:\s+\S*" + name + r"\S*\s*\n(?:.*\n){0,40}?\s+\.vgpr_count:\s+(\d+)", asm)]
        assert vg and max(vg) <= max_vgpr, (name, vg)
