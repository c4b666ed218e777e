"""CPU-side checks of the C ABI: the library loads, exports every symbol the
header declares, struct layouts match, and configuration errors are reported
without touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import torch  # noqa: F401  (HIP runtime first)
    from paper_2512_10576_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2512_10576_amd import build
        build.build()
    return binding.load()


def _declared():
    text = open(os.path.join(ROOT, "include", "ess.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ess_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert {"ess_index_score", "ess_topk", "ess_gather_latent", "ess_sparse_mla_decode", "ess_decode_step"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layouts():
    from paper_2512_10576_amd import binding as b
    assert C.sizeof(b.EssConfig) == 13 * 4
    assert C.sizeof(b.EssCache) == 5 * 8
    assert C.sizeof(b.EssStats) == 4 * 8
    assert b.EssStepArgs.B.offset == 48 and b.EssStepArgs.idx_out.offset == 64 and C.sizeof(b.EssStepArgs) == 112 and b.EssStepArgs.block_table.offset == 96


def test_config_validation_reports_errors(lib):
    from paper_2512_10576_amd import binding as b
    good = b.make_config(64, 1, 131072, 64, 128, 2048, 128, slots_per_seq=13108)
    n = b.workspace_bytes(good)
    assert n > 64 * 131072 * 4
    cases = [
        (dict(idx_dim=96), b.ESS_ERR_UNSUPPORTED),
        (dict(max_q_tokens=5), b.ESS_ERR_UNSUPPORTED),
        (dict(slots_per_seq=1000), b.ESS_ERR_CAPACITY),
        (dict(row_stride=1150), b.ESS_ERR_INVALID_ARG),
        (dict(max_ctx=1 << 20), b.ESS_ERR_INVALID_ARG),
        (dict(topk=0), b.ESS_ERR_INVALID_ARG),
        (dict(attn_heads=129), b.ESS_ERR_UNSUPPORTED),
    ]
    for change, code in cases:
        kw = dict(max_batch=64, max_q_tokens=1, max_ctx=131072, idx_heads=64, idx_dim=128, topk=2048,
                  attn_heads=128, slots_per_seq=13108)
        kw.update(change)
        with pytest.raises(b.EssError) as ei:
            b.workspace_bytes(b.make_config(**kw))
        assert ei.value.code == code and str(ei.value)
    bad = b.make_config(1, 1, 64, 4, 32, 8, 8)
    bad.struct_size = 8
    with pytest.raises(b.EssError):
        b.workspace_bytes(bad)


def test_attention_kernel_agprs_are_only_named_by_its_own_asm(tmp_path):
    """k_attn_partial_tr keeps its 256 output accumulators in AGPRs a0..a255 that its own asm statements name, and
    tells the compiler that the whole AGPR file is taken from a claim statement to a release statement.  Checked in
    the ISA the build flags produce, for all four instances: between claim and release no instruction outside an
    asm statement names an AGPR, nothing is spilled to scratch memory, and no asm MFMA has a vector ALU producer
    of one of its VGPR operands within eight wait states."""
    import collections
    import subprocess
    from paper_2512_10576_amd import build
    out = tmp_path / "sparse_mla.s"
    cmd = [build._hipcc(), *build.compile_flags("sparse_mla.hip"), "-S", "--cuda-device-only",
           os.path.join(build.CSRC, "sparse_mla.hip"), "-o", str(out)]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    lines = out.read_text().split("\n")
    starts = [i for i, l in enumerate(lines) if re.match(r"^_ZN\S*k_attn_partial_tr\S*:", l)]
    assert len(starts) == 4                      # one instance per entry format and per way of taking work
    num = r"(?:0x[0-9a-f]+|\d+)"               # the asm printer writes larger register numbers in hexadecimal
    agpr = re.compile(r"\ba\d+\b|\ba\[" + num + r"(:" + num + r")?\]")
    for start in starts:
        end = [i for i in range(start, len(lines)) if lines[i].startswith(".Lfunc_end")][0]
        tail = "\n".join(lines[end:end + 80])
        assert re.search(r"; ScratchSize: 0\b", tail), "the attention kernel spills registers to scratch memory"
        assert re.search(r"; NumAgprs: 256\b", tail)
        in_asm = claimed = False
        own = collections.Counter()
        n_claim = n_release = 0
        body = []                                # (text, inside an asm statement) between claim and release
        for l in lines[start:end]:
            t = l.strip()
            if t.startswith(";;#ASMSTART"):
                in_asm = True
                continue
            if t.startswith(";;#ASMEND"):
                in_asm = False
                continue
            if in_asm and "ess_agpr_claim" in t:
                claimed, n_claim = True, n_claim + 1
            if in_asm and "ess_agpr_release" in t:
                claimed, n_release = False, n_release + 1
            if not t or t.startswith((";", ".")):
                continue
            if claimed:
                body.append((t, in_asm))
            if agpr.search(t):
                if in_asm:
                    own[t.split()[0]] += 1
                    if t.startswith("v_mfma"):  # accumulate in place: a[x:y], v, v, a[x:y]
                        assert re.search(r"a\[(%s):(%s)\], v\[\d+:\d+\], v\[\d+:\d+\], a\[\1:\2\]" % (num, num), t), t
                else:
                    assert not claimed, "the compiler uses an AGPR of its own where the kernel holds its accumulators: " + t
        assert n_claim >= 1 and n_claim == n_release
        # in every copy of the tile loop the 32 accumulating MFMAs; 256 zero writes, 256 rescale writes and reads per
        # rescale site, 256 final reads
        assert own["v_mfma_f32_32x32x16_bf16"] % 32 == 0 and own["v_mfma_f32_32x32x16_bf16"] >= 32, own
        assert own["v_accvgpr_write_b32"] >= 512 and own["v_accvgpr_read_b32"] >= 512, own
        # hazards of the asm MFMAs (the compiler's hazard logic does not see inside asm statements)
        texts = [t for t, _ in body]
        for i, (t, inside) in enumerate(body):
            m = re.match(r"v_mfma\S* a\[%s:%s\], v\[(\d+):(\d+)\], v\[(\d+):(\d+)\], a\[" % (num, num), t)
            if not (inside and m):
                continue
            used = set(range(int(m[1]), int(m[2]) + 1)) | set(range(int(m[3]), int(m[4]) + 1))
            states = 0
            for prev in reversed(texts[max(0, i - 8):i]):
                if prev.startswith("s_nop"):
                    states += int(prev.split()[1]) + 1
                    continue
                states += 1
                if states > 8 or not prev.startswith("v_") or prev.startswith("v_mfma"):
                    continue
                dst = re.match(r"v_\S+ v(?:\[(\d+):(\d+)\]|(\d+))", prev)
                if dst:
                    wr = set(range(int(dst[1]), int(dst[2]) + 1)) if dst[1] else {int(dst[3])}
                    assert not (wr & used), (prev, t)
