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
    """k_attn_partial_tr keeps its 128 output accumulators in AGPRs a0..a127 that it names itself; the
    compiler must not use any AGPR in that kernel.  Checked in the ISA the build flags produce."""
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
    for start in starts:
        end = [i for i in range(start, len(lines)) if lines[i].startswith(".Lfunc_end")][0]
        seen = collections.Counter()
        for l in lines[start:end]:
            t = l.strip()
            if not t or t.startswith((";", ".")):
                continue
            if re.search(r"\ba\d+\b|\ba\[\d+:\d+\]", t):
                seen[t.split()[0]] += 1
                if t.startswith("v_mfma"):      # accumulate in place: a[x:y], v, v, a[x:y]
                    assert re.search(r"a\[(\d+):(\d+)\], v\[\d+:\d+\], v\[\d+:\d+\], a\[\1:\2\]", t), t
        # 32 accumulating MFMAs; 128 zero writes + 128 rescale writes; 128 rescale reads + 128 final reads
        assert seen == {"v_mfma_f32_16x16x32_bf16": 32, "v_accvgpr_write_b32": 256, "v_accvgpr_read_b32": 256}, seen
        # The compiler's hazard logic does not see inside those asm statements.  No vector ALU instruction
        # may write a VGPR operand of such an MFMA in the instructions just before it unless wait states
        # (s_nop) stand between: without them the MFMA was seen to read the register's old value.
        body = [l.strip() for l in lines[start:end] if l.strip() and not l.strip().startswith((";", "."))]
        for i, t in enumerate(body):
            m = re.match(r"v_mfma\S* a\[\d+:\d+\], v\[(\d+):(\d+)\], v\[(\d+):(\d+)\], a\[", t)
            if not m:
                continue
            used = set(range(int(m[1]), int(m[2]) + 1)) | set(range(int(m[3]), int(m[4]) + 1))
            states = 0
            for prev in reversed(body[max(0, i - 8):i]):
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
