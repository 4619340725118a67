"""Measured ceilings of the GPU at hand: a streaming copy (HBM) and a register-only fp32 MFMA loop.

    python -m paper_2012_15667_amd.ceilings

prints one JSON line.  bench.py quotes its roofline fractions against the published peaks and, beside them,
against these.

    python -m paper_2012_15667_amd.ceilings --share

prints, as a table, how waves that issue fp32 MFMAs and waves that issue plain VALU instructions share one SIMD:
the clock ticks per instruction of each wave when it runs alone and beside the others.
"""
import json
import sys

HBM_PEAK_GBPS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3


def measure(copy_bytes=1 << 30, copy_reps=5, mfma_iters=20000, mfma_reps=3):
    import torch
    from . import binding as B
    src = torch.zeros(copy_bytes // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    ms_copy = B.probe_hbm_copy(src, dst, copy_reps)
    del src, dst
    sink = torch.empty(B.probe_mfma_sink_bytes() // 4, dtype=torch.float32, device="cuda")
    ms_mfma, flop = B.probe_mfma_f32(sink, mfma_iters, mfma_reps)
    copy_gbps = 2.0 * copy_bytes / ms_copy / 1e6
    mfma_tflops = flop / ms_mfma / 1e9
    return {"hbm_copy_GBps": round(copy_gbps, 1), "hbm_copy_frac_of_published": round(copy_gbps / HBM_PEAK_GBPS, 4),
            "mfma_f32_TFLOPs": round(mfma_tflops, 2), "mfma_f32_frac_of_published": round(mfma_tflops / MFMA_F32_PEAK_TFLOPS, 4),
            "copy_bytes": copy_bytes, "mfma_ms": round(ms_mfma, 3)}


def pipeline_share(iters=2000):
    """Rows of (mix, ms, [(role, ticks per instruction)]) for the wave mixes below; an MFMA round is 8
    instructions, a VALU round 64."""
    from . import binding as B
    M, V = B.PROBE_ROLE_MFMA, B.PROBE_ROLE_VALU
    mixes = [[M], [M, M], [M, M, M, M], [V], [V, V], [M, V], [V, M], [M, M, V], [M, V, V], [M, M, M, V], [M, M, V, V]]
    rows = []
    for roles in mixes:
        ms, ticks = B.probe_pipeline_share(roles, iters)
        rows.append(("+".join("MFMA" if r == M else "VALU" for r in roles), ms,
                     [("MFMA" if r == M else "VALU", t / (iters * (8.0 if r == M else 64.0))) for r, t in zip(roles, ticks)]))
    return rows


def share_report(rows):
    lines = ["# How fp32 MFMA waves and VALU waves share one SIMD (one MI355X)", "",
             "Written by `python -m paper_2012_15667_amd.ceilings --share > profiles/pipeline_share.md` (from the repository root",
             "on the GPU box).  One launch of 256 workgroups; every SIMD holds the waves listed; an MFMA wave issues 16000",
             "`v_mfma_f32_32x32x2_f32` (64 matrix cycles each), a VALU wave 128000 `v_fma_f32`; ticks = `s_memtime` counts (core",
             "clock) per instruction of that wave.  Reading: a wave of MFMAs runs at its full rate whatever runs beside it; a",
             "VALU wave beside it needs the MFMA wave's whole time plus its own solo time (about (16000 x 64 + 128000 x 5.3) /",
             "128000 = 13.3 ticks per instruction): plain vector instructions make no progress while another wave of the SIMD",
             "streams fp32 MFMAs -- the two share one pipeline, and vector work next to matrix work is paid in full.", "",
             "| waves of one SIMD | launch ms | ticks per instruction, wave by wave |", "|---|---|---|"]
    for name, ms, per in rows:
        lines.append("| %s | %.3f | %s |" % (name, ms, ", ".join("%s %.1f" % (r, t) for r, t in per)))
    return "\n".join(lines)


if __name__ == "__main__":
    if "--share" in sys.argv[1:]:
        print(share_report(pipeline_share()))
    else:
        print(json.dumps(measure()))
    sys.exit(0)
