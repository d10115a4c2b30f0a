"""The bf16 matrix rate of the GPU against the number of busy CUs (include/chunk_attn.h: chunk_attn_measure_mfma_rate_on).

    python -m paper_2509_21275_amd.mfma_rate_scan [--markdown out.md]

Each row runs the library's MFMA-only kernel (independent v_mfma_f32_32x32x16_bf16 on signed random operands, four waves
per workgroup, one workgroup per busy CU) for half a second and reports the rate of the last launch.  An MFMA of this
shape takes 32 cycles of a SIMD's matrix pipe, so the rate per CU is also a clock.
"""
from __future__ import annotations

import argparse

import paper_2509_21275_amd as ca

FLOP_PER_CU_CLOCK = 4 * 2 * 32 * 32 * 16 / 32   # 4 SIMDs x one 32x32x16 MFMA per 32 cycles


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--markdown", default=None)
    args = ap.parse_args()
    full = ca.chunk_attn_measure_mfma_rate(500)          # brings the chip to its sustained state; also the last row's check
    lines = ["| busy CUs | TFLOP/s | TFLOP/s per busy CU | implied clock GHz |", "|---|---|---|---|"]
    for n in (8, 32, 64, 128, 160, 192, 224, 256):
        t = ca.chunk_attn_measure_mfma_rate_on(n, 500)
        lines.append(f"| {n} | {t:.1f} | {t / n:.3f} | {t * 1e12 / n / FLOP_PER_CU_CLOCK / 1e9:.3f} |")
        print(lines[-1], flush=True)
    lines.append("")
    lines.append(f"chunk_attn_measure_mfma_rate (one workgroup per CU, before the scan): {full:.1f} TFLOP/s")
    print(lines[-1], flush=True)
    if args.markdown:
        with open(args.markdown, "w") as fh:
            fh.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
