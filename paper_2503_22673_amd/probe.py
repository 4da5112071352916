"""Prints the two ceilings the GEMM is measured against: sustained bf16 MFMA rate and the
global -> LDS feed rate for L2-, MALL- and HBM-resident spans.

    python -m paper_2503_22673_amd.probe
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    import torch
    import synth
    from paper_2503_22673_amd import binding as B
    ctx = B.Context(B.make_config(synth.CONFIGS[3]))
    print("bf16 MFMA, register resident: %.0f TFLOP/s sustained" % ctx.probe_mfma_peak(100000, 2048))
    buf = torch.ones(8 << 30, dtype=torch.uint8, device="cuda")
    for span_mb, what in ((2, "L2-resident"), (64, "MALL-resident"), (8192, "HBM")):
        for k in (4, 8):
            g = ctx.probe_lds_feed(k, span_mb << 20, buf=buf)
            print("global->LDS feed, %-13s span %5d MB, %2d KB in flight per CU: %8.0f GB/s chip, %5.1f GB/s per CU"
                  % (what, span_mb, 8 * k, g, g / 256))


if __name__ == "__main__":
    main()
