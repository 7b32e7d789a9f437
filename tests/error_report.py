#!/usr/bin/env python3
"""Numerical error of the GPU path against the fp64 oracle, one JSON line per input type and benchmark
configuration.  Run on an MI355X from the repository root: python tests/error_report.py"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def error_report(torch, inputs, mla, dev):
    """Numerical error against the fp64 oracle in the manner of the paper's Table 1 (Section 4.3: RMSE of
    the FP16 outputs against a double-precision reference), for both input types over the five benchmark
    configurations.  The library's outputs are fp32; the paper's kernels deliver FP16, so the error of the
    output rounded to the input type is given as well."""
    import math
    import numpy as np
    from oracle import mla_oracle
    for name, dt, tag in (("fp16", torch.float16, mla_oracle.F16), ("bf16", torch.bfloat16, mla_oracle.BF16)):
        for cfg in sorted(inputs.CONFIGS):
            q, kv, lens = inputs.make_config(cfg, dtype=dt)
            out, lse = mla.mla_decode(q.to(dev), kv.to(dev), lens.to(dev), inputs.SCALE)
            torch.cuda.synchronize()
            ref_o, ref_l = mla_oracle.decode_general(inputs.bits16(q), inputs.bits16(kv), lens.numpy(), inputs.SCALE,
                                                     inputs.D_V, dtype=tag)
            ref_o = ref_o.reshape(out.shape[0], 16, 512)
            o32 = out.cpu().reshape(out.shape[0], 16, 512)
            e32 = o32.numpy().astype(np.float64) - ref_o
            e16 = o32.to(dt).float().numpy().astype(np.float64) - ref_o
            print(json.dumps({"dtype": name, "config": cfg, "batch": int(out.shape[0]), "total_kv_tokens": int(lens.sum()),
                              "rmse_fp32_out": math.sqrt(float((e32 ** 2).mean())), "max_abs_fp32_out": float(np.abs(e32).max()),
                              "rmse_out_rounded_to_input_type": math.sqrt(float((e16 ** 2).mean())),
                              "rms_of_reference_out": math.sqrt(float((ref_o ** 2).mean())),
                              "max_abs_lse": float(np.abs(lse.cpu().numpy().reshape(-1, 16) - ref_l.reshape(-1, 16)).max())}),
                  flush=True)
            del q, kv, out



if __name__ == "__main__":
    import torch
    from paper_2506_01969_amd import inputs, mla
    assert torch.cuda.is_available(), "needs a GPU"
    mla.lib()
    error_report(torch, inputs, mla, torch.device("cuda:0"))
