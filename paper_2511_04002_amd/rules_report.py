"""What Algorithm 1's two return rules cost and buy on the synthetic workloads, measured on the GPU path.

    python -m paper_2511_04002_amd.rules_report

For each workload and budget, compresses and restores with tsq_config.return_rule = TSQ_RETURN_LAST_PASSING
(the default) and TSQ_RETURN_AS_PRINTED, and prints one JSON line per case: mean width, compression ratio
and the relative RMS error of the restored inliers (outliers come back exactly under both rules).
"""
from __future__ import annotations

import json

import numpy as np


def widen(bits16: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f16":
        return bits16.view(np.float16).astype(np.float64)
    return (bits16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def main():
    import torch
    from . import synth, tsq
    tsq.lib()
    cases = [("C1", synth.make_c1()), ("C2", synth.make_c2()), ("C3", synth.make_c3(0)), ("C4", synth.make_c4(tokens=2048))]
    for name, x in cases:
        w = synth.WORKLOADS[name]
        T, H = x.shape
        xd = torch.from_numpy(x.view(np.int16)).cuda()
        v = widen(x, w.dtype)
        inl = np.abs(v) < w.tau
        for eps in (0.05, 0.2):
            row = {"workload": "%s %dx%d %s" % (name, T, H, w.dtype), "budget": "%.3g x row RMS" % eps}
            for rule in ("last_passing", "as_printed"):
                plan = tsq.Plan(T, H, w.dtype, w.tau, w.bit_set, eps, max_outliers=max(1, T * H // 8), return_rule=rule)
                blob = plan.compress(xd)
                info = plan.info(blob)
                out = widen(plan.decompress(blob).cpu().numpy().view(np.uint16), w.dtype)
                err = np.sqrt(((out[inl] - v[inl]) ** 2).sum() / max((v[inl] ** 2).sum(), 1e-300))
                row[rule] = {"mean_width": round(8.0 * info.payload_bytes / (T * H), 3),
                             "compression_ratio": round(2.0 * T * H / info.compressed_bytes, 3),
                             "rel_rms_error_of_inliers": float("%.4g" % err)}
            print(json.dumps(row))


if __name__ == "__main__":
    main()
