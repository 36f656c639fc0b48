"""Attention-level diagnostics on synthetic chunks: attention stealing and its repair without any model.

For one benchmark-shaped workload the cached chunks are quantized on the GPU, a sample of query rows of
the current chunk attends to them, and kvq_attention_diagnostics compares every row with attention over
the same tokens kept in BF16 (the paper's equation for Delta P_S and its appendices on the Jensen-Shannon
divergence of the attention weights and on the attention-output MSE).  Printed per setting: the mean of
Delta P_S = P^_S - P_S, of |Delta P_S|, of the divergence and of the output MSE, with the correction off
and on.  Everything numeric runs in the library's kernels; this module only generates inputs, calls
them and averages the per-row results.

    python -m paper_2605_26266_amd.diagnostics --workload small --rows 256
"""
from __future__ import annotations

import argparse
import json
from dataclasses import replace
from typing import Dict, List, Optional

import numpy as np
import torch

from . import binding as B
from . import workloads as wl


def _dev(x: np.ndarray, io_dtype: str, device: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)
    return t.to(torch.bfloat16) if io_dtype == "bf16" else t


def run(workload: str = "small", rows: int = 256, heads: Optional[int] = None, cached_chunks: Optional[int] = None,
        settings=((2, None), (2, 32), (2, "channel"), (4, None), (4, 32), (4, "channel")), corrections=(0, 1),
        device: str = "cuda:0") -> List[Dict]:
    """settings: (bits, group) pairs; group None = one fp32 (scale, zero-point) per token, an integer = FP8/BF16
    metadata per group of that many rotated channels, "channel" = keys quantized per channel over each cached
    chunk (values per token).  Returns one record per (setting, correction)."""
    base = wl.WORKLOADS[workload]
    n_heads = base.num_heads if heads is None else min(heads, base.num_heads)
    n_chunks = base.cached_chunks if cached_chunks is None else cached_chunks
    head_ids = range(n_heads)
    io = base.io_dtype
    chunks = [wl.chunk_kv(base, c, heads=head_ids) for c in range(n_chunks)]
    k_ref = torch.cat([_dev(k, io, device) for k, _ in chunks])
    v_ref = torch.cat([_dev(v, io, device) for _, v in chunks])
    k_cur, v_cur = (_dev(x, io, device) for x in wl.chunk_kv(base, n_chunks, heads=head_ids))
    row_ids = wl.sample_rows(base, rows)
    q = _dev(wl.chunk_q(replace(base, cached_chunks=n_chunks), heads=head_ids, rows=row_ids), io, device)
    records = []
    for bits, group in settings:
        per_channel = group == "channel"
        group = None if per_channel else group
        meta = B.KVQ_META_FP32 if group is None else B.KVQ_META_FP8_BF16
        cache = B.Cache(B.make_desc(n_heads, base.head_dim, bits, k_ref.shape[0],
                                    B.KVQ_BF16 if io == "bf16" else B.KVQ_FP32, group_size=group, meta_format=meta,
                                    key_axis=B.KVQ_KEYS_PER_CHANNEL if per_channel else B.KVQ_KEYS_PER_TOKEN),
                        device)
        n_chunk = base.chunk_tokens
        for c in range(n_chunks):      # one append per cached chunk, as a generation loop would do
            B.kvq_quantize_append(cache, k_ref[c * n_chunk:(c + 1) * n_chunk], v_ref[c * n_chunk:(c + 1) * n_chunk])
        for correction in corrections:
            diag = torch.empty((n_heads, q.shape[0], 4), dtype=torch.float32, device=device)
            B.kvq_attention_diagnostics(cache, 0, len(cache), q, k_ref, v_ref, k_cur, v_cur, diag, correction=correction)
            torch.cuda.synchronize()
            d = diag.double().cpu().numpy().reshape(-1, 4)
            steal = d[:, 1] - d[:, 0]
            records.append({"workload": workload, "bits": bits, "group": group or base.head_dim,
                            "metadata": "per-chan" if per_channel else "fp32" if group is None else "fp8/bf16",
                            "correction": correction,
                            "rows": int(d.shape[0]), "cached_tokens": int(k_ref.shape[0]),
                            "current_tokens": int(k_cur.shape[0]),
                            "mean_P_S": float(d[:, 0].mean()), "mean_stealing": float(steal.mean()),
                            "mean_abs_stealing": float(np.abs(steal).mean()), "mean_jsd": float(d[:, 2].mean()),
                            "mean_output_mse": float(d[:, 3].mean())})
        cache.close()
    return records


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workload", default="small", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--rows", type=int, default=256, help="query rows sampled from the current chunk")
    ap.add_argument("--heads", type=int, default=None)
    ap.add_argument("--cached-chunks", type=int, default=None)
    ap.add_argument("--json", action="store_true", help="one JSON record per line instead of the table")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("diagnostics: no GPU (the kernels are the only implementation)")
    recs = run(args.workload, args.rows, args.heads, args.cached_chunks)
    if args.json:
        for r in recs:
            print(json.dumps(r))
        return
    print("%s: %d rows x heads, %d cached + %d current tokens, mean P_S %.4f" % (
        args.workload, recs[0]["rows"], recs[0]["cached_tokens"], recs[0]["current_tokens"], recs[0]["mean_P_S"]))
    print("%-5s %-6s %-9s %-10s %12s %12s %12s %12s" % ("bits", "group", "metadata", "correction", "mean dP_S",
                                                         "mean |dP_S|", "mean JSD", "output MSE"))
    for r in recs:
        print("%-5d %-6d %-9s %-10s %12.5f %12.5f %12.5f %12.3e" % (
            r["bits"], r["group"], r["metadata"], ("off", "Taylor", "exact")[r["correction"]], r["mean_stealing"],
            r["mean_abs_stealing"], r["mean_jsd"], r["mean_output_mse"]))


if __name__ == "__main__":
    main()
