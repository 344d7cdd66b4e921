"""End-to-end size of a checkpoint chain: search + quantize + delta on the GPU, entropy stage on the
host, with and without the regrouping by the previous symbol (Sec. 6; the shape of the paper's delta
ablation).  Synthetic GPT-2-medium-shaped weights with Adam state, five steps.

    python -m paper_2306_11800_amd.ratio_report [--scale 0.25] [--threads 16] [--bins sketch]

--bins sketch keeps the prune / protect fractions the grid search chose and takes the bins from the
sketch + weighted K-Means rule with the fewest bits that meet eps (inshr_search_sketch; the same
uniform numbers at every step).

Prints one JSON line per step and a summary line.  Bytes of a step = entropy-coded delta streams +
codebooks + protected values (index and value, 8 bytes each) + group offsets.
"""
import argparse
import json
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from . import api, synth


def unpack(words: torch.Tensor, n: int, w: int) -> torch.Tensor:
    """Value i = bits [w*i, w*i + w) of the little-endian word stream (w <= 9)."""
    b = torch.cat([words.view(torch.uint8), torch.zeros(8, dtype=torch.uint8, device=words.device)])
    out = torch.empty(n, dtype=torch.int16, device=words.device)
    step = 1 << 24
    for i0 in range(0, n, step):
        i = torch.arange(i0, min(n, i0 + step), device=words.device, dtype=torch.int64)
        bit = i * w
        byte = bit >> 3
        two = b[byte].to(torch.int32) | (b[byte + 1].to(torch.int32) << 8)
        out[i0:i0 + i.numel()] = ((two >> (bit & 7).to(torch.int32)) & ((1 << w) - 1)).to(torch.int16)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--scale", type=float, default=1.0, help="shrinks the first dimension of every tensor")
    ap.add_argument("--threads", type=int, default=16)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--bins", choices=["equal", "sketch"], default="equal")
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    ctx = api.Context(dev)
    grid, eps = synth.grid_full(), synth.EPS_DEFAULT
    items = list(synth.gpt2_medium_steps(scale=args.scale, n_steps=args.steps))
    n_total = sum(st[0].size for _, st in items)
    q_prev = None
    totals = dict(fp32=0, quantized=0, regrouped=0, index_order=0)
    for t in range(args.steps):
        ts = [torch.from_numpy(st[t]).to(dev) for _, st in items]
        best, _, _ = ctx.search(ts, grid, eps, want_scores=False)
        if args.bins == "sketch":
            uni = np.random.default_rng(0).uniform(size=(len(ts), 256))
            q_cur, choices, _ = ctx.search_sketch(ts, [grid[b] for b in best], uni, eps, reuse_search=True)
        else:
            q_cur = ctx.quantize(ts, [grid[b] for b in best], reuse_search=True)
        side = sum(4 * (1 << q.bits) + 8 * q.n_outlier for q in q_cur)  # codebooks, protected values
        quantized = sum((q.n * q.sym_bits + 7) // 8 for q in q_cur) + side
        line = dict(step=t, fp32_bytes=4 * n_total, quantized_bytes=quantized,
                    mean_symbol_bits=round(sum(q.n * q.sym_bits for q in q_cur) / n_total, 3))
        if q_prev is not None:
            ds = ctx.delta(q_prev, q_cur, want_perm=True)
            ctx.sync()
            jobs, changed = [], 0
            for d, qp in zip(ds, q_prev):
                e = unpack(d.packed, d.n, d.delta_bits)
                changed += int((e != 0).sum())
                idx = torch.empty_like(e)
                idx[d.perm.to(torch.int64) & 0xFFFFFFFF] = e  # the delta in index order
                goff = d.group_off[:(1 << qp.bits) + 3].cpu().numpy().view(np.uint64)
                jobs.append((goff, d.delta_bits, d.packed.cpu().numpy().view(np.uint64), None))
                jobs.append((np.array([0, d.n], np.uint64), d.delta_bits, None,
                             idx.cpu().numpy().view(np.uint16)))
            t0 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=args.threads) as ex:
                sizes = list(ex.map(lambda j: api.entropy_encode(j[0], j[1], packed=j[2], values=j[3])[0].size,
                                    jobs))
            dt = time.perf_counter() - t0
            line.update(regrouped_bytes=sum(sizes[0::2]) + side, index_order_bytes=sum(sizes[1::2]) + side,
                        changed_fraction=round(changed / n_total, 4),
                        host_encode_s=round(dt, 2), host_threads=args.threads)
            totals["regrouped"] += line["regrouped_bytes"]
            totals["index_order"] += line["index_order_bytes"]
            totals["fp32"] += 4 * n_total
            totals["quantized"] += quantized
            line["ratio_regrouped"] = round(4 * n_total / line["regrouped_bytes"], 2)
            line["ratio_index_order"] = round(4 * n_total / line["index_order_bytes"], 2)
        line["ratio_quantized"] = round(4 * n_total / quantized, 2)
        print(json.dumps(line), flush=True)
        q_prev = q_cur
    if totals["fp32"]:
        print(json.dumps(dict(summary="steps 1.." + str(args.steps - 1), values_per_step=n_total,
                              ratio_quantized=round(totals["fp32"] / totals["quantized"], 2),
                              ratio_delta_index_order=round(totals["fp32"] / totals["index_order"], 2),
                              ratio_delta_regrouped=round(totals["fp32"] / totals["regrouped"], 2))))


if __name__ == "__main__":
    main()
