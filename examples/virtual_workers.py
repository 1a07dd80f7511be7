"""Algorithm 2 of the paper (quantized fully-sharded data parallelism) with P VIRTUAL workers on
one GPU: the data flow of a multi-GPU run, with the collectives replaced by views into shared
buffers, so that the codec entry points can be seen (and tested) working together.

Per step, for a layer of n parameters sharded P ways (shard = a multiple of the bucket size):
  1. weight gather: every owner's slot of the gather buffer holds the packed Q^w codes of its
     shard; a worker decodes all slots with one qsdp_dequantize_gathered call;
  2. every worker computes its local gradient on the decoded weights (here the toy objective
     f_p(w) = 1/2 |w - t_p|^2, so g_p = w - t_p; plain torch arithmetic, not part of the library);
  3. every worker quantizes its whole gradient with qsdp_quantize_grad (its own seed);
  4. gradient exchange: owner s needs slice s of every worker's codes, a strided view here;
  5. owner s runs qsdp_recv_step (or qsdp_recv_adamw_step): decode-and-average the P slices, SGD
     (AdamW) step on its fp32 master shard, Q^w of the result, whose codes go straight into its
     slot of the gather buffer.

    python examples/virtual_workers.py            # prints the loss per step
"""
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_2302_02390_amd import binding as qb  # noqa: E402


def layout(n, workers, bucket, wbits, gbits):
    """Sizes of the sharded layer: elements per shard and words per slot / per gradient slice."""
    if (bucket * wbits) % 128 or (bucket * gbits) % 128:
        raise ValueError("this example keeps every slice 16-byte aligned: bucket * bits must be a multiple of 128")
    per_worker = -(-n // workers)
    shard = -(-per_worker // bucket) * bucket
    nshards = -(-n // shard)
    return {
        "shard": shard, "nshards": nshards,
        "wwords": shard * wbits // 32, "gwords": shard * gbits // 32, "mfloats": 2 * (shard // bucket),
    }


def run(x0, targets, steps, lr, wbits=8, gbits=4, bucket=1024, delta=0.0, seed0=0, trace=None, keep_master=False,
        adamw=None):
    """x0: float32[n] initial weights on the GPU; targets: float32[P, n] (worker p pulls towards
    targets[p]). Returns (final master weights float32[n], [loss after every step]). `trace`, if
    given, receives (step, decoded weights) before every update. keep_master: the owners' shards stay
    in full precision (Algorithm 2 as written) instead of living on the quantization grid (the
    iteration the paper analyses). adamw: None for the SGD step, or (beta1, beta2, eps, weight_decay) for the
    owners' AdamW (moments live with the master shards)."""
    flags = qb.QSDP_FLAG_KEEP_MASTER if keep_master else 0
    dev = x0.device
    workers, n = targets.shape
    lay = layout(n, workers, bucket, wbits, gbits)
    shard, nshards = lay["shard"], lay["nshards"]
    if nshards != workers:
        raise ValueError("the layer is too small for this many workers")
    x = x0.clone()                                                   # fp32 master shards, back to back
    slot_codes = torch.zeros((nshards, (lay["wwords"] + 3) // 4 * 4), dtype=torch.int32, device=dev)
    slot_meta = torch.zeros((nshards, (lay["mfloats"] + 3) // 4 * 4), dtype=torch.float32, device=dev)
    bounds = [(s * shard, min((s + 1) * shard, n)) for s in range(nshards)]
    for s, (a, b) in enumerate(bounds):                              # initial Q^w of every shard
        nb = -(-(b - a) // bucket)
        qb.qsdp_quantize_weight(x[a:b], wbits, bucket, delta, seed0, slot_codes[s, :nb * bucket * wbits // 32],
                                slot_meta[s, :2 * nb])
    # every worker's quantized gradient of the whole layer; rows padded to 16 bytes
    nb_all = nshards * (shard // bucket)
    gcodes = torch.zeros((workers, nb_all * bucket * gbits // 32), dtype=torch.int32, device=dev)
    gmeta = torch.zeros((workers, (2 * nb_all + 3) // 4 * 4), dtype=torch.float32, device=dev)
    w = torch.empty(n, dtype=torch.float32, device=dev)
    mom = torch.zeros(n, dtype=torch.float32, device=dev) if adamw else None
    var = torch.zeros(n, dtype=torch.float32, device=dev) if adamw else None
    mean_target = targets.double().mean(dim=0)
    losses = []
    for t in range(steps):
        qb.qsdp_dequantize_gathered(slot_codes, slot_meta, nshards, n, shard, wbits, bucket, w)         # 1
        if trace is not None:
            trace(t, w)
        for p in range(workers):
            g = w - targets[p]                                                                          # 2
            nb = -(-n // bucket)
            qb.qsdp_quantize_grad(g, gbits, bucket, seed0 + 1000 * (t + 1) + p, 0,
                                  gcodes[p, :nb * bucket * gbits // 32], gmeta[p, :2 * nb])              # 3
        for s, (a, b) in enumerate(bounds):
            nb = -(-(b - a) // bucket)
            gw = nb * bucket * gbits // 32
            slices = gcodes[:, s * lay["gwords"]: s * lay["gwords"] + gw]                                # 4
            metas = gmeta[:, s * lay["mfloats"]: s * lay["mfloats"] + 2 * nb]
            out_codes, out_meta = slot_codes[s, :nb * bucket * wbits // 32], slot_meta[s, :2 * nb]
            if adamw:                                                                                    # 5
                b1, b2, eps, wd = adamw
                qb.qsdp_recv_adamw_step(x[a:b], mom[a:b], var[a:b], slices, metas, workers, 1.0 / workers, lr, b1, b2,
                                        eps, wd, 1.0 - b1 ** (t + 1), 1.0 - b2 ** (t + 1), wbits, gbits, bucket, delta,
                                        seed0 + t, flags, out_codes, out_meta)
            else:
                qb.qsdp_recv_step(x[a:b], slices, metas, workers, 1.0 / workers, lr, wbits, gbits, bucket, delta,
                                  seed0 + t, flags, out_codes, out_meta)
        losses.append(float(0.5 * ((x.double() - mean_target) ** 2).sum()))
    return x, losses


def main():
    if not torch.cuda.is_available():
        print("virtual_workers.py needs a GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev).manual_seed(0)
    n, workers = 1 << 20, 8
    x0 = 0.02 * torch.randn(n, device=dev, generator=gen)
    targets = 0.02 * torch.randn((workers, n), device=dev, generator=gen) + 0.01
    _, losses = run(x0, targets, steps=30, lr=0.3)
    for t, v in enumerate(losses):
        print(f"step {t + 1:3d}  loss {v:.6e}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
