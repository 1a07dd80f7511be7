"""The quantized iteration x <- Q^w(x - lr * Q^g(g)) driving a real (if small) training loop on one GPU.

A student MLP learns a fixed teacher MLP on synthetic inputs. Forward and backward run in PyTorch; all
parameters live in ONE flat fp32 buffer (the layers are views into it, so are their gradients), and the
update of every step is a single call of the library: `qsdp_fused_step` on that buffer, W8 G4, bucket
1024, seed = step index. The same loop with a plain SGD update is the baseline.

    python examples/train_mlp.py            # prints both loss curves
"""
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_2302_02390_amd import binding as qb  # noqa: E402

DIMS = (256, 512, 512, 64)


def flat_model(device, seed):
    """Weights and biases of the MLP as views into one flat parameter buffer (and one flat gradient buffer)."""
    gen = torch.Generator(device=device).manual_seed(seed)
    shapes = []
    for a, b in zip(DIMS[:-1], DIMS[1:]):
        shapes += [(b, a), (b,)]
    n = sum(int(torch.tensor(s).prod()) for s in shapes)
    n_pad = -(-n // 8) * 8
    flat = torch.zeros(n_pad, device=device)
    grad = torch.zeros(n_pad, device=device)
    params, off = [], 0
    for s in shapes:
        k = int(torch.tensor(s).prod())
        p = flat[off:off + k].view(s)
        if len(s) == 2:
            p.copy_(torch.randn(s, device=device, generator=gen) / s[1] ** 0.5)
        p.requires_grad_(True)
        p.grad = grad[off:off + k].view(s)
        params.append(p)
        off += k
    return flat, grad, params


def forward(params, inp):
    h = inp
    for i in range(0, len(params), 2):
        h = torch.nn.functional.linear(h, params[i], params[i + 1])
        if i + 2 < len(params):
            h = torch.tanh(h)
    return h


def train(steps=300, lr=0.3, quantized=True, wbits=8, gbits=4, bucket=1024, device="cuda:0", trace=None):
    device = torch.device(device)
    _, _, teacher = flat_model(device, 1)
    flat, grad, student = flat_model(device, 2)
    gen = torch.Generator(device=device).manual_seed(3)
    losses = []
    for step in range(steps):
        inp = torch.randn(512, DIMS[0], device=device, generator=gen)
        with torch.no_grad():
            target = forward(teacher, inp)
        grad.zero_()
        loss = torch.nn.functional.mse_loss(forward(student, inp), target)
        loss.backward()                      # accumulates into the views of `grad`
        with torch.no_grad():
            if quantized:
                qb.qsdp_fused_step(flat, grad, lr, wbits, gbits, bucket, 0.0, step)
            else:
                flat.add_(grad, alpha=-lr)
        losses.append(float(loss.detach()))
        if trace is not None and step % trace == 0:
            print(f"step {step:4d}  loss {losses[-1]:.6f}")
    return losses


if __name__ == "__main__":
    if not torch.cuda.is_available():
        print("train_mlp.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    print("quantized iteration, W8 G4:")
    q = train(trace=50)
    print("plain SGD:")
    s = train(quantized=False, trace=50)
    print(f"final loss (mean of the last 20 steps): quantized {sum(q[-20:]) / 20:.6f}, plain {sum(s[-20:]) / 20:.6f}")
