"""Algorithmic FLOP counts of the gradient kernels, per launch, for the roofline line of
the benchmark.  A GEMM of shape M x N x K counts 2 M N K; one workload launch covers all
N workers.  Kernel names are the ones the library reports through dbw_get_timing."""
from __future__ import annotations

from . import inputs


def _head(B, n, h, c, with_input_gradient):
    """The fused classifier head (last layer h -> c, c <= 16): logits, weight gradient and, below a
    hidden layer, the input gradient."""
    return n * 2 * B * h * c * (3 if with_input_gradient else 2)


def _mlp(cfg, dims):
    B, n = cfg.batch, cfg.n
    L = len(dims) - 1
    last = L - 1 if dims[-1] <= 16 else L           # layers [0, last) go through the GEMM kernels
    fwd = [2 * B * dims[l] * dims[l + 1] for l in range(last)]
    dgrad = [2 * B * dims[l] * dims[l + 1] for l in range(1, last)]
    table = {"fc_head_kernel": _head(B, n, dims[-2], dims[-1], L > 1)}
    if fwd:
        table.update({"mlp_forward_gemm": n * sum(fwd) / len(fwd), "mlp_wgrad_gemm": n * sum(fwd) / len(fwd),
                      "mlp_thin_forward": n * sum(fwd) / len(fwd)})
    if dgrad:
        table["mlp_dgrad_gemm"] = n * sum(dgrad) / len(dgrad)
    # the same products when the whole chain of layers runs in one launch and the weight gradients in another
    table["mlp_chain_kernel"] = n * (sum(fwd) + sum(dgrad)) + table["fc_head_kernel"]
    table["mlp_wgrad_kernel"] = n * sum(fwd)
    return table


def _cnn(cfg, desc):
    B, n = cfg.batch, cfg.n
    c0, h, w = desc["in"]
    c1, c2, k, f, nc = desc["c1"], desc["c2"], desc["k"], desc["fc"], desc["classes"]
    conv1 = 2 * B * h * w * c1 * c0 * k * k
    conv2 = 2 * B * (h // 2) * (w // 2) * c2 * c1 * k * k
    flat = c2 * (h // 4) * (w // 4)
    fc = [2 * B * flat * f, 2 * B * f * nc]
    table = {"conv1_forward": n * conv1, "conv1_wgrad": n * conv1,
             "conv2_forward": n * conv2, "conv2_wgrad": n * conv2, "conv2_dgrad": n * conv2}
    table["fc_head_kernel"] = _head(B, n, f, nc, True)
    if B == 32 and flat % 512 == 0 and f % 32 == 0:      # the first FC layer runs on the batch-32 kernels
        table.update({"fc32_forward": n * fc[0], "fc32_wgrad": n * fc[0], "fc32_dgrad": n * fc[0]})
    else:
        table.update({"mlp_forward_gemm": n * fc[0], "mlp_wgrad_gemm": n * fc[0], "mlp_dgrad_gemm": n * fc[0]})
    return table


def kernel_flops(cfg, kernel_name: str) -> float:
    desc = inputs.model_dims(cfg.model)
    table = _mlp(cfg, desc["dims"]) if desc["kind"] == "mlp" else _cnn(cfg, desc)
    for key, val in table.items():
        if kernel_name.startswith(key):
            return float(val)
    return 0.0
