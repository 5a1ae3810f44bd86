"""Seeded synthetic inputs shaped like the paper's DiT linear layers.

Holds no arithmetic of the method: only random draws, an activation function used to shape a
distribution, and the cast to bf16. Both the tests' CPU oracle and the HIP library are fed from
here (the oracle always receives the exact bf16 bit patterns, copied to the host).

Stand-ins for Qwen-Image tensors (appendix table of tensor shapes; the motivation section's
remarks that activations concentrate near zero with few active channels while weights are
quasi-Gaussian): no model weights or real activations are available offline.
"""
import torch

# (M, K, N) of the named workloads. M = 4096 image tokens (+512 text tokens where stated).
WORKLOADS = {
    "tiny": dict(M=256, K=512, N=512, x="laplace_outlier"),
    "mlp_down": dict(M=4096, K=12288, N=3072, x="gelu"),
    "fc1": dict(M=4608, K=3072, N=12288, x="laplace"),
    "qkv": dict(M=4608, K=3072, N=9216, x="laplace"),
    "out_proj": dict(M=4608, K=3072, N=3072, x="laplace"),
    "fc2": dict(M=4608, K=12288, N=3072, x="gelu"),
    "hr_mlp_down": dict(M=16896, K=12288, N=3072, x="gelu"),
    "hr_fc1": dict(M=16896, K=3072, N=12288, x="laplace"),
    "hr_qkv": dict(M=16896, K=3072, N=9216, x="laplace"),
    "hr_out_proj": dict(M=16896, K=3072, N=3072, x="laplace"),
    # other models of the paper's appendix (layer-shape tables of FLUX.1-dev and Z-Image), 4096 image tokens
    "flux_single_in": dict(M=4096, K=3072, N=21504, x="laplace"),     # single-stream fused QKV + MLP-up
    "flux_single_out": dict(M=4096, K=15360, N=3072, x="gelu"),       # single-stream fused out + MLP-down
    "zimage_up": dict(M=4096, K=3840, N=10240, x="laplace"),
    "zimage_down": dict(M=4096, K=10240, N=3840, x="gelu"),
    "zimage_attn": dict(M=4096, K=3840, N=3840, x="laplace"),
    # non-square images (aspect-ratio generality of the appendix): the same four linears at
    # 1536x1024 (96 x 64 = 6144 image tokens) and 2304x1024 (144 x 64 = 9216), + 512 text tokens;
    # 26 and 38 row panels of 256, i.e. ragged tile counts on 256 compute units
    "ar32_mlp_down": dict(M=6656, K=12288, N=3072, x="gelu"),
    "ar32_fc1": dict(M=6656, K=3072, N=12288, x="laplace"),
    "ar32_qkv": dict(M=6656, K=3072, N=9216, x="laplace"),
    "ar32_out_proj": dict(M=6656, K=3072, N=3072, x="laplace"),
    "ar94_mlp_down": dict(M=9728, K=12288, N=3072, x="gelu"),
    "ar94_fc1": dict(M=9728, K=3072, N=12288, x="laplace"),
    "ar94_qkv": dict(M=9728, K=3072, N=9216, x="laplace"),
    "ar94_out_proj": dict(M=9728, K=3072, N=3072, x="laplace"),
}
SWEEP_BLOCKS = 60
SWEEP_LAYERS = ("qkv", "out_proj", "fc1", "fc2")


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _laplace(shape, g, device):
    u = torch.rand(shape, generator=g, device=device, dtype=torch.float32) - 0.5
    return -torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp(max=0.49999997))


def activations(kind, M, K, seed, device="cpu"):
    """bf16 [M,K] activations.

    laplace          rows Laplace(0,1) times a per-channel scale exp(N(0,1))
    laplace_outlier  the same with 1 % of the channels multiplied by 20
    gelu             exact-erf GELU of N(0,1) pre-activations (post-GELU MLP hidden state)
    normal           N(0,1)
    """
    g = _gen(seed, device)
    if kind in ("laplace", "laplace_outlier"):
        x = _laplace((M, K), g, device)
        scale = torch.exp(torch.randn((K,), generator=g, device=device, dtype=torch.float32))
        if kind == "laplace_outlier":
            n_out = max(1, K // 100)
            perm = torch.randperm(K, generator=g, device=device)[:n_out]
            scale[perm] *= 20.0
        x = x * scale
    elif kind == "gelu":
        z = torch.randn((M, K), generator=g, device=device, dtype=torch.float32)
        x = torch.nn.functional.gelu(z, approximate="none")
    elif kind == "normal":
        x = torch.randn((M, K), generator=g, device=device, dtype=torch.float32)
    else:
        raise ValueError(kind)
    return x.to(torch.bfloat16).contiguous()


def weights(N, K, seed, device="cpu", std=0.02):
    """bf16 [N,K] weights ~ N(0, std)."""
    g = _gen(seed, device)
    w = torch.randn((N, K), generator=g, device=device, dtype=torch.float32) * std
    return w.to(torch.bfloat16).contiguous()


def bias(N, seed, device="cpu", std=0.02):
    g = _gen(seed, device)
    return (torch.randn((N,), generator=g, device=device, dtype=torch.float32) * std).to(
        torch.bfloat16)


def workload(name, seed=0, device="cpu", M=None):
    """(X, W) of a named workload; M overrides the row count (row slices for slow checkers)."""
    w = WORKLOADS[name]
    m = w["M"] if M is None else M
    # distinct streams per tensor: seed*4+{1,2}
    X = activations(w["x"], m, w["K"], seed * 4 + 1, device)
    W = weights(w["N"], w["K"], seed * 4 + 2, device)
    return X, W


def layer_seed(block, layer_kind, base_seed=0):
    """Seed of one linear of the 60-block denoising-step sweep."""
    return base_seed * 100003 + block * 16 + SWEEP_LAYERS.index(layer_kind) + 1000


def bits(t):
    """bf16 tensor -> numpy uint16 bit patterns on the host."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view("uint16")


def from_bits(a, device="cpu"):
    """numpy uint16 bit patterns -> bf16 tensor."""
    import numpy as np
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)


def lora(N, K, R, seed, device="cpu", std_a=0.02, std_b=0.02):
    """LoRA factors L_A bf16 [N,R], L_B bf16 [R,K] ~ N(0, std). (The paper initialises trained
    factors near zero; random factors of weight-like scale exercise the kernel harder.)"""
    g = _gen(seed, device)
    la = torch.randn((N, R), generator=g, device=device, dtype=torch.float32) * std_a
    lb = torch.randn((R, K), generator=g, device=device, dtype=torch.float32) * std_b
    return la.to(torch.bfloat16).contiguous(), lb.to(torch.bfloat16).contiguous()
