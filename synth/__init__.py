"""Seeded synthetic inputs for the five workloads.

Serves both the CPU oracle's tests and the HIP path's tests/benchmark.  It holds
no arithmetic of the method: only random draws with the shapes and value
distributions of the workloads (ResNet-18/50 layer shapes standing in for the
ImageNet runs of the paper's Section 6, which need data that is not available).

Convention for "N(0, v)" in the workload descriptions: v is the VARIANCE for
weights (He initialisation, var = 2/fan_in) and the STANDARD DEVIATION for
gradients.
"""
import numpy as np


def rng(seed):
    return np.random.default_rng(int(seed))


def normal(g, shape, std=1.0, mean=0.0):
    return (g.standard_normal(shape, dtype=np.float32) * np.float32(std)
            + np.float32(mean)).astype(np.float32)


def fc_layer(seed=0, M=64, K=256, N=128):
    """Config 0: X[M,K]~N(0,1), W[K,N]~N(0, var 1/K), dY[M,N]~N(0, std 1e-3)."""
    g = rng(seed)
    x = normal(g, (M, K))
    w = normal(g, (K, N), std=(1.0 / K) ** 0.5)
    dy = normal(g, (M, N), std=1e-3)
    return x, w, dy


def range_bn_input(seed=0, N=128, C=64, H=56, W=56):
    """Config 1: first half of the channels ~N(mu_c, sigma_c), mu_c~U(-2,2),
    sigma_c~U(0.1,3); second half ~Laplace(0,1); upstream gradient ~N(0, std 1e-2)."""
    g = rng(seed)
    half = C // 2
    mu = g.uniform(-2.0, 2.0, size=half).astype(np.float32)
    sigma = g.uniform(0.1, 3.0, size=half).astype(np.float32)
    x = np.empty((N, C, H, W), np.float32)
    for c in range(half):
        x[:, c] = normal(g, (N, H, W), std=sigma[c], mean=mu[c])
    for c in range(half, C):
        x[:, c] = g.laplace(0.0, 1.0, size=(N, H, W)).astype(np.float32)
    dy = normal(g, (N, C, H, W), std=1e-2)
    return x, dy


def conv_layer(seed=0, N=128, C=64, H=56, W=56, K=64, R=3, S=3, stride=1, pad=1, relu_input=True):
    """Config 2 (and every conv of configs 3/4): X=|N(0,1)| (post-ReLU) or N(0,1),
    He-normal W (var 2/(C*R*S)), dY~N(0, std 1e-3) of the output shape."""
    g = rng(seed)
    x = normal(g, (N, C, H, W))
    if relu_input:
        x = np.abs(x)
    w = normal(g, (K, C, R, S), std=(2.0 / (C * R * S)) ** 0.5)
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    dy = normal(g, (N, K, P, Q), std=1e-3)
    return x, w, dy


def bottleneck_block(seed=0, N=128, H=56, W=56, Cin=256, Cmid=64):
    """Config 3: input |N(0,1)| [N,Cin,H,W]; He-normal weights of 1x1 Cin->Cmid,
    3x3 Cmid->Cmid, 1x1 Cmid->Cin; output gradient ~N(0, std 1e-3)."""
    g = rng(seed)
    x = np.abs(normal(g, (N, Cin, H, W)))
    w1 = normal(g, (Cmid, Cin, 1, 1), std=(2.0 / Cin) ** 0.5)
    w2 = normal(g, (Cmid, Cmid, 3, 3), std=(2.0 / (Cmid * 9)) ** 0.5)
    w3 = normal(g, (Cin, Cmid, 1, 1), std=(2.0 / Cmid) ** 0.5)
    dout = normal(g, (N, Cin, H, W), std=1e-3)
    return x, (w1, w2, w3), dout


# (Cin, Cout, R, stride, pad, H_in) of every conv of ResNet-18 at 224x224 input (config 4)
RESNET18_CONVS = (
    [(3, 64, 7, 2, 3, 224)]
    + [(64, 64, 3, 1, 1, 56)] * 4
    + [(64, 128, 3, 2, 1, 56), (128, 128, 3, 1, 1, 28), (64, 128, 1, 2, 0, 56)]
    + [(128, 128, 3, 1, 1, 28)] * 2
    + [(128, 256, 3, 2, 1, 28), (256, 256, 3, 1, 1, 14), (128, 256, 1, 2, 0, 28)]
    + [(256, 256, 3, 1, 1, 14)] * 2
    + [(256, 512, 3, 2, 1, 14), (512, 512, 3, 1, 1, 7), (256, 512, 1, 2, 0, 14)]
    + [(512, 512, 3, 1, 1, 7)] * 2
)
