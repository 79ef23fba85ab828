"""Seeded synthetic inputs for the DiLoCoX outer step.

This module holds NO arithmetic of the method: it only draws the tensors that
stand in for the paper's training runs (trained weights, H inner steps on a
text corpus), in the shapes of the benchmark configurations.  The same bytes
are handed to the GPU library and to the CPU oracle.

Recipe (all configurations):
  theta_g            ~ N(0, 0.02^2), fp32
  raw pseudo-gradient of worker i:  G_i = U diag(s_i) V^T + E_i
      U, V           Q-factors of Gaussian matrices (k = min(m, n, 512) columns)
      s_k            k^-alpha ; worker i sees s_k * (1 + 0.1 u_ik), u ~ U(-1, 1)
      E_i            N(0, sigma^2) elementwise
  theta_l,i          cast(theta_g - G_i)  (fp32 or bf16)
  Q_in (round 1)     N(0, 1), shared by the workers
"""
import numpy as np

MASK64 = (1 << 64) - 1


def splitmix64(x):
    x = (x + 0x9E3779B97F4A7C15) & MASK64
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def seed_for(*fields):
    """One 64-bit seed from (config, round, worker, layer, matrix, tag ...)."""
    s = 0x2506_2126_3
    for f in fields:
        s = splitmix64(s ^ (int(f) & MASK64))
    return s


# ---------------------------------------------------------------------------
# Benchmark configurations (shapes are [out, in] = m x n, row-major)
# ---------------------------------------------------------------------------
def _opt13b_layer():
    return [(2048, 2048)] * 4 + [(2048, 8192), (8192, 2048)]


def _dense100b_layer():
    return [(8192, 8192), (8192, 8192), (8192, 1024), (8192, 1024),
            (8192, 28672), (8192, 28672), (28672, 8192)]


CONFIGS = {
    0: dict(name="cfg0-512x512", layers=1, layer_shapes=[(512, 512)], K=2, r=8, qbits=4,
            group=64, theta_l="f32", rounds=1, sigma=1e-3, alpha=1.0),
    1: dict(name="cfg1-opt1.3b-stage", layers=24, layer_shapes=_opt13b_layer(), K=4, r=32,
            qbits=4, group=128, theta_l="f32", rounds=3, sigma=1e-3, alpha=None),
    2: dict(name="cfg2-100b-stage", layers=10, layer_shapes=_dense100b_layer(), K=4, r=64,
            qbits=4, group=128, theta_l="bf16", rounds=1, sigma="scaled", alpha=None),
    3: dict(name="cfg3-100b-adaptive", layers=10, layer_shapes=_dense100b_layer(), K=4, r=256,
            qbits=4, group=128, theta_l="bf16", rounds=8, sigma="scaled", alpha="per-round",
            rmin=4, rmax=256, window=5),
    4: dict(name="cfg4-100b-overlap", layers=10, layer_shapes=_dense100b_layer(), K=8, r=64,
            qbits=8, group=64, theta_l="bf16", rounds=16, sigma="scaled", alpha=None),
}
LR, MU = 0.7, 0.9


def stage_shapes(cfg):
    c = CONFIGS[cfg]
    return [s for _ in range(c["layers"]) for s in c["layer_shapes"]]


def stage_params(cfg):
    return sum(m * n for m, n in stage_shapes(cfg))


def noise_sigma(cfg, m, n):
    """Elementwise noise std.  "scaled": same spectral noise floor as a 512x512 matrix at 1e-3."""
    s = CONFIGS[cfg]["sigma"]
    if s == "scaled":
        return 1e-3 * 45.25 / (np.sqrt(m) + np.sqrt(n))
    return float(s)


# ---------------------------------------------------------------------------
# numpy generator (tests, smoke, cpu baseline): everything on the host
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(x):
    """Round-to-nearest-even bf16 bit patterns (uint16) of a float32 array."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    rounded = u + 0x7FFF + ((u >> 16) & 1)
    return (rounded >> 16).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (b.astype(np.uint32) << 16).view(np.float32)


def orthonormal_columns(rng, rows, k):
    q, r = np.linalg.qr(rng.standard_normal((rows, k)))
    return q * np.sign(np.diag(r))


class MatrixInputs:
    """Inputs of one matrix: theta_g, K local replicas per round, the round-1 basis."""

    def __init__(self, m, n, K, r, seed, sigma=1e-3, alpha=1.0, theta_l="f32", kmax=512):
        self.m, self.n, self.K, self.r = m, n, K, r
        self.sigma, self.alpha, self.theta_l_kind, self.seed = sigma, alpha, theta_l, seed
        rng = np.random.default_rng(seed_for(seed, 1))
        self.k = min(m, n, kmax)
        self.U = orthonormal_columns(rng, m, self.k)
        self.V = orthonormal_columns(rng, n, self.k)
        self.theta_g = (0.02 * rng.standard_normal((m, n))).astype(np.float32)
        self.q_in = rng.standard_normal((r, n)).astype(np.float32)

    def spectrum(self, alpha=None):
        a = self.alpha if alpha is None else alpha
        return np.arange(1, self.k + 1, dtype=np.float64) ** (-a)

    def raw_pseudo_gradient(self, rnd, worker, alpha=None, noise=True):
        rng = np.random.default_rng(seed_for(self.seed, 2, rnd, worker))
        s = self.spectrum(alpha) * (1.0 + 0.1 * rng.uniform(-1.0, 1.0, self.k))
        G = (self.U * s) @ self.V.T
        if noise and self.sigma > 0:
            G = G + self.sigma * rng.standard_normal((self.m, self.n))
        return G

    def theta_local(self, theta_g_now, rnd, worker, alpha=None):
        """Local replica after the inner steps of round `rnd`, starting from theta_g_now."""
        tl = theta_g_now.astype(np.float64) - self.raw_pseudo_gradient(rnd, worker, alpha)
        tl = tl.astype(np.float32)
        if self.theta_l_kind == "bf16":
            return f32_to_bf16_bits(tl)
        return tl

    def fresh_basis_columns(self, rnd, count):
        rng = np.random.default_rng(seed_for(self.seed, 3, rnd))
        return rng.standard_normal((count, self.n)).astype(np.float32)


# ---------------------------------------------------------------------------
# torch generator (bench at full size): tensors are drawn directly in HBM
# ---------------------------------------------------------------------------
def torch_matrix_inputs(m, n, K, r, seed, sigma, alpha, theta_l, device, kmax=512, keep_uv=False):
    """Same recipe with torch ops on `device`.  Returns a dict of device tensors:
    theta_g (m,n) f32, theta_l list of K (m,n) f32|bf16, q_in (r,n) f32; with keep_uv also U, V,
    sigma and the generator, which torch_redraw_replicas needs to draw a later round."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(seed_for(seed, 1) & 0x7FFFFFFFFFFFFFFF)
    k = min(m, n, kmax)

    def orth(rows):
        a = torch.randn(rows, k, generator=g, device=device, dtype=torch.float32)
        q, _ = torch.linalg.qr(a)
        return q

    U, V = orth(m), orth(n)
    theta_g = 0.02 * torch.randn(m, n, generator=g, device=device, dtype=torch.float32)
    q_in = torch.randn(r, n, generator=g, device=device, dtype=torch.float32)
    dt = torch.bfloat16 if theta_l == "bf16" else torch.float32
    replicas = [torch.empty(m, n, device=device, dtype=dt) for _ in range(K)]
    out = dict(theta_g=theta_g, theta_l=replicas, q_in=q_in, U=U, V=V, sigma=sigma, gen=g)
    torch_redraw_replicas(out, theta_g, alpha)
    if not keep_uv:
        for key in ("U", "V", "gen", "sigma"):
            del out[key]
    return out


def torch_redraw_replicas(t, theta_g_now, alpha):
    """Local replicas of a new round, written over t["theta_l"]: theta_l,i = cast(theta_g_now -
    G_i) with G_i = U diag(s_i) V^T + E_i, s_k = k^-alpha perturbed by +-10 % per worker, fresh
    noise E_i -- the recipe of torch_matrix_inputs with this round's spectrum exponent."""
    import torch

    U, V, g, sigma = t["U"], t["V"], t["gen"], t["sigma"]
    k, dev = U.shape[1], U.device
    s0 = torch.arange(1, k + 1, device=dev, dtype=torch.float32) ** (-alpha)
    for tl in t["theta_l"]:
        s = s0 * (1.0 + 0.1 * (2.0 * torch.rand(k, generator=g, device=dev) - 1.0))
        G = (U * s) @ V.T
        G.add_(torch.randn(G.shape, generator=g, device=dev, dtype=torch.float32), alpha=sigma)
        torch.sub(theta_g_now, G, out=G)
        tl.copy_(G)
        del G


def hadamard(k):
    """Sylvester matrix of order 2^k: entries +-1, mutually orthogonal columns."""
    H = np.ones((1, 1))
    for _ in range(k):
        H = np.block([[H, H], [H, -H]])
    return H


def exact_lowrank_case(qmax, K):
    """delta = sum_c s_c h_c g_c^T with +-1 vectors h_c (length 16), g_c (length 64) and
    s_c = qmax * 2^-c: every factor entry the compressor meets is +-qmax times a power of two, so
    both quantisations, the mean, the orthonormalisation (column norms are powers of two times
    qmax) and all three products are exact.  Closed form: Delta == delta, bit for bit."""
    m, n, r = 16, 64, 4
    Hm, Hn = hadamard(4), hadamard(6)
    h, g = Hm[:, [1, 2, 5, 9]], Hn[:, [3, 7, 20, 41]]
    s = qmax * 2.0 ** -np.arange(r)
    delta = (h * s) @ g.T
    assert np.array_equal(delta, delta.astype(np.float32))
    theta0 = np.zeros((m, n), np.float32)
    tl = [(-delta).astype(np.float32) for _ in range(K)]     # theta_l = theta - delta
    q_in = np.ascontiguousarray(g.T, np.float32)             # r x n: the basis is V itself
    return m, n, r, theta0, tl, q_in, delta.astype(np.float32)
