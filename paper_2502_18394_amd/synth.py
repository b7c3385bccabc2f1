"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds none of the method's arithmetic: it only draws random tensors of the
shapes the paper's workloads have (Llama-3.2-1B head shape H=32, d=64 over the
length grid of Fig. 1; the decode setting of Table 1; a 14x14 ViT patch grid)
and rounds values to bf16 where a configuration stores them that way.  The same
arrays are handed to the CPU oracle and to the GPU library.

Base seed 42 is the seed the paper fixes for its runs (App. D, Reproducibility).
"""
import numpy as np

BASE_SEED = 42

# name -> shape of the workload
CONFIGS = {
    "single_head_1k": dict(B=1, H=1, L=1024, d=64, io="f32"),
    "llama1b_8k": dict(B=1, H=32, L=8192, d=64, io="bf16"),
    "llama1b_128k": dict(B=1, H=32, L=131072, d=64, io="bf16"),
    "decode_32k": dict(B=8, H=32, N_max=32768, d=64, steps=256, io="f32"),
    "vit_196": dict(B=256, H=12, L=196, d=64, io="f32"),
}
SWEEP_L = (512, 1024, 4096, 8192, 32768, 131072)
D_GATE = 64        # hidden width of the gate MLP in every configuration
LN_EPS = 1e-5


def f32_to_bf16_bits(x):
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def tokens(seed, shape, io="f32"):
    """N(0,1) rows.  Returns (values as float32 exactly as stored, storage array):
    for io == 'bf16' the storage array holds uint16 bit patterns and the float32
    array their exact values; for 'f32' both are the same array."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(shape, dtype=np.float32)
    if io == "bf16":
        bits = f32_to_bf16_bits(x)
        return bf16_bits_to_f32(bits), bits
    if io != "f32":
        raise ValueError(io)
    return x, x


def gate_params(seed, Hg, d, n_fft, d_g=D_GATE, modrelu=True, std=0.02):
    """Gate parameters: W1, b1, W2, b2, modReLU bias ~ N(0, std); LayerNorm
    gamma = 1 + N(0, std), beta ~ N(0, std).  float32, shapes as in the header."""
    rng = np.random.default_rng(seed)
    F = n_fft // 2 + 1

    def nrm(*s):
        return (std * rng.standard_normal(s, dtype=np.float32)).astype(np.float32)

    p = dict(
        Hg=Hg, d=d, d_g=d_g, n_fft=n_fft, ln_eps=LN_EPS,
        ln_gamma=(1.0 + nrm(Hg, d)).astype(np.float32), ln_beta=nrm(Hg, d),
        W1=nrm(Hg, d, d_g), b1=nrm(Hg, d_g),
        W2=nrm(Hg, d_g, 2 * F), b2=nrm(Hg, 2 * F),
        modrelu_bias=nrm(Hg, F) if modrelu else None,
    )
    return p


def wrm_params(seed, Hg, d, levels, d_w=D_GATE, std=0.02, gate_std=0.5):
    """Wavelet-refinement MLP (Sec. 3.5 step b): W1, b1 ~ N(0, std), LayerNorm as for the gate; the output
    layer ~ N(0, gate_std) so that the level gates are O(1) and every band visibly matters.
    W2 [Hg, d_w, (levels+1)*d], b2 [Hg, (levels+1)*d], float32."""
    rng = np.random.default_rng(seed)
    nout = (levels + 1) * d

    def nrm(sd, *s):
        return (sd * rng.standard_normal(s, dtype=np.float32)).astype(np.float32)

    return dict(Hg=Hg, d=d, d_w=d_w, levels=levels, ln_eps=LN_EPS,
                ln_gamma=(1.0 + nrm(std, Hg, d)).astype(np.float32), ln_beta=nrm(std, Hg, d),
                W1=nrm(std, Hg, d, d_w), b1=nrm(std, Hg, d_w),
                W2=nrm(gate_std, Hg, d_w, nout), b2=nrm(gate_std, Hg, nout))


def max_wavelet_levels(n):
    """How many times 2 divides n: the deepest Haar analysis of an n-point column."""
    J = 0
    while n > 1 and n % 2 == 0:
        n //= 2
        J += 1
    return J


def toeplitz_taps(seed, Hg, r, std=0.02):
    """Complex taps t_{-r..r} ~ N(0, std) for the optional low-rank gate update, complex64 [Hg, 2r+1]."""
    rng = np.random.default_rng(seed)
    t = std * rng.standard_normal((Hg, 2 * r + 1, 2), dtype=np.float32)
    return np.ascontiguousarray(t[..., 0] + 1j * t[..., 1]).astype(np.complex64)


def random_gate(seed, B, H, n_fft):
    """A stand-alone complex gate [B,H,F] with O(1) entries (for mixer-only tests)."""
    rng = np.random.default_rng(seed)
    F = n_fft // 2 + 1
    g = rng.standard_normal((B, H, F, 2), dtype=np.float32)
    return np.ascontiguousarray(g[..., 0] + 1j * g[..., 1]).astype(np.complex64)
