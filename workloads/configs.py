"""The five benchmark configurations and a few small parity shapes.

Field names follow the paper's notation (Section 3.3): `Li` = L_init sink
tokens, `Lw` = L_local recent-window tokens, `N` = compressed middle segment,
`Dkc`/`Dvc` = number of compressed K / V head dimensions, `M` = number of real
Fourier states kept per compressed dimension, `T` = period of the basis.
"""

from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class FAConfig:
    name: str
    index: int          # selects the seeds (1000+index tensors, 2000+index masks)
    B: int
    Hq: int
    Hkv: int
    D: int
    dtype: str          # "f32" or "bf16"
    Li: int
    Lw: int
    N: int
    Dkc: int
    Dvc: int
    M: int
    num_splits: int = 0  # 0 = library chooses
    period: int = 0      # basis period T; 0 = one period spans the compressed segment
    t0: int = 0          # basis position of the first middle row

    @property
    def W(self) -> int:
        return self.Li + self.Lw

    @property
    def L(self) -> int:
        return self.Li + self.N + self.Lw

    @property
    def T(self) -> int:
        # By default one period spans the compressed segment (the only choice
        # for which the basis is orthogonal on it); never shorter than the band.
        # The paper sets T to the maximum context length: `period` > N.
        return self.period if self.period > 0 else max(self.N, self.M)

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def tol(self) -> float:
        return 1e-5 if self.dtype == "f32" else 2e-3

    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def decode_bytes(self) -> int:
        """Algorithmic bytes of one decode step: q, coefficients (fp32), kept
        middle dims, full-width sink/window rows, masks, output (fp32)."""
        e = self.elem_bytes()
        bh = self.B * self.Hkv
        return (self.B * self.Hq * self.D * e
                + bh * self.M * (self.Dkc + self.Dvc) * 4
                + bh * self.N * ((self.D - self.Dkc) + (self.D - self.Dvc)) * e
                + bh * self.W * self.D * 2 * e
                + bh * self.D * 2
                + self.B * self.Hq * self.D * 4)

    def compress_bytes(self, Dc: int) -> int:
        """Algorithmic bytes of one fa_compress call (K or V): read full rows,
        write coefficients, write kept dims."""
        e = self.elem_bytes()
        bh = self.B * self.Hkv
        return bh * (self.N * self.D * e + self.M * Dc * 4 + self.N * (self.D - Dc) * e + self.D)

    def compress_flops(self, Dc: int) -> int:
        return 2 * self.B * self.Hkv * self.N * self.M * Dc


CONFIGS = (
    FAConfig("tiny", 1, B=1, Hq=4, Hkv=1, D=64, dtype="f32", Li=4, Lw=128, N=380,
             Dkc=48, Dvc=48, M=32),
    FAConfig("llama3_8b_32k", 2, B=1, Hq=32, Hkv=8, D=128, dtype="bf16", Li=4, Lw=1024,
             N=31740, Dkc=96, Dvc=96, M=256),
    FAConfig("batched_16x8k", 3, B=16, Hq=32, Hkv=8, D=128, dtype="bf16", Li=4, Lw=512,
             N=7676, Dkc=96, Dvc=96, M=128),
    FAConfig("long_128k", 4, B=1, Hq=32, Hkv=8, D=128, dtype="bf16", Li=4, Lw=2048,
             N=129020, Dkc=112, Dvc=112, M=512, num_splits=64),
    FAConfig("llama2_7b_mha_prefill", 5, B=8, Hq=32, Hkv=32, D=128, dtype="bf16", Li=4,
             Lw=512, N=4096, Dkc=96, Dvc=96, M=256),
)


# The setting the paper ran (Section 4.1: L_init 4, L_local 1024, k = 512, 32K context) on two KV heads
# of a LLaMA-3-8B-shaped layer: not a benchmark line, a full-size parity case.
PAPER_SETTING = FAConfig("paper_k512_32k", 6, B=1, Hq=8, Hkv=2, D=128, dtype="bf16", Li=4, Lw=1024,
                         N=31740, Dkc=96, Dvc=96, M=1023)


def one_launch_variants():
    """Shapes of the one-launch decode form (bf16, D = 128, at most four query heads per KV head,
    1 .. 32 kept dims on both sides, M <= 256, compressed counts in multiples of 4), covering its
    compiled variants: series of 128 / 256 slots, one or two tiles of kept V dims, one or several
    query heads per KV head; ragged row counts, no full-width rows, a period longer than the
    segment that starts inside it, a sequence of many steps."""
    base = CONFIGS[0]
    return (
        replace(base, name="ol_g4_m200", index=41, B=2, Hq=8, Hkv=2, D=128, N=1500, Lw=300,
                Dkc=96, Dvc=100, M=200, dtype="bf16", num_splits=1),
        replace(base, name="ol_mha_m100", index=42, B=3, Hq=3, Hkv=3, D=128, N=701, Lw=40,
                Dkc=112, Dvc=112, M=100, dtype="bf16", num_splits=1),
        replace(base, name="ol_g2_m256_nowindow", index=43, B=1, Hq=4, Hkv=2, D=128, N=2049, Lw=0, Li=0,
                Dkc=100, Dvc=120, M=256, dtype="bf16", num_splits=1),
        replace(base, name="ol_g3_m31_t0", index=44, B=2, Hq=3, Hkv=1, D=128, N=517, Lw=259, Li=1,
                Dkc=124, Dvc=96, M=31, dtype="bf16", num_splits=1, period=3000, t0=1400),
        replace(base, name="ol_mha_m129_short", index=45, B=1, Hq=2, Hkv=2, D=128, N=130, Lw=5,
                Dkc=96, Dvc=108, M=129, dtype="bf16", num_splits=1),
        # more than 32 steps of 256 rows in one workgroup (the register-resident series coefficients are
        # taken afresh every 32 steps)
        replace(base, name="ol_g4_long", index=46, B=1, Hq=4, Hkv=1, D=128, N=17111, Lw=20,
                Dkc=104, Dvc=112, M=90, dtype="bf16", num_splits=1),
    )


def get_config(key) -> FAConfig:
    """Look a config up by 1-based index or by name."""
    for c in CONFIGS:
        if key == c.index or key == c.name or str(key) == str(c.index):
            return c
    raise KeyError(key)


def small_variants():
    """Parity shapes the oracle finishes in seconds: several tiles, ragged
    tails, K/V with different compressed counts, odd M, degenerate splits."""
    base = CONFIGS[0]
    return (
        base,
        replace(base, name="tiny_bf16", index=11, dtype="bf16"),
        replace(base, name="gqa8_oddM", index=12, Hq=8, Hkv=1, D=128, N=777, Lw=61,
                Dkc=96, Dvc=112, M=63, dtype="bf16"),
        replace(base, name="mha_ragged", index=13, B=2, Hq=3, Hkv=3, D=128, N=1301, Lw=37,
                Dkc=80, Dvc=64, M=128, dtype="bf16"),
        replace(base, name="no_compress", index=14, B=2, Hq=4, Hkv=2, D=64, N=300, Lw=20,
                Dkc=0, Dvc=0, M=16, dtype="f32"),
        replace(base, name="all_compress", index=15, B=1, Hq=2, Hkv=2, D=64, N=515, Lw=0, Li=1,
                Dkc=64, Dvc=64, M=17, dtype="f32"),
        replace(base, name="window_only", index=16, B=1, Hq=4, Hkv=2, D=128, N=0, Lw=200,
                Dkc=96, Dvc=96, M=8, dtype="bf16"),
        replace(base, name="middle_only", index=17, B=1, Hq=4, Hkv=2, D=128, N=2100, Lw=0, Li=0,
                Dkc=104, Dvc=88, M=200, dtype="bf16"),
        replace(base, name="odd_dims", index=19, B=1, Hq=6, Hkv=2, D=128, N=900, Lw=33,
                Dkc=91, Dvc=101, M=40, dtype="bf16"),
        replace(base, name="g2_m1", index=18, B=3, Hq=4, Hkv=2, D=64, N=130, Lw=7,
                Dkc=8, Dvc=56, M=1, dtype="f32"),
        replace(base, name="wide_d256", index=20, B=1, Hq=2, Hkv=1, D=256, N=700, Lw=300, Li=3,
                Dkc=168, Dvc=200, M=24, dtype="bf16"),
        replace(base, name="gqa16", index=21, B=1, Hq=16, Hkv=1, D=64, N=450, Lw=150,
                Dkc=40, Dvc=32, M=32, dtype="bf16"),
        replace(base, name="wide_d256_f32", index=22, B=1, Hq=4, Hkv=2, D=256, N=260, Lw=90,
                Dkc=128, Dvc=192, M=16, dtype="f32"),
        replace(base, name="all_compress_bf16", index=24, B=2, Hq=4, Hkv=2, D=128, N=650, Lw=30,
                Dkc=128, Dvc=128, M=33, dtype="bf16"),
        # a short period with a tone next to the Nyquist order (the bf16 basis takes few distinct
        # values) and a long fp32 segment whose band (the mean alone) misses every tone
        replace(base, name="short_period", index=25, B=1, Hq=2, Hkv=2, D=128, N=80, Lw=12,
                Dkc=96, Dvc=96, M=72, dtype="bf16"),
        replace(base, name="f32_mean_only", index=26, B=2, Hq=3, Hkv=1, D=64, N=1878, Lw=113, Li=3,
                Dkc=55, Dvc=23, M=1, dtype="f32"),
        # a diffuse softmax (few compressed K dims, so small scores) over unstructured kept V dims:
        # the output is a near-cancelling average and shows any rounding of the probabilities
        replace(base, name="diffuse_kept_v", index=827, B=2, Hq=6, Hkv=3, D=64, N=2329, Lw=137, Li=2,
                Dkc=6, Dvc=3, M=304, dtype="bf16"),
        replace(base, name="m512", index=23, B=1, Hq=4, Hkv=1, D=128, N=1500, Lw=40,
                Dkc=112, Dvc=112, M=512, dtype="bf16"),
        # the paper's own state size: k = 512 complex orders = 1023 live real functions (1024 with the
        # unpaired cosine), Section 4.1
        replace(base, name="m1023_paper", index=31, B=1, Hq=4, Hkv=1, D=128, N=3000, Lw=64,
                Dkc=96, Dvc=96, M=1023, dtype="bf16"),
        replace(base, name="m1024_g2", index=32, B=1, Hq=4, Hkv=2, D=128, N=2500, Lw=10,
                Dkc=112, Dvc=104, M=1024, dtype="bf16"),
        # the paper's regime: the period is the maximum context length, the segment covers part of it
        replace(base, name="period_2n", index=27, B=1, Hq=4, Hkv=1, D=128, N=1111, Lw=70,
                Dkc=96, Dvc=104, M=96, dtype="bf16", period=2222),
        replace(base, name="period_n37_f32", index=28, B=2, Hq=4, Hkv=2, D=64, N=600, Lw=50,
                Dkc=40, Dvc=48, M=48, dtype="f32", period=637),
        # a segment that starts inside the period (what a chunked prefill hands over)
        replace(base, name="t0_offset", index=29, B=1, Hq=8, Hkv=2, D=128, N=900, Lw=33,
                Dkc=96, Dvc=88, M=130, dtype="bf16", period=4000, t0=1237),
        replace(base, name="t0_offset_f32", index=30, B=1, Hq=2, Hkv=1, D=64, N=333, Lw=9,
                Dkc=48, Dvc=32, M=31, dtype="f32", period=1000, t0=667),
    )


def random_variants(seed: int, count: int):
    """`count` random small shapes (seeded): both element types, head dims 64 to 256, any
    split of the head dims between kept and compressed, segment lengths 0 to 2600 with 1 <= M <= N,
    sink and window lengths from zero up, periods equal to or longer than the segment.  Nothing
    here knows the limits of any implementation: callers decide what to do with a shape their
    kernels do not cover.  The parity tests run them next to the hand-picked shapes above; they
    are what found the short-period and mean-only cases."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        D = int(rng.choice([64, 128, 128, 128, 192, 256]))
        Hkv = int(rng.integers(1, 4))
        G = int(rng.choice([1, 2, 3, 4, 8]))
        B = int(rng.integers(1, 3))
        N = int(rng.integers(1, 2600))
        Li = int(rng.integers(0, 5))
        Lw = int(rng.integers(0, 300))
        if rng.random() < 0.1:
            N = 0
        if N + Li + Lw == 0:
            Lw = 5
        Dkc = int(rng.integers(0, D + 1))
        Dvc = int(rng.integers(0, D + 1))
        if rng.random() < 0.5:
            Dkc, Dvc = (Dkc // 8) * 8, (Dvc // 8) * 8
        m_hi = 1100 if rng.random() < 0.35 else 300      # mostly M << N, the regime the method is meant for
        M = int(rng.integers(1, min(m_hi, max(N, 1)) + 1)) if N > 0 else int(rng.integers(1, 64))
        period, t0 = 0, 0
        if N > 0 and rng.random() < 0.3:      # a period longer than the segment, the segment anywhere inside it
            period = N + int(rng.integers(1, 3 * N + 2))
            t0 = int(rng.integers(0, period - N + 1))
        out.append(FAConfig(f"random{seed}_{i}", 500 + i, B, Hkv * G, Hkv, D, dtype, Li, Lw, N, Dkc, Dvc, M,
                            period=period, t0=t0))
    return tuple(out)
