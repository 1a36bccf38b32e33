"""The five workload shapes (logical tensors, SBP signatures, distributions).

Signatures are spelled as short strings: "S0", "S1", "B", "Psum", "Pmax".
dist: ("uniform", lo, hi) | ("normal", std) | ("pattern",).
"""

CONFIGS = {
    # k = 2, fp32: X S(1) x W S(0) -> Y P(sum); boxing P->B and P->S(0)
    "tiny": dict(
        k=2, dtype="f32",
        X=dict(id=0, shape=(64, 128), sbp="S1", dist=("uniform", -1.0, 1.0)),
        W=dict(id=1, shape=(128, 96), sbp="S0", dist=("uniform", -1.0, 1.0)),
    ),
    # Megatron-style MLP block, k = 8, bf16
    "mlp": dict(
        k=8, dtype="bf16",
        X=dict(id=0, shape=(8192, 4096), sbp="B", dist=("normal", 1.0)),
        W1=dict(id=1, shape=(4096, 16384), sbp="S1", dist=("normal", 0.02)),
        W2=dict(id=2, shape=(16384, 4096), sbp="S0", dist=("normal", 0.02)),
    ),
    # data-parallel weight gradient, k = 8, bf16: dW = X^T dY
    "dp_grad": dict(
        k=8, dtype="bf16",
        X=dict(id=0, shape=(16384, 1024), sbp="S0", dist=("normal", 1.0)),
        dY=dict(id=1, shape=(16384, 4096), sbp="S0", dist=("normal", 1.0)),
    ),
    # model-parallel classifier head, k = 8, bf16
    "classifier": dict(
        k=8, dtype="bf16",
        F=dict(id=0, shape=(1024, 512), sbp="B", dist=("normal", 1.0)),
        W=dict(id=1, shape=(512, 1000000), sbp="S1", dist=("normal", 0.01)),
    ),
    # pure relayout boxing, k = 16, raw 16-bit words
    "relayout": dict(
        k=16, dtype="bf16",
        T=dict(id=0, shape=(65536, 8192), sbp="S0", dist=("pattern",)),
    ),
}
