"""Seeded synthetic inputs for the breadth-first training-step path.

Serves both the HIP path's tests/benchmark and the CPU oracle; holds none of the
method's arithmetic: only random draws and the storage rounding of inputs.

Recipe (stands in for the text corpus the paper trains on; timing and gradient
parity do not depend on token statistics):
  activations X_m ~ N(0, 1), upstream gradients dY_m ~ N(0, 1),
  weights ~ N(0, init_std = 0.02),
  biases ~ N(0, bias_std), LayerNorm gain 1 + N(0, ln_std), LayerNorm bias N(0, ln_std).
bias_std = ln_std = 0 gives the plain initialisation (biases 0, gain 1); parity
tests use non-zero values so that every term of the layer is exercised.
"""
import numpy as np

PARAM_NAMES = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2",
)


def param_shapes(S_hidden, S_mlp):
    h, f = S_hidden, S_mlp
    return {
        "ln1_g": (h,), "ln1_b": (h,),
        "w_qkv": (h, 3 * h), "b_qkv": (3 * h,),
        "w_o": (h, h), "b_o": (h,),
        "ln2_g": (h,), "ln2_b": (h,),
        "w_fc1": (h, f), "b_fc1": (f,),
        "w_fc2": (f, h), "b_fc2": (h,),
    }


def round_bf16(a):
    """Round-to-nearest-even to bfloat16 precision, returned as float32."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def make_params(seed, N_layers, S_hidden, S_mlp, init_std=0.02, bias_std=0.02, ln_std=0.1, bf16=False):
    """List (one per layer) of dicts name -> float32 array."""
    out = []
    shapes = param_shapes(S_hidden, S_mlp)
    for l in range(N_layers):
        p = {}
        for i, name in enumerate(PARAM_NAMES):
            rng = np.random.Generator(np.random.PCG64([seed, l, i]))
            shp = shapes[name]
            if name.startswith("w_"):
                a = rng.standard_normal(shp, dtype=np.float32) * np.float32(init_std)
            elif name.endswith("_g"):
                a = np.float32(1.0) + rng.standard_normal(shp, dtype=np.float32) * np.float32(ln_std)
            elif name.startswith("ln"):
                a = rng.standard_normal(shp, dtype=np.float32) * np.float32(ln_std)
            else:
                a = rng.standard_normal(shp, dtype=np.float32) * np.float32(bias_std)
            p[name] = round_bf16(a) if bf16 else a
        out.append(p)
    return out


def make_batch(seed, N_mb, S_mb, S_seq, S_hidden, bf16=False):
    """(x, dy), each float32 [N_mb, S_mb, S_seq, S_hidden] ~ N(0, 1)."""
    shp = (N_mb, S_mb, S_seq, S_hidden)
    x = np.random.Generator(np.random.PCG64([seed, 1000, 0])).standard_normal(shp, dtype=np.float32)
    dy = np.random.Generator(np.random.PCG64([seed, 1000, 1])).standard_normal(shp, dtype=np.float32)
    if bf16:
        x, dy = round_bf16(x), round_bf16(dy)
    return x, dy


def normal(seed, tag, shape, std=1.0, bf16=False):
    """A single N(0, std) float32 tensor for per-kernel tests."""
    a = np.random.Generator(np.random.PCG64([seed, 2000, tag])).standard_normal(shape, dtype=np.float32)
    a = a * np.float32(std)
    return round_bf16(a) if bf16 else a


VOCAB_PARAM_NAMES = ("e_tok", "e_pos", "lnf_g", "lnf_b", "w_out")


def make_vocab_params(seed, S_voc, S_seq, S_hidden, init_std=0.02, ln_std=0.1, bf16=False):
    """Input / output layer parameters, dict name -> float32 array: token and position
    embeddings and the output projection ~ N(0, init_std), final LayerNorm as the layers' ones."""
    shapes = {"e_tok": (S_voc, S_hidden), "e_pos": (S_seq, S_hidden), "lnf_g": (S_hidden,), "lnf_b": (S_hidden,),
              "w_out": (S_voc, S_hidden)}
    p = {}
    for i, name in enumerate(VOCAB_PARAM_NAMES):
        rng = np.random.Generator(np.random.PCG64([seed, 3000, i]))
        a = rng.standard_normal(shapes[name], dtype=np.float32)
        if name == "lnf_g":
            a = np.float32(1.0) + a * np.float32(ln_std)
        elif name == "lnf_b":
            a = a * np.float32(ln_std)
        else:
            a = a * np.float32(init_std)
        p[name] = round_bf16(a) if bf16 else a
    return p


def make_tokens(seed, N_mb, S_mb, S_seq, S_voc, zipf=1.1):
    """(tokens, labels) int32 [N_mb, S_mb, S_seq].  Token ids follow a Zipf-like law over the vocabulary
    (text has a few very frequent tokens and a long tail, so rows of the embedding repeat inside a
    micro-batch); labels are the next token of the same stream."""
    rng = np.random.Generator(np.random.PCG64([seed, 4000]))
    w = 1.0 / np.arange(1, S_voc + 1, dtype=np.float64) ** zipf
    perm = rng.permutation(S_voc)
    stream = perm[rng.choice(S_voc, size=N_mb * S_mb * (S_seq + 1), p=w / w.sum())].astype(np.int32)
    stream = stream.reshape(N_mb, S_mb, S_seq + 1)
    return np.ascontiguousarray(stream[..., :-1]), np.ascontiguousarray(stream[..., 1:])
