"""Seeded synthetic inputs for decode attention.

This module only draws numbers and lays them out; it contains none of the
attention arithmetic.  Both the CPU oracle's tests and the GPU tests/benchmark
take their inputs from here so that the two sides see identical bits.

Layouts: q ``[B, Hq, D]``, k and v ``[B, Hkv, Smax, D]`` (float16, C-contiguous),
seq_lens ``[B]`` int32.  Values are i.i.d. N(0,1) rounded to float16
(round-to-nearest-even), standing in for a trained model's KV cache: with
D = 128 and scale 1/sqrt(128) the logits are roughly N(0,1), inside the range
the paper reports for Llama2-7B (Section 3, "Analysis and Insights").
"""
import math

import numpy as np

# The workloads the benchmark and the parity tests are sized for.  "ragged"
# gives the inclusive range sequence lengths are drawn from.
CONFIGS = {
    "c0_b1_h32_s1024": dict(B=1, Hq=32, Hkv=32, D=128, Smax=1024, seed=1000, chunk=256),
    "c1_b1_h32_s8192": dict(B=1, Hq=32, Hkv=32, D=128, Smax=8192, seed=2000, chunk=256),
    "c2_b16_h32_ragged4096": dict(B=16, Hq=32, Hkv=32, D=128, Smax=4096, seed=3000, chunk=256,
                                  ragged=(512, 4096)),
    "c3_b32_gqa64x8_s4096": dict(B=32, Hq=64, Hkv=8, D=128, Smax=4096, seed=4000, chunk=256),
    "c4_b4_h32_s32768_overflow": dict(B=4, Hq=32, Hkv=32, D=128, Smax=32768, seed=5000, chunk=256,
                                      plant_frac=0.01, plant_seed=5999, plant_gamma=36.0),
}
PHI = 3.0
BOUNDS = (-60.0, 20.0)


def default_scale(D):
    return float(np.float32(1.0 / math.sqrt(D)))


def _normal_f16(rng, shape):
    """N(0,1) as float16, generated in slabs to bound the float32 temporary."""
    out = np.empty(shape, dtype=np.float16)
    flat = out.reshape(-1)
    step = 1 << 24
    for i in range(0, flat.size, step):
        n = min(step, flat.size - i)
        flat[i:i + n] = rng.standard_normal(n, dtype=np.float32).astype(np.float16)
    return out


def make_case(B, Hq, Hkv, D, Smax, seed, ragged=None, seq_lens=None, poison_padding=False, **_):
    """Draw one decode-attention problem.

    Order of draws from ``default_rng(seed)``: lengths (if ragged), q, k, v.
    ``poison_padding`` overwrites K and V at positions >= seq_len with NaN so a
    test can prove padding never reaches the result.
    """
    rng = np.random.default_rng(seed)
    if seq_lens is not None:
        sl = np.asarray(seq_lens, dtype=np.int32).reshape(B)
    elif ragged is not None:
        sl = rng.integers(ragged[0], ragged[1], size=B, endpoint=True).astype(np.int32)
    else:
        sl = np.full(B, Smax, dtype=np.int32)
    q = _normal_f16(rng, (B, Hq, D))
    k = _normal_f16(rng, (B, Hkv, Smax, D))
    v = _normal_f16(rng, (B, Hkv, Smax, D))
    if poison_padding:
        for b in range(B):
            n = int(np.clip(sl[b], 0, Smax))
            k[b, :, n:, :] = np.float16(np.nan)
            v[b, :, n:, :] = np.float16(np.nan)
    return dict(q=q, k=k, v=v, seq_lens=sl, B=B, Hq=Hq, Hkv=Hkv, D=D, Smax=Smax,
                scale=default_scale(D))


def make_config(name, layer=0, **overrides):
    """Problem for one of CONFIGS; ``layer`` offsets the seed (one KV set per layer)."""
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    cfg["seed"] = cfg["seed"] + layer
    case = make_case(**cfg)
    case["chunk"] = cfg["chunk"]
    case["planted"] = []
    if cfg.get("plant_frac"):
        rows = cfg["B"] * cfg["Hq"]
        n_rows = int(math.ceil(cfg["plant_frac"] * rows))
        case["planted"] = plant_keys(case, n_rows, cfg["plant_gamma"], cfg["plant_seed"] + layer)
    return case


def plant_keys(case, n_rows, gamma, seed, allow_shared_kv=False):
    """Overwrite one key in each of ``n_rows`` distinct (b, hq) rows with
    ``gamma * q / ||q||`` (float16), at a seeded position among the valid keys.

    With shared KV heads (Hq != Hkv) the planted key also enters the other rows
    of the group (with a logit of about gamma * N(0,1) / sqrt(D)); this must be
    asked for with ``allow_shared_kv``.  Returns the list of (b, hq, position).
    The V row at that position keeps its random value.
    """
    if case["Hq"] != case["Hkv"] and not allow_shared_kv:
        raise ValueError("plant_keys needs Hq == Hkv unless allow_shared_kv is set")
    G = case["Hq"] // case["Hkv"]
    rng = np.random.default_rng(seed)
    rows = case["B"] * case["Hq"]
    picked = rng.choice(rows, size=n_rows, replace=False)
    planted = []
    originals = case.setdefault("planted_original_keys", [])
    for r in sorted(int(x) for x in picked):
        b, h = divmod(r, case["Hq"])
        n = int(np.clip(case["seq_lens"][b], 0, case["Smax"]))
        if n == 0:
            continue
        pos = int(rng.integers(0, n))
        qv = case["q"][b, h].astype(np.float64)
        originals.append(case["k"][b, h // G, pos, :].copy())
        case["k"][b, h // G, pos, :] = (gamma * qv / np.linalg.norm(qv)).astype(np.float16)
        planted.append((b, h, pos))
    return planted


def to_pages(case, page_size, seed, spare_pages=3, poison_unused=True):
    """Lay a drawn case's K and V out as a paged cache.

    Returns (k_pool, v_pool, table): pools ``[n_pages, Hkv, page_size, D]`` float16 and
    ``table [B, Smax / page_size]`` int32.  The pages that hold valid tokens get distinct,
    seeded-random places in the pool; table entries of pages without a valid token are -1;
    pool pages nobody uses (``spare_pages`` extra ones, and the unused tail of the last page
    of a sequence when ``poison_unused``) hold NaN, so a test can prove they are never read.
    Only copies bytes: no attention arithmetic here.
    """
    k, v, sl = case["k"], case["v"], case["seq_lens"]
    B, Hkv, Smax, D = k.shape
    P = int(page_size)
    if Smax % P:
        raise ValueError("Smax must be a multiple of the page size")
    T = Smax // P
    used = [(b, j) for b in range(B) for j in range((int(np.clip(sl[b], 0, Smax)) + P - 1) // P)]
    n_pages = len(used) + spare_pages
    rng = np.random.default_rng(seed)
    place = rng.permutation(n_pages)[:len(used)]
    k_pool = np.full((n_pages, Hkv, P, D), np.float16(np.nan), dtype=np.float16)
    v_pool = np.full((n_pages, Hkv, P, D), np.float16(np.nan), dtype=np.float16)
    table = np.full((B, T), -1, dtype=np.int32)
    for (b, j), pid in zip(used, place):
        k_pool[pid] = k[b, :, j * P:(j + 1) * P, :]
        v_pool[pid] = v[b, :, j * P:(j + 1) * P, :]
        table[b, j] = pid
        n = int(np.clip(sl[b], 0, Smax))
        if poison_unused and (j + 1) * P > n:
            k_pool[pid, :, n - j * P:, :] = np.float16(np.nan)
            v_pool[pid, :, n - j * P:, :] = np.float16(np.nan)
    return k_pool, v_pool, table
