"""Counter-based generator for synthetic weights and prompts.

Every element is a pure function of (seed, tensor name, element index), so any tensor
can be produced independently, on the CPU or on the GPU, with bit-identical results:
only 64-bit integer arithmetic, one table gather, one fp32 multiply and one
round-to-nearest-even conversion to bf16 are involved.

Normal deviates come from a 65536-entry inverse-CDF table (mid-point rule), i.e. a
standard normal discretised to 16 bits and truncated at about +-4.3 sigma.
"""
import numpy as np
import torch

_MASK64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the same bit pattern as a signed 64-bit value."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _C1) & _MASK64
    z = ((z ^ (z >> 27)) * _C2) & _MASK64
    return z ^ (z >> 31)


def _name_key(seed: int, name: str) -> int:
    h = 0xCBF29CE484222325
    for ch in name.encode():
        h = ((h ^ ch) * 0x100000001B3) & _MASK64
    return _mix_int(h ^ _mix_int(seed + _GOLD))


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix_t(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def _hash_block(key: int, first: int, count: int, device) -> torch.Tensor:
    """64-bit hashes of counters first .. first+count-1 under `key` (int64 bit patterns)."""
    ctr = torch.arange(first, first + count, dtype=torch.int64, device=device)
    return _mix_t(ctr * _s64(_GOLD) + _s64(key))


_TABLE = None


def _normal_table() -> torch.Tensor:
    global _TABLE
    if _TABLE is None:
        from scipy.special import ndtri
        u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
        _TABLE = torch.from_numpy(ndtri(u).astype(np.float32))
    return _TABLE


def gen_normal_bf16(seed: int, name: str, numel: int, std: float, device="cpu",
                    chunk: int = 1 << 26) -> torch.Tensor:
    """numel bf16 values ~ std * N(0,1) (discretised), as a flat bf16 tensor on `device`."""
    key = _name_key(seed, name)
    table = _normal_table().to(device)
    out = torch.empty(numel, dtype=torch.bfloat16, device=device)
    std32 = torch.tensor(std, dtype=torch.float32, device=device)
    done = 0
    while done < numel:
        n = min(chunk, numel - done)            # elements in this chunk; chunk is a multiple of 4
        nh = (n + 3) // 4
        h = _hash_block(key, done // 4, nh, device)
        idx = torch.stack([h & 0xFFFF, _lsr(h, 16) & 0xFFFF, _lsr(h, 32) & 0xFFFF, _lsr(h, 48) & 0xFFFF], dim=1)
        vals = table[idx.reshape(-1)[:n]] * std32
        out[done:done + n] = vals.to(torch.bfloat16)
        done += n
    return out


def gen_uniform_int(seed: int, name: str, numel: int, lo: int, hi: int) -> np.ndarray:
    """numel integers uniform on [lo, hi) (int64 numpy, host)."""
    key = _name_key(seed, name)
    h = _hash_block(key, 0, numel, "cpu")
    r = (_lsr(h, 11) % (hi - lo)) + lo
    return r.numpy().astype(np.int64)


def weight_specs(model):
    """[(name, shape, kind)] for every tensor of the model; kind in {'normal','lm','ones'}."""
    d, hd = model.d_model, model.head_dim
    nq, nkv, f, v = model.n_q_heads * hd, model.n_kv_heads * hd, model.d_ffn, model.vocab
    specs = [("tok_emb", (v, d), "normal")]
    for i in range(model.n_layers):
        p = f"l{i}."
        specs += [(p + "attn_norm", (d,), "ones"),
                  (p + "wq", (nq, d), "normal"), (p + "wk", (nkv, d), "normal"), (p + "wv", (nkv, d), "normal")]
        if model.qkv_bias:
            specs += [(p + "bq", (nq,), "normal"), (p + "bk", (nkv,), "normal"), (p + "bv", (nkv,), "normal")]
        specs += [(p + "wo", (d, nq), "normal"), (p + "ffn_norm", (d,), "ones"),
                  (p + "w_gate", (f, d), "normal"), (p + "w_up", (f, d), "normal"), (p + "w_down", (d, f), "normal")]
    specs += [("final_norm", (d,), "ones"), ("lm_head", (v, d), "lm")]
    return specs


def gen_tensor(model, seed: int, name: str, shape, kind: str, device="cpu") -> torch.Tensor:
    numel = int(np.prod(shape))
    if kind == "ones":
        return torch.ones(shape, dtype=torch.bfloat16, device=device)
    std = model.lm_head_std if kind == "lm" else model.w_std
    return gen_normal_bf16(seed, name, numel, std, device).reshape(shape)


def gen_weights(model, seed: int = 0, device="cpu"):
    """Yield (name, bf16 tensor) for every tensor of the model, one at a time."""
    for name, shape, kind in weight_specs(model):
        yield name, gen_tensor(model, seed, name, shape, kind, device)


def gen_prompt(model, seed: int, request: int, length: int) -> np.ndarray:
    """Prompt of `length` token ids uniform on [0, vocab-1): never the mask id."""
    return gen_uniform_int(seed, f"prompt{request}", length, 0, model.vocab - 1).astype(np.int32)


def gen_prompt_lengths(seed: int, n: int, lo: int, hi: int):
    """n prompt lengths uniform on [lo, hi] (inclusive)."""
    return [int(x) for x in gen_uniform_int(seed, "prompt_lengths", n, lo, hi + 1)]
