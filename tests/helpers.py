"""Small helpers shared by the tests (no method arithmetic beyond what a pin states itself)."""
import numpy as np

from paper_2604_09562_amd import synth


def gather_kv(inp, b, kind):
    """Contiguous [kv_len, Hkv, D] float64 view of request b's keys or values.

    Decoding goes through torch's dtype conversions (synth.decode_storage), which
    is independent of the oracle's own C decoders.
    """
    cache = inp["k_cache"] if kind == "k" else inp["v_cache"]
    scale = inp["k_scale"] if kind == "k" else inp["v_scale"]
    L = int(inp["kv_len"][b])
    bs = inp["block_size"]
    nblk = (L + bs - 1) // bs
    ids = inp["block_table"][b, :nblk]
    x = synth.decode_storage(cache[ids], inp["kv_dtype"]).astype(np.float64)  # [nblk,Hkv,bs,D]
    if scale is not None:
        x = x * scale[ids].astype(np.float64)[:, :, None, None]
    x = x.transpose(0, 2, 1, 3).reshape(nblk * bs, inp["num_kv_heads"], inp["head_dim"])
    return x[:L]


def q_values(inp):
    return synth.decode_storage(inp["q"], inp["q_dtype"]).astype(np.float64)


def softmax64(logits, T):
    z = np.asarray(logits, dtype=np.float64) / float(T)
    w = np.exp(z - z.max())
    return w / w.sum()
