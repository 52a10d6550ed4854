"""Helpers of the GPU parity tests: run the HIP path through the binding and bring results back as
numpy.  Nothing here computes any step of the method."""
import numpy as np
import torch

from paper_2605_21226_amd import binding, layout, synth

DEV = "cuda:0"


def to_dev(x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(DEV, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)


def sign_bits_dev(signs_pm1):
    return torch.from_numpy(synth.sign_bits(signs_pm1)).to(DEV)


def new_cache(cb, n_seq, n_kv, t_capacity, fill=0):
    n = binding.octopus_cache_bytes(cb, n_seq, n_kv, t_capacity)
    assert n > 0
    return torch.full((n,), fill, dtype=torch.uint8, device=DEV)


def gpu_encode(cb, keys, dtype, signs_pm1, t_capacity, start_pos=None, cache=None):
    """keys numpy [n_seq, n_new, n_kv, d] -> (canonical records [n_seq, n_kv, t_capacity, rb], padding, cache)"""
    n_seq, n_new, n_kv, _ = keys.shape
    if cache is None:
        cache = new_cache(cb, n_seq, n_kv, t_capacity)
    sp = None if start_pos is None else torch.tensor(start_pos, dtype=torch.int32, device=DEV)
    binding.octopus_encode(cb, to_dev(keys, dtype), sign_bits_dev(signs_pm1), cache, t_capacity, sp)
    torch.cuda.synchronize()
    rec, pad = layout.cache_to_records(cache.cpu().numpy(), n_seq, n_kv, t_capacity, cb.plan.granules,
                                       cb.plan.record_bytes)
    return rec, pad, cache


def cache_from_records(cb, records, t_capacity):
    """canonical records numpy [n_seq, n_kv, n_tok, rb] -> device cache tensor"""
    img = layout.records_to_cache(records, cb.plan.granules, t_capacity)
    return torch.from_numpy(img).to(DEV)


def gpu_decode(cb, q, q_dtype, signs_pm1, cache, t_capacity, v, v_dtype, seq_lens, scale, want_scores=True,
               max_len=None):
    """q numpy [n_seq, n_q, n_qh, d], v numpy [n_seq, n_kv, t_capacity, d] -> (out, scores) numpy"""
    n_seq, n_q, n_qh, d = q.shape
    n_kv = v.shape[1]
    max_len = int(max(seq_lens)) if max_len is None else max_len
    ws_bytes = binding.octopus_attn_decode_workspace(cb, n_seq, n_qh, n_kv, n_q, max_len)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    out = torch.full((n_seq, n_q, n_qh, d), float("nan"), dtype=torch.float32, device=DEV)
    scores = torch.full((n_seq, n_q, n_qh, t_capacity), float("nan"), dtype=torch.float32, device=DEV) if want_scores else None
    lens = torch.tensor(np.asarray(seq_lens), dtype=torch.int32, device=DEV)
    binding.octopus_attn_decode(cb, to_dev(q, q_dtype), sign_bits_dev(signs_pm1), cache, t_capacity,
                                to_dev(v, v_dtype), lens, max_len, scale, out, ws, scores)
    torch.cuda.synchronize()
    return out.cpu().numpy(), (scores.cpu().numpy() if want_scores else None)


def score_floor(q_vec, gamma, scale):
    """The size a score of this query has against a key of norm gamma whatever their relative direction:
    s_t = scale * gamma_t * (q_rot . u_t) with u_t a unit vector (Eq. (score-exact)), and q_rot . u has root mean
    square ||q|| / sqrt(d) over directions.  The yardstick of a row too short for its own rms to be one."""
    q_vec = np.asarray(q_vec, dtype=np.float64)
    return scale * np.linalg.norm(q_vec) * np.asarray(gamma, dtype=np.float64) / np.sqrt(q_vec.size)


def check_scores(got, ref, floor=None):
    """|s - s_ref| <= 1e-3 * max(|s_ref|, rms(s_ref), floor) per score row; `floor` (score_floor) or None"""
    rms = np.sqrt(np.mean(ref ** 2))
    bound = 1e-3 * np.maximum(np.abs(ref), rms)
    if floor is not None:
        bound = np.maximum(bound, 1e-3 * np.asarray(floor))
    err = np.abs(got - ref)
    assert np.all(err <= bound), f"score error {np.max(err / bound):.3g} x tolerance"
    return float(np.max(err / bound))


def record_gammas(records):
    """gamma (fp32, the first four bytes) of records [..., record_bytes] -> float64 [...]"""
    return np.ascontiguousarray(records[..., :4]).view(np.float32)[..., 0].astype(np.float64)


def check_out(got, ref):
    """||out - ref||_inf <= 1e-3 * ||ref||_inf per output row"""
    e = np.max(np.abs(got - ref))
    r = np.max(np.abs(ref))
    assert e <= 1e-3 * r, f"output error {e / r:.3g} relative to the row's max"
    return float(e / max(r, 1e-300))
