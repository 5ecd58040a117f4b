"""TEST INFRASTRUCTURE -- plain numpy statement of what surrounds the decoder layers in the first and last
pipeline stage (arxiv 2504.14775, section 2.1): the embedding layer that turns token ids into hidden states, the
linear projection of the final hidden states to logits over the vocabulary, and the sampling strategy (greedy,
top-k, nucleus) that selects the next token.  Only tests/ and benchmark baseline legs may import this module.

Everything is float64 unless the data itself is bf16 (tables, weights).  Readings (the paper names the operations
and nothing more):
  H1  the final hidden states are normalised like every layer input (RMSNorm, eps inside the root, gain last)
      before the projection -- the public Llama/Qwen head the stage shapes name; no bias in the projection.
  H2  sampling order: divide the logits by the temperature, keep the top-k logits, softmax over what is kept, keep
      the smallest set of most probable tokens whose mass reaches top-p, renormalise, draw.
  H3  ties are kept whole: every logit equal to the k-th largest stays, and so does every token as probable as the
      one with which the nucleus reaches top-p.  (A sort would keep an arbitrary subset of equals.)
  H4  the draw maps a uniform number u in [0,1) to the first token, IN INDEX ORDER, at which the running sum of
      the kept probabilities exceeds u times their total (so token i is drawn with probability p_i exactly).
      Any fixed order gives a correct sampler; index order needs no sort.  temperature <= 0 means greedy;
      greedy ties go to the lowest index.
  H5  a token id outside the table embeds to zeros.
"""
import numpy as np


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def embedding(table_bits: np.ndarray, ids: np.ndarray) -> np.ndarray:
    """table_bits: uint16 [V, H] (bf16 bit patterns); ids: int [T] -> uint16 [T, H]."""
    V, H = table_bits.shape
    out = np.zeros((len(ids), H), dtype=np.uint16)
    for t, i in enumerate(ids):
        if 0 <= int(i) < V:
            out[t] = table_bits[int(i)]
    return out


def final_logits(x: np.ndarray, rows, gamma_bits: np.ndarray, w_bits: np.ndarray, eps: float) -> np.ndarray:
    """x: float64 [T, H] residual stream leaving the last layer; rows: which of its rows get a next token
    -> float64 [len(rows), V]: rmsnorm(x[r]) . W^T."""
    g = bf16_to_f64(gamma_bits)
    w = bf16_to_f64(w_bits)
    out = np.empty((len(rows), w.shape[0]))
    for i, r in enumerate(rows):
        v = np.asarray(x[int(r)], dtype=np.float64)
        h = v / np.sqrt(np.mean(v * v) + eps) * g
        out[i] = w @ h
    return out


def greedy(logits: np.ndarray) -> int:
    return int(np.argmax(logits))           # numpy returns the first maximum


def kept_distribution(logits: np.ndarray, temperature: float, top_k: int, top_p: float):
    """(kept mask, probabilities renormalised over the kept tokens) after H2/H3.  top_k <= 0 or >= V keeps all;
    top_p >= 1 keeps all."""
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    V = z.shape[0]
    keep = np.ones(V, dtype=bool)
    if 0 < top_k < V:
        kth = np.sort(z)[V - top_k]
        keep &= z >= kth
    p = np.where(keep, np.exp(z - z.max()), 0.0)
    p /= p.sum()
    if top_p < 1.0:
        order = np.argsort(-p, kind="stable")
        cum = np.cumsum(p[order])
        cross = int(np.searchsorted(cum, top_p, side="left"))      # first position where the mass reaches top_p
        cross = min(cross, V - 1)
        keep &= p >= p[order[cross]]
        p = np.where(keep, p, 0.0)
        p /= p.sum()
    return keep, p


def sample(logits: np.ndarray, temperature: float, top_k: int, top_p: float, u: float) -> int:
    if temperature <= 0.0:
        return greedy(logits)
    keep, p = kept_distribution(logits, temperature, top_k, top_p)
    cum = np.cumsum(p)                      # index order (H4)
    idx = int(np.searchsorted(cum, u * cum[-1], side="right"))
    if idx >= len(p):                       # u * total rounded up to the total: the last kept token
        idx = int(np.nonzero(p > 0)[0][-1])
    return idx
