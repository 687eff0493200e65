"""CPU oracle for the sparse-sparse MoE expert-FFN path (Samoyeds, arxiv 2503.10725).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition of what the
GPU library computes.  Only the test-suite, the smoke check and the benchmark's
CPU-baseline leg may import it; the product path never does.  It shares no code
with the HIP sources and imports nothing from the product package.

Everything is numpy on the host, floating point in fp64.  bf16 tensors are
carried as ``uint16`` bit patterns so that "bit-exact" has a meaning here.

What is defined where (paper passages):

* weight sparsity pattern -- blocks of M rows x V reduction columns, keep N
  Sub-Rows per block, then 2:4 inside what is kept: section 4.1, "Dual-sided
  Sparse Data Format", and section 2.3 for the 2:4 unit itself;
* encoding into data / indices / metadata: section 4.1 (third paragraph after
  figure "Samoyeds Dual-side Sparse Data Format");
* selection array SEL (per-expert token list): section 4.1 last paragraph and
  section 3.1;
* expert = gate_proj, up_proj, activation, down_proj, weighted accumulation:
  section 4.5 (figure "Output Sparsity in MoE Layer") and section 2.1;
* shared experts take every token: section 6.2.

The paper fixes no pruning criterion for inference, no tie-break, no router
formula and no activation; the readings used here are listed in the design
notes of the repository and repeated in each docstring.

Pins (see tests/): every function below is pinned by brute-force loops on
tiny inputs, by structural invariants, by hand-encoded examples under
tests/golden/ and, for the FFN, by independent dense fp64 routines.  No
function in this file is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------
# bf16 <-> fp64 on bit patterns
# --------------------------------------------------------------------------


def bf16_bits_to_f64(bits):
    """uint16 bf16 bit patterns -> float64 (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):   # signalling NaN patterns are legal inputs
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x):
    """float64 -> bf16 bits, round-to-nearest-even on the fp32 image of x.

    Used only by the diagnostic mode that rounds the intermediate ``h``; the
    parity reference itself never rounds.
    """
    f = np.ascontiguousarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    return u.astype(np.uint16)


# --------------------------------------------------------------------------
# Format
# --------------------------------------------------------------------------


class Format:
    """Weight sparsity format (N, M, V) of section 4.1 stacked on 2:4.

    ``Format(1, 1, 0)`` is plain 2:4 (no vector-wise pruning, no index array).
    Otherwise blocks are M consecutive rows x V consecutive reduction columns
    and N of the M Sub-Rows of each block are kept.
    """

    def __init__(self, N=1, M=1, V=0):
        self.N, self.M, self.V = int(N), int(M), int(V)
        if self.N < 1 or self.M < self.N:
            raise ValueError("need 1 <= N <= M")
        if self.vectorwise and (self.V < 4 or self.V % 4):
            raise ValueError("V must be a positive multiple of 4")

    @property
    def vectorwise(self):
        return self.N < self.M

    def check(self, rows, K):
        if K % 4:
            raise ValueError("K must be a multiple of 4")
        if self.vectorwise and (K % self.V or rows % self.M):
            raise ValueError("K %% V and rows %% M must be 0")

    def compressed_rows(self, rows):
        return rows * self.N // self.M if self.vectorwise else rows


def compressed_sizes(rows, K, fmt):
    """Byte sizes of (values, metadata, indices): section 4.1 gives data and
    metadata as (m/M) x (k/2) items and indices as (m/M) x (k/V) for N = 1;
    for general N the row count is m*N/M.  Values are bf16 (2 B), a metadata
    item is 2 bits, an index is one byte."""
    fmt.check(rows, K)
    rc = fmt.compressed_rows(rows)
    values = rc * (K // 2) * 2
    meta_bits = rc * (K // 2) * 2
    meta = ((K // 4 + 7) // 8) * 4 * rc          # rows are padded to whole 32-bit words
    assert meta * 8 >= meta_bits
    index = rc * (K // fmt.V) if fmt.vectorwise else 0
    return values, meta, index


# --------------------------------------------------------------------------
# Selection rules (magnitude criterion; ties go to the lower position)
# --------------------------------------------------------------------------


def _kept_subrows(w, fmt):
    """For every block (M rows x V columns) the offsets of the N kept Sub-Rows,
    ascending.  Score = sum of squares of the V unpruned values, added in
    ascending column order in fp64; the N highest scores win, equal scores
    going to the lower row.  A score that is not a number (a NaN weight, or
    infinities of both signs... cannot occur: squares) ranks like +infinity: a
    Sub-Row that holds a NaN is kept, so the NaN shows in the layer's output
    instead of being pruned away.  Returns int array [rows/M][K/V][N]."""
    rows, K = w.shape
    M, V, N = fmt.M, fmt.V, fmt.N
    blk = w.reshape(rows // M, M, K // V, V)
    score = np.zeros(blk.shape[:3], dtype=np.float64)
    for v in range(V):
        score = score + blk[..., v] * blk[..., v]
    score = np.where(np.isnan(score), np.inf, score)
    score = np.moveaxis(score, 1, 2)                       # [rows/M][K/V][M]
    order = np.argsort(-score, axis=-1, kind="stable")     # stable: lower row first on ties
    return np.sort(order[..., :N], axis=-1)


def _kept_2of4(w):
    """For every group of 4 consecutive reduction elements the 2 positions kept:
    the two largest |v|, equal magnitudes going to the lower position; a NaN
    ranks like an infinity (it is kept and stays visible); returned ascending.
    Shape [rows][K/4][2]."""
    rows, K = w.shape
    a = np.abs(w.reshape(rows, K // 4, 4))
    a = np.where(np.isnan(a), np.inf, a)
    order = np.argsort(-a, axis=-1, kind="stable")
    return np.sort(order[..., :2], axis=-1)


# --------------------------------------------------------------------------
# prune / compress / decompress
# --------------------------------------------------------------------------


def prune(w_bits, fmt):
    """Dense bf16 [rows][K] -> the pruned dense matrix (bits).

    Order of section 4.1: Sub-Row selection first (on the unpruned values),
    then 2:4 inside what survives.  Kept values keep their bits (-0.0
    included), pruned positions become +0.0.
    """
    w_bits = np.ascontiguousarray(w_bits, dtype=np.uint16)
    rows, K = w_bits.shape
    fmt.check(rows, K)
    w = bf16_bits_to_f64(w_bits)
    live = np.ones((rows, K), dtype=bool)
    if fmt.vectorwise:
        M, V = fmt.M, fmt.V
        kept = _kept_subrows(w, fmt)                       # [rows/M][K/V][N]
        sub = np.zeros((rows // M, K // V, M), dtype=bool)
        np.put_along_axis(sub, kept, True, axis=-1)
        live = np.repeat(np.moveaxis(sub, 2, 1).reshape(rows, K // V), V, axis=1)
    pos = _kept_2of4(np.where(live, w, 0.0))
    m24 = np.zeros((rows, K // 4, 4), dtype=bool)
    np.put_along_axis(m24, pos, True, axis=-1)
    keep = live & m24.reshape(rows, K)
    return np.where(keep, w_bits, np.uint16(0)).astype(np.uint16)


def compress(w_bits, fmt):
    """Dense bf16 [rows][K] (pruned or not) -> (values, meta, index).

    * compressed row r' = b*N + j holds, for every reduction segment of V
      columns, the j-th kept Sub-Row (ascending row offset) of block-row b;
      ``index[r'][s]`` is that row offset in [0, M).  Plain 2:4: r' = r and
      ``index`` is empty.
    * ``values[r'][2g], values[r'][2g+1]`` are the two kept elements of group g
      in ascending position: "ordered sequentially" (section 4.1).
    * metadata: 2 bits per kept value = its position in the group of 4
      (section 2.3).  Packing: group g of a row is the nibble at bits
      [4*(g%8), 4*(g%8)+3] of little-endian uint32 word g//8 of that row; low
      two bits = first kept position, high two bits = second.
    """
    w_bits = np.ascontiguousarray(w_bits, dtype=np.uint16)
    rows, K = w_bits.shape
    fmt.check(rows, K)
    w = bf16_bits_to_f64(w_bits)
    if fmt.vectorwise:
        N, M, V = fmt.N, fmt.M, fmt.V
        kept = _kept_subrows(w, fmt)                       # [rows/M][K/V][N]
        index = np.moveaxis(kept, 2, 1).reshape(rows * N // M, K // V).astype(np.uint8)
        blk = w_bits.reshape(rows // M, M, K // V, V)
        src = np.moveaxis(kept, 2, 1)[..., None]           # [rows/M][N][K/V][1]
        gathered = np.take_along_axis(blk, np.broadcast_to(src, src.shape[:3] + (V,)), axis=1)
        cw_bits = gathered.reshape(rows * N // M, K)
    else:
        index = np.zeros((0,), dtype=np.uint8)
        cw_bits = w_bits
    rc = cw_bits.shape[0]
    pos = _kept_2of4(bf16_bits_to_f64(cw_bits))            # [rc][K/4][2]
    values = np.take_along_axis(cw_bits.reshape(rc, K // 4, 4), pos, axis=-1).reshape(rc, K // 2)
    nib = (pos[..., 0] | (pos[..., 1] << 2)).astype(np.uint32)      # [rc][K/4]
    words = (K // 4 + 7) // 8
    padded = np.zeros((rc, words * 8), dtype=np.uint32)
    padded[:, : K // 4] = nib
    shifts = (np.arange(8, dtype=np.uint32) * np.uint32(4))[None, None, :]
    meta = np.bitwise_or.reduce(padded.reshape(rc, words, 8) << shifts, axis=-1).astype(np.uint32)
    return np.ascontiguousarray(values, dtype=np.uint16), meta, index


def decompress(values, meta, index, rows, K, fmt):
    """Inverse of :func:`compress`: the pruned dense matrix as bf16 bits."""
    fmt.check(rows, K)
    rc = fmt.compressed_rows(rows)
    values = np.asarray(values, dtype=np.uint16).reshape(rc, K // 4, 2)
    meta = np.asarray(meta, dtype=np.uint32).reshape(rc, -1)
    shifts = (np.arange(8, dtype=np.uint32) * np.uint32(4))[None, None, :]
    nib = ((meta[:, :, None] >> shifts) & np.uint32(0xF)).reshape(rc, -1)[:, : K // 4]
    pos = np.stack([nib & 3, (nib >> 2) & 3], axis=-1).astype(np.int64)
    cw = np.zeros((rc, K // 4, 4), dtype=np.uint16)
    np.put_along_axis(cw, pos, values, axis=-1)
    cw = cw.reshape(rc, K)
    if not fmt.vectorwise:
        return cw
    N, M, V = fmt.N, fmt.M, fmt.V
    index = np.asarray(index, dtype=np.uint8).reshape(rows // M, N, K // V).astype(np.int64)
    out = np.zeros((rows // M, M, K // V, V), dtype=np.uint16)
    np.put_along_axis(out, np.broadcast_to(index[..., None], index.shape + (V,)),
                      cw.reshape(rows // M, N, K // V, V), axis=1)
    return out.reshape(rows, K)


# --------------------------------------------------------------------------
# routing and bucketing
# --------------------------------------------------------------------------


def route(logits, topk, n_shared=0, renormalize=True):
    """Router of section 2.1 ("a routing mechanism selects experts per token ...
    weighted sum"); the paper gives no formula, so: p = softmax(logits[t]) over
    all E experts in fp64; the k experts with the largest logits (fp32 compare,
    equal logits -> lower expert id) in descending-logit order; weight = p of
    each, divided by their sum when ``renormalize``.  Shared experts (section
    6.2) follow as ids E..E+S-1 with weight 1 in slots k..k+S-1.
    A NaN logit counts as -infinity (a masked expert): it has weight 0 and is
    chosen only when fewer than k logits are above -infinity, then in ascending
    id order like any other tie.  A token without any logit above -infinity
    has no defined weights (NaN); its ids are 0..k-1.

    Returns ids int32 [T][k+S], w float64 [T][k+S].
    """
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = lg.shape
    if not 1 <= topk <= E:
        raise ValueError("need 1 <= topk <= E")
    l64 = lg.astype(np.float64)
    l64 = np.where(np.isnan(l64), -np.inf, l64)
    with np.errstate(invalid="ignore"):
        p = np.exp(l64 - l64.max(axis=1, keepdims=True))
    p = p / p.sum(axis=1, keepdims=True)
    order = np.argsort(-l64, axis=1, kind="stable")[:, :topk]
    w = np.take_along_axis(p, order, axis=1)
    if renormalize:
        w = w / w.sum(axis=1, keepdims=True)
    ids = np.concatenate([order, np.broadcast_to(E + np.arange(n_shared), (T, n_shared))], axis=1)
    w = np.concatenate([w, np.ones((T, n_shared))], axis=1)
    return ids.astype(np.int32), w


def bucket(ids, n_experts_total):
    """Selection arrays of section 4.1: for every expert the ascending list of
    the tokens routed to it, stored back to back.

    Returns offsets int32 [E_total+1] (exclusive scan of the per-expert counts),
    sel int32 [P] (token id of every bucket position), slot int32 [P] (which
    of the token's slots put it there) and inv int32 [T][slots] (bucket
    position of every (token, slot))."""
    ids = np.asarray(ids, dtype=np.int64)
    T, slots = ids.shape
    counts = np.bincount(ids.reshape(-1), minlength=n_experts_total)
    offsets = np.concatenate([[0], np.cumsum(counts)])
    sel = np.zeros(T * slots, dtype=np.int32)
    slot = np.zeros(T * slots, dtype=np.int32)
    inv = np.zeros((T, slots), dtype=np.int32)
    fill = offsets[:-1].copy()
    for t in range(T):                       # ascending token id inside every bucket
        for j in range(slots):
            e = ids[t, j]
            sel[fill[e]] = t
            slot[fill[e]] = j
            inv[t, j] = fill[e]
            fill[e] += 1
    return offsets.astype(np.int32), sel, slot, inv


# --------------------------------------------------------------------------
# expert FFN and the layer
# --------------------------------------------------------------------------


def silu(g):
    return g / (1.0 + np.exp(-g))


ACTIVATIONS = ("silu", "gelu_tanh", "relu")


def activation(g, kind="silu"):
    """The expert's activation function.  The paper says only "activation function"
    (section 2.1, section 4.5); its models use SiLU (Mixtral, Qwen2-MoE, DeepSeek-MoE, MiniCPM-MoE)
    and, for OpenMoE (section 6.2), a GELU-family gate; the three kinds here:
    silu      g * sigmoid(g)
    gelu_tanh 0.5 g (1 + tanh(sqrt(2/pi) (g + 0.044715 g^3)))   (the tanh form of GELU)
    relu      max(g, 0)"""
    if kind == "silu":
        return silu(g)
    if kind == "gelu_tanh":
        return 0.5 * g * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (g + 0.044715 * g ** 3)))
    if kind == "relu":
        return np.maximum(g, 0.0)
    raise ValueError(f"unknown activation {kind!r}")


def router_logits(x_bits, wr_bits):
    """Router ("gate network", section 2.1): one linear layer without bias from the hidden
    state to one logit per routed expert, logits[t][e] = sum over k of x[t][k] * Wr[e][k].
    x_bits uint16 [T][H], wr_bits uint16 [E][H] (bf16 bit patterns); returns fp64 [T][E]."""
    return bf16_bits_to_f64(np.asarray(x_bits)) @ bf16_bits_to_f64(np.asarray(wr_bits)).T


def expert_ffn(x64, wg64, wu64, wd64, round_h=False, act="silu", gated=True):
    """One expert on its bucket: x64 [n][H]; wg64, wu64 [F][H]; wd64 [H][F]
    (weights stored as the transposed operand A = W^T of section 4.5: rows are
    output features).  Gated (the paper's models): h = act(gate) * up; not gated
    (``gated`` False, wu64 ignored): h = act(W1 x) with W1 = wg64; out = down(h).
    fp64 throughout; ``round_h`` (diagnostic only) rounds h to bf16 as the GPU
    path stores it."""
    g = x64 @ wg64.T
    h = activation(g, act)
    if gated:
        h = h * (x64 @ wu64.T)
    if round_h:
        h = bf16_bits_to_f64(f64_to_bf16_bits(h))
    return h @ wd64.T


def ssmm(enc_a, rows, K, fmt, b_bits, sel=None):
    """The sparse-sparse matrix multiplication of section 4.1 by its definition:
    C = A x B[:, SEL], with A the encoded weight (decoded here to its pruned dense
    form, rows x K) and B given with one row per column of the paper's B (K
    contiguous per token: the "transposed packing" of section 4.4).  Returns
    C^T as [len(sel)][rows] fp64 -- the compressed output layout of section 4.5: only
    the selected columns exist, in selection order.  ``sel`` None selects every
    column in order."""
    a64 = bf16_bits_to_f64(decompress(enc_a[0], enc_a[1], enc_a[2], rows, K, fmt))
    b64 = bf16_bits_to_f64(np.asarray(b_bits))
    if sel is not None:
        b64 = b64[np.asarray(sel, dtype=np.int64)]
    return b64 @ a64.T


def moe_layer(x_bits, logits, enc_gate, enc_up, enc_down, H, F, fmt, topk, n_shared=0,
              renormalize=True, round_h=False, act="silu", gated=True):
    """Whole hot path on the CPU.

    x_bits uint16 [T][H]; logits float32 [T][E]; enc_* are lists over the
    E + S experts of ``(values, meta, index)`` triples as :func:`compress`
    returns them (gate/up: F rows, K = H; down: H rows, K = F).

    route -> bucket -> per expert: decompress, gate/up, act(gate)*up (``gated`` False:
    act(W1 x), enc_up ignored), down -> y[t] = sum over the token's slots, in slot order, of w * out.

    Returns dict with y float64 [T][H] and the routing/bucketing arrays.
    """
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
    T = x_bits.shape[0]
    E_total = len(enc_gate)
    ids, w = route(logits, topk, n_shared, renormalize)
    offsets, sel, slot, inv = bucket(ids, E_total)
    x64 = bf16_bits_to_f64(x_bits)
    P = sel.shape[0]
    out = np.zeros((P, H), dtype=np.float64)
    for e in range(E_total):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        wg = bf16_bits_to_f64(decompress(*enc_gate[e], F, H, fmt))
        wu = bf16_bits_to_f64(decompress(*enc_up[e], F, H, fmt)) if gated else None
        wd = bf16_bits_to_f64(decompress(*enc_down[e], H, F, fmt))
        out[lo:hi] = expert_ffn(x64[sel[lo:hi]], wg, wu, wd, round_h, act, gated)
    y = np.zeros((T, H), dtype=np.float64)
    for j in range(ids.shape[1]):
        y = y + w[:, j:j + 1] * out[inv[:, j]]
    sel_w = w[sel, slot]
    return {"y": y, "ids": ids, "w": w, "offsets": offsets, "sel": sel, "sel_w": sel_w,
            "inv": inv, "pair_out": out}
