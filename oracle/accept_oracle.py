"""CPU oracle for the bit-level compression / decompression scheme (TEST INFRASTRUCTURE).

This file is the slow, plain reference that the GPU library is checked against.  It is
test infrastructure only: nothing in the product path may import it, and it imports
nothing from the GPU package.  It is written from the paper's sections "Bit-level Fast
Compression Scheme" and "Bit-level Fast Decompression Scheme"; every function names the
passage it follows.  Arithmetic is NumPy float32 where the scheme works on 32-bit values
(one IEEE operation per written operation, no fusing), float64 for the least-squares
statistics, and plain integers for all bit work.

Two quantizer/encoder pairs are defined by the paper:

* scheme U ("backward", gradients): symmetric max-abs uniform quantization to k-bit
  signed integers, then a dense bit stream (paragraphs "Backward Quantizer", "Backward
  Encoder", "Backward Decoder", "Backward Dequantizer").
* scheme M ("forward", features): multi-bit quantization x ~ B alpha with B in {-1,+1},
  packed as bit planes along the batch dimension, plus a bias-correction mean
  (paragraphs "Forward Quantizer", "Forward Encoder", "Forward Decoder", "Forward
  Dequantizer"; eqs. (MBQ), (alpha solution), (alpha update), (biased error)).

Readings taken where the paper is silent are listed next to the code that takes them.

Parity pins (tests/test_oracle_*.py): worked encoder example (byte 54), size formulas
and the size table's payload column, beta's printed formula, the bit-width schedule's
printed averages, numpy.packbits as an independent packer, brute force over tiny
tensors, closed forms for k=1, normal-equation and mean-preservation invariants.
Unpinned by the paper (documented readings only): the order in which scheme U lays
codes into bytes for k other than 4 and 8, and which two elements share a byte at k=4
(flat neighbours in the packed layout, batch neighbours in LAYOUT_BATCH).
"""
from __future__ import annotations

import numpy as np

F32 = np.float32
SCHEME_UNIFORM = 0
SCHEME_MBQ = 1
# payload layouts: this library's packed forms (dense stream / bit planes); the paper's own
# backward layout (codes of 8/k consecutive batch entries share a byte); one byte per value,
# the paper's "w/o enc." rows
LAYOUT_PACKED = 0
LAYOUT_BATCH = 1
LAYOUT_UNENCODED = 2
TINY_RANGE = F32(2.0 ** -100)  # ranges below this are treated as an all-zero tensor


# --------------------------------------------------------------------------------------
# sizes, schedules (section "Transmission Data Comparison"; bit-width paragraphs)
# --------------------------------------------------------------------------------------
def packed_size(scheme, bits, n, m, channels=0, layout=LAYOUT_PACKED):
    """(header_bytes, payload_bytes) of one compressed tensor.

    Scheme M: alpha (k floats) + mean error (1 float); payload ceil(n/8)*m*k bytes
    (eq. (compress ratio) and the sentence before it).  Scheme U: one 32-bit scale (one
    per channel in the per-channel extension); payload ceil(n*m*k/8) bytes ("n/(8/k) x w
    x h x c" bytes in the paper, where 8/k is an integer).

    LAYOUT_BATCH (scheme U, k in 2, 4, 8): ceil(n/(8/k)) * m bytes, the paper's own count.
    LAYOUT_UNENCODED (the "w/o enc." rows of the size table): one byte per transmitted
    integer, i.e. n*m bytes for scheme U and n*m*k for scheme M.
    """
    n, m, k = int(n), int(m), int(bits)
    if scheme == SCHEME_MBQ:
        assert layout in (LAYOUT_PACKED, LAYOUT_UNENCODED)
        return 4 * (k + 1), (n * m * k if layout == LAYOUT_UNENCODED else ((n + 7) // 8) * m * k)
    c = max(int(channels), 1)
    if layout == LAYOUT_UNENCODED:
        return 4 * c, n * m
    if layout == LAYOUT_BATCH:
        assert 8 % k == 0
        per = 8 // k
        return 4 * c, ((n + per - 1) // per) * m
    return 4 * c, (n * m * k + 7) // 8


def compression_ratio_forward(n, m, k):
    """c_f of eq. (compress ratio): 32 n m / (ceil(n/8) m k 8 + 32 (k+1))."""
    return (n * m * 32) / (((n + 7) // 8) * m * k * 8 + 32 * (k + 1))


def bits_schedule(direction, lr_changes):
    """Adaptive bit width.  Forward: starts at 2, +1 per learning-rate change, at most 4
    (paragraph after eq. (biased error)).  Backward: 8 until the learning rate first
    changes, then 4 (paragraph after the stochastic-rounding equation)."""
    if direction == 0:
        return min(2 + int(lr_changes), 4)
    return 8 if int(lr_changes) == 0 else 4


def beta(t):
    """beta = min(0.9, (1+t)/(10+t)) (text after eq. (alpha update))."""
    return min(0.9, (1.0 + t) / (10.0 + t))


# --------------------------------------------------------------------------------------
# storage formats
# --------------------------------------------------------------------------------------
def widen_bf16(bits16):
    """bfloat16 bit patterns -> the float32 values they denote (exact)."""
    return (np.asarray(bits16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(F32)


def narrow_bf16(x32):
    """float32 -> bfloat16 bit patterns, round to nearest even (finite inputs)."""
    b = np.ascontiguousarray(x32, dtype=F32).view(np.uint32)
    return ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def _as_f32(x, in_bf16):
    return widen_bf16(x).reshape(-1) if in_bf16 else np.ascontiguousarray(x, dtype=F32).reshape(-1)


# --------------------------------------------------------------------------------------
# counter-based uniform numbers for stochastic rounding
# --------------------------------------------------------------------------------------
def counter_uniform(seed, idx):
    """u in [0,1) on a 2^-24 grid for element index idx: the splitmix64 output function
    applied to seed + (idx+1)*golden-ratio increment; the top 24 bits are used."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed) + (np.asarray(idx, dtype=np.uint64) + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return (z >> np.uint64(40)).astype(F32) * F32(2.0 ** -24)


# --------------------------------------------------------------------------------------
# scheme U: backward quantizer / encoder / decoder / dequantizer
# --------------------------------------------------------------------------------------
def uniform_range(x, n, m, channels=0):
    """c = max|g| ("Backward Quantizer"), one value per range group.

    Per tensor (channels <= 1) as the paper has it; per channel (extension): the channel
    of flat element i is ((i mod m) // (m/C)), i.e. dimension 1 of an n x C x ... tensor.
    """
    C = max(int(channels), 1)
    a = np.abs(np.asarray(x, dtype=F32).reshape(int(n), C, int(m) // C))
    return a.max(axis=(0, 2)).astype(F32)


def uniform_scale(c, k):
    """s = c / (2^(k-1) - 1) ("Backward Quantizer") and its reciprocal r = (2^(k-1)-1)/c,
    each one float32 division.  A range below 2^-100 (all-zero tensor) gives s = r = 0."""
    L = F32(2 ** (k - 1) - 1)
    c = np.asarray(c, dtype=F32)
    ok = c >= TINY_RANGE
    safe = np.where(ok, c, F32(1.0)).astype(F32)
    s = np.where(ok, safe / L, F32(0.0)).astype(F32)
    r = np.where(ok, L / safe, F32(0.0)).astype(F32)
    return s, r


def _per_element(v, n, m):
    """Broadcast per-channel values v[C] to the flat n*m element order."""
    C = v.shape[0]
    return np.broadcast_to(v.reshape(1, C, 1), (int(n), C, int(m) // C)).reshape(-1)


def uniform_quantize(x, r, k, n, m, rounding=0, seed=0):
    """g_q: scale into [-2^(k-1), 2^(k-1)-1] and round ("Backward Quantizer").

    The scaling g/s is carried out as one float32 multiply by r.  rounding=0 is round
    half to even (the reproducible rule the graded bit streams use); rounding=1 is the
    paper's stochastic rule: floor(v) + 1 with probability v - floor(v), else floor(v),
    the uniform number for element i coming from counter_uniform(seed, i).
    """
    x = np.asarray(x, dtype=F32).reshape(-1)
    v = (x * _per_element(np.asarray(r, dtype=F32).reshape(-1), n, m)).astype(F32)
    if rounding == 0:
        q = np.rint(v)
    else:
        f = np.floor(v)
        pr = (v - f).astype(F32)
        u = counter_uniform(seed, np.arange(x.size, dtype=np.uint64))
        q = f + (u < pr).astype(F32)
    lo, hi = -(2 ** (k - 1)), 2 ** (k - 1) - 1
    return np.clip(q, lo, hi).astype(np.int32)


def uniform_codes(q, k):
    """Unsigned k-bit codes ("Backward Encoder"): k = 8 is sent as the two's-complement
    byte itself; otherwise 2^(k-1) is added (the paper's "+8" at k = 4)."""
    q = np.asarray(q, dtype=np.int64)
    if k == 8:
        return (q & 0xFF).astype(np.uint64)
    return (q + 2 ** (k - 1)).astype(np.uint64)


def pack_stream(u, k):
    """Dense bit stream of k-bit codes in flat order: code i occupies stream bits
    [ik, (i+1)k), most significant bit first, and stream bit b is bit 7-(b mod 8) of byte
    b // 8.  Eight codes are exactly k bytes, so the stream is built 8 codes at a time as
    one 8k-bit integer written out big-endian.  Unused bits of the last byte are 0."""
    u = np.asarray(u, dtype=np.uint64).reshape(-1)
    N = u.size
    G = (N + 7) // 8
    pad = np.zeros(G * 8, dtype=np.uint64)
    pad[:N] = u
    pad = pad.reshape(G, 8)
    val = np.zeros(G, dtype=np.uint64)
    for i in range(8):
        val |= pad[:, i] << np.uint64(k * (7 - i))
    out = np.empty((G, k), dtype=np.uint8)
    for b in range(k):
        out[:, b] = ((val >> np.uint64(8 * (k - 1 - b))) & np.uint64(0xFF)).astype(np.uint8)
    return out.reshape(-1)[: (N * k + 7) // 8].copy()


def unpack_stream(payload, k, N):
    """Inverse of pack_stream ("Backward Decoder": split each byte into its codes)."""
    G = (N + 7) // 8
    buf = np.zeros(G * k, dtype=np.uint64)
    p = np.asarray(payload, dtype=np.uint8).reshape(-1)[: (N * k + 7) // 8]
    buf[: p.size] = p
    buf = buf.reshape(G, k)
    val = np.zeros(G, dtype=np.uint64)
    for b in range(k):
        val |= buf[:, b] << np.uint64(8 * (k - 1 - b))
    codes = np.empty((G, 8), dtype=np.uint64)
    for i in range(8):
        codes[:, i] = (val >> np.uint64(k * (7 - i))) & np.uint64(2 ** k - 1)
    return codes.reshape(-1)[:N].copy()


def pack_batch(u, k, n, m):
    """The paper's own backward layout ("Backward Encoder": the shifted codes of two
    tensors along the first dimension are combined into one at k = 4, so that g_c has
    n/2 x w x h x c bytes): byte (g, j) holds the codes of batch entries g*(8/k) ..
    g*(8/k) + 8/k - 1 of column j, first entry in the most significant bits, like the
    forward encoder's worked example.  k must divide 8; entries beyond n contribute 0
    bits.  Which entries pair up is a reading: the paper does not say."""
    n, m = int(n), int(m)
    assert 8 % k == 0
    per = 8 // k
    G = (n + per - 1) // per
    pad = np.zeros((G * per, m), dtype=np.uint64)
    pad[:n] = np.asarray(u, dtype=np.uint64).reshape(n, m)
    pad = pad.reshape(G, per, m)
    out = np.zeros((G, m), dtype=np.uint64)
    for i in range(per):
        out |= pad[:, i, :] << np.uint64(k * (per - 1 - i))
    return out.astype(np.uint8).reshape(-1)


def unpack_batch(payload, k, n, m):
    """Inverse of pack_batch."""
    n, m = int(n), int(m)
    per = 8 // k
    G = (n + per - 1) // per
    pl = np.asarray(payload, dtype=np.uint8).reshape(G, m).astype(np.uint64)
    u = np.zeros((G, per, m), dtype=np.uint64)
    for i in range(per):
        u[:, i, :] = (pl >> np.uint64(k * (per - 1 - i))) & np.uint64(2 ** k - 1)
    return u.reshape(G * per, m)[:n].reshape(-1)


def uniform_compress(x, k, n, m, channels=0, in_bf16=False, rounding=0, seed=0, layout=LAYOUT_PACKED):
    """(g, k) -> (s, g_c): header bytes (little-endian float32 scale per range group) and
    payload bytes."""
    assert 2 <= k <= 8
    x32 = _as_f32(x, in_bf16)
    c = uniform_range(x32, n, m, channels)
    s, r = uniform_scale(c, k)
    q = uniform_quantize(x32, r, k, n, m, rounding, seed)
    if layout == LAYOUT_UNENCODED:  # g_q itself, one two's-complement byte per value
        payload = (np.asarray(q, dtype=np.int64) & 0xFF).astype(np.uint8)
    elif layout == LAYOUT_BATCH:
        payload = pack_batch(uniform_codes(q, k), k, n, m)
    else:
        payload = pack_stream(uniform_codes(q, k), k)
    return s.astype("<f4").tobytes(), payload


def uniform_decode(payload, k, N, layout=LAYOUT_PACKED, n=None, m=None):
    """g_q from g_c ("Backward Decoder": subtract the offset; skipped at k = 8)."""
    if layout == LAYOUT_UNENCODED:
        return np.asarray(payload, dtype=np.uint8).reshape(-1)[:N].view(np.int8).astype(np.int32)
    if layout == LAYOUT_BATCH:
        u = unpack_batch(payload, k, n, m).astype(np.int64)
    else:
        u = unpack_stream(payload, k, N).astype(np.int64)
    if k == 8:
        return np.where(u >= 128, u - 256, u).astype(np.int32)
    return (u - 2 ** (k - 1)).astype(np.int32)


def uniform_decompress(header, payload, k, n, m, channels=0, out_bf16=False, layout=LAYOUT_PACKED):
    """g_hat = g_q * s ("Backward Dequantizer"), one float32 multiply per element."""
    N = int(n) * int(m)
    s = np.frombuffer(bytes(header), dtype="<f4").astype(F32)
    q = uniform_decode(payload, k, N, layout, n, m)
    xh = (q.astype(F32) * _per_element(s, n, m)).astype(F32)
    return narrow_bf16(xh) if out_bf16 else xh


# --------------------------------------------------------------------------------------
# scheme M: forward quantizer / encoder / decoder / dequantizer
# --------------------------------------------------------------------------------------
def mbq_levels(alpha):
    """The set P of all 2^k values sum_j (+-alpha_j) ("Forward Quantizer"), sorted.

    Pattern p has bit j set when basis j is +1 (the encoder's -1 -> 0 replacement).  Each
    level is a float32 sum taken in the order j = 0..k-1 starting from 0.  Returns
    (levels ascending, pattern at each sorted position, thresholds); equal levels are
    ordered by pattern.  Threshold i is the float32 midpoint 0.5*(lv_i + lv_{i+1}).
    """
    alpha = np.asarray(alpha, dtype=F32).reshape(-1)
    k = alpha.size
    P = 1 << k
    lv = np.zeros(P, dtype=F32)
    for j in range(k):
        bit = ((np.arange(P) >> j) & 1).astype(bool)
        lv = (lv + np.where(bit, alpha[j], -alpha[j]).astype(F32)).astype(F32)
    order = np.lexsort((np.arange(P), lv))  # primary key lv, ties by pattern
    lv_sorted = lv[order]
    tau = (F32(0.5) * (lv_sorted[:-1] + lv_sorted[1:]).astype(F32)).astype(F32)
    return lv_sorted, order.astype(np.int64), tau


def mbq_assign(x, alpha):
    """B^t: for every element the nearest value of P^(t-1) ("Forward Quantizer").

    Position in the sorted level list = number of thresholds strictly below x, so a value
    exactly on a midpoint takes the lower level and NaN takes level 0.  Returns the k-bit
    sign pattern of every element."""
    x = np.asarray(x, dtype=F32).reshape(-1)
    _, order, tau = mbq_levels(alpha)
    idx = np.zeros(x.size, dtype=np.int64)
    for t in tau:
        idx += (x > t)
    return order[idx]


def mbq_pack(code, k, n, m):
    """B_c ("Forward Encoder"): -1 -> 0, then eight consecutive entries along the batch
    dimension become one byte, first entry in the most significant bit (the worked
    example 0,0,1,1,0,1,1,0 -> 54).  Layout ceil(n/8) x m x k, k innermost; batch rows
    beyond n contribute 0 bits."""
    n, m = int(n), int(m)
    G = (n + 7) // 8
    code = np.asarray(code, dtype=np.int64).reshape(n, m)
    out = np.zeros((G, m, k), dtype=np.uint8)
    for p in range(k):
        bits = np.zeros((G * 8, m), dtype=np.uint8)
        bits[:n] = (code >> p) & 1
        bits = bits.reshape(G, 8, m)
        for i in range(8):
            out[:, :, p] |= (bits[:, i, :] << np.uint8(7 - i)).astype(np.uint8)
    return out.reshape(-1)


def mbq_unpack(payload, k, n, m):
    """"Forward Decoder": eight 1-bit values out of every byte; returns sign patterns."""
    n, m = int(n), int(m)
    G = (n + 7) // 8
    pl = np.asarray(payload, dtype=np.uint8).reshape(G, m, k)
    code = np.zeros((G * 8, m), dtype=np.int64)
    for p in range(k):
        for i in range(8):
            code[i::8] |= (((pl[:, :, p] >> np.uint8(7 - i)) & 1).astype(np.int64)) << p
    return code[:n].reshape(-1)


def mbq_pack_unencoded(code, k):
    """The "w/o enc." form of B: every binary base as an 8-bit integer of its own, +1 or
    -1, element-major with the k bases innermost (n*m*k bytes)."""
    code = np.asarray(code, dtype=np.int64).reshape(-1)
    out = np.empty((code.size, k), dtype=np.int8)
    for p in range(k):
        out[:, p] = np.where((code >> p) & 1, 1, -1)
    return out.reshape(-1).view(np.uint8)


def mbq_unpack_unencoded(payload, k, N):
    """Sign patterns back from the +-1 bytes."""
    b = np.asarray(payload, dtype=np.uint8).reshape(-1)[: N * k].view(np.int8).reshape(N, k)
    code = np.zeros(N, dtype=np.int64)
    for p in range(k):
        code |= (b[:, p] > 0).astype(np.int64) << p
    return code


def mbq_stats(x, code, k):
    """float64 sums needed by eq. (alpha solution) and the bias term: G = B^T B,
    h = B^T x, S_b = 1^T B, S_x = 1^T x, with b = +1 where the pattern bit is 1."""
    x64 = np.asarray(x, dtype=np.float64).reshape(-1)
    code = np.asarray(code, dtype=np.int64).reshape(-1)
    B = [(2.0 * ((code >> p) & 1) - 1.0) for p in range(k)]
    G = np.empty((k, k), dtype=np.float64)
    h = np.empty(k, dtype=np.float64)
    Sb = np.empty(k, dtype=np.float64)
    for p in range(k):
        h[p] = np.sum(B[p] * x64)
        Sb[p] = np.sum(B[p])
        for q in range(p, k):
            G[p, q] = G[q, p] = np.sum(B[p] * B[q])
    return G, h, Sb, float(np.sum(x64))


def solve_spd_pivot(G, h, n_elems):
    """Gaussian elimination with partial pivoting in float64.  Returns None when a pivot
    is below 1e-9 * N (B^T B singular: constant or duplicated planes)."""
    k = h.size
    A = np.array(G, dtype=np.float64)
    b = np.array(h, dtype=np.float64)
    for col in range(k):
        piv = col + int(np.argmax(np.abs(A[col:, col])))
        if abs(A[piv, col]) < 1e-9 * n_elems:
            return None
        if piv != col:
            A[[col, piv]] = A[[piv, col]]
            b[[col, piv]] = b[[piv, col]]
        for row in range(col + 1, k):
            f = A[row, col] / A[col, col]
            A[row, col:] -= f * A[col, col:]
            b[row] -= f * b[col]
    sol = np.zeros(k, dtype=np.float64)
    for row in range(k - 1, -1, -1):
        sol[row] = (b[row] - np.dot(A[row, row + 1:], sol[row + 1:])) / A[row, row]
    return sol


def mbq_alpha_update(alpha_prev, G, h, t, n_elems):
    """eq. (alpha solution): alpha_cur = (B^T B)^-1 B^T x; eq. (alpha update):
    alpha_t = beta alpha_(t-1) + (1-beta) alpha_cur, rounded to float32 at the end.  A
    singular B^T B keeps alpha_(t-1) as alpha_cur."""
    a_prev = np.asarray(alpha_prev, dtype=F32).astype(np.float64)
    cur = solve_spd_pivot(G, h, n_elems)
    if cur is None:
        cur = a_prev
    b = beta(t)
    return (b * a_prev + (1.0 - b) * cur).astype(F32), cur


def mbq_mean_error(alpha_t, Sb, Sx, n_elems):
    """m_q = E[n_q] = mean(B alpha_t - x) (eq. (biased error)), float64 then float32."""
    a = np.asarray(alpha_t, dtype=F32).astype(np.float64)
    return F32((np.dot(a, Sb) - Sx) / n_elems)


def mbq_compress(x, k, n, m, alpha_prev, t, in_bf16=False, layout=LAYOUT_PACKED):
    """(x, k, alpha_(t-1)) -> header [alpha_t (k floats), m_q] and payload B_c."""
    x32 = _as_f32(x, in_bf16)
    N = int(n) * int(m)
    code = mbq_assign(x32, alpha_prev)
    payload = mbq_pack_unencoded(code, k) if layout == LAYOUT_UNENCODED else mbq_pack(code, k, n, m)
    G, h, Sb, Sx = mbq_stats(x32, code, k)
    alpha_t, _ = mbq_alpha_update(alpha_prev, G, h, t, N)
    mq = mbq_mean_error(alpha_t, Sb, Sx, N)
    header = np.concatenate([alpha_t, np.array([mq], dtype=F32)]).astype("<f4").tobytes()
    return header, payload


def mbq_decompress(header, payload, k, n, m, out_bf16=False, layout=LAYOUT_PACKED):
    """"Forward Dequantizer": x_hat = B alpha - m_q.  The product is the float32 sum of
    +-alpha_p in the order p = 0..k-1 starting from 0, then one float32 subtraction."""
    hdr = np.frombuffer(bytes(header), dtype="<f4").astype(F32)
    alpha, mq = hdr[:k], hdr[k]
    if layout == LAYOUT_UNENCODED:
        code = mbq_unpack_unencoded(payload, k, int(n) * int(m))
    else:
        code = mbq_unpack(payload, k, n, m)
    acc = np.zeros(code.size, dtype=F32)
    for p in range(k):
        acc = (acc + np.where((code >> p) & 1, alpha[p], -alpha[p]).astype(F32)).astype(F32)
    xh = (acc - mq).astype(F32)
    return narrow_bf16(xh) if out_bf16 else xh


def mbq_residue_init(x, k):
    """Residue-based initialisation of (B^0, alpha^0) at batch 0 of an epoch ("Forward
    Quantizer"): greedily, for the current residue rho, the best single basis is
    b = sign(rho) (sign(0) = +1) with alpha = mean|rho|; the next residue is rho - alpha b.
    Returns (alpha^0 float32[k], sign patterns of B^0)."""
    rho = np.asarray(x, dtype=F32).reshape(-1).astype(np.float64)
    alpha = np.zeros(k, dtype=F32)
    code = np.zeros(rho.size, dtype=np.int64)
    for j in range(k):
        a = F32(np.mean(np.abs(rho)))
        pos = rho >= 0.0
        code |= pos.astype(np.int64) << j
        alpha[j] = a
        rho = rho - np.where(pos, np.float64(a), -np.float64(a))
    return alpha, code


def mbq_compress_first(x, k, n, m, in_bf16=False):
    """Batch 0 of an epoch ("Forward Quantizer": B^0 and alpha^0 come from the residue method and
    are what is transmitted; the search among the previous batch's levels starts at batch 1).
    Header [alpha^0 (k floats), m_q] with m_q = mean(B^0 alpha^0 - x) (eq. (biased error)),
    payload = the bit planes of B^0 ("Forward Encoder")."""
    x32 = _as_f32(x, in_bf16)
    N = int(n) * int(m)
    alpha0, code = mbq_residue_init(x32, k)
    _, _, Sb, Sx = mbq_stats(x32, code, k)
    mq = mbq_mean_error(alpha0, Sb, Sx, N)
    header = np.concatenate([alpha0, np.array([mq], dtype=F32)]).astype("<f4").tobytes()
    return header, mbq_pack(code, k, n, m)


def mbq_residue_signs(x, alpha):
    """The sign patterns of the residue method for GIVEN coefficients: b_j = sign(rho_j)
    (sign(0) = +1), rho_0 = x, rho_(j+1) = rho_j - alpha_j b_j, in float64 like
    mbq_residue_init.  (With alpha = mbq_residue_init's own alpha^0 this is its B^0.)"""
    alpha = np.asarray(alpha, dtype=F32).reshape(-1)
    rho = np.asarray(x, dtype=F32).reshape(-1).astype(np.float64)
    code = np.zeros(rho.size, dtype=np.int64)
    for j in range(alpha.size):
        pos = rho >= 0.0
        code |= pos.astype(np.int64) << j
        rho = rho - np.where(pos, np.float64(alpha[j]), -np.float64(alpha[j]))
    return code
