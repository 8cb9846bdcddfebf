"""CPU oracle for decode-step attention over a quantized, bit-packed KV cache.

TEST INFRASTRUCTURE ONLY.  This is the plain, slow definition the HIP kernels are
checked against.  Only tests, the smoke check and the benchmark's cpu_baseline leg
may import it; it shares no code with the HIP path and never calls it.

What it follows (BitDecoding, arxiv 2503.18773):
  * Fig. 2 caption:  Out = softmax(Q . D(K')^T) . D(V'),  D = dequantization.
  * Sec. III-A(2) / Sec. IV-B(1): the cache is split into a low-bit packed part of
    N_p = L - (L mod N_r) tokens and a half-precision residual of L mod N_r tokens;
    a decode step appends to the residual and quantizes it when it reaches N_r.
  * Sec. IV-B(1), Sec. IV-C(1): K is quantized channel-wise (one scale/zero per channel
    over the N_r tokens of a block, K_p shape (T_n/group, d)); V "tensor-wise" (one
    scale/zero per token over a group of channels, V_p shape (T_n, d/group)).
  * Sec. IV-B(2): scale and zero-point are kept as a half2.
  * Sec. IV-A: query heads h*g_q .. h*g_q+g_q-1 share KV head h.
  * Sec. IV-D(2): the MXFP4 variant (e2m1 elements, one e8m0 scale per 32 elements).
  * Alg. 1 is the online form of the softmax; the oracle evaluates the two-pass
    definition in float64 instead (they agree up to rounding order).

The paper never writes the quantizer out; the reading used here (asymmetric min/max,
zero = min, scale = (max-min)/(2^bits-1) rounded to fp16, round-half-even codes) is
listed with the other readings in the design notes.  Pins: tests/test_oracle_*.py.
Everything here is pinned there; nothing is "parity unpinned" except agreement with
the authors' own bytes, for which the paper prints no example.
"""
from __future__ import annotations

import numpy as np

BLOCK = 128          # N_r: residual block == quantization group along tokens (K) / channels (V)
MX_GROUP = 32        # elements per MX block
E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])   # magnitudes of codes 0..7


# --------------------------------------------------------------------------- int4 / int2

def qmax_of(bits: int) -> int:
    assert bits in (4, 2)
    return (1 << bits) - 1


def quant_params(mn: np.ndarray, mx: np.ndarray, bits: int):
    """Scale and zero-point of a group from its fp16 minimum and maximum.

    zero = min (a -0 minimum is stored as +0); scale = fp16((f32(max) - f32(min)) / qmax),
    one fp32 subtraction, one fp32 division, one round-to-nearest-even to fp16."""
    mn = np.asarray(mn, dtype=np.float16)
    mx = np.asarray(mx, dtype=np.float16)
    zero = (mn + np.float16(0.0)).astype(np.float16)            # -0 + +0 == +0
    diff = mx.astype(np.float32) - mn.astype(np.float32)
    scale = (diff / np.float32(qmax_of(bits))).astype(np.float16)
    return scale, zero


def quant_codes(x: np.ndarray, scale: np.ndarray, zero: np.ndarray, bits: int) -> np.ndarray:
    """codes = clamp(rint((f32(x) - f32(zero)) / f32(scale)), 0, qmax); 0 where scale == 0.
    x fp16; scale/zero broadcastable to x.  fp32 IEEE subtract and divide, ties to even."""
    x32 = np.asarray(x, dtype=np.float16).astype(np.float32)
    s32 = np.broadcast_to(np.asarray(scale, dtype=np.float16).astype(np.float32), x32.shape)
    z32 = np.broadcast_to(np.asarray(zero, dtype=np.float16).astype(np.float32), x32.shape)
    live = s32 != 0
    safe = np.where(live, s32, np.float32(1.0))
    q = np.rint((x32 - z32) / safe)
    q = np.clip(q, 0, qmax_of(bits))
    return np.where(live, q, 0).astype(np.uint8)


def quantize_k_block(kblk: np.ndarray, bits: int):
    """K block [128 tokens, D] fp16 -> codes [128, D], scale [D], zero [D] (channel-wise:
    statistics run over the 128 tokens of the block)."""
    assert kblk.shape[0] == BLOCK and kblk.dtype == np.float16
    scale, zero = quant_params(kblk.min(axis=0), kblk.max(axis=0), bits)
    return quant_codes(kblk, scale[None, :], zero[None, :], bits), scale, zero


def quantize_k_block_per_token(kblk: np.ndarray, bits: int):
    """The KT setting (Sec. IV-C(1), Sec. V: K quantized "tensor-wise" like V instead of
    channel-wise): K block [128 tokens, D=128] fp16 -> codes [128, D], scale [128], zero [128],
    statistics over the 128 channels of each token."""
    assert kblk.shape == (BLOCK, BLOCK) and kblk.dtype == np.float16
    scale, zero = quant_params(kblk.min(axis=1), kblk.max(axis=1), bits)
    return quant_codes(kblk, scale[:, None], zero[:, None], bits), scale, zero


def quantize_v_block(vblk: np.ndarray, bits: int):
    """V block [128 tokens, D=128] fp16 -> codes [128, D], scale [128], zero [128]
    (per token: statistics run over the group of 128 channels, i.e. the whole head)."""
    assert vblk.shape == (BLOCK, BLOCK) and vblk.dtype == np.float16
    scale, zero = quant_params(vblk.min(axis=1), vblk.max(axis=1), bits)
    return quant_codes(vblk, scale[:, None], zero[:, None], bits), scale, zero


def quantize_k_block_grouped(kblk: np.ndarray, bits: int, group: int):
    """Channel-wise K with a quantization group of `group` tokens (Sec. IV-C(1): K_p has shape
    (T_n / group_size, d)): K block [128 tokens, D] fp16 -> codes [128, D], scale and zero
    [128 / group, D]; the statistics of channel c, group j run over tokens j*group .. (j+1)*group-1."""
    assert kblk.shape[0] == BLOCK and kblk.dtype == np.float16 and BLOCK % group == 0
    ng = BLOCK // group
    codes = np.empty(kblk.shape, np.uint8)
    scale = np.empty((ng, kblk.shape[1]), np.float16)
    zero = np.empty((ng, kblk.shape[1]), np.float16)
    for j in range(ng):
        sub = kblk[j * group:(j + 1) * group]
        scale[j], zero[j] = quant_params(sub.min(axis=0), sub.max(axis=0), bits)
        codes[j * group:(j + 1) * group] = quant_codes(sub, scale[j][None, :], zero[j][None, :], bits)
    return codes, scale, zero


def quantize_v_block_grouped(vblk: np.ndarray, bits: int, group: int):
    """Per-token V with a quantization group of `group` channels (V_p has shape
    (T_n, d / group_size)): V block [128 tokens, D] fp16 -> codes [128, D], scale and zero
    [128, D / group]; the statistics of token t, group g run over channels g*group .. (g+1)*group-1."""
    assert vblk.shape[0] == BLOCK and vblk.dtype == np.float16 and vblk.shape[1] % group == 0
    ng = vblk.shape[1] // group
    codes = np.empty(vblk.shape, np.uint8)
    scale = np.empty((BLOCK, ng), np.float16)
    zero = np.empty((BLOCK, ng), np.float16)
    for g in range(ng):
        sub = vblk[:, g * group:(g + 1) * group]
        scale[:, g], zero[:, g] = quant_params(sub.min(axis=1), sub.max(axis=1), bits)
        codes[:, g * group:(g + 1) * group] = quant_codes(sub, scale[:, g][:, None], zero[:, g][:, None], bits)
    return codes, scale, zero


def quantize_k_block_per_token_grouped(kblk: np.ndarray, bits: int, group: int):
    """The KT setting with a quantization group (Sec. IV-C(1): tensor-wise parameters have shape
    (T_n, d / group_size)): K block [128 tokens, D] fp16 -> codes [128, D], scale and zero [128, D / group];
    the statistics of token t, group g run over channels g*group .. (g+1)*group-1 -- what
    quantize_v_block_grouped does to V, applied to K."""
    return quantize_v_block_grouped(kblk, bits, group)


def pack_words(codes: np.ndarray, bits: int) -> np.ndarray:
    """Pack the last axis: 32/bits codes per little-endian uint32, code n of a word at
    bit offset bits*n."""
    cpw = 32 // bits
    c = codes.astype(np.uint32).reshape(codes.shape[:-1] + (codes.shape[-1] // cpw, cpw))
    w = np.zeros(c.shape[:-1], dtype=np.uint32)
    for n in range(cpw):
        w |= c[..., n] << np.uint32(bits * n)
    return w


def unpack_words(words: np.ndarray, bits: int) -> np.ndarray:
    cpw = 32 // bits
    mask = np.uint32((1 << bits) - 1)
    out = np.stack([(words >> np.uint32(bits * n)) & mask for n in range(cpw)], axis=-1)
    return out.reshape(words.shape[:-1] + (words.shape[-1] * cpw,)).astype(np.uint8)


def pack_half2(scale: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """half2 (scale, zero) as one uint32: scale in the low 16 bits, zero in the high 16."""
    s = np.asarray(scale, dtype=np.float16).view(np.uint16).astype(np.uint32)
    z = np.asarray(zero, dtype=np.float16).view(np.uint16).astype(np.uint32)
    return s | (z << np.uint32(16))


def unpack_half2(p: np.ndarray):
    p = np.asarray(p, dtype=np.uint32)
    s = (p & np.uint32(0xFFFF)).astype(np.uint16).view(np.float16)
    z = (p >> np.uint32(16)).astype(np.uint16).view(np.float16)
    return s, z


class IntCache:
    """Packed int4/int2 cache + fp16 residual of one (batch, kv_head) grid, in the memory
    layout the library documents:

      k_codes  uint32 [B, H, NBcap, 128 tokens, D*bits/32]   words run along channels
      v_codes  uint32 [B, H, NBcap, D channels, 128*bits/32] words run along the block's tokens
      k_params uint32 [B, H, NBcap, D]        half2 (scale, zero) per channel
                                              (k_per_token: per token of the block, [.., 128])
      v_params uint32 [B, H, NBcap, 128]      half2 (scale, zero) per token
      k_res, v_res fp16 [B, H, 128, D]        residual tokens, slots [0, res_len) valid

    group (32 or 64; 128 is the above): the quantization group is smaller than the residual block.
    K statistics run over `group` tokens per channel, V statistics over `group` channels per
    token; the codes stay where they are and the parameter arrays grow to
      k_params uint32 [B, H, NBcap, 128/group, D]      v_params uint32 [B, H, NBcap, 128, D/group]
    (k_per_token with a group: K statistics over `group` channels per token like V's,
      k_params uint32 [B, H, NBcap, 128, D/group])
    """

    def __init__(self, batch: int, n_kv_heads: int, bits: int, capacity: int, head_dim: int = 128,
                 k_per_token: bool = False, group: int = BLOCK):
        assert capacity % BLOCK == 0 and head_dim == 128
        assert group in (32, 64, BLOCK)
        self.B, self.H, self.D, self.bits, self.capacity = batch, n_kv_heads, head_dim, bits, capacity
        self.k_per_token = k_per_token          # KT: K statistics per token instead of per channel
        self.group = group
        nbc = capacity // BLOCK
        wpr = head_dim * bits // 32
        self.k_codes = np.zeros((batch, n_kv_heads, nbc, BLOCK, wpr), np.uint32)
        self.v_codes = np.zeros((batch, n_kv_heads, nbc, head_dim, BLOCK * bits // 32), np.uint32)
        if group == BLOCK:
            self.k_params = np.zeros((batch, n_kv_heads, nbc, head_dim), np.uint32)
            self.v_params = np.zeros((batch, n_kv_heads, nbc, BLOCK), np.uint32)
        else:
            kshape = (BLOCK, head_dim // group) if k_per_token else (BLOCK // group, head_dim)
            self.k_params = np.zeros((batch, n_kv_heads, nbc) + kshape, np.uint32)
            self.v_params = np.zeros((batch, n_kv_heads, nbc, BLOCK, head_dim // group), np.uint32)
        self.k_res = np.zeros((batch, n_kv_heads, BLOCK, head_dim), np.float16)
        self.v_res = np.zeros((batch, n_kv_heads, BLOCK, head_dim), np.float16)
        self.packed_len = 0
        self.res_len = 0

    # -- Sec. IV-B(1): fused quantize + pack of one full block
    def _store_block(self, nb: int, kblk: np.ndarray, vblk: np.ndarray):
        for b in range(self.B):
            for h in range(self.H):
                if self.group != BLOCK:
                    quant_kg = quantize_k_block_per_token_grouped if self.k_per_token else quantize_k_block_grouped
                    kc, ks, kz = quant_kg(kblk[b, h], self.bits, self.group)
                    vc, vs, vz = quantize_v_block_grouped(vblk[b, h], self.bits, self.group)
                else:
                    quant_k = quantize_k_block_per_token if self.k_per_token else quantize_k_block
                    kc, ks, kz = quant_k(kblk[b, h], self.bits)
                    vc, vs, vz = quantize_v_block(vblk[b, h], self.bits)
                self.k_codes[b, h, nb] = pack_words(kc, self.bits)              # [token][channel words]
                self.v_codes[b, h, nb] = pack_words(vc.T.copy(), self.bits)     # [channel][token words]
                self.k_params[b, h, nb] = pack_half2(ks, kz)
                self.v_params[b, h, nb] = pack_half2(vs, vz)

    def quant_pack_kv(self, K: np.ndarray, V: np.ndarray):
        """Prefill: the first L - (L mod 128) tokens are quantized, the rest kept in fp16."""
        L = K.shape[2]
        assert K.shape == V.shape == (self.B, self.H, L, self.D) and K.dtype == np.float16
        nb, r = divmod(L, BLOCK)
        assert nb * BLOCK <= self.capacity
        for n in range(nb):
            self._store_block(n, K[:, :, n * BLOCK:(n + 1) * BLOCK], V[:, :, n * BLOCK:(n + 1) * BLOCK])
        self.k_res[:, :, :r] = K[:, :, nb * BLOCK:]
        self.v_res[:, :, :r] = V[:, :, nb * BLOCK:]
        self.packed_len, self.res_len = nb * BLOCK, r

    def append_kv(self, k_new: np.ndarray, v_new: np.ndarray, flush: bool = True):
        """Decode step: the new token goes to the residual; a residual that reaches 128
        tokens is quantized into the next packed block at once.

        flush=False is the order of the paper's Residual Kernel (Sec. III-A(1), Sec. IV-B(1): it attends
        the half-precision residual first and quantizes it afterwards, once it holds N_r tokens):
        the token is appended, a full residual (res_len == 128) stays in fp16 for the attention of this
        step, and flush_if_full() after that attention packs it."""
        assert k_new.shape == v_new.shape == (self.B, self.H, self.D)
        assert self.res_len < BLOCK, "a full residual must be flushed before the next append"
        if self.res_len == BLOCK - 1 and self.packed_len + BLOCK > self.capacity:
            raise OverflowError("cache capacity exceeded")
        self.k_res[:, :, self.res_len] = k_new
        self.v_res[:, :, self.res_len] = v_new
        self.res_len += 1
        if flush:
            self.flush_if_full()

    def flush_if_full(self):
        """Sec. IV-B(1): a residual of N_r = 128 tokens becomes the next packed block."""
        if self.res_len == BLOCK:
            self._store_block(self.packed_len // BLOCK, self.k_res, self.v_res)
            self.packed_len += BLOCK
            self.res_len = 0

    # -- D(.) of Fig. 2: x_hat = code * scale + zero, in float64
    def dequant(self, b: int, h: int):
        """K_hat, V_hat [L, D] float64 of one (batch, kv_head): packed tokens dequantized,
        residual tokens as stored."""
        nb = self.packed_len // BLOCK
        Kh = np.empty((self.packed_len + self.res_len, self.D), np.float64)
        Vh = np.empty_like(Kh)
        for n in range(nb):
            kc = unpack_words(self.k_codes[b, h, n], self.bits).astype(np.float64)      # [t][c]
            vc = unpack_words(self.v_codes[b, h, n], self.bits).astype(np.float64).T    # [c][t] -> [t][c]
            ks, kz = unpack_half2(self.k_params[b, h, n])
            vs, vz = unpack_half2(self.v_params[b, h, n])
            if self.group != BLOCK:      # ks, kz [128/group, D] (k_per_token: [128, D/group]); vs, vz [128, D/group]
                ks, kz, vs, vz = (x.astype(np.float64) for x in (ks, kz, vs, vz))
                kax = 1 if self.k_per_token else 0
                Kh[n * BLOCK:(n + 1) * BLOCK] = kc * np.repeat(ks, self.group, axis=kax) + np.repeat(kz, self.group, axis=kax)
                Vh[n * BLOCK:(n + 1) * BLOCK] = vc * np.repeat(vs, self.group, axis=1) + np.repeat(vz, self.group, axis=1)
                continue
            if self.k_per_token:
                Kh[n * BLOCK:(n + 1) * BLOCK] = kc * ks.astype(np.float64)[:, None] + kz.astype(np.float64)[:, None]
            else:
                Kh[n * BLOCK:(n + 1) * BLOCK] = kc * ks.astype(np.float64)[None, :] + kz.astype(np.float64)[None, :]
            Vh[n * BLOCK:(n + 1) * BLOCK] = vc * vs.astype(np.float64)[:, None] + vz.astype(np.float64)[:, None]
        Kh[self.packed_len:] = self.k_res[b, h, :self.res_len].astype(np.float64)
        Vh[self.packed_len:] = self.v_res[b, h, :self.res_len].astype(np.float64)
        return Kh, Vh


class PagedIntCache:
    """The page-managed cache of the paper's "Page" setting (Sec. V-A, Sec. V-B: kernels run on
    both a contiguous and a paged KV cache).  The paper names the setting without describing a
    layout; the reading used here: a page is one 128-token quantization block (so that a block's
    channel-wise K statistics stay inside one page), the packed blocks of all sequences live
    in one pool, block n of sequence b is page block_table[b, n], every sequence has its own
    length, and the fp16 residual stays per sequence.

      k_codes  uint32 [P, H, 128 tokens, D*bits/32]    v_codes  uint32 [P, H, D, 128*bits/32]
      k_params uint32 [P, H, D]                        v_params uint32 [P, H, 128]
      k_res, v_res fp16 [B, H, 128, D]
      block_table int32 [B, max_pages]                 seq_lens int32 [B]

    Paging is a pure relocation: every block holds exactly the bytes IntCache would hold
    (with group = 64 or 32: k_params uint32 [P, H, 128/group, D], v_params uint32 [P, H, 128, D/group];
    k_per_token with a group: k_params uint32 [P, H, 128, D/group]).
    """

    def __init__(self, batch: int, n_kv_heads: int, bits: int, num_pages: int, max_pages: int,
                 block_table: np.ndarray, head_dim: int = 128, k_per_token: bool = False, group: int = BLOCK):
        assert head_dim == 128 and block_table.shape == (batch, max_pages)
        assert group in (32, 64, BLOCK)
        self.B, self.H, self.D, self.bits = batch, n_kv_heads, head_dim, bits
        self.k_per_token = k_per_token
        self.group = group
        self.P, self.max_pages = num_pages, max_pages
        self.k_codes = np.zeros((num_pages, n_kv_heads, BLOCK, head_dim * bits // 32), np.uint32)
        self.v_codes = np.zeros((num_pages, n_kv_heads, head_dim, BLOCK * bits // 32), np.uint32)
        if group == BLOCK:
            self.k_params = np.zeros((num_pages, n_kv_heads, head_dim), np.uint32)
            self.v_params = np.zeros((num_pages, n_kv_heads, BLOCK), np.uint32)
        else:
            kshape = (BLOCK, head_dim // group) if k_per_token else (BLOCK // group, head_dim)
            self.k_params = np.zeros((num_pages, n_kv_heads) + kshape, np.uint32)
            self.v_params = np.zeros((num_pages, n_kv_heads, BLOCK, head_dim // group), np.uint32)
        self.k_res = np.zeros((batch, n_kv_heads, BLOCK, head_dim), np.float16)
        self.v_res = np.zeros((batch, n_kv_heads, BLOCK, head_dim), np.float16)
        self.block_table = block_table.astype(np.int32).copy()
        self.seq_lens = np.zeros(batch, np.int32)
        # lazy flush (append_kv(flush=False)): sequences whose residual holds 128 tokens that are not packed yet
        self.unflushed = np.zeros(batch, bool)

    def _page_of(self, b: int, n: int) -> int:
        if n >= self.max_pages:
            raise OverflowError("block table row is full")
        p = int(self.block_table[b, n])
        if not 0 <= p < self.P:
            raise IndexError("block table entry outside the pool")
        return p

    def _store_block(self, b: int, n: int, kblk: np.ndarray, vblk: np.ndarray):
        p = self._page_of(b, n)
        quant_k = quantize_k_block_per_token if self.k_per_token else quantize_k_block
        for h in range(self.H):
            if self.group != BLOCK:
                quant_kg = quantize_k_block_per_token_grouped if self.k_per_token else quantize_k_block_grouped
                kc, ks, kz = quant_kg(kblk[h], self.bits, self.group)
                vc, vs, vz = quantize_v_block_grouped(vblk[h], self.bits, self.group)
            else:
                kc, ks, kz = quant_k(kblk[h], self.bits)
                vc, vs, vz = quantize_v_block(vblk[h], self.bits)
            self.k_codes[p, h] = pack_words(kc, self.bits)
            self.v_codes[p, h] = pack_words(vc.T.copy(), self.bits)
            self.k_params[p, h] = pack_half2(ks, kz)
            self.v_params[p, h] = pack_half2(vs, vz)

    def quant_pack_kv(self, b: int, K: np.ndarray, V: np.ndarray):
        """Prefill of sequence b from K, V [H, L, D]: full blocks into its pages, the rest into
        its residual; the sequence's previous contents are replaced."""
        L = K.shape[1]
        assert K.shape == V.shape == (self.H, L, self.D) and K.dtype == np.float16
        nb, r = divmod(L, BLOCK)
        for n in range(nb):
            self._store_block(b, n, K[:, n * BLOCK:(n + 1) * BLOCK], V[:, n * BLOCK:(n + 1) * BLOCK])
        self.k_res[b, :, :r] = K[:, nb * BLOCK:]
        self.v_res[b, :, :r] = V[:, nb * BLOCK:]
        self.seq_lens[b] = L

    def append_kv(self, k_new: np.ndarray, v_new: np.ndarray, flush: bool = True):
        """One decode step of every sequence: token b goes to slot seq_lens[b] mod 128 of
        sequence b's residual; a residual that reaches 128 tokens is quantized into the
        sequence's next page at once.

        flush=False is the order of the paper's Residual Kernel (Sec. III-A(1), Sec. IV-B(1)), as in
        IntCache.append_kv: a sequence whose residual reaches 128 tokens keeps them in fp16 for the
        attention of this step, and flush_if_full() after that attention packs them into the page."""
        assert k_new.shape == v_new.shape == (self.B, self.H, self.D)
        assert not self.unflushed.any(), "a full residual must be flushed before the next append"
        for b in range(self.B):
            nb, r = divmod(int(self.seq_lens[b]), BLOCK)
            if r == BLOCK - 1:
                self._page_of(b, nb)            # raises before anything of this sequence is changed
            self.k_res[b, :, r] = k_new[b]
            self.v_res[b, :, r] = v_new[b]
            self.seq_lens[b] += 1
            if r == BLOCK - 1:
                self.unflushed[b] = True
                if flush:
                    self.flush_if_full()

    def flush_if_full(self):
        """Sec. IV-B(1): a residual of N_r = 128 tokens becomes the sequence's next packed block."""
        for b in range(self.B):
            if self.unflushed[b]:
                self._store_block(b, int(self.seq_lens[b]) // BLOCK - 1, self.k_res[b], self.v_res[b])
                self.unflushed[b] = False

    def dequant(self, b: int, h: int):
        """K_hat, V_hat [seq_lens[b], D] float64 of one (sequence, kv_head)."""
        nb, r = divmod(int(self.seq_lens[b]), BLOCK)
        if self.unflushed[b]:                  # the newest 128 tokens are still the fp16 residual
            nb, r = nb - 1, BLOCK
        Kh = np.empty((nb * BLOCK + r, self.D), np.float64)
        Vh = np.empty_like(Kh)
        for n in range(nb):
            p = self._page_of(b, n)
            kc = unpack_words(self.k_codes[p, h], self.bits).astype(np.float64)
            vc = unpack_words(self.v_codes[p, h], self.bits).astype(np.float64).T
            ks, kz = unpack_half2(self.k_params[p, h])
            vs, vz = unpack_half2(self.v_params[p, h])
            if self.group != BLOCK:      # ks, kz [128/group, D] (k_per_token: [128, D/group]); vs, vz [128, D/group]
                ks, kz, vs, vz = (x.astype(np.float64) for x in (ks, kz, vs, vz))
                kax = 1 if self.k_per_token else 0
                Kh[n * BLOCK:(n + 1) * BLOCK] = kc * np.repeat(ks, self.group, axis=kax) + np.repeat(kz, self.group, axis=kax)
                Vh[n * BLOCK:(n + 1) * BLOCK] = vc * np.repeat(vs, self.group, axis=1) + np.repeat(vz, self.group, axis=1)
                continue
            if self.k_per_token:
                Kh[n * BLOCK:(n + 1) * BLOCK] = kc * ks.astype(np.float64)[:, None] + kz.astype(np.float64)[:, None]
            else:
                Kh[n * BLOCK:(n + 1) * BLOCK] = kc * ks.astype(np.float64)[None, :] + kz.astype(np.float64)[None, :]
            Vh[n * BLOCK:(n + 1) * BLOCK] = vc * vs.astype(np.float64)[:, None] + vz.astype(np.float64)[:, None]
        Kh[nb * BLOCK:] = self.k_res[b, h, :r].astype(np.float64)
        Vh[nb * BLOCK:] = self.v_res[b, h, :r].astype(np.float64)
        return Kh, Vh


# --------------------------------------------------------------------------- MXFP4

def e2m1_decode(code: np.ndarray) -> np.ndarray:
    """Value of a 4-bit e2m1 code: bit 3 sign, bits 2..1 exponent, bit 0 mantissa."""
    code = np.asarray(code).astype(np.int64)
    mag = E2M1_GRID[code & 7]
    return np.where(code & 8, -mag, mag)


def e2m1_encode(v: np.ndarray) -> np.ndarray:
    """Nearest e2m1 code of v (float64): ties go to the neighbour whose mantissa bit is 0,
    magnitudes beyond 6 saturate to 6, and a result of magnitude 0 is stored as +0."""
    a = np.abs(np.asarray(v, dtype=np.float64))
    d = np.abs(a[..., None] - E2M1_GRID)                 # distance to each of the 8 magnitudes
    best = d.min(axis=-1, keepdims=True)
    cand = d == best                                      # one or two neighbouring entries
    idx = np.arange(8)
    even_first = np.where(cand & (idx % 2 == 0), idx, 99).min(axis=-1)
    any_first = np.where(cand, idx, 99).min(axis=-1)
    mag_idx = np.where(even_first < 99, even_first, any_first)
    mag_idx = np.where(a > 6.0, 7, mag_idx)
    sign = (np.asarray(v) < 0) & (mag_idx != 0)
    return (mag_idx | (sign.astype(np.int64) << 3)).astype(np.uint8)


def mx_quantize(x: np.ndarray):
    """x [..., 32*k] (values representable in bf16, held as float32/64) -> e2m1 codes of the
    same shape and e8m0 scale bytes [..., k].  Per 32 contiguous elements: amax == 0 gives
    byte 127 and zero codes; otherwise the shared exponent is floor(log2(amax)) - 2 (2 is
    the exponent of e2m1's largest binade), clamped to [-127, 127], stored biased by 127."""
    x = np.asarray(x, dtype=np.float64)
    g = x.reshape(x.shape[:-1] + (x.shape[-1] // MX_GROUP, MX_GROUP))
    amax = np.abs(g).max(axis=-1)
    nz = amax > 0
    _, ex = np.frexp(np.where(nz, amax, 1.0))            # amax = m * 2^ex, m in [0.5, 1)
    e = np.clip(ex - 1 - 2, -127, 127)
    e = np.where(nz, e, 0)
    codes = e2m1_encode(g * np.exp2(-e.astype(np.float64))[..., None])
    return codes.reshape(x.shape), (e + 127).astype(np.uint8)


def mx_dequantize(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    c = codes.reshape(codes.shape[:-1] + (codes.shape[-1] // MX_GROUP, MX_GROUP))
    val = e2m1_decode(c) * np.exp2(scales.astype(np.float64) - 127.0)[..., None]
    return val.reshape(codes.shape)


def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """Two 4-bit codes per byte along the last axis, even element in the low nibble."""
    c = codes.astype(np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << np.uint8(4))).astype(np.uint8)


def unpack_nibbles(b: np.ndarray) -> np.ndarray:
    out = np.empty(b.shape[:-1] + (b.shape[-1] * 2,), np.uint8)
    out[..., 0::2] = b & np.uint8(0xF)
    out[..., 1::2] = b >> np.uint8(4)
    return out


class MxCache:
    """MXFP4 cache.  Every token is quantized on arrival (an MX block lies inside one
    token), so there is no residual.  Layout:

      k_codes  uint8 [B, H, cap tokens, D/2]            byte j: channels 2j (low), 2j+1 (high)
      k_scales uint8 [B, H, cap tokens, D/32]           e8m0 per 32 channels
      v_codes  uint8 [B, H, cap/128, D channels, 64]    byte j of a channel row: tokens 2j, 2j+1
                                                         of that 128-token block
      v_scales uint8 [B, H, cap tokens, D/32]
    """

    def __init__(self, batch: int, n_kv_heads: int, capacity: int, head_dim: int = 128):
        assert capacity % BLOCK == 0 and head_dim == 128
        self.B, self.H, self.D, self.capacity = batch, n_kv_heads, head_dim, capacity
        self.k_codes = np.zeros((batch, n_kv_heads, capacity, head_dim // 2), np.uint8)
        self.k_scales = np.full((batch, n_kv_heads, capacity, head_dim // MX_GROUP), 127, np.uint8)
        self.v_codes = np.zeros((batch, n_kv_heads, capacity // BLOCK, head_dim, BLOCK // 2), np.uint8)
        self.v_scales = np.full((batch, n_kv_heads, capacity, head_dim // MX_GROUP), 127, np.uint8)
        self.length = 0

    def _store(self, t0: int, K: np.ndarray, V: np.ndarray):
        n = K.shape[2]
        kc, ks = mx_quantize(K)
        vc, vs = mx_quantize(V)
        self.k_codes[:, :, t0:t0 + n] = pack_nibbles(kc)
        self.k_scales[:, :, t0:t0 + n] = ks
        self.v_scales[:, :, t0:t0 + n] = vs
        for i in range(n):                      # V codes go channel-major inside their block
            t = t0 + i
            row = self.v_codes[:, :, t // BLOCK, :, (t % BLOCK) // 2]
            if t % 2 == 0:
                row[...] = (row & np.uint8(0xF0)) | vc[:, :, i, :]
            else:
                row[...] = (row & np.uint8(0x0F)) | (vc[:, :, i, :] << np.uint8(4))

    def quant_pack_kv(self, K: np.ndarray, V: np.ndarray):
        assert K.shape == V.shape and K.shape[2] <= self.capacity
        self._store(0, K, V)
        self.length = K.shape[2]

    def append_kv(self, k_new: np.ndarray, v_new: np.ndarray):
        if self.length + 1 > self.capacity:
            raise OverflowError("cache capacity exceeded")
        self._store(self.length, k_new[:, :, None, :], v_new[:, :, None, :])
        self.length += 1

    def dequant(self, b: int, h: int):
        L = self.length
        Kh = mx_dequantize(unpack_nibbles(self.k_codes[b, h, :L]), self.k_scales[b, h, :L])
        nb = -(-L // BLOCK)
        vc = unpack_nibbles(self.v_codes[b, h, :nb])                   # [nb][c][128 tokens]
        vc = vc.transpose(0, 2, 1).reshape(nb * BLOCK, self.D)[:L]     # [t][c]
        Vh = mx_dequantize(vc, self.v_scales[b, h, :L])
        return Kh, Vh


class PagedMxCache:
    """MXFP4 in the page-managed setting (same reading as PagedIntCache: a page is a 128-token
    block, block n of sequence b is page block_table[b, n], lengths per sequence).  Inside a
    page every array has the bytes the contiguous MxCache holds for that block:

      k_codes  uint8 [P, H, 128 tokens, D/2]     k_scales uint8 [P, H, 128, D/32]
      v_codes  uint8 [P, H, D channels, 64]      v_scales uint8 [P, H, 128, D/32]
    """

    def __init__(self, batch: int, n_kv_heads: int, num_pages: int, max_pages: int, block_table: np.ndarray,
                 head_dim: int = 128):
        assert head_dim == 128 and block_table.shape == (batch, max_pages)
        self.B, self.H, self.D, self.P, self.max_pages = batch, n_kv_heads, head_dim, num_pages, max_pages
        self.k_codes = np.zeros((num_pages, n_kv_heads, BLOCK, head_dim // 2), np.uint8)
        self.k_scales = np.full((num_pages, n_kv_heads, BLOCK, head_dim // MX_GROUP), 127, np.uint8)
        self.v_codes = np.zeros((num_pages, n_kv_heads, head_dim, BLOCK // 2), np.uint8)
        self.v_scales = np.full((num_pages, n_kv_heads, BLOCK, head_dim // MX_GROUP), 127, np.uint8)
        self.block_table = block_table.astype(np.int32).copy()
        self.seq_lens = np.zeros(batch, np.int32)

    def _page_of(self, b: int, n: int) -> int:
        if n >= self.max_pages:
            raise OverflowError("block table row is full")
        p = int(self.block_table[b, n])
        if not 0 <= p < self.P:
            raise IndexError("block table entry outside the pool")
        return p

    def _store_token(self, b: int, t: int, k: np.ndarray, v: np.ndarray):
        """Token t of sequence b from k, v [H, D] (bf16 values in float32)."""
        p, i = self._page_of(b, t // BLOCK), t % BLOCK
        kc, ks = mx_quantize(k)
        vc, vs = mx_quantize(v)
        self.k_codes[p, :, i] = pack_nibbles(kc)
        self.k_scales[p, :, i] = ks
        self.v_scales[p, :, i] = vs
        row = self.v_codes[p, :, :, i // 2]
        if i % 2 == 0:
            row[...] = (row & np.uint8(0xF0)) | vc
        else:
            row[...] = (row & np.uint8(0x0F)) | (vc << np.uint8(4))

    def quant_pack_kv(self, b: int, K: np.ndarray, V: np.ndarray):
        """Prefill of sequence b from K, V [H, L, D]; replaces what the sequence held."""
        L = K.shape[1]
        assert K.shape == V.shape == (self.H, L, self.D)
        for t in range(L):
            self._store_token(b, t, K[:, t], V[:, t])
        self.seq_lens[b] = L

    def append_kv(self, k_new: np.ndarray, v_new: np.ndarray):
        assert k_new.shape == v_new.shape == (self.B, self.H, self.D)
        for b in range(self.B):
            self._store_token(b, int(self.seq_lens[b]), k_new[b], v_new[b])
            self.seq_lens[b] += 1

    def dequant(self, b: int, h: int):
        L = int(self.seq_lens[b])
        Kh = np.empty((L, self.D), np.float64)
        Vh = np.empty((L, self.D), np.float64)
        for n in range(-(-L // BLOCK)):
            p = self._page_of(b, n)
            m = min(BLOCK, L - n * BLOCK)
            Kh[n * BLOCK:n * BLOCK + m] = mx_dequantize(unpack_nibbles(self.k_codes[p, h, :m]), self.k_scales[p, h, :m])
            vc = unpack_nibbles(self.v_codes[p, h]).T[:m]            # [c][128] -> [t][c]
            Vh[n * BLOCK:n * BLOCK + m] = mx_dequantize(vc, self.v_scales[p, h, :m])
        return Kh, Vh


# --------------------------------------------------------------------------- attention

def attention_weights(q: np.ndarray, Kh: np.ndarray, sm_scale: float) -> np.ndarray:
    """Softmax weights of one query vector over L keys, two-pass, float64."""
    s = sm_scale * (Kh @ q.astype(np.float64))
    p = np.exp(s - s.max())
    return p / p.sum()


def decode_attn(cache, q: np.ndarray, sm_scale: float, units=None) -> np.ndarray:
    """out[b, hq, :] = softmax(sm_scale * q[b,hq] . K_hat^T) . V_hat over all cached tokens
    of KV head hq // g_q (Fig. 2 caption; Sec. IV-A for the head grouping).  float64.
    `units`: optional iterable of (b, kv_head) pairs; rows of other units are left NaN."""
    B, Hq, D = q.shape
    g = Hq // cache.H
    out = np.full((B, Hq, D), np.nan, np.float64)
    todo = [(b, h) for b in range(B) for h in range(cache.H)] if units is None else list(units)
    for b, h in todo:
        Kh, Vh = cache.dequant(b, h)
        if Kh.shape[0] == 0:            # a sequence with no tokens: defined as a zero output
            out[b, h * g:(h + 1) * g] = 0.0
            continue
        for j in range(g):
            w = attention_weights(np.asarray(q[b, h * g + j], dtype=np.float64), Kh, sm_scale)
            out[b, h * g + j] = w @ Vh
    return out
