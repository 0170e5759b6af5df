"""Stage-wise, teacher-forced comparison of one encoder layer run on the GPU with the CPU oracle (no method
arithmetic here: every reference value comes from ``oracle``).

Every stage of the layer is recomputed by the oracle from the GPU's OWN output of the stage before it, on the
rows of the sequences that are asked for, so a mistake anywhere (a wrong row range at a sequence seam, one bad
head, a wrong hand-over of codes) shows in the stage where it happens:
  integer stages (quantizer of the input, the four linears' binary16 outputs)  -> bit-exact
  float stages (LayerNorm outputs)                                              -> |err| <= rtol |ref| + rtol rms(ref), rtol = 1e-2
  codes decided from a float that went through LayerNorm / softmax / GELU       -> equal, except by one step where the
      oracle's pre-rounding value lies within a band of a rounding boundary.
Bands (in units of one code), from the arithmetic of the kernels:
  LayerNorm and GELU outputs: the kernel works in binary32, the oracle in binary64 rounded once; the same
      relative perturbation of a value is 16 times more code units at 8 bits than at 4: 2^-10 at 4 bits, 2^-7 at 8.
  Attention context: both sides narrow the softmax probabilities to binary16 before P.v; the kernel's
      probabilities come from binary32 arithmetic, so a probability that sits at a binary16 rounding boundary may
      narrow the other way, moving it by one binary16 unit in the last place (<= 2^-10 p).  If every probability
      of a row did, the context element would move by at most 2^-10 sum_j p_j |v_j|; that bound, evaluated per
      element by the oracle (attention with |v| in place of v), divided by the step, is the band.
A band says where a difference is allowed, not that it is expected; the number of differing codes is also
bounded by the share of elements that lie inside their band.
"""
import numpy as np

import oracle
from helpers import RTOL, assert_codes_match_with_tie_band, assert_float_close


def qrange(bits):
    return dict(qmin=-8, qmax=7) if bits == 4 else dict(qmin=-128, qmax=127)


def attention_code_band(qkv_rows, length, hidden, heads, step):
    """Per-element band, in code units, of the context codes of one sequence (see the module docstring)."""
    absv = np.array(qkv_rows, np.float32, copy=True)
    absv[:, 2 * hidden:] = np.abs(absv[:, 2 * hidden:])
    bound = oracle.attention(absv, 1, length, hidden, heads)  # sum_j p_j |v_j|, probabilities in binary32/64
    return (2.0 ** -10 + 2.0 ** -16) * bound / float(step) + 2.0 ** -12


def codes_match(got, want, pre_round, step, band, what):
    band = np.broadcast_to(np.asarray(band, np.float64), np.shape(want))
    v = np.asarray(pre_round, np.float64) / float(step)
    inside = np.abs(v - np.floor(v) - 0.5) <= band
    # no more codes may differ than there are elements inside their band (plus the 1e-4 of the general rule)
    return assert_codes_match_with_tie_band(got, want, pre_round, step, band=band,
                                            max_frac=float(inside.mean()) + 1e-4, what=what)


def code_row_pitch(cols):
    """Codes per row of a 4-bit code buffer of the layer: rows whose length is no multiple of 32 are stored
    padded with zero codes to the next multiple of 128."""
    return cols if cols % 32 == 0 else (cols + 127) // 128 * 128


class LayerBuffers:
    """The layer's workspace and outputs as numpy arrays (read back once)."""

    def __init__(self, ws_bytes, layout, M, hidden, ffn, bits):
        self.M, self.hidden, self.ffn, self.bits = M, hidden, ffn, bits
        self.ws, self.L = ws_bytes, layout

    def codes(self, off, cols):
        if self.bits == 8:
            return self.ws[off: off + self.M * cols].view(np.int8).reshape(self.M, cols)
        pitch = code_row_pitch(cols)
        rows = oracle.unpack_nibbles(self.ws[off: off + self.M * pitch // 2], pitch)
        assert not rows[:, cols:].any(), "padding codes must be zero"
        return rows[:, :cols]

    def f16(self, off, cols):
        return self.ws[off: off + self.M * cols * 2].view(np.float16).reshape(self.M, cols).astype(np.float32)


def check_layer_stagewise(buf, q, h_in, h_out, sequences, *, c0_in=None, q_next=None, s_out_next=0.0, next_bits=0,
                          what=""):
    """buf: LayerBuffers of the run; q: the oracle's layer parameters (w_*, sw_*, b_*, sx_*, ln*, heads);
    h_in / h_out: [M, hidden] float32 values of the binary16 tensors; sequences: (first row, length) of every
    sequence to check; c0_in: the input codes if the caller handed them in (q_in), else the workspace's are
    checked against the quantizer; q_next: int8 codes [M, hidden] the layer wrote for the next one."""
    bits, H, F, heads = buf.bits, buf.hidden, buf.ffn, q["heads"]
    Q = qrange(bits)
    band = 2.0 ** -10 if bits == 4 else 2.0 ** -7
    L = buf.L
    c0_all = c0_in if c0_in is not None else buf.codes(L.c0, H)
    c1_all, c2_all, c3_all = buf.codes(L.c1, H), buf.codes(L.c2, H), buf.codes(L.c3, F)
    qkv_all, u_all, h1_all, d_all = buf.f16(L.qkv, 3 * H), buf.f16(L.u, H), buf.f16(L.h1, H), buf.f16(L.d, H)
    flips = 0
    for (r0, n) in sequences:
        rows = slice(r0, r0 + n)
        tag = f"{what} rows {r0}..{r0 + n - 1}: "
        hf = h_in[rows]
        c0 = c0_all[rows]
        if c0_in is None:
            assert np.array_equal(c0, oracle.quantize(hf, q["sx_qkv"], **Q)), tag + "input codes"
        r = oracle.linear_int4(c0, q["sx_qkv"], q["w_qkv"], q["sw_qkv"], q["b_qkv"], out_dtype=oracle.F16, **Q)
        assert np.array_equal(qkv_all[rows], r["y"]), tag + "qkv"
        ctx_ref = oracle.attention(qkv_all[rows], 1, n, H, heads, p_dtype=oracle.F16)
        flips += codes_match(c1_all[rows], oracle.quantize(ctx_ref, q["sx_ao"], **Q), ctx_ref, q["sx_ao"],
                             attention_code_band(qkv_all[rows], n, H, heads, q["sx_ao"]), tag + "context codes")
        r = oracle.linear_int4(c1_all[rows], q["sx_ao"], q["w_ao"], q["sw_ao"], q["b_ao"], residual=hf,
                               out_dtype=oracle.F16, **Q)
        assert np.array_equal(u_all[rows], r["y"]), tag + "attention output + residual"
        h1_ref = oracle.layernorm(u_all[rows], q["ln1_gamma"], q["ln1_beta"], q["ln_eps"])
        assert_float_close(h1_all[rows], oracle.round_storage(h1_ref, oracle.F16), RTOL[1], tag + "h1")
        flips += codes_match(c2_all[rows], oracle.quantize(h1_ref, q["sx_up"], **Q), h1_ref, q["sx_up"], band,
                             tag + "h1 codes")
        r = oracle.linear_int4(c2_all[rows], q["sx_up"], q["w_up"], q["sw_up"], q["b_up"], act=oracle.ACT_GELU,
                               s_next=q["sx_down"], **Q)
        flips += codes_match(c3_all[rows], r["q"], r["y"], q["sx_down"], band, tag + "ffn codes")
        r = oracle.linear_int4(c3_all[rows], q["sx_down"], q["w_down"], q["sw_down"], q["b_down"],
                               residual=h1_all[rows], out_dtype=oracle.F16, **Q)
        assert np.array_equal(d_all[rows], r["y"]), tag + "ffn output + residual"
        out_ref = oracle.layernorm(d_all[rows], q["ln2_gamma"], q["ln2_beta"], q["ln_eps"])
        assert_float_close(h_out[rows], oracle.round_storage(out_ref, oracle.F16), RTOL[1], tag + "layer output")
        if q_next is not None:
            nb = next_bits or bits
            flips += codes_match(q_next[rows], oracle.quantize(out_ref, s_out_next, **qrange(nb)), out_ref, s_out_next,
                                 2.0 ** -10 if nb == 4 else 2.0 ** -7, tag + f"next-layer codes ({nb} bits)")
    return flips
