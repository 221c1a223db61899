"""A decoder layer and a whole decode step composed in Python from the oracle's own functions (and nothing
else): fp64 reference contractions rounded once to bf16, the bit-exact CANON emulation everywhere else.
The layer returns its intermediate values as well, so that a test can bound the GPU's deviation element
by element from the roundings that lie on the path of each output.

TEST INFRASTRUCTURE ONLY (as the rest of this package): used by tests/, the smoke check and the CPU-baseline
leg of the benchmark; it calls the oracle's functions and never the HIP library."""
import numpy as np

from . import (attn_decode_f64, bf16_from_f64, bf16_to_f32, gemm_f64, residual, rmsnorm, rope, swiglu)


def _proj(a_bits, w_bits):
    """bf16( fp64 reference product ): the oracle's reading of a projection (sections 6.5 / task statement)."""
    c, _ = gemm_f64(a_bits, w_bits, want_abs=False)
    return bf16_from_f64(c)   # one rounding, fp64 -> bf16 (no intermediate fp32 rounding)


def ulp_bf16(bits):
    """One unit in the last place of each bf16 value (2^(e-7) for a normal number with exponent e)."""
    f = np.abs(bf16_to_f32(np.ascontiguousarray(bits)).astype(np.float64))
    e = np.floor(np.log2(np.maximum(f, 2.0 ** -126)))
    return 2.0 ** (e - 7)


def layer(x, w, kcache, vcache, positions, cos_t, sin_t, cfg):
    """One decoder layer (the steps of det_decoder_layer in its documented order).  x [B,H] bf16 bits;
    `w`: logical [K,N] bf16-bit weights norm1, wqkv, wo, norm2, wgu, wdown; caches [B,Hkv,Lmax,D] are
    updated in place.  Returns (x_out, dict of intermediates)."""
    B, H = x.shape
    Hq, Hkv, D, F = cfg["Hq"], cfg["Hkv"], cfg["D"], cfg["F"]
    positions = np.asarray(positions, dtype=np.int32)
    h = rmsnorm(x, w["norm1"], cfg["eps"])
    qkv = _proj(h, w["wqkv"])
    q_rot = rope(np.ascontiguousarray(qkv[:, :Hq * D]).reshape(B, Hq, D), positions, cos_t, sin_t)
    k_rot = rope(np.ascontiguousarray(qkv[:, Hq * D:(Hq + Hkv) * D]).reshape(B, Hkv, D), positions, cos_t, sin_t)
    v_new = qkv[:, (Hq + Hkv) * D:].reshape(B, Hkv, D)
    for b in range(B):
        kcache[b, :, positions[b]] = k_rot[b]
        vcache[b, :, positions[b]] = v_new[b]
    att, _ = attn_decode_f64(q_rot, kcache, vcache, positions + 1, cfg["scale"])
    att = bf16_from_f64(att).reshape(B, Hq * D)
    o = _proj(att, w["wo"])
    x1 = residual(x, o)
    h2 = rmsnorm(x1, w["norm2"], cfg["eps"])
    gu = _proj(h2, w["wgu"])
    mm = swiglu(np.ascontiguousarray(gu[:, :F]), np.ascontiguousarray(gu[:, F:]))
    dn = _proj(mm, w["wdown"])
    x2 = residual(x1, dn)
    return x2, dict(o=o, x1=x1, dn=dn, mm=mm, att=att)


def layer_bound(x2, inter, carried_rel=2.0 ** -8):
    """Element-wise bound on |gpu - oracle| for the layer output.

    The two sides differ in how a contraction is accumulated (fp32 on the matrix core against fp64), which
    moves a pre-rounding value by about 2^-23 relative; where that value sits next to a bf16 rounding
    boundary the rounded results land one bf16 ulp apart.  The output element x2 = bf16(x1 + dn),
    x1 = bf16(x + o) has four roundings on its path (o, x1, dn, x2), each of which may land one ulp of its
    own value away: the first four terms.
    Carried term.  One-ulp flips of earlier activations reach an output through a projection as noise: a
    fraction f of flipped inputs adds about sqrt(K f) 2^-8 |a||w| to an output whose own size is about
    sqrt(K) |a||w|, i.e. sqrt(f) 2^-8 relative, which in turn flips about sqrt(f) of the next stage's
    outputs.  Starting from the few 10^-4 of the first projection the fraction grows to a few percent
    after gate/up and to 10-25 % after the down projection (measured: a quarter of the outputs of the
    Llama-shaped layer differ from the oracle, nearly all by one ulp), and the noise on dn and o reaches a
    few tenths of an ulp of an rms-sized value, with a tail over thousands of outputs of about one such ulp:
    `carried_rel` * rms(x2), 2^-8 by default (1-2 ulps of an rms-sized branch value)."""
    f = bf16_to_f32(np.ascontiguousarray(x2)).astype(np.float64)
    rms = np.sqrt((f ** 2).mean())
    return (ulp_bf16(inter["o"]) + ulp_bf16(inter["x1"]) + ulp_bf16(inter["dn"]) + ulp_bf16(x2)
            + carried_rel * rms)


def model_step(weights, cfg, tokens, positions, kcaches, vcaches, cos_t, sin_t):
    """One decode step of the whole model (section 6.6's loop body as a pure function): embedding rows of
    `tokens`, every layer at `positions`, final RMSNorm, lm_head as the fp64 reference product.
    Returns fp64 logits [B, V]; the caches (one pair per layer) are updated in place."""
    x = np.ascontiguousarray(weights["embed"][np.asarray(tokens, dtype=np.int64)])
    for lw, kc, vc in zip(weights["layers"], kcaches, vcaches):
        x, _ = layer(x, lw, kc, vc, positions, cos_t, sin_t, cfg)
    xn = rmsnorm(x, weights["final_norm"], cfg["eps"])
    logits, _ = gemm_f64(xn, weights["lm_head"], want_abs=False)
    return logits
