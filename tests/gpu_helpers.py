"""Helpers for the -m gpu parity tests: build a context from a Workload, run the HIP path through
the C ABI, and compare with the CPU oracle."""
import numpy as np

from oracle import pie_oracle as O

MAX_ABS, MEAN_ABS = 2e-2, 2e-3  # tolerance on bf16 layer outputs


def make_ctx(w, with_head=True, max_dist_rows=None, max_top_k=256):
    from paper_2510_24051_amd import Pie
    b = w.batch
    n_dist = max_dist_rows if max_dist_rows is not None else (max(len(w.dist_rows), 1) if w.head is not None else 0)
    ctx = Pie(w.model, w.n_kv_pages, w.n_embeds, max_batch_tokens=b.n_tokens, max_batch_requests=b.n_requests,
              max_top_k=max_top_k, max_dist_rows=n_dist if (with_head and w.head is not None) else 0)
    ctx.load_layer(0, w.weights)
    if with_head and w.head is not None:
        ctx.load_head(w.head)
    seed_ctx(ctx, w)
    return ctx


def seed_ctx(ctx, w):
    ctx.embed_write(w.batch.in_embed_ids, w.embed_bits)
    if len(w.prior.page_ids):
        ctx.kv_write(0, w.prior.page_ids, w.prior.slots, w.prior.k_bits, w.prior.v_bits)


def dec(bits):
    return O.bf16_decode(bits)


def err_stats(got, ref):
    d = np.abs(np.asarray(got, dtype=np.float64) - np.asarray(ref, dtype=np.float64))
    return float(d.max()) if d.size else 0.0, float(d.mean()) if d.size else 0.0


def assert_close(got, ref, what, max_abs=MAX_ABS, mean_abs=MEAN_ABS):
    mx, mn = err_stats(got, ref)
    print(f"    {what}: max-abs {mx:.3e} mean-abs {mn:.3e} (limits {max_abs:.0e} / {mean_abs:.0e})", flush=True)
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), f"{what}: non-finite GPU output"
    assert mx <= max_abs and mn <= mean_abs, f"{what}: max-abs {mx} mean-abs {mn}"


def bf16_half_ulp(x):
    """Half the spacing of bf16 values at |x| (8 significand bits): 2**(floor(log2|x|) - 8)."""
    e = np.floor(np.log2(np.maximum(np.abs(np.asarray(x, dtype=np.float64)), 2.0 ** -126)))
    return 2.0 ** (e - 8)


# What the stated limits leave above the output format's own rounding step: 2e-2 is the half-ulp of bf16 in
# [4, 8) (2**-6) plus 4.4e-3, and 2e-3 is the mean rounding error of a unit-scale bf16 output (about 1.2e-3) plus 8e-4.
ALLOW_MAX, ALLOW_MEAN = MAX_ABS - 2.0 ** -6, 8e-4


def assert_y_close(got, ref, what, stored_as=None, allow_scale=1.0):
    """Stored bf16 layer outputs against the oracle's wide y: max-abs <= 2e-2 and mean-abs <= 2e-3.  Where the
    format itself cannot meet these (an element with |y| >= 8 has a half-ulp of 0.031 or more; a tensor whose own
    mean rounding error exceeds 1.2e-3), the limit is the rounding floor of the oracle's own y plus the allowance
    the stated limits leave above that floor for |y| < 8, never a wider blanket limit; the error is also printed as
    a multiple of the floor.
    `stored_as` (comparison against the wide-intermediate oracle): the y of the oracle with bf16 intermediates.  The
    floor is then the error that oracle's own stored output has against `ref`: the paper's activation precision
    bounds how close any bf16 pipeline can come to the wide value (rows that see a handful of keys have attention
    outputs of order one, whose bf16 rounding step alone moves y by more than the stated limits).
    `allow_scale`: the part of the error that is not the output's own rounding comes from bf16 intermediates that
    round the other way than the oracle's (their inputs differ in the last fp32 bits) and reaches y through the
    output and down projections, so it is proportional to the scale of those two weights; a draw whose residual
    projections are `allow_scale` times the depth-scaled ones gets that multiple of the allowance."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite GPU output"
    d = np.abs(got - ref)
    floor = np.abs(O.bf16_round(ref if stored_as is None else np.asarray(stored_as, dtype=np.float64)) - ref)
    if stored_as is None:
        lim = np.maximum(MAX_ABS, bf16_half_ulp(ref) + ALLOW_MAX * allow_scale)
    else:  # what the comparison with `stored_as` already bounds (both outputs rounded, then the triangle inequality)
        lim = np.maximum(MAX_ABS, floor + 2.0 * bf16_half_ulp(ref) + ALLOW_MAX * allow_scale)
    mean_lim = max(MEAN_ABS, float(floor.mean()) + ALLOW_MEAN * allow_scale)
    n_big = int((np.abs(ref) >= 8).sum())
    print(f"    {what}: max-abs {d.max():.3e} mean-abs {d.mean():.3e} (limits {MAX_ABS:.0e} / {mean_lim:.2e}); rounding "
          f"floor of {'the oracle with bf16 intermediates' if stored_as is not None else 'the oracle'}'s own y "
          f"{floor.max():.3e} / {floor.mean():.3e} -> {d.mean() / max(floor.mean(), 1e-30):.2f}x "
          f"the mean floor; {n_big} elements with |y| >= 8", flush=True)
    worst = int(np.argmax(d - lim))
    assert (d <= lim).all(), f"{what}: |err| {d.flat[worst]} > {lim.flat[worst]} at |y| = {abs(ref.flat[worst])}"
    assert d.mean() <= mean_lim, f"{what}: mean-abs {d.mean()} > {mean_lim}"


def assert_mlp_stages(w, h_gpu, act_bits, y_bits, rows, what, max_rows=256):
    """The MLP kernels one by one at their real width, each against the oracle's arithmetic applied to the GPU's
    own input of that stage (so no rounding decision of an earlier stage is compared twice):
      second norm + gate/up + SwiGLU: act recomputed from the GPU's fp32 residual; equal up to the last bf16 bit
        except where the normalised row itself rounds the other way (a handful of values),
      down projection + residual + output rounding: y recomputed from the GPU's residual and activation; the stored
        bf16 output is within its own half-ulp plus the fp32 accumulation error of the contraction."""
    m, wt = w.model, w.weights
    pick = np.arange(len(rows)) if len(rows) <= max_rows else np.linspace(0, len(rows) - 1, max_rows).astype(np.int64)
    h = np.asarray(h_gpu, dtype=np.float64)[pick]
    act_gpu = dec(act_bits[pick])
    hn = O.bf16_round(O.rmsnorm(h, dec(wt.g2), m.rms_eps))
    act_ref = O.bf16_round(O.silu(hn @ dec(wt.wgate).T) * (hn @ dec(wt.wup).T))
    ulp = 2.0 * bf16_half_ulp(np.maximum(np.abs(act_ref), 2.0 ** -20))
    diff = np.abs(act_gpu - act_ref)
    off = diff / ulp
    # fp32 accumulation over the hidden dimension leaves the sums a few 1e-6 from the float64 ones, which flips the
    # bf16 rounding of well under 1% of the products; about one element in ten rows of the normalised input rounds
    # the other way than the host's float64 norm (one ulp of a value of 3 times a 3-sigma weight moves a sum by 1e-3),
    # which a product near zero (silu(gate) or up passing through zero) shows as many of its own ulps: hence the
    # absolute term
    w2 = int(np.argmax(diff - ulp))
    print(f"    {what} gate/up + SwiGLU from the GPU's own residual ({len(pick)} rows x {m.mlp_dim}): "
          f"{np.mean(off > 0) * 100:.3f}% of values differ, {np.mean(off > 1.01) * 100:.4f}% by more than one ulp "
          f"(all near zero: largest excess over one ulp {max(diff.flat[w2] - ulp.flat[w2], 0):.2e} at |act| "
          f"{abs(act_ref.flat[w2]):.2e})", flush=True)
    assert np.mean(off > 0) < 0.02 and np.mean(off > 1.01) < 2e-3 and (diff <= 1.01 * ulp + 3e-3).all()
    y_ref = h + act_gpu @ dec(wt.wdown).T
    err = np.abs(dec(y_bits[pick]) - y_ref)
    lim = bf16_half_ulp(y_ref) * 1.001 + 1e-5 * (1.0 + np.abs(y_ref))
    print(f"    {what} down projection + residual from the GPU's own activation: worst excess over the output's "
          f"half-ulp {max((err - bf16_half_ulp(y_ref)).max(), 0):.2e}, |y| up to {np.abs(y_ref).max():.1f}", flush=True)
    assert (err <= lim).all()


def gpu_forward(ctx, w, validate=True):
    """Run pie_batch_create + pie_forward, return the stored output rows (uint16 bits) and their token indices."""
    pb = ctx.batch_create(w.batch, validate=validate)
    ctx.forward(0, pb)
    ctx.synchronize()
    stored = np.nonzero(w.batch.out_embed_ids >= 0)[0]
    y_bits = ctx.embed_read(w.batch.out_embed_ids[stored])
    return pb, stored, y_bits


def appended_positions(w):
    b, P = w.batch, w.model.page_size
    pages, slots = [], []
    for r in range(b.n_requests):
        n_new = b.tok_indptr[r + 1] - b.tok_indptr[r]
        pg = b.page_ids[b.page_indptr[r]:b.page_indptr[r + 1]]
        j = b.kv_len[r] - n_new + np.arange(n_new)
        pages.append(pg[j // P])
        slots.append(j % P)
    return np.concatenate(pages).astype(np.int32), np.concatenate(slots).astype(np.int32)


def assert_bf16_close(got_bits, ref_bits, what, ulps=1, frac=0.03):
    """bf16 tensors computed in different precisions: equal up to `ulps` units in the last place, and
    bit-identical for all but a small fraction."""
    g, r = dec(got_bits), dec(ref_bits)
    # the rotary step mixes two values, so a one-ulp flip of an input shows at the scale of the pair, not of
    # the (possibly cancelling) result: measure ulps at max(|ref|, rms of the tensor)
    ulp = np.maximum(np.abs(r), np.sqrt(np.mean(r * r)) + 2.0 ** -120) * 2.0 ** -7
    bad = np.abs(g - r) > ulps * ulp
    mism = float(np.mean(got_bits != ref_bits))
    print(f"    {what}: {mism * 100:.3f}% of bf16 values differ, {int(bad.sum())} by more than {ulps} ulp", flush=True)
    assert not bad.any(), f"{what}: {int(bad.sum())} values off by more than {ulps} ulp"
    assert mism <= frac, f"{what}: {mism} of values differ"
