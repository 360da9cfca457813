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
