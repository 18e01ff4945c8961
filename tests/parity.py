"""Shared parity checks: HIP library results against the fp64 oracle on the same seeded inputs.

Protocol
* masks: the oracle forward pass is run with the GPU's masks forced on all earlier layers, so
  that one fp32/fp64 sign disagreement near z = 0 does not cascade; the GPU mask of a layer must
  equal (z_oracle > 0) on every element with |z_oracle| > MASK_GUARD * rms(z_oracle).
* gradients: against fp64 backprop with the GPU's masks forced (the same piecewise-linear
  piece), per tensor, normwise relative error <= GRAD_TOL.
* integers (packed words, erased offsets, fragment bases and counts): bit-exact against the
  oracle's own packing/compaction applied to the GPU's masks.
* with the library's own pre-activations and Phase-II cotangents kept (debug_keep): the mask words
  are the oracle's packing of (z_gpu > 0) and the fragment store is the oracle's compaction of
  h_gpu, both bit for bit, inside the running network (check_kept_tensors).
"""
import numpy as np

from oracle import moonwalk_oracle as O

GRAD_TOL = 1e-3      # normwise relative, per tensor (the stated bar for fp32 gradients)
MASK_GUARD = 1e-4    # relative to the layer's rms pre-activation


def gpu_masks(net, wl):
    out = []
    for i in range(wl.depth):
        words = net.fetch_mask(i)
        n = wl.batch * wl.widths[i + 1]
        assert words.size == (n + 63) // 64
        if n % 64:
            assert int(words[-1]) >> (n % 64) == 0, "padding bits of the last mask word must be zero"
        out.append(O.unpack_mask(words, n).reshape(wl.batch, wl.widths[i + 1]))
    return out


def check_masks(wl, masks):
    _, zs, _ = O.forward(wl.W, wl.b, wl.alphas, wl.x, forced_masks=masks)
    in_band = 0
    for i, (z, m) in enumerate(zip(zs, masks)):
        rms = float(np.sqrt(np.mean(z * z)))
        sure = np.abs(z) > MASK_GUARD * rms
        bad = (m != (z > 0)) & sure
        assert not bad.any(), f"layer {i}: {int(bad.sum())} sign bits differ outside the guard band"
        in_band += int((~sure).sum())
    return in_band


def grads_to_numpy(res):
    return [g.detach().cpu().numpy() for g in res.dW], [g.detach().cpu().numpy() for g in res.db]


def check_gradients(wl, masks, res, tol=GRAD_TOL):
    ref = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t, forced_masks=masks)
    dW, db = grads_to_numpy(res)
    eW = [O.normwise_rel_err(a, b) for a, b in zip(dW, ref["dW"])]
    eb = [O.normwise_rel_err(a, b) for a, b in zip(db, ref["db"])]
    assert max(eW) <= tol, f"dW normwise errors per layer: {eW}"
    assert max(eb) <= tol, f"db normwise errors per layer: {eb}"
    loss = float(res.loss.item())
    assert abs(loss - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 1e-30, (loss, ref["loss"])
    return ref, max(eW), max(eb)


def check_fragment_index(net, wl, masks):
    """Erased offsets, counts and layer bases: bit-exact against the oracle's definitions."""
    running = 0
    for i in range(wl.depth - 1, -1, -1):
        if wl.alphas[i] != 0.0:
            continue
        off = net.fetch_frag_offsets(i)
        np.testing.assert_array_equal(off, O.erased_word_offsets(masks[i]))
        assert net.fetch_frag_base(i) == running
        n0 = masks[i].size - int(masks[i].sum())
        assert int(off[-1]) == n0
        assert net.fetch_fragments(i).size == n0
        running += n0
    return running


def check_moonwalk(net, wl, res, tol=GRAD_TOL, check_h0=True):
    masks = gpu_masks(net, wl)
    in_band = check_masks(wl, masks)
    ref, eW, eb = check_gradients(wl, masks, res, tol)
    stats = net.memory_stats()
    assert stats["sign_mismatches"] == 0 and stats["frag_overflow"] == 0
    if check_h0:
        h0 = net.fetch_h0() / wl.loss_scale
        assert O.normwise_rel_err(h0, ref["h"][0]) <= 1e-4
    total = check_fragment_index(net, wl, masks)
    assert stats["frag_used"] == total
    # fragment values: the erased part of the phase-II cotangent of that layer
    for i in range(wl.depth):
        if wl.alphas[i] == 0.0:
            got = net.fetch_fragments(i) / wl.loss_scale
            want = O.compact_fragments(ref["h"][i + 1], masks[i])
            assert O.normwise_rel_err(got, want) <= 1e-4
    return {"max_dW_err": eW, "max_db_err": eb, "guard_band": in_band}


def check_moonwalk_layerwise(net, wl, res, say=print, tol=GRAD_TOL):
    """check_moonwalk for a network too large to hold the oracle's whole state (256 layers of 4096 x 4096): the same
    protocol (GPU masks forced, guard band, loss, every dW and db, h_0), one layer in host memory at a time. `wl`
    may hold device tensors; each layer's parameters come to the host when the oracle asks for them. `say` reports
    progress (a long silent test looks hung)."""
    def host(a):
        return a if isinstance(a, np.ndarray) else a.detach().cpu().numpy()

    def layer(i):
        return host(wl.W[i]), host(wl.b[i])

    state = {"in_band": 0}

    def gpu_mask(i, z):
        words = net.fetch_mask(i)
        assert words.size == (z.size + 63) // 64
        m = O.unpack_mask(words, z.size).reshape(z.shape)
        rms = float(np.sqrt(np.mean(z * z)))
        sure = np.abs(z) > MASK_GUARD * rms
        bad = (m != O.sign_mask(z)) & sure
        assert not bad.any(), f"layer {i}: {int(bad.sum())} sign bits differ outside the guard band"
        state["in_band"] += int((~sure).sum())
        if i % 32 == 31:
            say(f"  oracle forward: {i + 1} layers")
        return m

    xs, masks = O.forward_layerwise(layer, wl.depth, wl.alphas, host(wl.x), gpu_mask)
    eW, eb = [], []
    for i, dW, db, h in O.backprop_layerwise(layer, wl.alphas, xs, masks, host(wl.t)):
        if i == wl.depth:
            loss = float(res.loss.item())
            assert abs(loss - dW) <= 1e-5 * abs(dW) + 1e-30, (loss, dW)
            continue
        eW.append(O.normwise_rel_err(res.dW[i].detach().cpu().numpy(), dW))
        eb.append(O.normwise_rel_err(res.db[i].detach().cpu().numpy(), db))
        assert eW[-1] <= tol and eb[-1] <= tol, f"layer {i}: dW {eW[-1]:.3e}, db {eb[-1]:.3e}"
        if i % 32 == 0:
            say(f"  oracle reverse: down to layer {i}, worst so far dW {max(eW):.2e} db {max(eb):.2e}")
    assert O.normwise_rel_err(net.fetch_h0() / wl.loss_scale, h) <= 1e-4
    stats = net.memory_stats()
    assert stats["sign_mismatches"] == 0 and stats["frag_overflow"] == 0
    return {"max_dW_err": max(eW), "max_db_err": max(eb), "guard_band": state["in_band"]}


def check_kept_tensors(net, wl, ref, masks, h_tol=1e-4, hf_tol=1e-3):
    """A network built with debug_keep: the GPU's own z, Phase-II h and Phase-III h of every layer.

    Integer and copy steps, bit-exact against the oracle's definitions applied to the GPU's OWN tensors:
    mask words = pack(z_gpu > 0); for a ReLU layer the stored fragments = compaction of h_gpu at the
    erased entries; for a layer with a re-seed checkpoint the checkpoint is h_gpu itself. Floating
    point, against the mask-forced fp64 oracle: z (given the GPU's masks below), Phase-II h, and the
    Phase-III h, whose error is the one that grows between re-seeds.
    Returns the per-layer normwise errors of the Phase-III cotangent.
    """
    xs, zs, _ = O.forward(wl.W, wl.b, wl.alphas, wl.x, forced_masks=masks)
    hf_err = []
    for i in range(wl.depth):
        n = wl.batch * wl.widths[i + 1]
        z = net.fetch_z(i)
        np.testing.assert_array_equal(O.pack_mask(O.sign_mask(z)), net.fetch_mask(i))
        assert O.normwise_rel_err(z, zs[i]) <= 2e-5, f"layer {i}: pre-activations"
        h = net.fetch_h(i)
        assert h.size == n
        assert O.normwise_rel_err(h / wl.loss_scale, ref["h"][i + 1]) <= h_tol, f"layer {i}: Phase-II cotangent"
        if wl.alphas[i] == 0.0:
            np.testing.assert_array_equal(net.fetch_fragments(i), O.compact_fragments(h, masks[i]))
        hf = net.fetch_h_forward(i)
        if wl.alphas[i] == 0.0:
            # restored entries are copies of the Phase-II cotangent
            erased = ~masks[i]
            np.testing.assert_array_equal(hf[erased], h[erased])
        hf_err.append(O.normwise_rel_err(hf / wl.loss_scale, ref["h"][i + 1]))
    assert max(hf_err) <= hf_tol, f"Phase-III cotangent errors per layer: {hf_err}"
    return hf_err
