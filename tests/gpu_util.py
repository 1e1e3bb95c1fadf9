"""Helpers shared by the GPU parity tests: oracle snapshot <-> device snapshot conversion."""
import numpy as np


def dist_bits_of(dist, is_float):
    """Oracle distances (float64 holding exact ints or float32 values) -> the 32 key bits."""
    if is_float:
        return dist.astype(np.float32).view(np.uint32)
    return dist.astype(np.int64).astype(np.uint32)


def snapshot_to_device(snap, is_float, R):
    """oracle.Snapshot -> (keys int64-typed cuda tensor [N,R], deg int32 cuda tensor)."""
    import torch
    import paper_2310_20419_amd as rn
    assert snap.ids.shape[1] == R
    keys = rn.pack_keys(snap.ids, dist_bits_of(snap.dist, is_float), snap.flags, snap.deg)
    return (torch.from_numpy(keys.view(np.int64)).cuda(), torch.from_numpy(snap.deg.copy()).cuda())


def device_to_arrays(keys, deg):
    """Device snapshot -> (ids, dist_bits, flags, deg) numpy, padded slots normalised (-1, 0, 0).  Large
    snapshots are unpacked on the device first (plain tensor bit operations: test tooling, three small copies
    instead of one large one); the packing itself is pinned by tests/test_abi.py on the host."""
    import torch
    import paper_2310_20419_amd as rn
    d = deg.cpu().numpy()
    if keys.numel() < (1 << 22):
        ids, bits, flags = rn.unpack_keys(keys.cpu().numpy().view(np.uint64), d)
        return ids, bits, flags, d
    W = keys.shape[1]
    pad = torch.arange(W, device=keys.device)[None, :] >= deg[:, None]
    ids = ((keys >> 1) & 0x7FFFFFFF).to(torch.int32).masked_fill_(pad, -1).cpu().numpy()
    bits = ((keys >> 32) & 0xFFFFFFFF).masked_fill_(pad, 0).to(torch.uint32).cpu().numpy() \
        if hasattr(torch, "uint32") else None
    if bits is None or bits.dtype != np.uint32:
        bits = ((keys >> 32) & 0xFFFFFFFF).masked_fill_(pad, 0).cpu().numpy().astype(np.uint32)
    flags = (keys & 1).to(torch.uint8).masked_fill_(pad, 0).cpu().numpy()
    return ids, bits, flags, d


FLOAT_REL_TOL = 1e-5      # stated bar for float data: distances within 1e-5 relative ...
FLOAT_EDGE_SHARE = 0.99   # ... and at least 99 % of the edges equal to the oracle's


def float_bar_report(snap, ids, bits, d, what):
    """The stated bar for float data, evaluated on a pair of graphs that are not bit-identical: share of the
    oracle's edges the GPU graph holds, and the largest relative difference of the distances stored with the
    edges both hold.  (The two sides round the same real number to float, but sum in different orders -- the
    oracle in index order, the GPU in 8 strided lanes joined by a fixed tree -- so the doubles they round can
    differ in their last bits, and with them, rarely, the float.)"""
    n, W = ids.shape
    base = np.arange(n, dtype=np.int64)[:, None] * (2 ** 31)
    valid_g = np.arange(W)[None, :] < d[:, None]
    valid_o = np.arange(W)[None, :] < snap.deg[:, None]
    code_g = (base + ids)[valid_g]
    code_o = (base + snap.ids)[valid_o]
    dist_g = bits[valid_g].view(np.float32).astype(np.float64)
    dist_o = snap.dist[valid_o]
    og, oo = np.argsort(code_g, kind="stable"), np.argsort(code_o, kind="stable")
    code_g, dist_g, code_o, dist_o = code_g[og], dist_g[og], code_o[oo], dist_o[oo]
    pos = np.searchsorted(code_g, code_o)
    pos[pos >= len(code_g)] = len(code_g) - 1 if len(code_g) else 0
    hit = code_g[pos] == code_o if len(code_g) else np.zeros(len(code_o), bool)
    share = hit.sum() / max(1, max(len(code_o), len(code_g)))
    rel = np.abs(dist_g[pos[hit]] - dist_o[hit]) / np.maximum(dist_o[hit], 1e-300)
    worst = float(rel.max()) if rel.size else 0.0
    print("%s: not bit-identical: %d of %d oracle edges present (share %.6f), %d distances differ, worst relative "
          "difference %.3g" % (what, hit.sum(), len(code_o), share, int((rel > 0).sum()), worst), flush=True)
    return share, worst


def assert_snapshot_equal(snap, is_float, keys, deg, what="", float_bar=None):
    """Bit-exact comparison of a device snapshot with the oracle's.  Integer data: always exact.  Float data
    (float_bar defaults to is_float): a mismatch is counted and printed, and the test fails only if the stated
    bar (distances within 1e-5 relative, at least 99 % of the edges) is missed as well."""
    ids, bits, flags, d = device_to_arrays(keys, deg)
    want_bits = dist_bits_of(snap.dist, is_float)
    valid = np.arange(ids.shape[1])[None, :] < d[:, None]
    same_deg = (d == snap.deg).all()
    exact = same_deg and (ids == snap.ids).all() and (bits[valid] == want_bits[valid]).all() and \
        (flags[valid] == snap.flags[valid]).all()
    if exact:
        return True
    if float_bar is None:
        float_bar = is_float
    if float_bar:
        share, worst = float_bar_report(snap, ids, bits, d, what)
        assert share >= FLOAT_EDGE_SHARE and worst <= FLOAT_REL_TOL, \
            "%s: float bar missed (edge share %.6f, worst relative distance difference %.3g)" % (what, share, worst)
        return False
    assert same_deg, "%s: degrees differ at %s" % (what, np.nonzero(d != snap.deg)[0][:10])
    bad = np.nonzero((ids != snap.ids).any(1))[0]
    assert bad.size == 0, "%s: ids differ in %d rows, first %d:\n gpu %s\n orc %s" % (
        what, bad.size, bad[0], ids[bad[0]], snap.ids[bad[0]])
    assert (bits[valid] == want_bits[valid]).all(), "%s: distances differ" % what
    assert (flags[valid] == snap.flags[valid]).all(), "%s: flags differ" % what
    return True
