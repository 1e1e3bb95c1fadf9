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
    """Device snapshot -> (ids, dist_bits, flags, deg) numpy, padded slots normalised."""
    import paper_2310_20419_amd as rn
    d = deg.cpu().numpy()
    ids, bits, flags = rn.unpack_keys(keys.cpu().numpy().view(np.uint64), d)
    return ids, bits, flags, d


def assert_snapshot_equal(snap, is_float, keys, deg, what=""):
    ids, bits, flags, d = device_to_arrays(keys, deg)
    assert (d == snap.deg).all(), "%s: degrees differ at %s" % (what, np.nonzero(d != snap.deg)[0][:10])
    bad = np.nonzero((ids != snap.ids).any(1))[0]
    assert bad.size == 0, "%s: ids differ in %d rows, first %d:\n gpu %s\n orc %s" % (
        what, bad.size, bad[0], ids[bad[0]], snap.ids[bad[0]])
    want_bits = dist_bits_of(snap.dist, is_float)
    valid = np.arange(ids.shape[1])[None, :] < d[:, None]
    assert (bits[valid] == want_bits[valid]).all(), "%s: distances differ" % what
    assert (flags[valid] == snap.flags[valid]).all(), "%s: flags differ" % what
