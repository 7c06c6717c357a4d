"""Host <-> device plumbing for the GPU parity tests (no arithmetic of the method)."""
import numpy as np
import torch

from paper_1910_00932_amd import binding as B

TDT = {"f32": torch.float32, "bf16": torch.bfloat16}
CDT = {"f32": B.TSM_F32, "bf16": B.TSM_BF16}
CLAY = {"ntchw": B.TSM_NTCHW, "nthwc": B.TSM_NTHWC}
TOL = {"f32": 1e-4, "bf16": 2e-2}   # relative L2 against the fp64 oracle (spec tolerances)


def to_dev(a, dtype, layout="ntchw"):
    """numpy [N,T,C,H,W] -> contiguous CUDA tensor in the requested memory order."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if layout == "nthwc":
        t = t.permute(0, 1, 3, 4, 2).contiguous()
    return t.to(TDT[dtype]).cuda()


def from_dev(t, layout="ntchw"):
    """CUDA tensor written in `layout` (viewed as [N,T,C,H,W] or [N,T,H,W,C]) -> float64 numpy [N,T,C,H,W]."""
    a = t.float().cpu().numpy().astype(np.float64)
    if layout == "nthwc":
        a = np.transpose(a, (0, 1, 4, 2, 3))
    return np.ascontiguousarray(a)


def empty_act(shape_ntchw, dtype, layout):
    N, T, C, H, W = shape_ntchw
    shp = (N, T, C, H, W) if layout == "ntchw" else (N, T, H, W, C)
    return torch.empty(shp, dtype=TDT[dtype], device="cuda")


def dev_vec(a, dtype="f32"):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(TDT[dtype]).cuda()


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device="cuda")


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / (nb if nb > 0 else 1.0))


# Element-wise bounds |a - b| <= atol_rel * rms(b) + rtol * |b| per storage type.  A bf16 result is an fp32 sum
# rounded once (2^-9 relative); the bound leaves a factor of two and an absolute term for values that cancel.
ELEM = {"f32": dict(rtol=1e-4, atol_rel=1e-4), "bf16": dict(rtol=2.0 ** -8, atol_rel=2.0 ** -8)}


def compare_local(a, b, tol, what, rows=None, tile=256, rtol=None, atol_rel=None, local_factor=1.0, max_outliers=0,
                  part_outliers=0.0, part_cap=None):
    """Parity of `a` (HIP path) with `b` (oracle) that can see a localised error, which one relative L2 norm over
    a whole tensor cannot (a wrong tile edge or clip-end frame is a fraction of a per cent of the energy):

      * relative L2 over the whole tensor < tol;
      * relative L2 of every slice along the first axis (frame, output channel of a weight gradient, ...) and of
        every block of `tile` consecutive rows of the row view < local_factor * tol, each against the larger of
        the oracle's norm on that part and a quarter of the share of the whole norm the part would have if the
        energy were spread evenly (so that a part that is zero in the oracle does not divide by zero);
        With part_outliers > 0 that fraction of the parts may lie above the bound as long as none exceeds
        part_cap * tol: a single ReLU decision that the two sides take differently (a value that rounds to either
        side of zero) moves one output channel's row of a weight gradient by a few per cent when the channel has
        only a few hundred pixels, while a wrong tile puts many neighbouring parts far out;
      * element-wise |a - b| <= atol_rel * rms(b) + rtol * |b| (skipped when rtol is None), at most
        `max_outliers` elements outside.

    a, b: arrays of equal shape, first axis = the slices; `rows` = an (R, C) view given as a (a_rows, b_rows)
    pair of arrays in the memory order the kernel tiles (channels-innermost pixel rows), or None to skip the tile
    check.  Returns the measured figures."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (what, a.shape, b.shape)
    nb = float(np.linalg.norm(b))
    out = {"l2": rel_l2(a, b)}
    assert out["l2"] < tol, (what, "whole tensor", out["l2"], tol)

    def parts_err(pa, pb):   # pa, pb: [parts, elements]
        floor = 0.25 * nb / np.sqrt(pa.shape[0])
        den = np.maximum(np.linalg.norm(pb, axis=1), floor if floor > 0 else 1.0)
        return np.linalg.norm(pa - pb, axis=1) / den

    def parts_ok(e, kind, n):
        over = int((e >= local_factor * tol).sum())
        allowed = int(part_outliers * n)
        assert over <= allowed, (what, "%d of %d %ss above %g (allowed %d); worst %s %d: %g"
                                 % (over, n, kind, local_factor * tol, allowed, kind, int(e.argmax()), float(e.max())))
        if part_cap is not None:
            assert float(e.max()) < part_cap * tol, (what, "%s %d" % (kind, int(e.argmax())), float(e.max()), part_cap * tol)

    if a.ndim >= 2 and a.shape[0] > 1:
        e = parts_err(a.reshape(a.shape[0], -1), b.reshape(b.shape[0], -1))
        out["slice_max"], out["slice_at"] = float(e.max()), int(e.argmax())
        parts_ok(e, "slice", a.shape[0])
    if rows is not None:
        ra, rb = (np.asarray(r, dtype=np.float64) for r in rows)
        R, C = ra.shape
        nt = (R + tile - 1) // tile
        pad = nt * tile - R
        if pad:
            ra = np.concatenate([ra, np.zeros((pad, C))])
            rb = np.concatenate([rb, np.zeros((pad, C))])
        e = parts_err(ra.reshape(nt, -1), rb.reshape(nt, -1))
        out["tile_max"], out["tile_at"] = float(e.max()), int(e.argmax())
        parts_ok(e, "tile of %d rows" % tile, nt)
    if rtol is not None:
        rms = nb / np.sqrt(max(b.size, 1))
        excess = np.abs(a - b) - (atol_rel * rms + rtol * np.abs(b))
        out["elem_worst"] = float((np.abs(a - b) / (atol_rel * rms + rtol * np.abs(b) + 1e-300)).max())
        nbad = int((excess > 0).sum())
        out["elem_outliers"] = nbad
        assert nbad <= max_outliers, (what, "element-wise", nbad, "outside; worst at",
                                     np.unravel_index(int(excess.argmax()), a.shape), out["elem_worst"])
    return out


def act_rows(a_ntchw):
    """[N,T,C,H,W] -> the (N*T*H*W, C) row view the kernels tile."""
    a = np.asarray(a_ntchw)
    N, T, C, H, W = a.shape
    return np.ascontiguousarray(np.transpose(a, (0, 1, 3, 4, 2))).reshape(-1, C)


def compare_act(a, b, tol, what, dtype, elem=True, **kw):
    """compare_local for activation tensors [N,T,C,H,W]: slices = frames, tiles = 256 pixel rows."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    N, T = a.shape[:2]
    e = ELEM[dtype] if elem else dict(rtol=None, atol_rel=None)
    e = dict(e)
    e.update(kw)
    return compare_local(a.reshape((N * T,) + a.shape[2:]), b.reshape((N * T,) + b.shape[2:]), tol, what,
                         rows=(act_rows(a), act_rows(b)), **e)
