"""Helpers of the GPU parity tests: move oracle-side numpy data to the device and back.

The packed device buffers fed to the library are produced from oracle levels by the oracle's own
packer; results coming back are unpacked by the oracle's unpacker.  Nothing here comes from the
HIP path.
"""
import numpy as np
import torch

from oracle import vqo
from paper_2504_18547_amd import vitq
from tests.oracle_cases import preln_case, quantized_weights  # noqa: F401  (re-exported for the GPU tests)


def storage_of(bits):
    """Smallest storage field (2, 4 or 8 bits) that holds b-bit levels."""
    return 2 if bits <= 2 else (4 if bits <= 4 else 8)


def to_qmat(levels, bits, storage_bits=None, row_stride=None):
    """numpy int8 (signed) or uint8 (unsigned) levels -> packed QMat on the GPU."""
    sb = storage_bits if storage_bits is not None else storage_of(bits)
    packed = vqo.pack(levels, sb, row_stride=row_stride)
    t = torch.from_numpy(packed).cuda()
    return vitq.QMat(t, levels.shape[1], bits, sb, unsigned=(levels.dtype == np.uint8))


def from_qmat(m):
    return vqo.unpack(m.data.cpu().numpy(), m.cols, m.storage_bits, unsigned=m.unsigned)


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def device_weights(wts, bits_w, prepack=False):
    """prepack: also make the expanded int8 copies (wp_*) with vq_prepack_weight, as bench.py does."""
    out = {}
    for k, v in wts.items():
        out[k] = to_qmat(v, bits_w) if k.startswith("w_") else dev(v)
    if prepack and storage_of(bits_w) in (2, 4):
        for k in [k for k in out if k.startswith("w_")]:
            out["wp_" + k[2:]] = vitq.vq_prepack_weight(out[k])
    return out


def assert_fp32_close(got, want, what=""):
    """The fp32 tolerance of the target: 1e-5 relative, 1e-6 absolute."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    err = np.abs(got - want)
    tol = 1e-5 * np.abs(want) + 1e-6
    bad = err > tol
    assert not bad.any(), "%s: %d of %d outside tolerance, worst %g" % (what, bad.sum(), bad.size, err.max())
