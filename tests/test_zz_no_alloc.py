"""The entry point that allocates nothing (jpgd_decode_static: the workspace is an array inside the library's device
image) against jpgd_decode, through the C ABI: same kernels, so coefficients and pixels must be identical.  Two calls
in a row, the second with a smaller image (the array keeps the first call's contents); sizes beyond the array are
refused before anything is launched."""
import numpy as np
import pytest

import paper_2111_09219_amd as J
from workloads import config_jpeg, encode_jpeg, small_image

pytestmark = pytest.mark.gpu


def _both(data, **cfg):
    import torch
    c = J.Config.make(**cfg)
    batch = J.prepare_batch([data], c)
    batch.d_coef.fill_(-3)
    batch.d_pixels.fill_(7)
    batch.decode()
    torch.cuda.synchronize()
    want_coef = batch.d_coef.clone()
    want_pix = batch.d_pixels.clone()
    batch.d_coef.fill_(-9)
    batch.d_pixels.fill_(7)       # (what a call leaves untouched -- padding, the rest behind a reduced image -- stays equal)
    torch.cuda.synchronize()
    rep = J.jpgd_decode_static(batch.infos[0], batch.d_scans, batch.d_coef, batch.d_pixels, c)
    torch.cuda.synchronize()
    assert torch.equal(batch.d_coef, want_coef), "coefficients differ from jpgd_decode"
    assert torch.equal(batch.d_pixels, want_pix), "pixels differ from jpgd_decode"
    return rep


def test_static_workspace_entry_point_matches_jpgd_decode():
    import torch
    assert torch.cuda.is_available()
    J.jpgd_init()
    J.jpgd_init()                                       # again: harmless
    assert J.jpgd_static_workspace_bytes() == J.STATIC_WORKSPACE_BYTES
    big = config_jpeg(2).data                           # 1920x1088 4:4:4, 738 KB of scan: about 1.6 MB of workspace
    small = encode_jpeg(small_image(7, 120, 168, sigma=9.0), 85, "420", True).data
    rst = encode_jpeg(small_image(8, 200, 333, sigma=12.0), 92, "422", False, restart_interval=5).data
    rep = _both(big)
    assert rep.n_sequences > 16
    _both(small)                                        # right after the large one, in the same array
    _both(rst, subseq_bits=1024)
    _both(big, subseq_bits=1024, flags=J.F_PLANAR)
    _both(small, flags=J.F_SCALE_4)
    # too large for the array: refused, nothing launched
    huge = config_jpeg(3).data
    info = J.jpgd_parse(huge)
    assert J.jpgd_workspace_bytes([info]) > J.STATIC_WORKSPACE_BYTES
    b = J.prepare_batch([huge])
    with pytest.raises(J.JpgdError) as e:
        J.jpgd_decode_static(b.infos[0], b.d_scans, b.d_coef, b.d_pixels, b.cfg)
    assert e.value.name == "WORKSPACE"
    with pytest.raises(J.JpgdError) as e:
        J.jpgd_decode_static(b.infos[0], b.d_scans, b.d_coef, b.d_pixels, J.Config.make(timing_mask=1))
    assert e.value.name == "ARG"
    _both(small)                                        # and the entry point still works after the refusals
