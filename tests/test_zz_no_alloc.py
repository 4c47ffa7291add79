"""The entry point that allocates nothing (haq_moe_w8a8_ffn_static): same bits as haq_moe_w8a8_ffn with a
caller workspace, on two calls in a row that share the library's built-in scratch array, the second with
a smaller input; and a problem beyond the array's size is refused on the host."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import paper_2508_07329_amd as haq
from paper_2508_07329_amd import binding
from tests import offline
from tests.gpu_util import bits_equal, dev, diff_report, host, upload_experts

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    H, I, E = 256, 1024, 8
    big = offline.small_moe(seed=91, T=200, H=H, I=I, E=E)      # grouped tiled GEMMs
    small = offline.small_moe(seed=92, T=7, H=H, I=I, E=E)      # weight-streaming kernels, fewer rows
    for m in (big, small):                                        # in this order: the second call finds the
        experts = upload_experts(m["experts"])                    # scratch as the larger first one left it
        X, logits, s_in = dev(m["X"]), dev(m["logits"]), dev(m["s_in"])
        ref = haq.haq_moe_w8a8_ffn(X, logits, s_in, experts, I)
        out = torch.zeros_like(ref)
        haq.haq_moe_w8a8_ffn_static(X, logits, s_in, experts, I, out=out)
        torch.cuda.synchronize()
        assert bits_equal(host(out), host(ref)), diff_report(host(out), host(ref))
        idx, gw = oracle.route_top2(m["logits"])
        assert bits_equal(host(out), oracle.moe_ffn(m["X"], idx, gw, m["s_in"], m["experts"]))
    # beyond the built-in array: refused on the host with the size it would have needed
    L = haq.lib()
    one = C.c_void_p(16)
    descs = (binding._ExpertDesc * 8)()
    rc = L.haq_moe_w8a8_ffn_static(one, C.c_int64(4096), one, C.c_int64(8), None, descs, 4096, 4096, 14336, 8, 2, one,
                                   C.c_int64(4096), None)
    assert rc == -3 and "built-in array" in L.haq_last_error().decode()
