"""ssnet_degree_reduce_static, the entry point that allocates nothing, against ssnet_degree_reduce:
same output shares, bit for bit, on two calls in a row, the second on a
smaller input (the fixed device array then still holds the first call's messages)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2406_02629_amd import SSNet, binding
from util import field_uniform, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,t,p", [(5, 2, binding.P61), (3, 1, binding.P61), (7, 3, binding.P61), (5, 2, binding.P45)])
def test_static_scratch_call_matches_workspace_call(n, t, p):
    ss = SSNet(n, t, f=13, seed=77, p=p)
    lib, ctx = ss.lib, ss._ctx
    words = (2 * t + 1) * (t + 1) + (t + 1) * n
    limit = binding.STATIC_SCRATCH_BYTES // 8 // words
    for call, count in enumerate([min(20000, limit), 777]):       # several kernels' size classes, then a smaller one
        c = field_uniform((n, count), seed=100 + call) % np.uint64(p)
        d_c = to_dev(c)
        want = ss.degree_reduce(d_c, stream_id=5 + call)          # workspace path (allocates through torch)
        got = torch.full_like(d_c, -1)
        rc = lib.ssnet_degree_reduce_static(ctx, C.c_void_p(d_c.data_ptr()), count, 5 + call, C.c_void_p(got.data_ptr()))
        assert rc == binding.OK, rc
        assert np.array_equal(to_np(got), to_np(want)), (n, t, count)
        # in place
        rc = lib.ssnet_degree_reduce_static(ctx, C.c_void_p(d_c.data_ptr()), count, 5 + call, C.c_void_p(d_c.data_ptr()))
        assert rc == binding.OK
        assert np.array_equal(to_np(d_c), to_np(want))


def test_static_scratch_call_rejects_what_does_not_fit():
    ss = SSNet(5, 2, f=13, seed=1)
    lib, ctx = ss.lib, ss._ctx
    limit = binding.STATIC_SCRATCH_BYTES // 8 // 30
    x = torch.zeros((5, 8), dtype=torch.int64, device="cuda")
    assert lib.ssnet_degree_reduce_static(ctx, C.c_void_p(x.data_ptr()), limit + 1, 0, C.c_void_p(x.data_ptr())) == binding.ESCRATCH
    assert lib.ssnet_degree_reduce_static(ctx, None, 8, 0, C.c_void_p(x.data_ptr())) == binding.EINVAL
    assert lib.ssnet_degree_reduce_static(ctx, C.c_void_p(x.data_ptr()), 0, 0, C.c_void_p(x.data_ptr())) == binding.EINVAL
