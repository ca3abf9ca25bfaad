"""The allocation-free entry point npas_run_stack_static against npas_run_stack: same stack, same inputs, two calls
in a row, the second on a smaller batch (the static workspace keeps the first call's contents)."""
import numpy as np
import pytest

from tests import helpers
from tests.helpers import new_dev, pack_layer, to_dev
from workloads import configs, dtypes

pytestmark = pytest.mark.gpu


def test_static_workspace_entry_point_matches_run_stack(npas):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    flags = npas.STACK_FUSE_POINTWISE | npas.STACK_FUSE_INVERTED_RESIDUAL | npas.STACK_FUSE_CONV_MAXPOOL
    results = []
    w_big = configs.config5(batch=3, HW=64, width=16)
    packed = [pack_layer(npas, L, w_big.dtype) if L.kind in ("conv", "fc", "dwconv") else None for L in w_big.layers]
    st = npas.Stack(helpers.stack_descs(npas, w_big.layers, packed), 64, 64, flags)
    for N in (3, 1):                               # the second call is the smaller one
        print(f"static workspace: batch {N}", flush=True)
        x = to_dev(np.ascontiguousarray(w_big.x_store[:N]), torch)
        wsb = st.workspace_bytes(N)
        assert 0 < wsb <= npas.STATIC_WORKSPACE_BYTES
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        y_ref = new_dev((N, 1000), w_big.dtype, torch, fill=0x7FC1)
        st.run(x, y_ref, N, ws, wsb)
        y = new_dev((N, 1000), w_big.dtype, torch, fill=0x7FC1)
        st.run_static(x, y, N)
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref), f"batch {N}: static-workspace result differs from npas_run_stack's"
        results.append(y.cpu().numpy().copy())
    assert not (results[0].view(np.uint16) == 0x7FC1).any()
    np.testing.assert_array_equal(results[0][:1], results[1])       # image 0 gives the same logits in both calls
    # a stack that does not fit is refused, not truncated
    N_big = npas.STATIC_WORKSPACE_BYTES // st.workspace_bytes(1) + 2
    assert st.workspace_bytes(N_big) > npas.STATIC_WORKSPACE_BYTES
    with pytest.raises(npas.NpasError) as e:
        st.run_static(x, y, N_big)
    assert e.value.code == npas.E_WORKSPACE and "static workspace" in str(e.value)
