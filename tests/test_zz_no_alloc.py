"""bs_stack_run_static -- the entry point for callers that cannot allocate -- against
bs_stack_run, through the C ABI.

The stacks here split into several sequences, so both entry points pass intermediate tensors
through a workspace: the caller's buffer for bs_stack_run, the library's static device array
for bs_stack_run_static.  Same kernels, same launch order: outputs and argmax indices must be
bit-identical (and are also held against the CPU oracle).  Two calls in a row, the second on a
smaller input, share the array.
"""
import numpy as np
import pytest
import torch

from oracle import breadth_first as bf
from paper_1804_08378_amd import brainslug as bs
from paper_1804_08378_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _blocks(c, n, seed):
    return sum(([wl.maxpool(3, 1, 1, i % 2 == 0), wl.bn_params(c, seed + i), wl.relu()] for i in range(n)), [])


def _both_entry_points(layers, x, label, **opts):
    print(f"[no-alloc] {label} shape={x.shape} opts={opts}", flush=True)
    st = bs.Stack(layers, x.shape, "f32").plan(**opts)
    info = st.info()
    assert info["n_sequences"] > 1 and info["workspace_bytes"] > 0, "the case must need a workspace"
    assert info["workspace_bytes"] <= bs.bs_static_workspace_capacity()
    xd = torch.from_numpy(x).cuda()
    # reference entry point: caller-owned workspace
    out_a, idx_a = st.alloc_outputs(xd.device)
    ws = torch.empty(info["workspace_bytes"], dtype=torch.uint8, device=xd.device)
    stream = torch.cuda.current_stream().cuda_stream
    bs.bs_stack_run(st.handle, xd.data_ptr(), [], out_a.data_ptr(), [t.data_ptr() for t in idx_a],
                    ws.data_ptr(), ws.numel(), stream)
    # the entry point under test: outputs allocated beforehand, nothing allocated by the call
    out_b, idx_b = st.alloc_outputs(xd.device)
    out_b.fill_(float("nan"))
    for t in idx_b:
        t.fill_(-7)
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    bs.bs_stack_run_static(st.handle, xd.data_ptr(), [], out_b.data_ptr(), [t.data_ptr() for t in idx_b], stream)
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before, "the call changed the device's free memory"
    a, b = out_a.cpu().numpy(), out_b.cpu().numpy()
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), label
    assert len(idx_a) == len(idx_b) > 0
    for p, q in zip(idx_a, idx_b):
        assert np.array_equal(p.cpu().numpy(), q.cpu().numpy()), label
    ref, ref_idx, _ = bf.run_stack(layers, x, [], "f32")
    assert np.array_equal(b.view(np.uint32), ref.view(np.uint32)), label
    for q, r in zip(idx_b, ref_idx):
        assert np.array_equal(q.cpu().numpy(), r), label
    st.close()


def test_static_workspace_matches_caller_workspace_on_two_calls_in_a_row():
    assert bs.bs_static_workspace_capacity() == 64 << 20
    # first call: 8 x 16 x 56 x 56 float32 through six one-step sequences (1.6 MB per workspace half)
    _both_entry_points(_blocks(16, 6, 300), wl.activation((8, 16, 56, 56), 11), "large", max_steps_per_sequence=1)
    # second call, smaller and ragged, on the array the first call left behind
    _both_entry_points(_blocks(4, 5, 320), wl.activation((2, 4, 33, 29), 12), "small", max_steps_per_sequence=1)
    # and a third with multi-step (LDS) sequences cut by a small on-chip budget
    _both_entry_points(_blocks(4, 9, 340), wl.activation((3, 4, 40, 36), 13), "lds", max_lds_bytes=8192)


def test_static_workspace_refuses_what_does_not_fit():
    layers = _blocks(64, 3, 360)
    shape = (64, 64, 56, 56)  # 51 MB per workspace half: more than the array holds
    st = bs.Stack(layers, shape, "f32").plan(max_steps_per_sequence=1)
    assert st.info()["workspace_bytes"] > bs.bs_static_workspace_capacity()
    x = torch.zeros(shape, device="cuda")
    out, idx = st.alloc_outputs(x.device)
    with pytest.raises(bs.BrainSlugError) as e:
        bs.bs_stack_run_static(st.handle, x.data_ptr(), [], out.data_ptr(), [t.data_ptr() for t in idx],
                               torch.cuda.current_stream().cuda_stream)
    assert e.value.status == bs.STATUS_BY_NAME["BS_ERR_WORKSPACE"]
    st.close()


def test_static_workspace_is_not_needed_by_single_sequence_stacks():
    layers, x, res = wl.inputs_for("tiny", 0, "f32", indices=True)
    st = bs.Stack(layers, x.shape, "f32").plan()
    assert st.info()["workspace_bytes"] == 0
    xd = torch.from_numpy(x).cuda()
    out, idx = st.alloc_outputs(xd.device)
    bs.bs_stack_run_static(st.handle, xd.data_ptr(), [], out.data_ptr(), [t.data_ptr() for t in idx],
                           torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ref, ref_idx, _ = bf.run_stack(layers, x, res, "f32")
    assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    assert np.array_equal(idx[0].cpu().numpy(), ref_idx[0])
    st.close()
