"""The entry point that allocates nothing (et_merge_select_static: the compression stage on the
library's static device scratch) against et_merge_select with a caller workspace, through the C
boundary: identical outputs bit for bit, on two calls in a row, the second on a smaller input (the
scratch keeps the first call's contents)."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2605_30010_amd as et
from paper_2605_30010_amd import binding as B
from et_inputs import make_hidden_states, scene_lengths_geometric
from tests._util import bits_to_dev

pytestmark = pytest.mark.gpu


def _outputs(T, L, D):
    bufs = B._alloc_outputs(T, L, D, torch.device("cuda:0"))
    for v in bufs.values():
        v.fill_(-1)                                   # stale contents must not pass for results
    return bufs


def _call_both(bits, tau, keep):
    T, L, D = bits.shape
    x = bits_to_dev(bits)
    lib = et.load_library()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    # the existing entry point, caller workspace
    ws = torch.empty((et.et_merge_workspace_bytes(T, L, D),), dtype=torch.uint8, device="cuda")
    ref_bufs = _outputs(T, L, D)
    o_ref = B._out_struct(ref_bufs)
    rc = lib.et_merge_select(C.c_void_p(x.data_ptr()), T, L, D, tau, keep, C.c_void_p(ws.data_ptr()), ws.numel(),
                             stream, C.byref(o_ref))
    assert rc == 0, et.et_last_error()
    # the new one: inputs and outputs only
    got_bufs = _outputs(T, L, D)
    o_got = B._out_struct(got_bufs)
    rc = lib.et_merge_select_static(C.c_void_p(x.data_ptr()), T, L, D, tau, keep, stream, C.byref(o_got))
    assert rc == 0, et.et_last_error()
    torch.cuda.synchronize()
    assert (o_got.n_frames_out, o_got.n_tokens) == (o_ref.n_frames_out, o_ref.n_tokens)
    n, nt = o_ref.n_frames_out, o_ref.n_tokens
    assert 1 <= n <= T and nt == n * et.et_keep_count(L, keep)
    assert torch.equal(got_bufs["tokens"][:nt].view(torch.int16), ref_bufs["tokens"][:nt].view(torch.int16))
    assert torch.equal(got_bufs["kept_idx"][:nt], ref_bufs["kept_idx"][:nt])
    assert torch.equal(got_bufs["cu_tokens"][:n + 1], ref_bufs["cu_tokens"][:n + 1])
    assert torch.equal(got_bufs["seg_start"][:n + 1], ref_bufs["seg_start"][:n + 1])
    assert torch.equal(got_bufs["frame_sim"][:T - 1], ref_bufs["frame_sim"][:T - 1])
    return n, nt


def test_static_scratch_entry_point_matches_the_workspace_one_twice():
    rng = np.random.default_rng(11)
    big = make_hidden_states(24, 300, 512, scene_lengths_geometric(rng, 24, 4), 71, sigma=0.1)
    small = make_hidden_states(7, 100, 256, scene_lengths_geometric(rng, 7, 3), 72, sigma=0.1)
    n1, _ = _call_both(big, 0.9, 0.3)
    n2, _ = _call_both(small, 0.9, 0.5)          # smaller input right after: the scratch still holds the first call's data
    assert 1 < n1 < 24 and 1 <= n2 <= 7
    # the headline clip's shape fits the static buffer; one frame, too
    c3 = make_hidden_states(32, 729, 1152, scene_lengths_geometric(rng, 32, 4), 73, sigma=0.1)
    _call_both(c3, 0.9, 0.5)
    _call_both(small[:1], 0.9, 0.5)
