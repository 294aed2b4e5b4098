"""The allocation-free entry point no_sage_layer_bwd_static (workspace in the library's static device array)
against no_sage_layer_bwd with a caller's workspace: same kernels, so the same bits, on two calls in a row, the
second with a smaller input (the array keeps the first call's contents, which must not leak into the second)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import oracle as ora

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def one_case(b, V, E, F, d_out, fanouts, B, seed, relu):
    src, dst = si.rmat_edges(V, E, seed)
    og = ora.build_csr(src, dst, V)
    seeds = si.train_split(V, 0.65, seed)[:B]
    blk = ora.sample_blocks(og, seeds, fanouts, seed, 0).blocks[-1]
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((blk.n_src, F)).astype(np.float32)
    (w_self, w_neigh, bias), = si.init_weights([F, d_out], seed)
    n_dst, n_src = blk.n_dst, blk.n_src
    cap_dst, cap_src = n_dst + 5, n_src + 9
    view = b.block_view_from_tensors(dev(np.array([n_dst], np.int32)), dev(np.array([n_src], np.int32)),
                                     dev(np.concatenate([blk.indptr, np.zeros(5, np.int32)])), dev(blk.indices), cap_dst,
                                     cap_src, dev(np.concatenate([blk.csc_indptr, np.zeros(9, np.int32)])), dev(blk.csc_dst))
    o_mean, o_h = ora.sage_layer_fwd(blk, x, w_self, w_neigh, bias, relu)
    xs, tws, twn = dev(x), dev(w_self), dev(w_neigh)
    hh = torch.zeros((cap_dst, d_out), device="cuda")
    hh[:n_dst] = dev(o_h.astype(np.float32))
    mm = torch.zeros((cap_dst, F), device="cuda")
    mm[:n_dst] = dev(o_mean.astype(np.float32))
    gh = torch.zeros((cap_dst, d_out), device="cuda")
    grad_h = rng.standard_normal((n_dst, d_out)).astype(np.float32)
    gh[:n_dst] = dev(grad_h)
    need = b.no_sage_layer_ws_bytes(cap_dst, cap_src, F, d_out)
    assert need <= b.NO_LAYER_STATIC_WS_BYTES
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    outs = []
    for static in (False, True):
        gws = torch.full((F, d_out), 9.0, device="cuda")
        gwn = torch.full((F, d_out), 9.0, device="cuda")
        gb = torch.full((d_out,), 9.0, device="cuda")
        gx = torch.full((cap_src, F), 3.0, device="cuda")
        if static:
            b.no_sage_layer_bwd_static(view, xs, mm, hh, gh, tws, twn, relu, gws, gwn, gb, gx)
        else:
            b.no_sage_layer_bwd(view, xs, mm, hh, gh, tws, twn, relu, gws, gwn, gb, gx, ws)
        torch.cuda.synchronize()
        outs.append((gws, gwn, gb, gx))
    for a, c in zip(*outs):
        assert torch.equal(a, c)
    # and against the oracle, to the tolerance of the layer tests
    r = ora.sage_layer_bwd(blk, x, o_mean.astype(np.float32), o_h.astype(np.float32), grad_h, w_self, w_neigh, relu, True)
    for got, ref in zip(outs[1], r):
        got = got.cpu().numpy().astype(np.float64)[: ref.shape[0]]
        assert np.all(np.abs(got - ref) <= 1e-4 * np.abs(ref) + 1e-4 * np.abs(ref).max())
    return need


def test_static_workspace_backward_matches_the_workspace_form_twice():
    from paper_2311_13225_amd import binding as b
    print("first call: 602 -> 256 over ~3000 destinations", flush=True)
    big = one_case(b, 6000, 90_000, 602, 256, (8, 6), 400, 21, True)
    print("second call: smaller input, 100 -> 47", flush=True)
    small = one_case(b, 3000, 30_000, 100, 47, (5, 4), 100, 22, False)
    assert small < big


def test_static_workspace_rejects_a_layer_that_does_not_fit():
    from paper_2311_13225_amd import binding as b
    n0 = dev(np.array([0], np.int32))
    cap = 200_000
    assert b.no_sage_layer_ws_bytes(cap, cap, 602, 256) > b.NO_LAYER_STATIC_WS_BYTES
    view = b.block_view_from_tensors(n0, n0, torch.zeros(cap + 1, dtype=torch.int32, device="cuda"),
                                     torch.zeros(4, dtype=torch.int32, device="cuda"), cap, cap)
    x = torch.zeros((4, 602), device="cuda")
    w = torch.zeros((602, 256), device="cuda")
    g = torch.zeros((602, 256), device="cuda")
    gb = torch.zeros(256, device="cuda")
    with pytest.raises(b.NoError) as ei:
        b.no_sage_layer_bwd_static(view, x, x, x, x, w, w, True, g, g, gb, None)
    assert ei.value.code == -3
