"""GPU parity of max-pool, transposed conv, head and the swap engine, through the C-ABI."""
import ctypes

import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ pool
@pytest.mark.parametrize("shape,dt", [((1, 8, 8, 8, 32), "bf16"), ((2, 6, 4, 10, 8), "bf16"), ((1, 4, 6, 2, 3), "bf16"),
                                      ((1, 4, 4, 4, 8), "f32"), ((2, 2, 6, 4, 5), "f32")])
def test_pool_fwd_bwd_exact(orc, shape, dt):
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty
    N, D, H, W, C = shape
    x = synth.activations(50, shape, dt)
    x[x < 0] = 0.0                           # post-ReLU statistics: many exact ties at zero
    x = np.round(x * 4) / 4 if dt == "bf16" else x   # and ties among positive values
    dy = synth.activations(51, (N, D // 2, H // 2, W // 2, C), dt)
    add = synth.activations(52, shape, dt)
    xd, dyd, addd = to_dev(x, dt), to_dev(dy, dt), to_dev(add, dt)
    y = empty((N, D // 2, H // 2, W // 2, C), dt)
    k3.pool3d_fwd(xd, y)
    dx = empty(shape, dt)
    k3.pool3d_bwd(xd, dyd, None, dx)
    dx2 = empty(shape, dt)
    k3.pool3d_bwd(xd, dyd, addd, dx2)
    dx3 = empty(shape, dt)
    k3.pool3d_bwd(xd, dyd, addd, dx3, relu_mask=True)
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(y), orc.pool3d_fwd(x.astype(np.float64)))
    ref = orc.pool3d_bwd(x.astype(np.float64), dy.astype(np.float64))
    assert np.array_equal(to_f64(dx), ref)
    ref2 = ref + add.astype(np.float64)
    ref3 = orc.relu_bwd(ref2, x.astype(np.float64))     # producer-side ReLU mask of x
    if dt == "bf16":
        assert np.array_equal(to_f64(dx2), orc.round_bf16(ref2))
        assert np.array_equal(to_f64(dx3), orc.round_bf16(ref3))
    else:
        np.testing.assert_allclose(to_f64(dx2), ref2, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(to_f64(dx3), ref3, rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("shape", [(1, 8, 8, 8, 32), (2, 6, 4, 10, 16), (1, 2, 2, 2, 48), (1, 20, 12, 36, 64), (3, 4, 2, 6, 128)])
def test_pool_with_route_bits_is_bit_exact(orc, shape):
    """Forward with routing bits, backward from the bits alone: y, the bits and dx equal the oracle's
    element for element, and dx equals what the x-reading backward pass with the ReLU mask gives."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty
    N, D, H, W, C = shape
    x = synth.activations(53, shape, "bf16")
    x[x < 0] = 0.0                           # post-ReLU statistics: windows that are all zero, ties at zero
    x = np.round(x * 4) / 4                  # and ties among positive values
    dy = synth.activations(54, (N, D // 2, H // 2, W // 2, C), "bf16")
    xd, dyd = to_dev(x, "bf16"), to_dev(dy, "bf16")
    y = empty((N, D // 2, H // 2, W // 2, C), "bf16")
    assert k3.relu_bits_bytes(xd) == x.size // 8
    bits = torch.full((N, D, H, W, C // 16), 0x5555, device="cuda", dtype=torch.int16)
    k3.pool3d_fwd_bits(xd, y, bits)
    dx = torch.full_like(xd, 7.0)
    k3.pool3d_bwd_bits(bits, dyd, dx)
    dx_ref = empty(shape, "bf16")
    k3.pool3d_bwd(xd, dyd, None, dx_ref, relu_mask=True)
    torch.cuda.synchronize()
    x64, dy64 = x.astype(np.float64), dy.astype(np.float64)
    assert np.array_equal(to_f64(y), orc.pool3d_fwd(x64))
    ref_bits = orc.pool3d_route_bits(x64)
    assert np.array_equal(bits.cpu().numpy().view(np.uint16), ref_bits)
    assert np.array_equal(to_f64(dx), orc.pool3d_bwd_bits(ref_bits, dy64))
    assert np.array_equal(to_f64(dx), orc.relu_bwd(orc.pool3d_bwd(x64, dy64), x64))
    assert torch.equal(dx, dx_ref)


def test_pool_with_route_bits_rejects_what_it_does_not_serve():
    from paper_1811_12174_amd import k3
    from gpu_util import empty
    import torch
    bits = torch.zeros(64, device="cuda", dtype=torch.int16)
    with pytest.raises(k3.K3Error) as e:      # 8 channels: no whole 16-channel word
        k3.pool3d_fwd_bits(empty((1, 4, 4, 4, 8), "bf16"), empty((1, 2, 2, 2, 8), "bf16"), bits)
    assert e.value.status == k3.E_UNSUPPORTED
    with pytest.raises(k3.K3Error) as e:      # fp32
        k3.pool3d_fwd_bits(empty((1, 4, 4, 4, 16), "f32"), empty((1, 2, 2, 2, 16), "f32"), bits)
    assert e.value.status == k3.E_UNSUPPORTED
    with pytest.raises(k3.K3Error) as e:
        k3.pool3d_bwd_bits(bits, empty((1, 2, 2, 3, 16), "bf16"), empty((1, 4, 4, 4, 16), "bf16"))
    assert e.value.status == k3.E_SHAPE
    with pytest.raises(k3.K3Error) as e:
        k3.pool3d_bwd_bits(None, empty((1, 2, 2, 2, 16), "bf16"), empty((1, 4, 4, 4, 16), "bf16"))
    assert e.value.status == k3.E_BADARG


def test_pool_odd_dim_is_rejected():
    from paper_1811_12174_amd import k3
    from gpu_util import empty
    with pytest.raises(k3.K3Error) as e:
        k3.pool3d_fwd(empty((1, 3, 4, 4, 8), "bf16"), empty((1, 1, 2, 2, 8), "bf16"))
    assert e.value.status == k3.E_SHAPE


# ------------------------------------------------------------------ upconv
UP_CASES = [((1, 3, 4, 5), 3, 5, "f32"), ((2, 2, 2, 2), 8, 4, "bf16"), ((1, 4, 4, 8), 64, 32, "bf16"),
            ((2, 5, 3, 7), 32, 32, "bf16"), ((1, 6, 5, 9), 128, 64, "bf16"), ((1, 2, 2, 2), 256, 128, "bf16"),
            ((1, 12, 10, 22), 64, 64, "bf16"), ((2, 9, 8, 8), 128, 32, "bf16"), ((1, 2, 2, 3), 512, 256, "bf16")]


def _up_packed(w):
    import torch
    from paper_1811_12174_amd import k3
    nb = k3.upconv3d_packed_bytes(w.shape[3], w.shape[4], k3.BF16 if w.dtype == torch.bfloat16 else k3.F32)
    if nb == 0:
        return None
    p = torch.empty(nb, device="cuda", dtype=torch.uint8)
    k3.upconv3d_pack_weights(w, p)
    return p


@pytest.mark.parametrize("sp,ci,co,dt", UP_CASES)
def test_upconv_all_passes(orc, sp, ci, co, dt):
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, rel_l2, TOL
    N, D, H, W = sp
    x = synth.activations(60, (N, D, H, W, ci), dt)
    w = synth.upconv_weights(61, ci, co, dt)
    b = (synth.normal(synth.SEED, 62, (co,), np.float64) * 0.5).astype(np.float32)
    dy = synth.activations(63, (N, 2 * D, 2 * H, 2 * W, co), dt)
    xd, wd, dyd, bd = to_dev(x, dt), to_dev(w, dt), to_dev(dy, dt), torch.from_numpy(b).cuda()
    pk = _up_packed(wd)
    y = empty((N, 2 * D, 2 * H, 2 * W, co), dt)
    y.fill_(float("nan"))
    k3.upconv3d_fwd(xd, wd, pk, bd, y)
    dx = empty((N, D, H, W, ci), dt)
    dx.fill_(float("nan"))
    k3.upconv3d_bwd_data(dyd, wd, pk, dx)
    om = synth.activations(64, (N, D, H, W, ci), dt)
    om[om < 0.2] = 0.0
    dxm = empty((N, D, H, W, ci), dt)
    k3.upconv3d_bwd_data(dyd, wd, pk, dxm, dx_mask=to_dev(om, dt))
    dW = torch.full((2, 2, 2, ci, co), float("nan"), device="cuda")
    db = torch.full((co,), float("nan"), device="cuda")
    ws = torch.empty(max(1, k3.upconv3d_bwd_weight_workspace_bytes(xd, dyd)), device="cuda", dtype=torch.uint8)
    k3.upconv3d_bwd_weight(xd, dyd, dW, db, ws)
    torch.cuda.synchronize()
    x64, w64, dy64 = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
    e = rel_l2(to_f64(y), orc.upconv3d_fwd(x64, w64, b.astype(np.float64)))
    assert e < TOL[dt] and (dt != "bf16" or e < 4e-3), e
    rdx = orc.upconv3d_bwd_data(dy64, w64)
    e = rel_l2(to_f64(dx), rdx)
    assert e < TOL[dt] and (dt != "bf16" or e < 4e-3), e
    e = rel_l2(to_f64(dxm), orc.relu_bwd(rdx, om.astype(np.float64)))
    assert e < TOL[dt] and (dt != "bf16" or e < 4e-3), e
    assert np.all(to_f64(dxm)[om <= 0] == 0)
    rW, rb = orc.upconv3d_bwd_weight(x64, dy64)
    assert rel_l2(to_f64(dW), rW) < 1e-5
    assert rel_l2(to_f64(db), rb) < 1e-5


# ------------------------------------------------------------------ head
@pytest.mark.parametrize("sp,C,dt", [((1, 8, 8, 8), 32, "bf16"), ((2, 5, 7, 9), 64, "bf16"), ((1, 4, 4, 4), 8, "f32"),
                                     ((1, 3, 3, 3), 2, "bf16"), ((1, 16, 16, 17), 32, "bf16"), ((1, 7, 9, 11), 16, "bf16"),
                                     ((2, 6, 5, 9), 128, "bf16"), ((1, 33, 30, 31), 64, "bf16")])
def test_head(orc, sp, C, dt):
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, rel_l2, TOL
    N, D, H, W = sp
    a = synth.activations(70, (N, D, H, W, C), dt)
    wh = synth.head_weights(71, C)
    bh = (synth.normal(synth.SEED, 72, (3,), np.float64) * 0.3).astype(np.float32)
    lab = (synth.uniform(synth.SEED, 73, N * D * H * W) * 3).astype(np.uint8).reshape(N, D, H, W)
    ad = to_dev(a, dt)
    whd, bhd = torch.from_numpy(wh).cuda(), torch.from_numpy(bh).cuda()
    labd = torch.from_numpy(lab).cuda()
    loss = torch.full((1,), float("nan"), device="cuda")
    da = empty(a.shape, dt)
    dW = torch.full((C, 3), float("nan"), device="cuda")
    db = torch.full((3,), float("nan"), device="cuda")
    logits = torch.full((N * D * H * W, 3), float("nan"), device="cuda")
    ws = torch.empty(k3.head_workspace_bytes(ad), device="cuda", dtype=torch.uint8)
    k3.head_softmax_ce_fwd_bwd(ad, whd, bhd, labd, loss, da, dW, db, logits, ws)
    dam = empty(a.shape, dt)
    k3.head_softmax_ce_fwd_bwd(ad, whd, bhd, labd, loss, dam, dW, db, logits, ws, relu_mask=True)
    torch.cuda.synchronize()
    ref = orc.head_softmax_ce(a.astype(np.float64), wh.astype(np.float64), bh.astype(np.float64), lab)
    assert abs(loss.item() - ref["loss"]) < 1e-5 * abs(ref["loss"])
    assert rel_l2(to_f64(logits), ref["logits"].reshape(-1, 3)) < 1e-5
    assert rel_l2(to_f64(da), ref["da"]) < TOL[dt]
    assert rel_l2(to_f64(dam), orc.relu_bwd(ref["da"], a.astype(np.float64))) < TOL[dt]
    assert rel_l2(to_f64(dW), ref["dW"]) < 1e-5
    assert np.abs(to_f64(db) - ref["db"]).max() < 1e-5 * max(1e-3, np.abs(ref["db"]).max()) + 1e-7
    # in place (da = a): every output is the one of the separate-buffer call, bit for bit
    for mask, want in ((False, da), (True, dam)):
        k3.head_softmax_ce_fwd_bwd(ad, whd, bhd, labd, loss, empty(a.shape, dt), dW, db, logits, ws, relu_mask=mask)
        inpl = ad.clone()
        loss2, dW2, db2 = torch.full_like(loss, float("nan")), torch.full_like(dW, float("nan")), torch.full_like(db, float("nan"))
        logits2 = torch.full_like(logits, float("nan"))
        k3.head_softmax_ce_fwd_bwd(inpl, whd, bhd, labd, loss2, inpl, dW2, db2, logits2, ws, relu_mask=mask)
        torch.cuda.synchronize()
        assert torch.equal(inpl, want) and torch.equal(loss2, loss) and torch.equal(dW2, dW) and torch.equal(db2, db)
        assert torch.equal(logits2, logits)


# ------------------------------------------------------------------ swap engine
def test_swap_round_trip_is_bit_exact_and_ordered():
    import torch
    from paper_1811_12174_amd import k3
    ctx = k3.lms_create(0)
    n = 8 << 20
    t = torch.randint(-32768, 32767, (n,), device="cuda", dtype=torch.int16)
    orig = t.clone()
    nbytes = n * 2
    host = k3.lms_host_alloc(nbytes)
    try:
        h = k3.lms_swap_out(ctx, t.data_ptr(), nbytes, host)
        assert k3.lms_handle_state(ctx, h) in (k3.LMS_OUT_IN_FLIGHT, k3.LMS_ON_HOST)
        k3.lms_release_after(ctx, h)
        t.fill_(-1)                                   # poison the device block (ordered after the copy)
        k3.lms_prefetch_in(ctx, h, t.data_ptr())
        out = t.clone()                               # consumer on the compute stream
        torch.cuda.synchronize()
        assert torch.equal(out, orig)
        assert k3.lms_handle_state(ctx, h) == k3.LMS_RESIDENT
        hb = (ctypes.c_int16 * 16).from_address(host)
        assert list(hb) == orig[:16].cpu().tolist()
        k3.lms_release(ctx, h)
        st = k3.lms_get_stats(ctx)
        assert st["bytes_out"] == nbytes and st["bytes_in"] == nbytes and st["live_handles"] == 0
    finally:
        k3.lms_sync(ctx)
        k3.lms_host_free(host)
        k3.lms_destroy(ctx)


def test_swap_errors_on_gpu():
    import torch
    from paper_1811_12174_amd import k3
    ctx = k3.lms_create(1 << 20)
    t = torch.zeros(1024, device="cuda", dtype=torch.uint8)
    pageable = np.zeros(1024, dtype=np.uint8)
    try:
        with pytest.raises(k3.K3Error) as e:
            k3.lms_swap_out(ctx, t.data_ptr(), 1024, pageable.ctypes.data)
        assert e.value.status == k3.E_NOT_PINNED
        with pytest.raises(k3.K3Error) as e:
            k3.lms_account_alloc(ctx, 2 << 20)
        assert e.value.status == k3.E_OOM
        with pytest.raises(k3.K3Error) as e:
            k3.lms_prefetch_in(ctx, 0, t.data_ptr())
        assert e.value.status == k3.E_BADARG
    finally:
        k3.lms_destroy(ctx)


def test_copy_busy_time_measurement():
    """With timing on, the engine reports how long each copy stream was busy; off, nothing is counted."""
    import torch
    from paper_1811_12174_amd import k3
    ctx = k3.lms_create(0)
    n = 64 << 20
    t = torch.zeros(n, device="cuda", dtype=torch.uint8)
    host = k3.lms_host_alloc(n)
    try:
        h = k3.lms_swap_out(ctx, t.data_ptr(), n, host)
        k3.lms_sync(ctx)
        assert k3.lms_copy_busy_ms(ctx) == (0.0, 0.0)
        k3.lms_release(ctx, h)
        k3.lms_set_copy_timing(ctx, True)
        for _ in range(3):
            h = k3.lms_swap_out(ctx, t.data_ptr(), n, host)
            k3.lms_release_after(ctx, h)
            k3.lms_prefetch_in(ctx, h, t.data_ptr())
            k3.lms_sync(ctx)
            torch.cuda.synchronize()
            k3.lms_release(ctx, h)
        out_ms, in_ms = k3.lms_copy_busy_ms(ctx)
        # 3 x 64 MiB each way: between 5 and 200 GB/s is a sane link
        for ms in (out_ms, in_ms):
            assert 3 * n / 200e9 * 1e3 < ms < 3 * n / 5e9 * 1e3, (out_ms, in_ms)
        k3.lms_set_copy_timing(ctx, False)
        h = k3.lms_swap_out(ctx, t.data_ptr(), n, host)
        k3.lms_sync(ctx)
        k3.lms_release(ctx, h)
        assert k3.lms_copy_busy_ms(ctx) == (out_ms, in_ms)
    finally:
        k3.lms_host_free(host)
        k3.lms_destroy(ctx)
