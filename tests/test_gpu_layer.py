"""Parity of the whole-layer entry points (hstu_layer_fwd / hstu_layer_bwd, through the C ABI) against the CPU fp64
layer oracle on the same seeded inputs.  bf16 storage of every activation: tolerance 2e-2 on the max error normalised
by the largest reference magnitude, as for the attention kernels."""
import numpy as np
import pytest
import torch

from oracle import layer as lorc
from paper_2602_16986_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-2


@pytest.fixture(scope="module")
def hb():
    assert torch.cuda.is_available(), "GPU tests need a GPU; deselect with -m 'not gpu'"
    from paper_2602_16986_amd import binding
    return binding


def f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def check(name, got, ref, tol=TOL, rms_tol=None):
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    if ref.size == 0:
        return
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    err = np.abs(got - ref).max()
    scale = np.abs(ref).max()
    rel = err / scale if scale > 0 else err
    rms = np.sqrt(np.mean((got - ref) ** 2)) / scale if scale > 0 else 0.0
    print(f"  {name}: max_abs_err={err:.3e} max|ref|={scale:.3e} normalised={rel:.3e} rms={rms:.3e}", flush=True)
    assert rel <= tol, f"{name}: normalised max error {rel:.3e} > {tol}"
    if rms_tol is not None:
        assert rms <= rms_tol, f"{name}: normalised rms error {rms:.3e} > {rms_tol}"


def attn_kw(c):
    return dict(num_targets=c.num_targets, K1=c.K1, K2=c.K2, alpha=c.alpha, inv_n=1.0 / c.N, table=c.table, bounds=c.bounds)


def run_case(c):
    from paper_2602_16986_amd.runner import DeviceLayer
    print(f"layer case {c.name}: lengths={c.lengths.tolist()} H={c.H} d={c.d} E={c.E} K1={c.K1} K2={c.K2} "
          f"targets={None if c.num_targets is None else c.num_targets.tolist()}", flush=True)
    dl = DeviceLayer(c)
    for t in (dl.out, dl.u_saved, dl.attn_saved, dl.dz, dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2):
        t.fill_(float("nan"))
    dl.fwd()
    torch.cuda.synchronize()
    kw = dict(norm_eps=c.eps, gated_eps=c.eps, **attn_kw(c))
    ref_out, s = lorc.layer_fwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, **kw)
    check("out", f64(dl.out), ref_out)
    check("U (saved)", f64(dl.u_saved), s["u"])
    check("A (saved)", f64(dl.attn_saved), s["a"])
    check("mean", f64(dl.mean), s["mean"], 1e-5)
    check("rstd", f64(dl.rstd), s["rstd"], 1e-5)
    dl.bwd()
    torch.cuda.synchronize()
    g = lorc.layer_bwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, c.dout, **kw)
    check("dZ", f64(dl.dz), g["dz"])
    check("d norm_w", f64(dl.d_norm_w), g["d_norm_w"])
    check("d W1", f64(dl.d_w1), g["d_w1"])
    check("d gated_norm_w", f64(dl.d_gated_norm_w), g["d_gated_norm_w"])
    check("d W2", f64(dl.d_w2), g["d_w2"])
    return dl


@pytest.mark.parametrize("name", wl.LAYER_SMALL)
def test_layer_small(hb, name):
    run_case(wl.layer_case(name))


def test_layer_wide_rows(hb):
    """Embedding width and H d above 512: both norms' backward passes share a row among the waves of a workgroup."""
    run_case(wl.build_layer("layer-wide", [70, 0, 33, 129], 8, 128, 1024, seed=3, K1=40, K2=8))


def test_layer_mid(hb):
    """Four sequences of 1024..2048 tokens, H=4, d=128, E=512: the layer shape of the benchmark at a size the oracle
    finishes in seconds."""
    run_case(wl.layer_case("layer-mid"))


@pytest.mark.parametrize("name", ["layer-long", "layer-long-sparse"])
def test_layer_long_sequences_against_the_oracle(hb, name):
    """Two sequences of 8,192 and 4,200 tokens (the first inside the benchmark's length range; 64 and 33 row blocks, cut and
    uncut work items, the pipelined kernels' long tile lists), H=4, d=128, E=512: forward and every gradient of the whole
    layer against the fp64 oracle, dense and under the semi-local mask."""
    run_case(wl.layer_case(name))


def test_layer_backward_twice_is_identical(hb):
    """The backward rebuilds its intermediates from (Z, U, A, statistics) alone: a second call after unrelated work in
    the same workspace returns bit-identical gradients (attention and norms are deterministic, the GEMM plans are fixed)."""
    from paper_2602_16986_amd.runner import DeviceLayer
    dl = DeviceLayer(wl.layer_case("layer-small-sparse-targets"))
    dl.fwd()
    dl.bwd()
    first = [t.clone() for t in (dl.dz, dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2)]
    dl.ws_bwd.fill_(0x5A)
    dl.bwd()
    torch.cuda.synchronize()
    for a, b in zip(first, (dl.dz, dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2)):
        assert torch.equal(a, b)


def test_layer_new_token_count_of_a_known_class_tunes_nothing(hb):
    """The GEMM kernels are chosen once per shape class (layer dimensions, token count rounded up to a power of two).
    A batch with another token count of the same class must not time candidates again (that would block the host on
    every jagged batch), and its results must still match the oracle."""
    run_case(wl.build_layer("class-a", [300, 0, 150, 210], 2, 64, 320, seed=11, K1=64, K2=16))     # T = 660: class 1024
    tuned = hb.hstu_layer_gemm_tunings()
    assert tuned > 0
    run_case(wl.build_layer("class-b", [401, 77, 333], 2, 64, 320, seed=12, K1=64, K2=16))         # T = 811: same class
    assert hb.hstu_layer_gemm_tunings() == tuned
    run_case(wl.build_layer("class-c", [700, 500], 2, 64, 320, seed=13, K1=64, K2=16))             # T = 1200: class 2048
    assert hb.hstu_layer_gemm_tunings() > tuned


def test_layer_empty_batch(hb):
    from paper_2602_16986_amd.runner import DeviceLayer
    dl = DeviceLayer(wl.build_layer("empty", [0, 0], 2, 64, 96))
    for t in (dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2):
        t.fill_(float("nan"))
    dl.fwd()
    dl.bwd()
    torch.cuda.synchronize()
    for t in (dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2):
        assert not t.any()


def test_layer_rejects_fp32_and_small_workspace(hb):
    from paper_2602_16986_amd.runner import DeviceLayer
    dl = DeviceLayer(wl.layer_case("layer-small-dense"))
    with pytest.raises(hb.HstuError):
        hb.hstu_layer_fwd(dl.problem, dl.z, dl.out, dl.u_saved, dl.attn_saved, dl.mean, dl.rstd, dl.ws_fwd[:4096])
    dl.problem.params.attn.dtype = hb.HSTU_FP32
    with pytest.raises(hb.HstuError):
        dl.fwd()


# ----------------------------------------------------------------------------------------------
# the benchmark's configuration (layer-C3: 8 sequences of 8k-16k tokens, H=4, d=128, E=512)
# ----------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def layer_c3(hb):
    from paper_2602_16986_amd.runner import DeviceLayer
    c = wl.layer_case("layer-C3")
    dl = DeviceLayer(c)
    dl.fwd()
    dl.bwd()
    torch.cuda.synchronize()
    return c, dl


def test_layer_full_size_forward_sampled_rows(layer_c3):
    """Output rows of the full-size layer that the oracle computes one by one: the projection is evaluated for every
    token (the sampled queries need all keys and values), attention, gated norm and output projection on the sample."""
    c, dl = layer_c3
    HD = c.H * c.d
    rng = np.random.default_rng(7)
    rows = np.sort(np.concatenate([rng.choice(c.T, size=96, replace=False), c.offsets[:-1], c.offsets[1:] - 1]))
    x, _, _ = lorc.layer_norm_fwd(c.z, c.norm_w, c.eps)
    pre = x @ c.w1.astype(np.float64).T
    act = pre * lorc.sigmoid(pre)
    u, v, q, k = (act[:, i * HD:(i + 1) * HD] for i in range(4))
    shp = (c.T, c.H, c.d)
    from oracle import hstu_oracle as orc
    a = orc.attn_fwd(q.reshape(shp), k.reshape(shp), v.reshape(shp), c.offsets, rows=rows, **attn_kw(c)).reshape(len(rows), HD)
    y, _, _ = orc.gated_norm_fwd(a, u[rows], c.gated_norm_w, None, c.eps)
    ref = y @ c.w2.astype(np.float64).T + c.z[rows].astype(np.float64)
    idx = torch.from_numpy(rows).to(dl.device)
    check("A rows", f64(dl.attn_saved[idx]), a)
    check("U rows", f64(dl.u_saved[idx]), u[rows])
    check("out rows", f64(dl.out[idx]), ref)


def test_layer_full_size_backward_against_composition(hb, layer_c3):
    """At full size the backward is checked against its own steps done separately: the standalone attention and
    gated-norm entry points (each checked against the oracle at this size elsewhere) for those two steps, torch fp32
    on the GPU for the norms, projections and SiLU.  Same inputs, independent arithmetic for everything the layer adds."""
    c, dl = layer_c3
    F = torch.nn.functional
    HD, T = c.H * c.d, c.T
    z32 = dl.z.float().requires_grad_(True)
    nw = dl.norm_w.clone().requires_grad_(True)
    w1 = dl.w1.float().requires_grad_(True)
    xn = F.layer_norm(z32, (c.E,), weight=nw, eps=c.eps)
    pre = xn @ w1.T
    act = F.silu(pre)
    act_bf = act.detach().to(torch.bfloat16)                          # what the kernels see: [T, 4 H d], U V Q K
    y_ref = F.layer_norm(dl.attn_saved.float(), (HD,), weight=dl.gated_norm_w, eps=c.eps) * dl.u_saved.float()
    dout32 = dl.dout.float()
    d_w2_ref = dout32.T @ y_ref
    dy = (dout32 @ dl.w2.float()).to(torch.bfloat16)
    # gated norm backward and attention backward through their own entry points
    dattn, du = torch.empty_like(dy), torch.empty_like(dy)
    dgw = torch.empty(HD, dtype=torch.float32, device=dl.device)
    ws_n = hb.new_workspace(hb.hstu_gated_norm_bwd_workspace_bytes(T, HD), dl.device)
    hb.hstu_gated_norm_bwd(dy, dl.attn_saved, dl.u_saved, dl.gated_norm_w, None, c.eps, dattn, du, dgw, None, ws_n)
    shp = (T, c.H, c.d)
    qv, kv, vv = (act_bf[:, i * HD:(i + 1) * HD].view(shp) for i in (2, 3, 1))
    dact = torch.empty_like(act_bf)
    dact[:, :HD] = du
    dqv, dkv, dvv = (dact[:, i * HD:(i + 1) * HD].view(shp) for i in (2, 3, 1))
    prob = hb.AttnProblem(qv, kv, vv, dattn.view(shp), dl.offsets, max_seqlen=c.max_seqlen, local_window=c.K1,
                          global_prefix=c.K2, alpha=c.alpha, inv_n=1.0 / c.N, rab_table=dl.table, rab_bounds=dl.bounds)
    ws_a = hb.new_workspace(hb.hstu_attn_workspace_bytes(prob, True), dl.device)
    hb.hstu_attn_bwd(prob, qv, kv, vv, dattn.view(shp), dqv, dkv, dvv, ws_a)
    torch.cuda.synchronize()
    act.backward(dact.float())                                        # SiLU', both projection gradients, the norm
    dz_ref = z32.grad + dout32
    check("d gated_norm_w", f64(dl.d_gated_norm_w), f64(dgw))
    check("d W2", f64(dl.d_w2), f64(d_w2_ref))
    check("d W1", f64(dl.d_w1), f64(w1.grad))
    check("d norm_w", f64(dl.d_norm_w), f64(nw.grad))
    check("dZ", f64(dl.dz), f64(dz_ref))


# ----------------------------------------------------------------------------------------------
# FP8 forward (Section 4.2.2): both projections on row-wise quantised operands
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,E", [("layer-small-sparse-targets", 256), ("layer-mid", 512)])
def test_layer_forward_fp8(hb, name, E):
    """hstu_layer_fwd with quantised weights against the oracle's FP8 forward.  Both sides quantise, but not the same
    numbers: the kernel's Y is computed from A and U that were rounded to bf16 (relative error 2^-9), the oracle's from fp64
    ones, so a value within that distance of a rounding boundary (a few percent of them: the E4M3 spacing is 2^-3 to 2^-4
    relative) gets the neighbouring code and moves its element by one step.  Hence two bounds: the largest error is a few such
    steps landing in one dot product (5e-2 of the output's magnitude), the root-mean-square error stays at 4e-3.  The
    quantiser itself is compared bit for bit in test_gpu_fp8.py.  The FP8 forward also differs from the bf16 forward
    (it is really taken)."""
    from paper_2602_16986_amd.runner import DeviceLayer
    c = wl.layer_case(name)
    assert c.E == E
    dl = DeviceLayer(c, fp8=True)
    dl.out.fill_(float("nan"))
    dl.fwd()
    torch.cuda.synchronize()
    kw = dict(norm_eps=c.eps, gated_eps=c.eps, **attn_kw(c))
    ref, s = lorc.layer_fwd_fp8(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, **kw)
    print(f"layer FP8 forward {name}", flush=True)
    check("out (fp8 forward)", f64(dl.out), ref, 5e-2, 4e-3)
    check("U (saved)", f64(dl.u_saved), s["u"], 5e-2, 4e-3)
    check("A (saved)", f64(dl.attn_saved), s["a"], 5e-2, 4e-3)
    check("mean", f64(dl.mean), s["mean"], 1e-5)
    bf = DeviceLayer(c)
    bf.fwd()
    torch.cuda.synchronize()
    assert not torch.equal(bf.out, dl.out)
    exact, _ = lorc.layer_fwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, **kw)
    rel = np.abs(f64(dl.out) - exact).max() / np.abs(exact).max()
    print(f"  FP8 forward against the unquantised layer: normalised max difference {rel:.3e}", flush=True)
    assert rel < 0.1
    # the backward rematerialises U, V, Q, K through the same FP8 projection and differentiates there in bf16
    dl.bwd()
    torch.cuda.synchronize()
    g = lorc.layer_bwd(c.z, c.norm_w, c.w1, c.gated_norm_w, c.w2, c.offsets, c.H, c.d, c.dout, pre_override=s["pre"], **kw)
    check("dZ", f64(dl.dz), g["dz"])
    check("d norm_w", f64(dl.d_norm_w), g["d_norm_w"])
    check("d W1", f64(dl.d_w1), g["d_w1"])
    check("d gated_norm_w", f64(dl.d_gated_norm_w), g["d_gated_norm_w"])
    check("d W2", f64(dl.d_w2), g["d_w2"])


def test_layer_fp8_needs_all_four_weight_tensors(hb):
    from paper_2602_16986_amd.runner import DeviceLayer
    dl = DeviceLayer(wl.layer_case("layer-small-sparse-targets"), fp8=True)
    dl.problem.params.w2_scale = None
    with pytest.raises(hb.HstuError):
        dl.fwd()
    small = DeviceLayer(wl.layer_case("layer-small-dense"))          # E = 96: no FP8 GEMM for that width
    q1 = torch.zeros((4 * 128, 96), dtype=torch.uint8, device=small.device)
    s1 = torch.ones(4 * 128, device=small.device)
    q2 = torch.zeros((96, 128), dtype=torch.uint8, device=small.device)
    s2 = torch.ones(96, device=small.device)
    p = small.problem.params
    p.w1_q, p.w1_scale, p.w2_q, p.w2_scale = q1.data_ptr(), s1.data_ptr(), q2.data_ptr(), s2.data_ptr()
    with pytest.raises(hb.HstuError):
        small.fwd()
