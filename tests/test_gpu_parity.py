"""GPU parity: libmxq (through its C ABI) against the CPU oracle on the same seeded inputs.

Bar: codes and scale bytes bit-exact; per-block SSE bit-exact (both sides use the same fp32
tree); per-tensor MSE within 1e-6 relative.
"""
import numpy as np
import pytest
import torch

from paper_2605_08565_amd import workloads as W

pytestmark = pytest.mark.gpu

FMT_NAMES = {0: "e8m0", 1: "e4m3", 2: "ue5m3"}
REC_NAMES = {0: "absmax", 1: "absmax_pz", 2: "4over6", 3: "4over6_pz", 4: "brute", 5: "brute_pruned"}
ORACLE_REC = {0: 0, 1: 1, 2: 2, 3: 3, 4: 4, 5: 4}      # the pruned search must equal the full one
BLOCKS = (2, 4, 8, 16, 32, 64, 128)
# pow2 MX, E4M3 abs-max, clamp, 4-over-6, UE5M3 abs-max, E4M3 brute force
CONFIG5_RECIPES = [(0, 0), (1, 0), (1, 1), (1, 2), (2, 0), (1, 4)]


@pytest.fixture(scope="module")
def mxq():
    from paper_2605_08565_amd import mxq as M
    assert torch.cuda.is_available(), "these tests need the GPU"
    M.lib()
    return M


def combos(brute=True):
    out = [(0, 0)] + ([(0, 4)] if brute else [])
    for fmt in (1, 2):
        for rec in (0, 1, 2, 3) + ((4, 5) if brute else ()):
            out.append((fmt, rec))
    return out


def run_gpu(mxq, x_np, block, fmt, rec, T=1.0):
    x = mxq.from_bits(x_np)
    c, s, e = mxq.quantize(x, block, fmt, rec, tensor_scale=T)
    torch.cuda.synchronize()
    return c.cpu().numpy(), s.cpu().numpy(), e.cpu().numpy()


def check(oracle, mxq, x_np, block, fmt, rec, T=1.0, tag=""):
    print(f"[parity] {tag} shape={x_np.shape} dtype={x_np.dtype} b={block} fmt={FMT_NAMES[fmt]} "
          f"recipe={REC_NAMES[rec]} T={T}", flush=True)
    gc, gs, ge = run_gpu(mxq, x_np, block, fmt, rec, T)
    oc, os_, oe = oracle.quantize(x_np, block, fmt, ORACLE_REC[rec], tensor_scale=T)
    assert (gs == os_).all(), f"scale bytes differ in {(gs != os_).sum()} blocks"
    assert (gc == oc).all(), f"code bytes differ in {(gc != oc).sum()} bytes"
    assert (ge.view(np.uint32) == oe.view(np.uint32)).all(), "block SSE not bit-identical"
    if x_np.size:            # the same call with the clipping-only SSE as a fourth output
        x = mxq.from_bits(x_np)
        clip = torch.full((x_np.shape[0], x_np.shape[1] // block), -1.0, dtype=torch.float32, device="cuda")
        c2, s2, e2 = mxq.quantize(x, block, fmt, rec, tensor_scale=T, clip_sse_out=clip)
        torch.cuda.synchronize()
        assert (c2.cpu().numpy() == oc).all() and (s2.cpu().numpy() == os_).all()
        assert (e2.cpu().numpy().view(np.uint32) == oe.view(np.uint32)).all()
        want = oracle.clip_sse(x_np, os_, block, fmt, tensor_scale=T)
        assert (clip.cpu().numpy().view(np.uint32) == want.view(np.uint32)).all(), "clipping-only SSE differs"
    if x_np.size:
        m_g, m_o = oracle.tensor_mse(ge, x_np.size, T), oracle.tensor_mse(oe, x_np.size, T)
        if np.isfinite(m_o):
            assert abs(m_g - m_o) <= 1e-6 * abs(m_o)


# ------------------------------------------------------------------ small, every combination

@pytest.mark.parametrize("block", BLOCKS)
def test_all_recipes_bf16_weights(oracle, mxq, block):
    """37 x 1152 spans several workgroup tiles (9 wavefronts of chunks per 2 rows) and ends
    inside a wavefront."""
    x = W.student_t_weights(37, 1152, seed=100 + block)
    for fmt, rec in combos():
        check(oracle, mxq, x, block, fmt, rec, tag="weights")


@pytest.mark.parametrize("block", BLOCKS)
def test_all_recipes_f32_normal(oracle, mxq, block):
    x = W.normal_f32(19, 640, seed=200 + block, sigma=0.004)
    x[3] *= 300.0
    x[7] *= 1e-3
    for fmt, rec in combos():
        check(oracle, mxq, x, block, fmt, rec, tag="normal-f32")


@pytest.mark.parametrize("block", (4, 16, 64))
def test_hierarchical_small(oracle, mxq, block):
    x = W.outlier_activations(48, 1024, seed=300 + block)
    xt = mxq.from_bits(x)
    A = float(mxq.tensor_absmax(xt).cpu()[0])
    assert A == oracle.tensor_absmax(x)
    for fmt in (1, 2):
        T = mxq.tensor_scale_from_absmax(A, fmt)
        assert T == oracle.tensor_scale(A, fmt)
        for rec in (0, 1, 2, 3, 4, 5):
            check(oracle, mxq, x, block, fmt, rec, T=T, tag="hierarchical")
    check(oracle, mxq, W.bf16_bits_to_f32(x), block, 1, 2, T=mxq.tensor_scale_from_absmax(A, 1),
          tag="hierarchical-f32")


def check_hier(oracle, mxq, x_np, block, fmt, rec, tag=""):
    """mxq_quantize_hier against the oracle run with the oracle's own T."""
    print(f"[parity] hier-device {tag} shape={x_np.shape} dtype={x_np.dtype} b={block} "
          f"fmt={FMT_NAMES[fmt]} recipe={REC_NAMES[rec]}", flush=True)
    x = mxq.from_bits(x_np)
    amax = mxq.tensor_absmax(x)
    gc, gs, ge, gT = mxq.quantize_hier(x, block, fmt, rec, amax)
    torch.cuda.synchronize()
    T = np.float32(oracle.tensor_scale(oracle.tensor_absmax(x_np), fmt))
    assert gT.cpu().numpy().view(np.uint32)[0] == T.view(np.uint32), (float(gT.cpu()[0]), float(T))
    oc, os_, oe = oracle.quantize(x_np, block, fmt, ORACLE_REC[rec], tensor_scale=float(T))
    assert (gs.cpu().numpy() == os_).all() and (gc.cpu().numpy() == oc).all()
    assert (ge.cpu().numpy().view(np.uint32) == oe.view(np.uint32)).all()
    # de-quantise with the scale still in device memory
    for dt, tdt in ((oracle.DT_F32, torch.float32), (oracle.DT_BF16, torch.bfloat16)):
        got = mxq.dequantize(gc, gs, block, fmt, gT, tdt).cpu()
        want = oracle.dequantize(oc, os_, block, fmt, float(T), dt)
        if tdt == torch.float32:
            assert (got.numpy().view(np.uint32) == want.view(np.uint32)).all()
        else:
            assert (got.view(torch.int16).numpy().view(np.uint16) == want).all()


@pytest.mark.parametrize("block", (2, 4, 16, 128))
def test_hierarchical_scale_taken_from_device_memory(oracle, mxq, block):
    """The per-tensor scale derived by the kernels from the abs-max in device memory: every
    division path (T = 1 for a zero tensor and for power-of-two scales, the reciprocal-refined
    range, plain division beyond it), ragged sizes whose only launch is the tail kernel, fp32."""
    acts = W.outlier_activations(48, 1024, seed=700 + block)
    huge = (W.normal_f32(9, 256, seed=701, sigma=1.0) * np.float32(1e30)).astype(np.float32)   # T > 2^20
    tiny = (W.normal_f32(9, 256, seed=702, sigma=1.0) * np.float32(1e-12)).astype(np.float32)  # T < 2^-20
    zeros = np.zeros((4, 256), np.float32)
    for x_np, tag in ((acts, "activations"), (W.bf16_bits_to_f32(acts), "activations-f32"), (huge, "huge"),
                      (tiny, "tiny"), (zeros, "zeros")):
        for fmt, rec in ((1, 0), (1, 2), (1, 3), (2, 0), (2, 2), (0, 0), (1, 4), (2, 5)):
            check_hier(oracle, mxq, x_np, block, fmt, rec, tag)
    if block <= 4:
        for shape in ((5, 12), (1, 4)):                     # 60 elements: main + tail; 4: tail only
            x_np = W.normal_f32(shape[0], shape[1], seed=703, sigma=0.3)
            for fmt, rec in ((1, 0), (1, 2), (2, 4), (0, 0)):
                check_hier(oracle, mxq, x_np, block, fmt, rec, "ragged")


def test_hierarchical_division_paths(oracle, mxq):
    """The per-tensor division has a reciprocal-refined path (2^-20 <= T <= 2^20), a per-wavefront
    fall-back for blocks of very small or very large adjusted values, and a plain-division path
    for every other T; all must give the IEEE quotient."""
    rng = np.random.default_rng(55)
    x = (rng.standard_normal((24, 512)) * 0.3).astype(np.float32)
    x[2] *= 1e-30          # adjusted abs-max far below 2^-40: fall-back
    x[3] *= 1e-38          # sub-normal inputs
    x[5] *= 1e30           # adjusted abs-max above 2^90 for small T: fall-back (stays finite)
    x[7, ::3] = 0.0
    x[8] = 0.0
    x[9, 1::2] = -0.0
    all_ones = float(np.float32(1.99999988) * np.float32(0.0625))     # mantissa 0x7FFFFF
    for T in (0.0917, 3.0e-7, 2.0 ** 21, 2.0 ** -20, 2.0 ** 20, all_ones, 1.0000001, 7.5e-4):
        for block, fmt, rec in [(16, 1, 0), (4, 1, 2), (64, 2, 3), (32, 0, 0), (8, 1, 4), (2, 2, 1), (16, 2, 5)]:
            check(oracle, mxq, x, block, fmt, rec, T=T, tag="division-paths")
    xb = W.f32_to_bf16_bits(x)
    for T in (0.0917, 3.0e-7):
        check(oracle, mxq, xb, 16, 1, 2, T=T, tag="division-paths-bf16")


def test_config1_full(oracle, mxq):
    """fp32 1024 x 4096, N(0,1), E2M1, block 16, unsigned E4M3, abs-max: the whole tensor."""
    x = W.config1()
    check(oracle, mxq, x, 16, 1, 0, tag="config1")


# ------------------------------------------------------------------ several tensors per launch

@pytest.mark.parametrize("block", BLOCKS)
def test_quantize_batch(oracle, mxq, block):
    """mxq_quantize_batch against the oracle run tensor by tensor: eleven tensors (two launches)
    of very different sizes -- one chunk, ragged last slices, several tiles per workgroup, an empty
    tensor, for b = 2 and 4 element counts that are not a multiple of 8 -- both dtypes, every
    streaming recipe and scale format, and one tensor without an SSE output."""
    rng = np.random.default_rng(900 + block)
    m = 3 if block < 8 else 1
    shapes = [(1, block * m), (37, 1152), (3, 128 * 5), (0, 256), (513, 2048), (2, 128), (64, 4096), (7, block * 3 * m),
              (1, 128), (300, 384), (2100, 1024)]
    for to_bits in (W.f32_to_bf16_bits, lambda a: a):
        xs_np = [to_bits((rng.standard_normal(sh) * 10.0 ** rng.uniform(-3, 1)).astype(np.float32)) for sh in shapes]
        xs = [mxq.from_bits(a) if a.size else torch.empty(a.shape, dtype=torch.bfloat16 if a.dtype == np.uint16 else torch.float32,
                                                        device="cuda") for a in xs_np]
        for fmt, rec in [(0, 0), (1, 0), (1, 1), (1, 2), (1, 3), (2, 0), (2, 2)]:
            print(f"[parity] batch b={block} dtype={xs_np[0].dtype} fmt={FMT_NAMES[fmt]} recipe={REC_NAMES[rec]}", flush=True)
            outs = mxq.quantize_batch(xs, block, fmt, rec)
            torch.cuda.synchronize()
            for a, (c, s_, e) in zip(xs_np, outs):
                if a.size == 0:
                    continue
                oc, os_, oe = oracle.quantize(a, block, fmt, rec)
                assert (c.cpu().numpy() == oc).all() and (s_.cpu().numpy() == os_).all(), a.shape
                assert (e.cpu().numpy().view(np.uint32) == oe.view(np.uint32)).all(), a.shape
        outs = mxq.quantize_batch(xs[:3], block, 1, 2, want_sse=False)
        assert all(o[2] is None for o in outs)
        oc, os_, _ = oracle.quantize(xs_np[1], block, 1, 2)
        assert (outs[1][0].cpu().numpy() == oc).all() and (outs[1][1].cpu().numpy() == os_).all()
    with pytest.raises(mxq.MxqError):
        mxq.quantize_batch(xs[:2], block, 1, 4)


def test_quantize_batch_one_layer_equals_single_calls(mxq):
    """The seven matrices of a model layer in one launch: the same bytes as seven mxq_quantize
    calls (which the layer tests compare with the oracle)."""
    from paper_2605_08565_amd import sweep
    layer = sweep.host_layer(3)
    xs = [mxq.from_bits(a) for a in layer.values()]
    for block, fmt, rec in [(16, 1, 0), (32, 0, 0), (4, 1, 2), (128, 2, 1), (2, 1, 3)]:
        outs = mxq.quantize_batch(xs, block, fmt, rec)
        for x, (c, s_, e) in zip(xs, outs):
            c1, s1, e1 = mxq.quantize(x, block, fmt, rec)
            assert torch.equal(c, c1) and torch.equal(s_, s1) and torch.equal(e.view(torch.int32), e1.view(torch.int32))


# ------------------------------------------------------------------ edge cases

def test_ragged_and_tiny_shapes(oracle, mxq):
    rng = np.random.default_rng(7)
    for rows, cols, block in [(1, 2, 2), (3, 6, 2), (1, 4, 4), (5, 12, 4), (7, 10, 2), (1, 8, 8),
                              (3, 24, 8), (1, 16, 16), (1, 128, 128), (65, 20, 4), (513, 18, 2)]:
        x32 = (rng.standard_normal((rows, cols)) * 0.05).astype(np.float32)
        for x in (x32, W.f32_to_bf16_bits(x32)):
            for fmt, rec in combos():
                check(oracle, mxq, x, block, fmt, rec, tag="ragged")


def test_binding_refuses_buffers_that_are_too_small(mxq):
    """The library trusts its pointers, so the binding checks every caller-supplied buffer."""
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    u8 = lambda n: torch.empty(n, dtype=torch.uint8, device="cuda")
    f32 = lambda n: torch.empty(n, dtype=torch.float32, device="cuda")
    with pytest.raises(ValueError):
        mxq.quantize(x, 16, 1, 0, codes_out=u8(127))
    with pytest.raises(ValueError):
        mxq.quantize(x, 16, 1, 0, scales_out=u8(15))
    with pytest.raises(ValueError):
        mxq.quantize(x, 16, 1, 0, sse_out=f32(15))
    with pytest.raises(TypeError):
        mxq.quantize(x, 16, 1, 0, sse_out=u8(64))
    c, s_, _ = mxq.quantize(x, 16, 1, 0)
    with pytest.raises(ValueError):
        mxq.dequantize(c, s_[:3], 16, 1)
    with pytest.raises(ValueError):
        mxq.dequantize(c, s_, 16, 1, out=f32(255))
    with pytest.raises(ValueError):
        mxq.clip_sse(x, s_[:3], 16, 1)
    with pytest.raises(ValueError):
        mxq.histogram(c, s_[:3], 16)
    with pytest.raises(ValueError):
        mxq.quantize(x.cpu(), 16, 1, 0)


def test_empty(mxq):
    x = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    c, s, e = mxq.quantize(x, 16, 1, 0)
    assert c.shape == (0, 32) and s.shape == (0, 4) and e.shape == (0, 4)
    out = mxq.dequantize(c, s, 16, 1)
    assert out.shape == (0, 64)
    assert float(mxq.tensor_absmax(x).cpu()[0]) == 0.0


def test_special_values(oracle, mxq):
    """Zero blocks, signed zeros, sub-normals, values that clip the scale format, exact ties."""
    rows = []
    rows.append(np.zeros(128, np.float32))
    z = np.zeros(128, np.float32); z[1::2] = -0.0; rows.append(z)
    rows.append(np.full(128, 1e-41, np.float32))
    rows.append(np.full(128, 2.0 ** -126, np.float32))
    rows.append(np.tile(np.float32([3e4, -1e6, 2.5e5, 7e9, -3e38, 1e38, 6 * 448.0, 6 * 448.1]), 16))
    ties = np.float32([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0])
    rows.append(np.tile(ties, 16))
    rows.append(np.tile(-ties * 0.8125, 16))
    rows.append(np.tile(np.nextafter(ties * np.float32(1.375), np.float32(0)), 16))
    rows.append(np.tile(np.float32([2 ** -10 * 6, 2 ** -10 * 4, 2 ** -9, 2 ** -11, 0, 0, 0, 0]), 16))
    rows.append(np.tile(np.float32([2 ** -18 * 6, 2 ** -18 * 4, 2 ** -17, 2 ** -19, 0, 0, 0, 0]), 16))
    x = np.stack(rows)
    for block in (2, 8, 16, 128):
        for fmt, rec in combos():
            check(oracle, mxq, x, block, fmt, rec, tag="special")
    xb = W.f32_to_bf16_bits(x)
    for block in (4, 32):
        for fmt, rec in combos():
            check(oracle, mxq, xb, block, fmt, rec, tag="special-bf16")


def test_randomised_wide_dynamic_range(oracle, mxq):
    """Seeded random tensors whose magnitudes spread over many binades (log-uniform exponents,
    per-row and per-element), with zeros and repeated values mixed in, under random per-tensor
    scales: every recipe, both dtypes.  Stresses the scale-format limits, the pruning bounds of
    the pruned search and the fall-backs of the per-tensor division."""
    rng = np.random.default_rng(20260508)
    for case in range(30):
        rows, cols = int(rng.integers(3, 20)), 128 * int(rng.integers(1, 5))
        row_exp = rng.uniform(-36, 30, size=(rows, 1))
        elem_exp = rng.uniform(-6, 6, size=(rows, cols)) * rng.integers(0, 2, size=(rows, 1))
        x = (rng.standard_normal((rows, cols)) * np.exp2(row_exp + elem_exp)).astype(np.float32)
        x[rng.random((rows, cols)) < 0.05] = 0.0
        x[rng.random((rows, cols)) < 0.05] *= -1.0
        rep = rng.random((rows, cols)) < 0.1
        x[rep] = np.float32(x[0, 0])
        T = float(np.float32(np.exp2(rng.uniform(-30, 30)))) if case % 2 else 1.0
        data = x if case % 3 else W.f32_to_bf16_bits(x)
        with np.errstate(over="ignore", divide="ignore", invalid="ignore"):
            adj = np.abs(W.bf16_bits_to_f32(data) if data.dtype == np.uint16 else data).astype(np.float64) / T
        if not np.isfinite(adj.astype(np.float32)).all():        # adjusted inputs must stay finite
            T = 1.0
        for block in (2, 4, 8, 16, 32, 64, 128)[case % 3::3]:
            for fmt, rec in combos():
                check(oracle, mxq, data, block, fmt, rec, T=T if fmt else 1.0, tag=f"random-{case}")


def test_nan_and_inf_stay_inside_their_blocks(oracle, mxq):
    """NaN / Inf elements give unspecified results for their own block only (every table index
    and loop bound in the kernels is clamped, so nothing can fault): all other blocks equal the
    oracle's.  Rows 1, 3 and 5 carry the special values; blocks never straddle rows."""
    x = W.normal_f32(8, 256, seed=12, sigma=0.05)
    x[1, 7] = np.nan
    x[3, 100] = np.inf
    x[5, 31] = -np.inf
    x[5, 200] = np.nan
    clean = [0, 2, 4, 6, 7]
    for data in (x, W.f32_to_bf16_bits(x)):
        for block in (2, 16, 128):
            for fmt, rec in combos():
                print(f"[parity] specials dtype={data.dtype} b={block} fmt={FMT_NAMES[fmt]} recipe={REC_NAMES[rec]}",
                      flush=True)
                gc, gs, ge = run_gpu(mxq, data, block, fmt, rec)
                oc, os_, oe = oracle.quantize(np.ascontiguousarray(data[clean]), block, fmt, ORACLE_REC[rec])
                assert (gc[clean] == oc).all() and (gs[clean] == os_).all()
                assert (ge[clean].view(np.uint32) == oe.view(np.uint32)).all()


def test_sse_out_may_be_null(oracle, mxq):
    x_np = W.student_t_weights(16, 256, seed=5)
    x = mxq.from_bits(x_np)
    for rec in (0, 2, 4):
        c, s, e = mxq.quantize(x, 16, 1, rec, want_sse=False)
        assert e is None
        oc, os_, _ = oracle.quantize(x_np, 16, 1, rec)
        assert (c.cpu().numpy() == oc).all() and (s.cpu().numpy() == os_).all()


def test_non_default_stream_and_determinism(mxq):
    x = mxq.from_bits(W.student_t_weights(256, 2048, seed=6))
    st = torch.cuda.Stream()
    ref = None
    for _ in range(3):
        with torch.cuda.stream(st):
            c, s, e = mxq.quantize(x, 16, 1, 2)
        st.synchronize()
        cur = (c.cpu(), s.cpu(), e.cpu())
        if ref is not None:
            assert all(torch.equal(a, b) for a, b in zip(ref, cur))
        ref = cur


# ------------------------------------------------------------------ de-quantise, abs-max

@pytest.mark.parametrize("block", (2, 16, 128))
def test_dequantize(oracle, mxq, block):
    rng = np.random.default_rng(block)
    rows, cols = 9, 384
    codes = rng.integers(0, 256, size=(rows, cols // 2), dtype=np.uint8)
    for fmt, hi in ((0, 255), (1, 0x7F), (2, 0xFF)):
        lo = 110 if fmt == 0 else 0
        top = 140 if fmt == 0 else hi
        scales = rng.integers(lo, top, size=(rows, cols // block), dtype=np.uint8)
        for T in (1.0, 0.0731):
            for dt, tdt in ((oracle.DT_F32, torch.float32), (oracle.DT_BF16, torch.bfloat16)):
                want = oracle.dequantize(codes, scales, block, fmt, T, dt)
                got = mxq.dequantize(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda(),
                                     block, fmt, T, tdt)
                g = got.cpu()
                g = g.numpy() if tdt == torch.float32 else g.view(torch.int16).numpy().view(np.uint16)
                if tdt == torch.float32:
                    assert (g.view(np.uint32) == want.view(np.uint32)).all()
                else:
                    assert (g == want).all()


@pytest.mark.parametrize("block", (2, 4, 8, 16, 32, 64, 128))
def test_dequantize_ragged_and_multi_pass(oracle, mxq, block):
    """Element counts that leave a partial lane (fp32 output: 4 elements per lane, bf16: 8) and a
    tensor large enough that the fp32 kernel's grid-stride loop runs more than once."""
    rng = np.random.default_rng(100 + block)
    shapes = [(3, block * (3 if block < 8 else 1)), (1, block), (1536, 2048)]
    for rows, cols in shapes:
        codes = rng.integers(0, 256, size=(rows, cols // 2), dtype=np.uint8)
        scales = rng.integers(0, 0x7F, size=(rows, cols // block), dtype=np.uint8)
        for dt, tdt in ((oracle.DT_F32, torch.float32), (oracle.DT_BF16, torch.bfloat16)):
            want = oracle.dequantize(codes, scales, block, 1, 0.37, dt)
            got = mxq.dequantize(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda(),
                                 block, 1, 0.37, tdt).cpu()
            if tdt == torch.float32:
                assert (got.numpy().view(np.uint32) == want.view(np.uint32)).all(), (rows, cols)
            else:
                assert (got.view(torch.int16).numpy().view(np.uint16) == want).all(), (rows, cols)


def test_dequantize_roundtrip_ragged(oracle, mxq):
    x = W.student_t_weights(5, 12, seed=8)
    c, s, _ = oracle.quantize(x, 4, 1, 0)
    want = oracle.dequantize(c, s, 4, 1)
    got = mxq.dequantize(torch.from_numpy(c).cuda(), torch.from_numpy(s).cuda(), 4, 1).cpu().numpy()
    assert (got == want).all()


def test_tensor_absmax(oracle, mxq):
    for x in (W.config1()[:37], W.student_t_weights(33, 1000, seed=9), W.normal_f32(1, 6, 3)):
        got = float(mxq.tensor_absmax(mxq.from_bits(x)).cpu()[0])
        assert got == oracle.tensor_absmax(x)


def test_tensor_absmax_running_maximum(oracle, mxq):
    """mxq_tensor_absmax_acc: two words used alternately, each call clearing the other one's word
    (no clear launch anywhere); a tensor fed in row shards accumulates to the whole tensor's
    maximum; an empty tensor leaves the word alone."""
    words = torch.zeros(2, dtype=torch.float32, device="cuda")
    big = W.config3()
    cases = [big, W.bf16_bits_to_f32(big[:2048]), W.config1()[:37] * np.float32(0.01), W.student_t_weights(33, 1000, seed=9),
             W.normal_f32(1, 6, 3) * np.float32(1e-3), np.zeros((3, 40), np.float32), big[:7]]
    got = []
    for k, x_np in enumerate(cases):            # no host synchronisation between the calls
        mxq.tensor_absmax_acc(mxq.from_bits(x_np), words[k % 2:k % 2 + 1], clear_word=words[(k + 1) % 2:(k + 1) % 2 + 1])
        got.append(words[k % 2:k % 2 + 1].clone())
    for k, x_np in enumerate(cases):
        assert float(got[k].cpu()[0]) == oracle.tensor_absmax(x_np), k
    acc = torch.zeros(1, dtype=torch.float32, device="cuda")
    xb = mxq.from_bits(big)
    for r0 in range(0, big.shape[0], 1000):
        mxq.tensor_absmax_acc(xb[r0:r0 + 1000], acc)
    assert float(acc.cpu()[0]) == oracle.tensor_absmax(big)
    mxq.tensor_absmax_acc(torch.empty((0, 8), dtype=torch.float32, device="cuda"), acc, clear_word=words[0:1])
    assert float(acc.cpu()[0]) == oracle.tensor_absmax(big) and float(words.cpu()[0]) == 0.0


def test_tensor_absmax_one_launch(oracle, mxq):
    """mxq_tensor_absmax_ws: one workspace reused over tensors of very different sizes (1 to 256
    workgroups, ragged tails, both dtypes, an empty tensor, decreasing maxima so that a value
    left behind by an earlier call would show), stale output words, and the workspace back at
    zero after every call."""
    ws = mxq.absmax_workspace()
    out = torch.full((1,), 123.0, dtype=torch.float32, device="cuda")
    big = W.config3()
    cases = [big, W.bf16_bits_to_f32(big[:2048]), W.config1()[:37] * np.float32(0.01), W.student_t_weights(33, 1000, seed=9),
             W.normal_f32(1, 6, 3) * np.float32(1e-3), np.zeros((3, 40), np.float32), big[:7],
             W.normal_f32(2049, 4099, 5) * np.float32(1e-5)]
    for x_np in cases:
        print(f"[absmax-ws] shape={x_np.shape} dtype={x_np.dtype}", flush=True)
        mxq.tensor_absmax(mxq.from_bits(x_np), out=out, workspace=ws)
        assert float(out.cpu()[0]) == oracle.tensor_absmax(x_np)
        assert int(ws.cpu().to(torch.int64).sum()) == 0
    empty = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    mxq.tensor_absmax(empty, out=out, workspace=ws)
    assert float(out.cpu()[0]) == 0.0
    # back-to-back calls on one stream without a host synchronisation in between
    xs = [mxq.from_bits(c) for c in cases[:4]]
    outs = torch.zeros(16, dtype=torch.float32, device="cuda")
    for rep in range(4):
        for i, x in enumerate(xs):
            mxq.tensor_absmax(x, out=outs[4 * rep + i:4 * rep + i + 1], workspace=ws)
    got = outs.cpu().numpy()
    for rep in range(4):
        for i in range(4):
            assert got[4 * rep + i] == oracle.tensor_absmax(cases[i])


# ------------------------------------------------------------------ full benchmark sizes

def sample_rows(n_rows, k, seed):
    rng = np.random.default_rng(seed)
    mid = rng.choice(np.arange(1, n_rows - 1), size=k - 2, replace=False)
    return np.sort(np.concatenate([[0, n_rows - 1], mid]))


def check_rows(oracle, x_np, rows, gpu_out, block, fmt, rec, T=1.0):
    gc, gs, ge = gpu_out
    idx = torch.from_numpy(rows).cuda()
    gc, gs, ge = gc[idx].cpu().numpy(), gs[idx].cpu().numpy(), ge[idx].cpu().numpy()
    oc, os_, oe = oracle.quantize(np.ascontiguousarray(x_np[rows]), block, fmt, ORACLE_REC[rec], tensor_scale=T)
    assert (gs == os_).all() and (gc == oc).all()
    assert (ge.view(np.uint32) == oe.view(np.uint32)).all()


def check_full(oracle, x_np, gpu_out, block, fmt, rec, T=1.0):
    """Every byte of a full-size run against the oracle, and the tensor MSE (1e-6 relative)."""
    gc, gs, ge = (t.cpu().numpy() for t in gpu_out)
    oc, os_, oe = oracle.quantize(x_np, block, fmt, ORACLE_REC[rec], tensor_scale=T)
    assert (gs == os_).all(), f"scale bytes differ in {(gs != os_).sum()} blocks"
    assert (gc == oc).all(), f"code bytes differ in {(gc != oc).sum()} bytes"
    assert (ge.view(np.uint32) == oe.view(np.uint32)).all(), "block SSE not bit-identical"
    m_g, m_o = oracle.tensor_mse(ge, x_np.size, T), oracle.tensor_mse(oe, x_np.size, T)
    assert abs(m_g - m_o) <= 1e-6 * abs(m_o)


def test_config2_full_size(oracle, mxq):
    """bf16 4096 x 14336 Student-t weights, the launch configuration the benchmark times:
    all 12 runs (b in {8,16,32,64} x abs-max, prevent-zero, 4-over-6) compared with the oracle
    on the WHOLE tensor; the SSE chain abs-max >= 4-over-6 holds on every block."""
    x_np = W.config2()
    x = mxq.from_bits(x_np)
    for block in (8, 16, 32, 64):
        outs = {}
        for rec in (0, 1, 2):
            print(f"[parity] config2 b={block} recipe={REC_NAMES[rec]}", flush=True)
            outs[rec] = mxq.quantize(x, block, 1, rec)
            torch.cuda.synchronize()
            check_full(oracle, x_np, outs[rec], block, 1, rec)
        assert bool((outs[0][2] >= outs[2][2]).all())
        assert bool((outs[0][2] >= outs[1][2]).all())
    # the fused clipping-only SSE at full size: equal to the separate pass on the same scales and
    # to the oracle's, for abs-max and for 4-over-6
    for block, rec in ((16, 0), (16, 2), (64, 2), (8, 1)):
        print(f"[parity] config2 fused clip b={block} recipe={REC_NAMES[rec]}", flush=True)
        clip = torch.empty((x_np.shape[0], x_np.shape[1] // block), dtype=torch.float32, device="cuda")
        c, s, e = mxq.quantize(x, block, 1, rec, clip_sse_out=clip)
        sep = mxq.clip_sse(x, s, block, 1)
        torch.cuda.synchronize()
        assert torch.equal(clip.view(torch.int32), sep.view(torch.int32))
        want = oracle.clip_sse(x_np, s.cpu().numpy(), block, 1)
        assert (clip.cpu().numpy().view(np.uint32) == want.view(np.uint32)).all()


def test_config3_full_size(oracle, mxq):
    """bf16 8192 x 4096 activations with outlier channels, hierarchical scaling: all 10 runs
    (b in {4,8,16,32,64} x abs-max, 4-over-6) compared with the oracle on the WHOLE tensor."""
    x_np = W.config3()
    x = mxq.from_bits(x_np)
    A = float(mxq.tensor_absmax(x).cpu()[0])
    assert A == oracle.tensor_absmax(x_np)
    T = mxq.tensor_scale_from_absmax(A, 1)
    for block in (4, 8, 16, 32, 64):
        for rec in (0, 2):
            print(f"[parity] config3 b={block} recipe={REC_NAMES[rec]} T={T}", flush=True)
            out = mxq.quantize(x, block, 1, rec, tensor_scale=T)
            torch.cuda.synchronize()
            check_full(oracle, x_np, out, block, 1, rec, T=T)


@pytest.mark.parametrize("fmt,block", [(1, 16), (1, 4), (2, 16), (2, 4)])
def test_config4_brute_full_size(oracle, mxq, fmt, block):
    """Brute-force search (126 / 254 candidates) on the full 4096 x 14336 weights, compared with
    the oracle on the WHOLE tensor (in chunks of 512 rows); brute-force SSE <= 4-over-6 SSE <=
    abs-max SSE on every block; the pruned search returns the same bytes."""
    x_np = W.config2()
    x = mxq.from_bits(x_np)
    out = mxq.quantize(x, block, fmt, 4)
    torch.cuda.synchronize()
    gc, gs, ge = (t.cpu().numpy() for t in out)
    for r0 in range(0, x_np.shape[0], 512):
        print(f"[parity] config4 b={block} fmt={FMT_NAMES[fmt]} brute rows {r0}..{r0 + 511}", flush=True)
        sl = slice(r0, r0 + 512)
        oc, os_, oe = oracle.quantize(np.ascontiguousarray(x_np[sl]), block, fmt, 4)
        assert (gs[sl] == os_).all() and (gc[sl] == oc).all()
        assert (ge[sl].view(np.uint32) == oe.view(np.uint32)).all()
    if fmt == 1:
        ab = mxq.quantize(x, block, 1, 0)[2]
        f6 = mxq.quantize(x, block, 1, 2)[2]
        assert bool((out[2] <= f6).all()) and bool((f6 <= ab).all())
    pr = mxq.quantize(x, block, fmt, 5)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(out, pr))


def test_pruned_search_equals_full_search_on_activations_full_size(oracle, mxq):
    """The pruned search against the full enumeration on the whole 8192 x 4096 activation tensor
    (outlier channels: blocks of very different magnitude share a wavefront, some blocks hold one
    outlier and otherwise tiny values), with and without the per-tensor scale, both scale formats,
    small and large blocks: identical bytes.  The full enumeration of the same tensor is checked
    against the oracle on 256 whole rows."""
    x_np = W.config3()
    x = mxq.from_bits(x_np)
    T = oracle.tensor_scale(oracle.tensor_absmax(x_np), 1)
    rows = sample_rows(x_np.shape[0], 256, seed=45)
    for fmt in (1, 2):
        for block in (2, 4, 16, 64):
            for t in ((1.0, T) if fmt == 1 else (1.0,)):
                print(f"[parity] config3 pruned-vs-full fmt={FMT_NAMES[fmt]} b={block} T={t}", flush=True)
                full = mxq.quantize(x, block, fmt, 4, tensor_scale=t)
                pr = mxq.quantize(x, block, fmt, 5, tensor_scale=t)
                torch.cuda.synchronize()
                assert all(torch.equal(a, b) for a, b in zip(full, pr))
                if block in (4, 16) and fmt == 1:
                    check_rows(oracle, x_np, rows, full, block, fmt, 4, T=t)


def test_binade_shift_invariance_full_size(mxq):
    """A property that holds at any size, on the full 4096 x 14336 weights in the launch
    configuration the benchmark times: multiplying the inputs by 4 (exact in bf16) leaves every
    element code as it is, moves every UE5M3 scale byte up by two binades (16 codes) and multiplies
    every block SSE by 16 exactly -- for all streaming recipes, the full search and the pruned one."""
    x = mxq.from_bits(W.config2())
    x4 = x * 4
    for block in (4, 16):
        for rec in (0, 1, 2, 3, 4, 5):
            print(f"[parity] shift invariance b={block} recipe={REC_NAMES[rec]}", flush=True)
            c0, s0, e0 = mxq.quantize(x, block, 2, rec)
            c1, s1, e1 = mxq.quantize(x4, block, 2, rec)
            torch.cuda.synchronize()
            normal = s0 >= 16                                    # a binade of margin above the sub-normal codes
            assert float(normal.float().mean()) > 0.99
            assert torch.equal(s1[normal].to(torch.int32), s0[normal].to(torch.int32) + 16)
            assert torch.equal(e1[normal], e0[normal] * 16)
            keep = normal.repeat_interleave(block // 2, dim=1)
            assert torch.equal(c1[keep], c0[keep])


def test_brute_force_over_power_of_two_scales_full_size(oracle, mxq):
    """The search over all 255 power-of-two scales on the full 4096 x 14336 weights (b = 32, the
    MX block size): 1 024 whole rows against the oracle; on every block its SSE is at most that of
    the floor rule of Eq. 1, which is one of its candidates."""
    x_np = W.config2()
    x = mxq.from_bits(x_np)
    for block in (32, 4):
        out = mxq.quantize(x, block, 0, 4)
        floor_rule = mxq.quantize(x, block, 0, 0)
        torch.cuda.synchronize()
        assert bool((out[2] <= floor_rule[2]).all())
        rows = sample_rows(x_np.shape[0], 1024 if block == 32 else 256, seed=44)
        print(f"[parity] e8m0 brute b={block} rows={len(rows)}", flush=True)
        check_rows(oracle, x_np, rows, out, block, 0, 4)


def test_config5_layer0(oracle, mxq):
    """Layer 0 of the synthetic 32-layer model, every matrix, every recipe and block size.  The
    streaming recipes are compared on the whole k and v matrices (1024 x 4096) and on 512 whole
    rows of the larger ones; the brute-force search on 129 whole rows per matrix."""
    for name in W.LAYER_SHAPES:
        x_np = W.layer_matrix(0, name)
        x = mxq.from_bits(x_np)
        rows = sample_rows(x_np.shape[0], 512, seed=5)
        for block in BLOCKS:
            for fmt, rec in CONFIG5_RECIPES:
                print(f"[parity] config5 {name} b={block} fmt={FMT_NAMES[fmt]} "
                      f"recipe={REC_NAMES[rec]}", flush=True)
                out = mxq.quantize(x, block, fmt, rec)
                torch.cuda.synchronize()
                if rec == 4:
                    check_rows(oracle, x_np, np.union1d(rows[::4], rows[-1:]), out, block, fmt, rec)
                elif x_np.shape[0] <= 1024:
                    check_full(oracle, x_np, out, block, fmt, rec)
                else:
                    check_rows(oracle, x_np, rows, out, block, fmt, rec)


@pytest.mark.parametrize("layer", (1, 15, 31))
def test_config5_later_layers(oracle, mxq, layer):
    """Layers beyond the first: the GPU quantises every whole matrix of the layer (the bytes
    `workloads.layer_matrix` draws, which are also what the sweep driver quantises) with all six
    recipes at all seven block sizes; 16 seeded whole rows per matrix -- first and last row
    included, so every block size sees whole blocks -- are compared with the oracle bit for bit."""
    from paper_2605_08565_amd import sweep
    layer_np = sweep.host_layer(layer)
    for name, x_np in layer_np.items():
        x = mxq.from_bits(x_np)
        rows = sample_rows(x_np.shape[0], 16, seed=1000 * layer + len(name))
        for block in BLOCKS:
            for fmt, rec in CONFIG5_RECIPES:
                print(f"[parity] config5 layer={layer} {name} b={block} fmt={FMT_NAMES[fmt]} "
                      f"recipe={REC_NAMES[rec]}", flush=True)
                out = mxq.quantize(x, block, fmt, rec)
                torch.cuda.synchronize()
                check_rows(oracle, x_np, rows, out, block, fmt, rec)


# ------------------------------------------------------------------ fp32 input beyond one tile per workgroup

def test_f32_input_grid_stride_ragged(oracle, mxq):
    """fp32 input whose 5 147 slices of 256 chunks exceed the 2 048 workgroups of the launch, so
    every workgroup runs the double-buffered loop (and its wavefront-private LDS re-formation)
    two or three times, with a ragged last slice; the whole tensor against the oracle."""
    x_np = W.normal_f32(2563, 4112, seed=1101)
    x_np[5] *= np.float32(1e-3)
    x_np[100] *= np.float32(40.0)
    x_np[2000, ::7] = 0.0
    assert (x_np.size // 8) % 256 != 0 and x_np.size // 8 > 2 * 2048 * 256
    x = mxq.from_bits(x_np)
    A = float(mxq.tensor_absmax(x).cpu()[0])
    assert A == oracle.tensor_absmax(x_np)
    T = mxq.tensor_scale_from_absmax(A, 1)
    slow_T = float(np.float32(1.99999988) * np.float32(2.0 ** -7))       # plain-division kernel
    for block, fmt, rec, t in [(16, 1, 0, 1.0), (16, 1, 2, 1.0), (16, 1, 0, T), (16, 1, 3, T), (8, 1, 2, slow_T),
                               (16, 0, 0, 1.0), (8, 2, 2, 1.0), (4, 1, 1, 1.0), (2, 1, 2, 1.0), (2, 2, 0, T)]:
        print(f"[parity] f32-grid-stride b={block} fmt={FMT_NAMES[fmt]} recipe={REC_NAMES[rec]} T={t}", flush=True)
        out = mxq.quantize(x, block, fmt, rec, tensor_scale=t)
        torch.cuda.synchronize()
        check_full(oracle, x_np, out, block, fmt, rec, T=t)
    # the same tensor through mxq_quantize_hier (T taken from device memory inside the kernel)
    out = mxq.quantize_hier(x, 16, 1, 2, mxq.tensor_absmax(x))
    torch.cuda.synchronize()
    check_full(oracle, x_np, out[:3], 16, 1, 2, T=T)
    rows = sample_rows(x_np.shape[0], 257, seed=11)
    for block, fmt, rec, t in [(16, 1, 4, 1.0), (4, 2, 4, 1.0), (8, 1, 5, T)]:
        print(f"[parity] f32-grid-stride brute b={block} fmt={FMT_NAMES[fmt]} recipe={REC_NAMES[rec]} T={t}", flush=True)
        out = mxq.quantize(x, block, fmt, rec, tensor_scale=t)
        torch.cuda.synchronize()
        check_rows(oracle, x_np, rows, out, block, fmt, rec, T=t)


def test_f32_activations_full_size(oracle, mxq):
    """The 8192 x 4096 activation tensor widened to fp32 (33.5 M elements, 16 384 slices: eight
    tiles per workgroup): abs-max, 4-over-6, hierarchical abs-max and 4-over-6, power-of-two scales
    and the widest blocks on the WHOLE tensor; the brute-force search on 512 whole rows."""
    x_np = W.bf16_bits_to_f32(W.config3())
    x = mxq.from_bits(x_np)
    A = float(mxq.tensor_absmax(x).cpu()[0])
    assert A == oracle.tensor_absmax(x_np)
    T = mxq.tensor_scale_from_absmax(A, 1)
    for block, fmt, rec, t in [(16, 1, 0, 1.0), (16, 1, 2, 1.0), (16, 1, 0, T), (32, 1, 2, T), (32, 0, 0, 1.0),
                               (128, 1, 2, 1.0), (64, 2, 1, 1.0)]:
        print(f"[parity] f32-activations b={block} fmt={FMT_NAMES[fmt]} recipe={REC_NAMES[rec]} T={t}", flush=True)
        out = mxq.quantize(x, block, fmt, rec, tensor_scale=t)
        torch.cuda.synchronize()
        check_full(oracle, x_np, out, block, fmt, rec, T=t)
    rows = sample_rows(x_np.shape[0], 512, seed=12)
    for block, fmt, rec, t in [(16, 1, 4, 1.0), (32, 1, 4, T)]:
        print(f"[parity] f32-activations brute b={block} T={t}", flush=True)
        out = mxq.quantize(x, block, fmt, rec, tensor_scale=t)
        torch.cuda.synchronize()
        check_rows(oracle, x_np, rows, out, block, fmt, rec, T=t)
    # de-quantise to fp32 and bf16 at this size (several passes of the grid-stride loops)
    c, s, _ = mxq.quantize(x, 16, 1, 0, tensor_scale=T)
    oc, os_, _ = oracle.quantize(x_np, 16, 1, 0, tensor_scale=T)
    got = mxq.dequantize(c, s, 16, 1, T, torch.float32).cpu().numpy()
    assert (got.view(np.uint32) == oracle.dequantize(oc, os_, 16, 1, T, oracle.DT_F32).view(np.uint32)).all()
    got = mxq.dequantize(c, s, 16, 1, T, torch.bfloat16).cpu().view(torch.int16).numpy().view(np.uint16)
    assert (got == oracle.dequantize(oc, os_, 16, 1, T, oracle.DT_BF16)).all()


# ------------------------------------------------------------------ appendix diagnostics

def test_clip_sse_and_histograms(oracle, mxq):
    """Clipping-only SSE (bit-exact) and the entry / scale histograms (exact counts) on the
    outputs of every recipe, incl. ragged shapes, a per-tensor scale and fp32 input."""
    cases = [(W.student_t_weights(37, 1152, seed=400), 1.0),
             (W.normal_f32(19, 640, seed=401, sigma=0.004), 1.0),
             (W.outlier_activations(16, 1024, seed=402), None),
             (W.f32_to_bf16_bits(W.normal_f32(5, 12, seed=403, sigma=0.05)), 1.0),
             (W.normal_f32(3, 6, seed=404, sigma=0.05), 0.37)]
    for x_np, T in cases:
        x = mxq.from_bits(x_np)
        if T is None:
            T = mxq.tensor_scale_from_absmax(float(mxq.tensor_absmax(x).cpu()[0]), 1)
        for block in (2, 4, 8, 16, 32, 64, 128):
            if x_np.shape[1] % block:
                continue
            for fmt, rec in [(0, 0), (1, 0), (1, 1), (1, 2), (1, 4), (2, 3)]:
                print(f"[diag] shape={x_np.shape} b={block} fmt={fmt} rec={rec} T={T}", flush=True)
                c, s, _ = mxq.quantize(x, block, fmt, rec, tensor_scale=T)
                clip = mxq.clip_sse(x, s, block, fmt, tensor_scale=T).cpu().numpy()
                eh, sh = mxq.histogram(c, s, block)
                oc, os_, _ = oracle.quantize(x_np, block, fmt, rec, tensor_scale=T)
                want = oracle.clip_sse(x_np, os_, block, fmt, tensor_scale=T)
                assert (clip.view(np.uint32) == want.view(np.uint32)).all()
                weh, wsh = oracle.histograms(oc, os_)
                assert (eh.cpu().numpy().astype(np.uint64) == weh).all()
                assert (sh.cpu().numpy().astype(np.uint64) == wsh).all()


def test_histogram_full_size(oracle, mxq):
    x_np = W.config2()
    x = mxq.from_bits(x_np)
    for block, rec in [(16, 0), (4, 2)]:
        c, s, _ = mxq.quantize(x, block, 1, rec)
        eh, sh = mxq.histogram(c, s, block)
        torch.cuda.synchronize()
        weh, wsh = oracle.histograms(c.cpu().numpy(), s.cpu().numpy())
        assert (eh.cpu().numpy().astype(np.uint64) == weh).all()
        assert (sh.cpu().numpy().astype(np.uint64) == wsh).all()
        assert int(eh.sum()) == x_np.size and int(sh.sum()) == x_np.size // block


def test_histogram_unaligned_and_multi_pass(oracle, mxq):
    """Pointers that are 4- but not 16-byte aligned (the kernel reads 128-bit vectors between a
    serial head and tail), sizes around the vector and the grid-stride boundaries."""
    rng = np.random.default_rng(77)
    for rows, cols, block, c_off, s_off in [(1, 2, 2, 4, 4), (3, 34, 2, 4, 8), (7, 96, 16, 8, 12), (5, 1000, 4, 12, 4),
                                            (640, 4096, 2, 4, 12), (2048, 8192, 16, 0, 4)]:
        n = rows * cols
        codes = rng.integers(0, 256, size=(rows, cols // 2), dtype=np.uint8)
        scales = rng.integers(0, 256, size=(rows, cols // block), dtype=np.uint8)
        cbuf = torch.zeros(n // 2 + 64, dtype=torch.uint8, device="cuda")
        sbuf = torch.zeros(n // block + 64, dtype=torch.uint8, device="cuda")
        c = cbuf[c_off:c_off + n // 2].view(rows, cols // 2)
        s = sbuf[s_off:s_off + n // block].view(rows, cols // block)
        c.copy_(torch.from_numpy(codes))
        s.copy_(torch.from_numpy(scales))
        assert c.data_ptr() % 16 == c_off % 16 and s.data_ptr() % 16 == s_off % 16
        eh, sh = mxq.histogram(c, s, block)
        weh, wsh = oracle.histograms(codes, scales)
        assert (eh.cpu().numpy().astype(np.uint64) == weh).all(), (rows, cols, block)
        assert (sh.cpu().numpy().astype(np.uint64) == wsh).all(), (rows, cols, block)


# ------------------------------------------------------------------ graphs, very large tensors

def test_graph_capture_and_replay(oracle, mxq):
    """The whole path (tensor abs-max, hierarchical quantise with the scale taken from device
    memory, quantise, de-quantise, clip SSE) captured in
    a HIP graph and replayed with new input contents between replays, with eager work and
    synchronisation in between; every replay must equal the oracle on the current contents."""
    rows, cols, block = 64, 1024, 16
    x = torch.zeros((rows, cols), dtype=torch.bfloat16, device="cuda")
    amax = torch.zeros(1, dtype=torch.float32, device="cuda")
    codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device="cuda")
    scales = torch.empty((rows, cols // block), dtype=torch.uint8, device="cuda")
    sse = torch.empty((rows, cols // block), dtype=torch.float32, device="cuda")
    deq = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
    clip = torch.empty((rows, cols // block), dtype=torch.float32, device="cuda")
    codes_h, scales_h, sse_h = torch.empty_like(codes), torch.empty_like(scales), torch.empty_like(sse)
    t_dev = torch.zeros(1, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside capture
        mxq.quantize(x, block, 1, 2, codes_out=codes, scales_out=scales, sse_out=sse)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    ws = mxq.absmax_workspace()
    amax2 = torch.zeros(1, dtype=torch.float32, device="cuda")
    with torch.cuda.graph(g):
        mxq.tensor_absmax(x, out=amax)
        mxq.tensor_absmax(x, out=amax2, workspace=ws)                 # the one-launch form
        mxq.quantize_hier(x, block, 1, 2, amax2, tensor_scale_out=t_dev, codes_out=codes_h, scales_out=scales_h,
                          sse_out=sse_h)
        mxq.quantize(x, block, 1, 2, codes_out=codes, scales_out=scales, sse_out=sse)
        mxq.dequantize(codes, scales, block, 1, 1.0, out=deq)
        mxq.clip_sse(x, scales, block, 1, out=clip)
    for it in range(4):
        x_np = W.student_t_weights(rows, cols, seed=900 + it)
        x.copy_(mxq.from_bits(x_np))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        oc, os_, oe = oracle.quantize(x_np, block, 1, 2)
        assert float(amax.cpu()[0]) == oracle.tensor_absmax(x_np) == float(amax2.cpu()[0])
        assert (codes.cpu().numpy() == oc).all() and (scales.cpu().numpy() == os_).all()
        assert (sse.cpu().numpy().view(np.uint32) == oe.view(np.uint32)).all()
        want = oracle.dequantize(oc, os_, block, 1, 1.0, oracle.DT_BF16)
        assert (deq.cpu().view(torch.int16).numpy().view(np.uint16) == want).all()
        assert (clip.cpu().numpy().view(np.uint32) == oracle.clip_sse(x_np, os_, block, 1).view(np.uint32)).all()
        # hierarchical scaling inside the graph: T follows the data from replay to replay
        T = np.float32(oracle.tensor_scale(oracle.tensor_absmax(x_np), 1))
        assert t_dev.cpu().numpy().view(np.uint32)[0] == T.view(np.uint32)
        hc, hs, he = oracle.quantize(x_np, block, 1, 2, tensor_scale=float(T))
        assert (codes_h.cpu().numpy() == hc).all() and (scales_h.cpu().numpy() == hs).all()
        assert (sse_h.cpu().numpy().view(np.uint32) == he.view(np.uint32)).all()
        # eager work between replays
        e = mxq.quantize(x, block, 1, 0)[2]
        assert bool((e >= sse).all())


def test_more_than_2_to_32_elements(oracle, mxq):
    """64-bit indexing: a bf16 tensor of 65 544 x 65 536 = 2^32 + 2^19 elements (8.6 GB).
    Rows at the start, around the 2^32-element boundary and at the end are checked against the
    oracle; tensor abs-max against the maximum of the planted values."""
    rows, cols, block = 65544, 65536, 16
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    x = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
    step = 4096
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        x[r0:r1] = (torch.randn((r1 - r0, cols), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    x[rows - 1, cols - 3] = 7.5
    x[65536, 5] = -9.25                                 # first row past 2^32 elements
    torch.cuda.synchronize()
    print("[large] tensor ready", flush=True)
    assert float(mxq.tensor_absmax(x).cpu()[0]) == 9.25
    pick = np.array([0, 1, 32767, 65535, 65536, 65537, rows - 2, rows - 1])
    idx = torch.from_numpy(pick).cuda()
    x_np = x[idx].cpu().view(torch.int16).numpy().view(np.uint16)
    for rec in (0, 2):
        print(f"[large] recipe {rec}", flush=True)
        c, s, e = mxq.quantize(x, block, 1, rec)
        torch.cuda.synchronize()
        oc, os_, oe = oracle.quantize(x_np, block, 1, rec)
        assert (c[idx].cpu().numpy() == oc).all() and (s[idx].cpu().numpy() == os_).all()
        assert (e[idx].cpu().numpy().view(np.uint32) == oe.view(np.uint32)).all()
    d = mxq.dequantize(c, s, block, 1, 1.0, torch.bfloat16)
    torch.cuda.synchronize()
    want = oracle.dequantize(oc, os_, block, 1, 1.0, oracle.DT_BF16)
    assert (d[idx].cpu().view(torch.int16).numpy().view(np.uint16) == want).all()
    eh, sh = mxq.histogram(c, s, block)
    assert int(eh.sum()) == rows * cols and int(sh.sum()) == rows * cols // block
    del x, c, s, e, d
    torch.cuda.empty_cache()
