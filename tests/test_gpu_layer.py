"""GPU parity of mmtrain_layer_fwd / mmtrain_layer_bwd against the fp64 oracle, element by element,
on the same seeded inputs: small cases that span several tiles with ragged tails, the edge
cases, and the five workloads at full size."""
import numpy as np
import pytest
import torch

from paper_2408_04275_amd import binding as mm
from paper_2408_04275_amd import workloads as wl
from paper_2408_04275_amd.harness import LayerRunner, check
from util import compare_layer, gpu_run, oracle_run, say, storage_floors, summary

pytestmark = pytest.mark.gpu


def run_case(shape, cu, modes, seed=0, std=0.02, what="", bars=None):
    W = wl.make_weights(shape, seed, std=std)
    x, dy = wl.make_activations(shape, int(cu[-1]), seed)
    ref = oracle_run(shape, cu, modes, W, x, dy)
    floors = storage_floors(shape, cu, modes, W, x, dy, ref)        # bf16: what storage alone costs this very case
    got = gpu_run(shape, cu, modes, W, x, dy)
    errs = compare_layer(shape, got, ref, what, bars, floors)
    say(f"{what or shape.name}: worst over {len(errs)} tensors: {summary(errs, floors)}")
    return errs


# ---- workload 1 (fp32), both readings of the image span's mask ------------------------
@pytest.mark.parametrize("image_bidir", [False, True])
def test_config1_fp32(image_bidir):
    cu, modes, _ = wl.make_segments(1, image_bidir=image_bidir)
    run_case(wl.SHAPES[1], cu, modes, what=f"config1 image_bidir={image_bidir} ")


# ---- reduced shapes: several tiles, ragged tails, every code path ----------------------
RAGGED_CU = np.array([0, 1, 1, 70, 199, 200, 457, 648], dtype=np.int32)
RAGGED_MODES = np.array([0, 1, 1, 0, 1, 0, 1], dtype=np.uint8)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("nh,nkv,d,H,F", [(4, 2, 64, 272, 688), (2, 1, 128, 256, 528)])
def test_small_decoder(dtype, nh, nkv, d, H, F):
    shape = wl.LayerShape("small-dec", wl.DECODER, dtype, H, nh, nkv, d, F, 648)
    run_case(shape, RAGGED_CU, RAGGED_MODES, seed=1, std=0.05, what=f"small decoder dtype={dtype} d={d} ")


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_small_encoder(dtype):
    shape = wl.LayerShape("small-enc", wl.ENCODER, dtype, 272, 4, 4, 64, 528, 648)
    run_case(shape, RAGGED_CU, np.ones(7, dtype=np.uint8), seed=2, std=0.05, what=f"small encoder dtype={dtype} ")


def test_peaky_softmax_decoder():
    # large weights make the softmax far from uniform, so masking and max-subtraction mistakes show
    shape = wl.LayerShape("peaky", wl.DECODER, wl.F32, 256, 4, 2, 64, 512, 648)
    run_case(shape, RAGGED_CU, RAGGED_MODES, seed=3, std=0.15, what="peaky decoder ")


# ---- many rows on a narrow layer: the row-walking kernels take several rows per workgroup --------------------
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("kind", [wl.DECODER, wl.ENCODER])
def test_many_rows_narrow_layer(kind, dtype):
    # 5003 tokens, 144 wide: more rows than the normalisation kernels have workgroups (each walks several rows, the
    # next one requested ahead), a last workgroup with fewer rows, and column counts that end inside a thread's chunk
    rng = np.random.default_rng(11)
    T = 5003
    cuts = np.sort(rng.choice(np.arange(1, T), size=47, replace=False))
    cu = np.concatenate([[0], cuts, [T]]).astype(np.int32)
    modes = (np.ones(48, dtype=np.uint8) if kind == wl.ENCODER else rng.integers(0, 2, size=48).astype(np.uint8))
    shape = wl.LayerShape("rows", kind, dtype, 144, 2, 2 if kind == wl.ENCODER else 1, 64, 272, T)
    run_case(shape, cu, modes, seed=5, std=0.05, what=f"many rows kind={kind} dtype={dtype} ")


# ---- edge cases ----------------------------------------------------------------------
def test_empty_pack():
    shape = wl.LayerShape("e", wl.DECODER, wl.BF16, 256, 4, 2, 64, 512, 0)
    W = wl.make_weights(shape, 0)
    r = LayerRunner(shape, W, np.array([0, 0], dtype=np.int32))
    for g in r.g.values():
        g.fill_(1.0)
    r.step()
    torch.cuda.synchronize()
    assert all(float(g.abs().max()) == 0.0 for g in r.g.values())      # an empty pack contributes zero gradients


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_single_token_segments_only(dtype):
    # nine tokens, each its own segment: attention is the identity on v
    shape = wl.LayerShape("one", wl.DECODER, dtype, 256, 4, 2, 64, 512, 16)
    run_case(shape, np.arange(0, 10, dtype=np.int32), np.zeros(9, dtype=np.uint8), seed=4,
             what=f"single-token segments dtype={dtype} ")


def test_accumulate_and_frozen():
    shape = wl.LayerShape("acc", wl.DECODER, wl.BF16, 256, 4, 2, 64, 512, 648)
    W = wl.make_weights(shape, 5, std=0.05)
    x, dy = wl.make_activations(shape, 648, 5)
    y, dx, G = oracle_run(shape, RAGGED_CU, RAGGED_MODES, W, x, dy)
    floors = storage_floors(shape, RAGGED_CU, RAGGED_MODES, W, x, dy, (y, dx, G))
    # two accumulating backward passes give twice the gradient
    r = LayerRunner(shape, W, RAGGED_CU, RAGGED_MODES)
    r.set_inputs(x, dy)
    r.step()
    check(r.backward(mm.BWD_ACCUMULATE_WGRAD), "bwd accumulate")
    gy, gdx, gG = r.results()
    compare_layer(shape, (gy, gdx, gG), (y, dx, {k: 2 * v for k, v in G.items()}), "accumulate ", floors=floors)
    # frozen module: no weight gradients requested, input gradient still produced
    r2 = LayerRunner(shape, W, RAGGED_CU, RAGGED_MODES, grad_names=[])
    r2.set_inputs(x, dy)
    r2.step()
    _, fdx, fG = r2.results()
    assert fG == {} and np.array_equal(fdx, gdx)
    # partially frozen: only the MLP matrices
    gy3, gdx3, gG3 = gpu_run(shape, RAGGED_CU, RAGGED_MODES, W, x, dy, grad_names=["w_fc1", "w_fc2"])
    compare_layer(shape, (gy3, gdx3, gG3), (y, dx, {k: G[k] for k in ("w_fc1", "w_fc2")}), "partial ", floors=floors)


@pytest.mark.parametrize("names", [["b_o"], ["b_fc2", "norm2_w"], ["b_fc1"], ["b_qkv", "norm1_b"], ["norm2_b", "b_o", "b_fc2"]])
def test_encoder_partially_frozen(names):
    # the encoder's bias gradients are summed inside kernels that also serve other gradients: every subset must still
    # give the requested ones, bit-identical to the run that requests them all, and the same input gradient
    shape = wl.LayerShape("enc-frozen", wl.ENCODER, wl.BF16, 272, 4, 4, 64, 528, 648)
    W = wl.make_weights(shape, 9, std=0.05)
    x, dy = wl.make_activations(shape, 648, 9)
    modes = np.ones(7, dtype=np.uint8)
    y, dx, G = gpu_run(shape, RAGGED_CU, modes, W, x, dy)
    y2, dx2, G2 = gpu_run(shape, RAGGED_CU, modes, W, x, dy, grad_names=names)
    assert sorted(G2) == sorted(names)
    assert np.array_equal(y, y2) and np.array_equal(dx, dx2)
    for k in names:
        assert np.array_equal(G[k], G2[k]), k


def test_segment_order_invariance_on_gpu():
    # Section 5.2: reordering subsequences permutes outputs block-wise; summed weight gradients agree to rounding
    shape = wl.LayerShape("perm", wl.DECODER, wl.BF16, 256, 4, 2, 64, 512, 648)
    W = wl.make_weights(shape, 6, std=0.05)
    x, dy = wl.make_activations(shape, 648, 6)
    y, dx, G = gpu_run(shape, RAGGED_CU, RAGGED_MODES, W, x, dy)
    perm = [5, 0, 3, 6, 2, 1, 4]
    blocks = [(RAGGED_CU[s], RAGGED_CU[s + 1]) for s in perm]
    xp = np.concatenate([x[a:b] for a, b in blocks]); dyp = np.concatenate([dy[a:b] for a, b in blocks])
    cup = np.concatenate([[0], np.cumsum([b - a for a, b in blocks])]).astype(np.int32)
    yp, dxp, Gp = gpu_run(shape, cup, RAGGED_MODES[perm], W, xp, dyp)
    from paper_2408_04275_amd.parity import check as bars
    bars("y", yp, np.concatenate([y[a:b] for a, b in blocks]), wl.BF16)
    bars("dx", dxp, np.concatenate([dx[a:b] for a, b in blocks]), wl.BF16)
    for k in G:
        bars(k, Gp[k], G[k], wl.BF16)


@pytest.mark.parametrize("kind", [wl.DECODER, wl.ENCODER])
def test_fp32_main_gradient_buffers(kind):
    # mixed-precision training keeps accumulated gradients of bf16 parameters in fp32: with BWD_WGRAD_F32 the
    # gradient buffers are fp32, are written without the rounding to bf16, and accumulate exactly
    shape = wl.LayerShape("g32", kind, wl.BF16, 512, 8, 8 if kind == wl.ENCODER else 2, 64, 1024, 1300)
    rng = np.random.default_rng(31)
    cu, modes = wl.random_segments(rng, 1300, 6)
    W = wl.make_weights(shape, 7, std=0.05)
    x, dy = wl.make_activations(shape, 1300, 7)
    ref = oracle_run(shape, cu, modes, W, x, dy)
    r16 = LayerRunner(shape, W, cu, modes); r16.set_inputs(x, dy); r16.step()
    y16, dx16, G16 = r16.results()
    r32 = LayerRunner(shape, W, cu, modes, grads_f32=True); r32.set_inputs(x, dy)
    check(r32.forward(), "fwd"); check(r32.backward(mm.BWD_WGRAD_F32), "bwd, fp32 gradients")
    y32, dx32, G32 = r32.results()
    assert np.array_equal(y16, y32) and np.array_equal(dx16, dx32)
    floors = storage_floors(shape, cu, modes, W, x, dy, ref, round_param_grads=False)
    errs = compare_layer(shape, (y32, dx32, G32), ref, f"fp32 gradients kind={kind} ", floors=floors)
    for k in G32:
        # same products, one rounding fewer: rounding the fp32 result to bf16 gives the bf16 run's bits
        assert np.array_equal(wl.round_bf16(G32[k]), G16[k]), k
        e16 = np.linalg.norm(G16[k] - ref[2][k]) / np.linalg.norm(ref[2][k])
        assert errs[k]["l2_err"] <= e16 * 1.001 + 1e-7, (k, errs[k]["l2_err"], e16)
    # accumulation in fp32 is exact for a repeated microbatch: g + g = 2 g
    check(r32.backward(mm.BWD_WGRAD_F32 | mm.BWD_ACCUMULATE_WGRAD), "bwd, fp32 gradients, accumulate")
    G2 = r32.results()[2]
    for k in G32:
        assert np.array_equal(G2[k], 2.0 * G32[k]), k


def test_fp32_main_gradient_flag_with_fp32_storage():
    shape = wl.LayerShape("g32f", wl.DECODER, wl.F32, 128, 4, 2, 64, 352, 300)
    rng = np.random.default_rng(32)
    cu, modes = wl.random_segments(rng, 300, 4)
    W = wl.make_weights(shape, 8, std=0.05)
    x, dy = wl.make_activations(shape, 300, 8)
    a = gpu_run(shape, cu, modes, W, x, dy)
    r = LayerRunner(shape, W, cu, modes, grads_f32=True); r.set_inputs(x, dy)
    check(r.forward(), "fwd"); check(r.backward(mm.BWD_WGRAD_F32), "bwd")
    b = r.results()
    assert np.array_equal(a[1], b[1])
    for k in a[2]:
        assert np.array_equal(a[2][k], b[2][k]), k


@pytest.mark.parametrize("kind", [wl.ENCODER, wl.DECODER])
def test_head_dim_80(kind):
    # ViT-Huge-like proportions at reduced width (4 heads of 80); the decoder variant exercises the rotary
    # embedding on a head dimension that the attention kernels pad (separate rotation pass in backward)
    shape = wl.LayerShape("hd80", kind, wl.BF16, 320, 4, 4 if kind == wl.ENCODER else 2, 80, 1280, 900)
    rng = np.random.default_rng(41)
    cu, modes = wl.random_segments(rng, 900, 5)
    if kind == wl.ENCODER:
        modes[:] = wl.BIDIR
    run_case(shape, cu, modes, seed=9, what=f"head_dim 80 kind={kind} ")


def test_hip_graph_capture_and_replay():
    # the library neither allocates nor synchronises, so a caller may capture forward + backward in a HIP graph;
    # every replay (with new inputs, and eager work between replays) must reproduce the eager result bit for bit
    shape = wl.LayerShape("graph", wl.ENCODER, wl.BF16, 512, 8, 8, 64, 1024, 1400)
    rng = np.random.default_rng(51)
    cu, modes = wl.random_segments(rng, 1400, 6)
    W = wl.make_weights(shape, 10, std=0.05)
    r = LayerRunner(shape, W, cu, modes)
    inputs = [wl.make_activations(shape, 1400, 20 + i) for i in range(3)]
    eager = []
    for x, dy in inputs:
        r.set_inputs(x, dy)
        r.step()
        eager.append(r.results())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the capture stream (one-time kernel attributes)
        check(r.forward(side.cuda_stream), "fwd warm-up")
        check(r.backward(0, side.cuda_stream), "bwd warm-up")
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        st = torch.cuda.current_stream().cuda_stream
        check(r.forward(st), "fwd under capture")
        check(r.backward(0, st), "bwd under capture")
    for (x, dy), want in zip(inputs, eager):
        r.set_inputs(x, dy)
        torch.cuda.synchronize()
        g.replay()
        got = r.results()
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
        for k in want[2]:
            assert np.array_equal(got[2][k], want[2][k]), k
        # eager work between replays
        r.step()
        torch.cuda.synchronize()
