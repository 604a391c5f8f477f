"""GPU parity of the velocity network: single ops against numpy fp64 on the same
inputs, and the whole forward against the oracle, teacher-forced (fp32: relative
L2 error <= 1e-4; bf16: <= 2e-2)."""
import numpy as np
import pytest
import torch

from oracle import dit
from paper_2509_06040_amd import binding as br
from paper_2509_06040_amd import synth
from gpu_util import DEV, assert_velocity, bytes_buffer, cond_dev, dev, host, make_model, rel_l2

pytestmark = pytest.mark.gpu


def _bf(a):
    return synth.from_bf16_bits(synth.to_bf16_bits(a))


@pytest.mark.parametrize("M,N,K", [(37, 64, 16), (130, 192, 64), (300, 100, 256)])
def test_gemm_fp32(lib, M, N, K):
    rng = np.random.default_rng(M)
    A, W, b = (rng.standard_normal(s).astype(np.float32) for s in ((M, K), (N, K), (N,)))
    ref = A.astype(np.float64) @ W.astype(np.float64).T + b
    out = torch.empty((M, N), device=DEV)
    br.op_gemm(br.F32, 0, dev(A), dev(W), dev(b), out)
    assert rel_l2(host(out), ref) < 1e-6
    br.op_gemm(br.F32, 1, dev(A), dev(W), dev(b), out)
    assert rel_l2(host(out), dit.gelu_tanh(ref)) < 1e-5


@pytest.mark.parametrize("variant", [4, 5, 6, 7, 7 | (2 << 4), 4 | (3 << 4), 6 | (1 << 4), -1])
@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (129, 64, 64), (1101, 384, 128), (2 * 1101 + 5, 1024, 256), (700, 36, 192), (515, 640, 320), (5000, 4096, 128), (9000, 1280, 384)])
def test_gemm_bf16_every_tile_shape(lib, variant, M, N, K):
    rng = np.random.default_rng(M + N)
    A, W = _bf(rng.standard_normal((M, K)).astype(np.float32)), _bf(rng.standard_normal((N, K)).astype(np.float32) * 0.05)
    b = rng.standard_normal(N).astype(np.float32)
    ref = A.astype(np.float64) @ W.astype(np.float64).T + b
    Ad, Wd = dev(A, torch.bfloat16), dev(W, torch.bfloat16)
    out32 = torch.full((M, N), -9.0, device=DEV)
    if variant >= 0 and (variant & 15) == 7 and K % 128:
        with pytest.raises(br.BranchRolloutError) as e:      # the streaming kernel needs K % 128 == 0
            br.op_gemm(br.BF16, 4, Ad, Wd, dev(b), out32, variant=variant)
        assert e.value.code == -3
        return
    br.op_gemm(br.BF16, 4, Ad, Wd, dev(b), out32, variant=variant)
    assert rel_l2(host(out32), ref) < 1e-5, rel_l2(host(out32), ref)
    out16 = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    br.op_gemm(br.BF16, 0, Ad, Wd, dev(b), out16, variant=variant)
    assert np.array_equal(host(out16), _bf(host(out32)))          # same accumulators, rounded once
    br.op_gemm(br.BF16, 1, Ad, Wd, dev(b), out16, variant=variant)
    assert rel_l2(host(out16), dit.gelu_tanh(ref)) < 4e-3


def test_gemm_gated_residual_epilogue(lib):
    rng = np.random.default_rng(0)
    L, B, N, K, C, Astr = 50, 3, 128, 64, 2, 700
    M = L * B
    A, W = _bf(rng.standard_normal((M, K)).astype(np.float32)), _bf(rng.standard_normal((N, K)).astype(np.float32) * 0.1)
    b, x0 = rng.standard_normal(N).astype(np.float32), rng.standard_normal((M, N)).astype(np.float32)
    mods = rng.standard_normal((C, Astr)).astype(np.float32)
    cond = np.array([1, 0, 1], np.int32)
    gate = mods[cond][:, 256:256 + N]
    ref = x0 + np.repeat(gate, L, axis=0) * (A.astype(np.float64) @ W.astype(np.float64).T + b)
    for dt, tol in ((br.BF16, 1e-5), (br.F32, 1e-6)):
        x = dev(x0.copy())
        tdt = torch.bfloat16 if dt == br.BF16 else torch.float32
        br.op_gemm(dt, 2, dev(A, tdt), dev(W, tdt), dev(b), x, mods=dev(mods), gate_off=256, cond=dev(cond), L=L)
        assert rel_l2(host(x), ref) < tol


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_gemm_two_launch_cut_matches_one_launch_and_fp64(lib, mode):
    """16 samples of 1101 tokens and 1024 output columns are 1.08 rounds of 256x256 tiles on 256
    compute units: the library cuts the rows between two samples into a launch of the persistent
    kernel and one of 256x128 tiles.  Same bits as the persistent kernel alone, and right against
    fp64 on sampled rows on both sides of the cut (each sample with its own gate)."""
    rng = np.random.default_rng(mode)
    L, B, N, K, C = 1101, 16, 1024, 256, 5
    M = L * B
    A, W = _bf(rng.standard_normal((M, K)).astype(np.float32)), _bf(rng.standard_normal((N, K)).astype(np.float32) * 0.05)
    b = rng.standard_normal(N).astype(np.float32)
    Ad, Wd, bd = dev(A, torch.bfloat16), dev(W, torch.bfloat16), dev(b)
    rows = np.concatenate([np.arange(0, 3), np.arange(14 * L - 2, 14 * L + 3), np.arange(15 * L - 2, 15 * L + 2), np.arange(16382, 16387), np.arange(M - 3, M)])
    lin = A[rows].astype(np.float64) @ W.astype(np.float64).T + b
    if mode == 2:
        x0 = rng.standard_normal((M, N)).astype(np.float32)
        mods = rng.standard_normal((C, N)).astype(np.float32)
        cond = (np.arange(B) * 3 % C).astype(np.int32)
        outs = []
        for variant in (-1, 7):
            x = dev(x0.copy())
            br.op_gemm(br.BF16, 2, Ad, Wd, bd, x, mods=dev(mods), gate_off=0, cond=dev(cond), L=L, variant=variant)
            outs.append(x)
        ref = x0[rows] + mods[cond[rows // L]] * lin
        tol = 1e-5
    else:
        outs = []
        for variant in (-1, 7):
            out = torch.full((M, N), 3.0, dtype=torch.bfloat16, device=DEV)
            br.op_gemm(br.BF16, mode, Ad, Wd, bd, out, variant=variant)
            outs.append(out)
        ref = dit.gelu_tanh(lin) if mode == 1 else lin
        tol = 4e-3
    assert torch.equal(outs[0], outs[1])
    assert rel_l2(host(outs[0].float())[rows], ref) < tol


def _attention_ref(qkv, nh):
    B, L, H3 = qkv.shape
    H = H3 // 3
    return np.stack([dit.attention(qkv[b, :, :H], qkv[b, :, H:2 * H], qkv[b, :, 2 * H:], nh) for b in range(B)])


@pytest.mark.parametrize("dh,nh,L,B", [(16, 4, 24, 2), (32, 2, 100, 1), (64, 2, 77, 1), (128, 1, 130, 2)])
def test_attention_fp32(lib, dh, nh, L, B):
    rng = np.random.default_rng(dh + L)
    qkv = rng.standard_normal((B, L, 3 * nh * dh)).astype(np.float32)
    out = torch.empty((B, L, nh * dh), device=DEV)
    br.op_attention(br.F32, dev(qkv), out, nh)
    assert rel_l2(host(out), _attention_ref(qkv.astype(np.float64), nh)) < 2e-6


# the last four: enough (sample, head) pairs for the XCD-grouped tile order, with ragged query
# and key tiles, one key tile only, and the last sample ending at the end of the buffer
@pytest.mark.parametrize("dh,nh,L,B", [(64, 2, 1, 1), (64, 3, 77, 2), (64, 2, 1101, 1), (128, 2, 130, 2), (128, 1, 640, 1),
                                        (64, 1, 128, 1), (64, 16, 203, 3), (128, 8, 150, 5), (64, 12, 63, 3),
                                        (128, 9, 257, 4)])
def test_attention_bf16(lib, dh, nh, L, B):
    rng = np.random.default_rng(dh + L)
    qkv = _bf(rng.standard_normal((B, L, 3 * nh * dh)).astype(np.float32) * 1.5)
    out = torch.full((B, L, nh * dh), 3.0, dtype=torch.bfloat16, device=DEV)
    br.op_attention(br.BF16, dev(qkv, torch.bfloat16), out, nh)
    ref = _attention_ref(qkv.astype(np.float64), nh)
    err = rel_l2(host(out), ref)
    assert err < 3e-3, err                       # bf16 probabilities and output rounding (measured 1.8e-3)


@pytest.mark.parametrize("dh,nh,L,B", [(64, 2, 77, 2), (64, 4, 1101, 1), (128, 2, 130, 2), (128, 9, 257, 4), (64, 12, 63, 3)])
def test_attention_bf16_prescaled_queries(lib, dh, nh, L, B):
    """The layout the network's QKV projection writes: q * log2(e) / sqrt(dh) in the q third.  The
    result is softmax attention of the q that these bf16 values stand for."""
    rng = np.random.default_rng(dh + L)
    H = nh * dh
    c = np.log2(np.e) / np.sqrt(dh)
    qkv = rng.standard_normal((B, L, 3 * H)).astype(np.float32) * 1.5
    qkv[..., :H] *= c
    qkv = _bf(qkv)
    out = torch.full((B, L, H), 3.0, dtype=torch.bfloat16, device=DEV)
    br.op_attention(br.BF16, dev(qkv, torch.bfloat16), out, nh, q_prescaled=1)
    plain = qkv.astype(np.float64)
    plain[..., :H] /= c
    err = rel_l2(host(out), _attention_ref(plain, nh))
    assert err < 3e-3, err
    raw = br.load()
    import ctypes as C
    p = C.c_void_p(out.data_ptr())
    assert raw.br_op_attention(br.F32, p, p, 1, 16, 2, 64, 1, None) == -1     # fp32 has no prescaled layout


@pytest.mark.parametrize("jump", [40.0, -200.0])
def test_attention_bf16_reference_follows_the_scores(lib, jump):
    """jump > 0: keys 300.. score about `jump` (in powers of two) above everything before them, so
    the kernel's softmax reference has to move mid-sequence.  jump < 0: every score sits that far
    below zero, so the first tile must not start from a reference of zero."""
    rng = np.random.default_rng(7)
    dh, nh, L, B = 64, 2, 400, 1
    H = nh * dh
    qkv = rng.standard_normal((B, L, 3 * H)).astype(np.float32)
    u = rng.standard_normal(dh).astype(np.float32)
    u /= np.linalg.norm(u)
    a = 4.0
    b = jump * np.sqrt(dh) / np.log2(np.e) / a          # a b / sqrt(dh) * log2(e) = jump
    for h in range(nh):
        qkv[0, :, h * dh:(h + 1) * dh] += a * u
        first = 300 if jump > 0 else 0
        qkv[0, first:, H + h * dh:H + (h + 1) * dh] += b * u
    qkv = _bf(qkv)
    out = torch.full((B, L, H), 3.0, dtype=torch.bfloat16, device=DEV)
    br.op_attention(br.BF16, dev(qkv, torch.bfloat16), out, nh)
    got = host(out)
    assert np.isfinite(got).all()
    err = rel_l2(got, _attention_ref(qkv.astype(np.float64), nh))
    assert err < 3e-3, err


def test_attention_bf16_rejects_what_it_cannot_address(lib):
    import ctypes as C
    raw = br.load()
    buf = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    p = C.c_void_p(buf.data_ptr())
    # rows of one sample beyond 4 GiB (the check precedes any launch; the buffers are never touched)
    assert raw.br_op_attention(br.BF16, p, p, 1, 400000, 16, 128, 0, None) == -3
    assert b"4 GiB" in raw.br_last_error()
    assert raw.br_op_attention(br.BF16, p, p, 1, 16, 2, 32, 0, None) == -3          # head dim 32 in bf16
    assert raw.br_op_attention(br.BF16, p, p, 1, 0, 2, 64, 0, None) == -1


@pytest.mark.parametrize("dt", [br.F32, br.BF16])
def test_ln_modulate(lib, dt):
    rng = np.random.default_rng(1)
    B, L, n_img, H, C, Astr = 3, 9, 7, 192, 2, 1000
    x = (rng.standard_normal((B * L, H)) * 3 + 1).astype(np.float32)
    mods = rng.standard_normal((C, Astr)).astype(np.float32) * 0.3
    cond = np.array([0, 1, 1], np.int32)
    tdt = torch.bfloat16 if dt == br.BF16 else torch.float32
    tol = 4e-3 if dt == br.BF16 else 2e-6
    for rows, so, co in ((L, 0, H), (n_img, 400, 600)):
        out = torch.empty((B * rows, H), dtype=tdt, device=DEV)
        br.op_ln_modulate(dt, dev(x), out, rows, L, dev(mods), so, co, dev(cond))
        xs = x.reshape(B, L, H)[:, :rows].astype(np.float64)
        m = mods[cond].astype(np.float64)
        ref = dit.layer_norm(xs) * (1 + m[:, None, co:co + H]) + m[:, None, so:so + H]
        assert rel_l2(host(out).reshape(B, rows, H), ref) < tol


def _velocity_case(cfg, n_cond, B, t, seed, std=0.02):
    W = synth.make_weights(cfg, seed, std)
    D = synth.model_sizes(cfg)["D"]
    z = synth.random_latents(B, D, seed + 1)
    cond = synth.cond_tokens(cfg, n_cond, seed + 2)
    cidx = np.arange(B) % n_cond
    model = make_model(cfg, W)
    ws = bytes_buffer(br.workspace_bytes(None, model, B))
    v = torch.full((B, D), 5.0, device=DEV)
    br.velocity(model, dev(z), t, cond_dev(cfg, cond), cidx, v, ws)
    rnd = dit.round_bf16 if cfg["dtype"] == synth.BF16 else dit.identity
    ref = dit.forward(cfg, W, z, t, cond, cidx, act_round=rnd)
    return host(v), ref, (model, W, z, cond, cidx)


def test_velocity_tiny_fp32_matches_oracle(lib):
    cfg = synth.WORKLOADS["tiny"]["model"]
    for t, std in ((1.0, 0.02), (0.37, 0.02), (0.05, 0.2)):
        got, ref, _ = _velocity_case(cfg, 2, 5, t, 0, std)
        for b in range(5):
            assert_velocity(cfg, got[b], ref[b], 1e-4, "tiny t=%g b=%d" % (t, b))   # stated fp32 tolerance


def test_velocity_fp32_other_shapes(lib):
    # temporal patches, head dim 32, ragged token count
    cfg = synth.model_cfg(2, 64, 2, (3, 4, 6, 10), (2, 2, 2), 5, synth.F32)
    got, ref, _ = _velocity_case(cfg, 3, 4, 0.6, 3, 0.1)
    for b in range(4):
        assert_velocity(cfg, got[b], ref[b], 1e-4, "fp32 shapes b=%d" % b)


def test_velocity_small_bf16_matches_oracle(lib):
    for cfg in (synth.model_cfg(2, 128, 2, (16, 1, 16, 20), (1, 2, 2), 13, synth.BF16),          # d_h 64, L = 93
                synth.model_cfg(1, 256, 2, (16, 2, 8, 12), (1, 2, 2), 70, synth.BF16)):         # d_h 128, L = 166
        got, ref, _ = _velocity_case(cfg, 2, 3, 0.5, 1, 0.05)
        for b in range(3):
            assert_velocity(cfg, got[b], ref[b], 2e-2, "small bf16 b=%d" % b)                   # stated bf16 tolerance


def test_velocity_chunked_batches_agree(lib):
    cfg = synth.WORKLOADS["tiny"]["model"]
    got, ref, (model, W, z, cond, cidx) = _velocity_case(cfg, 2, 5, 0.5, 4)
    small = bytes_buffer(br.workspace_bytes(None, model, 2) + 64)       # forces chunks of <= 2
    v2 = torch.empty_like(torch.from_numpy(got)).to(DEV)
    br.velocity(model, dev(z), 0.5, cond_dev(cfg, cond), cidx, v2, small)
    assert np.array_equal(host(v2), got)
    with pytest.raises(br.BranchRolloutError) as e:
        br.velocity(model, dev(z), 0.5, cond_dev(cfg, cond), cidx, v2, bytes_buffer(256))
    assert e.value.code == -4
