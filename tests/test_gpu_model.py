"""GPU parity of the bctm_ entry points (include/bct_model.h) and of the decoder stack built
from them, against oracle/model_ref, element by element on the same seeded inputs.

Tolerances.  The kernels accumulate in fp32 and round once to bf16; the oracle computes in
fp64 and rounds once.  The two bf16 results therefore differ by at most one bf16 spacing
where the exact value lies near a rounding boundary, plus the fp32 accumulation error,
bounded here by 2^-20 * sum_k |x_k w_k| (a pairwise-like split-K sum of fp32 products is
far inside it).  Arg-max and embedding are integer / byte work: bit-exact.
"""
import numpy as np
import pytest

import bct_synth as syn
from _util import bf16_ulp, to_dev, to_np
from oracle import model_ref as R

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def M():
    from paper_2411_15785_amd import model
    model.mlib()
    return model


def dev(a):
    return to_dev(a, "bf16")


def host(t):
    return to_np(t, "bf16")


def draw(tid, shape, std=1.0):
    return syn.pack(std * syn.normal(11, 9, tid, shape), "bf16")


def check_close(got_bits, ref_bits, slack, what):
    got, ref = R.bf16_to_f64(got_bits), R.bf16_to_f64(ref_bits)
    tol = bf16_ulp(ref) + slack
    bad = np.abs(got - ref) > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} beyond 1 ulp + slack, worst " \
                          f"{np.max(np.abs(got - ref) / tol):.2f}x at {np.unravel_index(np.argmax(np.abs(got - ref) / tol), got.shape)}"


LIN_SHAPES = [  # rows, K, N
    (1, 32, 16), (5, 64, 96), (32, 192, 48), (33, 320, 32), (70, 1024, 160), (32, 4096, 256), (3, 11008, 64),
    (17, 2336, 16),    # 73 K tiles: uneven shares for the wavefronts, whole rounds plus a masked one
    (33, 96, 16416),   # wide output (an output head): two feature tiles per workgroup
    (33, 96, 12288), (7, 2336, 12336),   # three feature tiles per workgroup (the fused q | wq | wv projection)
]


@pytest.mark.parametrize("rows,K,N", LIN_SHAPES)
@pytest.mark.parametrize("with_res", [False, True])
def test_linear(M, rows, K, N, with_res):
    x, w = draw(1, (rows, K)), draw(2, (N, K), K ** -0.5)
    res = draw(3, (rows, N)) if with_res else None
    out = M.bctm_linear(dev(x), M.bctm_pack_weight(dev(w)), dev(res) if with_res else None)
    mass = np.abs(R.bf16_to_f64(x)) @ np.abs(R.bf16_to_f64(w)).T
    check_close(host(out), R.linear(x, w, res), 2.0 ** -20 * mass, f"linear {rows}x{K}x{N}")


# Many rows (a prefill chunk): the 128 x 128 matrix-core kernel.  Ragged row counts, several row bands,
# one K step and many, feature counts that make the last XCD round partial.
ROWS_SHAPES = [(128, 32, 128), (130, 320, 256), (257, 4096, 384), (300, 96, 128), (1100, 64, 640), (129, 2336, 1152),
               (1100, 64, 768), (1024, 4096, 256), (2050, 96, 512)]   # the last three: 256 x 256 workgroups


@pytest.mark.parametrize("rows,K,N", ROWS_SHAPES)
@pytest.mark.parametrize("with_res", [False, True])
@pytest.mark.parametrize("tiled", [False, True])
def test_linear_many_rows(M, rows, K, N, with_res, tiled):
    x, w = draw(1, (rows, K)), draw(2, (N, K), K ** -0.5)
    res = draw(3, (rows, N)) if with_res else None
    xin = M.bctm_pack_rows(dev(x)) if tiled else dev(x)
    out = M.bctm_linear(xin, M.bctm_pack_weight(dev(w)), dev(res) if with_res else None)
    mass = np.abs(R.bf16_to_f64(x)) @ np.abs(R.bf16_to_f64(w)).T
    check_close(host(out), R.linear(x, w, res), 2.0 ** -20 * mass, f"linear {rows}x{K}x{N}")


def test_linear_many_rows_selects_the_right_operands(M):
    # one-hot weight rows pick input features, distinct per output feature and row: exact
    rows, K, N = 200, 256, 256
    x = draw(4, (rows, K))
    sel = (np.arange(N) * 37 + 5) % K
    w = np.zeros((N, K), dtype=np.float32)
    w[np.arange(N), sel] = 1.0
    wb = (w.view(np.uint32) >> 16).astype(np.uint16)
    for xin in (dev(x), M.bctm_pack_rows(dev(x))):
        out = host(M.bctm_linear(xin, M.bctm_pack_weight(dev(wb))))
        assert np.array_equal(out, x[:, sel])


def test_linear_many_rows_in_place_residual_and_split(M):
    import torch
    rows, K = 150, 192
    x, res = draw(1, (rows, K)), draw(3, (rows, 256))
    w = draw(2, (256, K), K ** -0.5)
    buf = dev(res)
    M.bctm_linear(dev(x), M.bctm_pack_weight(dev(w)), buf, buf)
    mass = np.abs(R.bf16_to_f64(x)) @ np.abs(R.bf16_to_f64(w)).T
    check_close(host(buf), R.linear(x, w, res), 2.0 ** -20 * mass, "in place, many rows")
    # three outputs whose borders fall inside a workgroup's 128 features
    widths = (144, 48, 64)
    ws = [draw(20 + i, (n, K), K ** -0.5) for i, n in enumerate(widths)]
    outs = [torch.zeros((rows, n), dtype=torch.bfloat16, device="cuda") for n in widths]
    M.bctm_linear_split(M.bctm_pack_rows(dev(x)), M.bctm_pack_weight(*[dev(a) for a in ws]), outs)
    for o, wi in zip(outs, ws):
        m = np.abs(R.bf16_to_f64(x)) @ np.abs(R.bf16_to_f64(wi)).T
        check_close(host(o), R.linear(x, wi, None), 2.0 ** -20 * m, "split, many rows")


@pytest.mark.parametrize("rows,K,N", [(128, 64, 64), (200, 544, 192), (260, 4096, 320), (1030, 96, 384), (1300, 1024, 128)])
def test_swiglu_many_rows(M, rows, K, N):
    x, wg, wu = draw(5, (rows, K)), draw(6, (N, K), 2.0 * K ** -0.5), draw(7, (N, K), K ** -0.5)
    pg, pu = M.bctm_pack_weight(dev(wg)), M.bctm_pack_weight(dev(wu))
    out = M.bctm_swiglu(dev(x), pg, pu)
    xa = np.abs(R.bf16_to_f64(x))
    g, u = R.linear_f64(x, wg), R.linear_f64(x, wu)
    mg, mu = xa @ np.abs(R.bf16_to_f64(wg)).T, xa @ np.abs(R.bf16_to_f64(wu)).T
    slack = 2.0 ** -20 * (1.1 * mg * np.abs(u) + (np.abs(g) + 1.0) * mu + np.abs(g * u))
    check_close(host(out), R.swiglu(x, wg, wu), slack, f"swiglu {rows}x{K}x{N}")
    if N % 32 == 0:
        t = M.bctm_swiglu(M.bctm_pack_rows(dev(x)), pg, pu, tiled=True)
        assert np.array_equal(untile(t, rows, N), host(out))


def tiled_offsets(rows, K):
    """bf16 offset of element (r, k) in the tiled activation layout, written out from its definition."""
    r, k = np.meshgrid(np.arange(rows), np.arange(K), indexing="ij")
    block = (r // 32) * (K // 32) + k // 32
    return block * 1024 + ((r % 32) // 16) * 512 + 8 * (16 * ((k % 32) // 8) + r % 16) + k % 8


def untile(t, rows, K):
    return host(t.data.view(1, -1))[0][tiled_offsets(rows, K)]


@pytest.mark.parametrize("rows,K", [(1, 32), (16, 64), (33, 96), (70, 4096)])
def test_pack_rows_layout(M, rows, K):
    x = draw(13, (rows, K))
    t = M.bctm_pack_rows(dev(x))
    assert t.data.numel() == 32 * ((rows + 31) // 32) * K
    assert np.array_equal(untile(t, rows, K), x)


@pytest.mark.parametrize("rows,K,N", [(1, 32, 16), (32, 4096, 256), (45, 320, 64), (3, 11008, 64), (17, 2336, 16),
                                      (5, 160, 16416)])
def test_linear_tiled_input_is_bitwise_the_row_major_result(M, rows, K, N):
    x, w, res = draw(1, (rows, K)), M.bctm_pack_weight(dev(draw(2, (N, K), K ** -0.5))), dev(draw(3, (rows, N)))
    a = M.bctm_linear(dev(x), w, res)
    b = M.bctm_linear(M.bctm_pack_rows(dev(x)), w, res)
    assert np.array_equal(host(a), host(b))


@pytest.mark.parametrize("rows,K,N", [(5, 64, 32), (32, 4096, 352), (40, 544, 64)])
def test_swiglu_tiled_in_and_out(M, rows, K, N):
    x = draw(5, (rows, K))
    wg, wu = M.bctm_pack_weight(dev(draw(6, (N, K), 2.0 * K ** -0.5))), M.bctm_pack_weight(dev(draw(7, (N, K), K ** -0.5)))
    plain = host(M.bctm_swiglu(dev(x), wg, wu))
    t = M.bctm_swiglu(M.bctm_pack_rows(dev(x)), wg, wu, tiled=True)
    assert np.array_equal(untile(t, rows, N), plain)


@pytest.mark.parametrize("rows,dim", [(3, 64), (32, 4096), (37, 512)])
def test_rmsnorm_tiled_out(M, rows, dim):
    x, g = draw(8, (rows, dim), 3.0), syn.pack(1.0 + 0.1 * syn.normal(11, 9, 9, (dim,)), "bf16")
    plain = host(M.bctm_rmsnorm(dev(x), dev(g), 1e-5))
    t = M.bctm_rmsnorm(dev(x), dev(g), 1e-5, tiled=True)
    assert np.array_equal(untile(t, rows, dim), plain)


@pytest.mark.parametrize("rows,K,widths", [(32, 4096, (512, 128, 128)), (7, 320, (48, 16, 32)), (33, 64, (16, 64)),
                                           (5, 64, (6144, 3072, 3072))])
def test_linear_split_is_bitwise_the_separate_projections(M, rows, K, widths):
    import torch
    x = dev(draw(1, (rows, K)))
    ws = [dev(draw(20 + i, (n, K), K ** -0.5)) for i, n in enumerate(widths)]
    outs = [torch.empty((rows, n), dtype=torch.bfloat16, device="cuda") for n in widths]
    for xin in (x, M.bctm_pack_rows(x)):
        for o in outs:
            o.zero_()
        M.bctm_linear_split(xin, M.bctm_pack_weight(*ws), outs)
        for o, w in zip(outs, ws):
            assert np.array_equal(host(o), host(M.bctm_linear(x, M.bctm_pack_weight(w))))


def test_linear_in_place_residual(M):
    rows, K, N = 7, 256, 128
    x, w, res = draw(1, (rows, K)), draw(2, (N, K), K ** -0.5), draw(3, (rows, N))
    buf = dev(res)
    out = M.bctm_linear(dev(x), M.bctm_pack_weight(dev(w)), buf, buf)
    assert out.data_ptr() == buf.data_ptr()
    mass = np.abs(R.bf16_to_f64(x)) @ np.abs(R.bf16_to_f64(w)).T
    check_close(host(buf), R.linear(x, w, res), 2.0 ** -20 * mass, "linear in place")


def test_pack_weight_layout(M):
    # the documented layout, element by element: tile (n/16, k/32), lane 16*((k%32)/8) + n%16, 8 inputs per lane
    N, K = 48, 96
    w = np.arange(N * K, dtype=np.uint16).reshape(N, K)          # every element distinct
    got = M.bctm_pack_weight(dev(w)).data
    got = host(got.view(1, -1))[0]
    n, k = np.meshgrid(np.arange(N), np.arange(K), indexing="ij")
    off = ((n // 16) * (K // 32) + k // 32) * 512 + 8 * (16 * ((k % 32) // 8) + n % 16) + k % 8
    want = np.empty(N * K, dtype=np.uint16)
    want[off.ravel()] = w.ravel()
    assert np.array_equal(got, want)


def test_linear_selects_the_right_operands(M):
    # one-hot weight rows pick input features: exact, and fails for a transposed or shifted operand
    rows, K, N = 9, 128, 64
    x = draw(4, (rows, K))
    sel = (np.arange(N) * 37 + 5) % K
    w = np.zeros((N, K), dtype=np.float32)
    w[np.arange(N), sel] = 1.0
    wb = (w.view(np.uint32) >> 16).astype(np.uint16)
    out = host(M.bctm_linear(dev(x), M.bctm_pack_weight(dev(wb))))
    assert np.array_equal(out, x[:, sel])


@pytest.mark.parametrize("rows,K,N", [(1, 32, 16), (6, 192, 96), (32, 4096, 352), (40, 544, 64)])
def test_swiglu(M, rows, K, N):
    x, wg, wu = draw(5, (rows, K)), draw(6, (N, K), 2.0 * K ** -0.5), draw(7, (N, K), K ** -0.5)
    out = M.bctm_swiglu(dev(x), M.bctm_pack_weight(dev(wg)), M.bctm_pack_weight(dev(wu)))
    xa = np.abs(R.bf16_to_f64(x))
    g, u = R.linear_f64(x, wg), R.linear_f64(x, wu)
    mg, mu = xa @ np.abs(R.bf16_to_f64(wg)).T, xa @ np.abs(R.bf16_to_f64(wu)).T
    # d(silu)/dg is at most 1.1; the fast exponential adds a relative 2^-20 to silu
    slack = 2.0 ** -20 * (1.1 * mg * np.abs(u) + (np.abs(g) + 1.0) * mu + np.abs(g * u))
    check_close(host(out), R.swiglu(x, wg, wu), slack, f"swiglu {rows}x{K}x{N}")


@pytest.mark.parametrize("rows,dim", [(1, 8), (3, 64), (5, 520), (32, 4096), (9, 16384)])
def test_rmsnorm(M, rows, dim):
    x, g = draw(8, (rows, dim), 3.0), syn.pack(1.0 + 0.1 * syn.normal(11, 9, 9, (dim,)), "bf16")
    out = M.bctm_rmsnorm(dev(x), dev(g), 1e-5)
    ref = R.rmsnorm(x, g, 1e-5)
    check_close(host(out), ref, 2.0 ** -20 * np.abs(R.bf16_to_f64(ref)), f"rmsnorm {rows}x{dim}")


def test_embed_and_argmax_are_exact(M):
    import torch
    vocab, dim = 1000, 264
    table = draw(10, (vocab, dim))
    ids = np.array([0, 999, 5, 5, 1000, -1, 123], dtype=np.int32)
    out = host(M.bctm_embed(torch.from_numpy(ids).cuda(), dev(table)))
    assert np.array_equal(out, R.embed(ids, table))
    for rows, N in [(1, 32), (4, 1000), (33, 32000), (2, 7), (3, 1003), (2, 8200)]:   # N not a multiple of 8: element loads
        lg = draw(12, (rows, N))
        lg[0, : min(N, 5)] = 0x7F00            # several equal maxima: the lowest index wins
        lg[rows - 1, N - 1] = 0x7F00
        if rows > 2:
            lg[1, N // 3] = lg[1, N // 2] = lg[1, N - 2] = 0x7F00     # equal maxima held by different threads
        got = M.bctm_argmax(dev(lg)).cpu().numpy()
        assert np.array_equal(got, R.argmax(lg)), (rows, N)
        assert got[0] == 0 and (rows <= 2 or got[1] == N // 3)


def test_argument_errors(M):
    import torch
    w = torch.zeros((32, 72), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.BctModelError) as e:
        M.bctm_pack_weight(w)                    # K not a multiple of 32
    assert e.value.status == 2
    w = torch.zeros((40, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.BctModelError):
        M.bctm_pack_weight(w)                    # N not a multiple of 16
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ValueError):
        M.bctm_linear(x, w)                      # a row-major tensor where a packed weight is expected
    with pytest.raises(ValueError):
        M.bctm_linear(x, M.bctm_pack_weight(torch.zeros((32, 96), dtype=torch.bfloat16, device="cuda")))


# ---------------------------------------------------------------- the stack

def stack_pair(M, shape, seed, max_prefill_T=0):
    w = syn.make_stack_weights(shape, seed=seed)
    wd = {"embed": dev(w["embed"]), "final_norm": dev(w["final_norm"]), "head": dev(w["head"]),
          "layers": [{k: dev(v) for k, v in lw.items()} for lw in w["layers"]],
          "keys": [dev(k) for k in w["keys"]]}
    return R.RefStack(shape, w), M.BctStack(shape, wd, max_prefill_T=max_prefill_T)


def check_logits(got_bits, ref_bits, got_ids, ref_ids, rel, what):
    got, ref = R.bf16_to_f64(got_bits), R.bf16_to_f64(ref_bits)
    scale = np.max(np.abs(ref), axis=1, keepdims=True)
    err = np.max(np.abs(got - ref) / scale)
    assert err <= rel, f"{what}: logits differ by {err:.3e} of the row maximum (allowed {rel:.1e})"
    # the greedy token must agree wherever the oracle's winner leads by more than the allowed error
    srt = np.sort(ref, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 2 * rel * scale[:, 0]
    assert np.array_equal(got_ids[clear], ref_ids[clear]), what
    # and every token the GPU picked is within the allowed error of the oracle's best logit
    assert np.all(ref[np.arange(len(ref)), got_ids] >= srt[:, -1] - 2 * rel * scale[:, 0]), what
    return int(clear.sum())


def test_stack_decode_teacher_forced(M):
    """Eight decode steps of a 3-layer stack (GQA 2:1), both sides fed the same token ids.
    Each operation is within one bf16 spacing of the oracle's; through 3 layers of ~10 roundings each the
    logits stay within 2% of the row maximum (measured ~0.5%), which is what bf16 activations allow."""
    import torch
    s = M.StackShape(n_layers=3, dim=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=704, vocab=512,
                     capacity_M=128, batch=5)
    ref, gpu = stack_pair(M, s, seed=4)
    n_clear = 0
    for t in range(8):
        ids = syn.make_token_ids(4, t, s.batch, s.vocab)
        r_ids, r_lg = ref.forward(ids)
        g_ids, g_lg = gpu.forward(torch.from_numpy(ids).cuda())
        n_clear += check_logits(host(g_lg), r_lg, g_ids.cpu().numpy(), r_ids, 2e-2, f"step {t}")
    assert n_clear >= 20         # the token comparison was not vacuous


def test_stack_prefill_then_decode(M):
    """A 37-token chunk through bct_prefill (row b*T + t), then two decode steps on the state it left."""
    import torch
    s = M.StackShape(n_layers=2, dim=128, n_q_heads=2, n_kv_heads=2, head_dim=64, ffn=256, vocab=256,
                     capacity_M=192, batch=2)
    T = 37
    ref, gpu = stack_pair(M, s, seed=5, max_prefill_T=T)
    ids = syn.make_token_ids(5, 0, s.batch * T, s.vocab)
    r_ids, r_lg = ref.forward(ids, T=T)
    g_ids, g_lg = gpu.forward(torch.from_numpy(ids).cuda(), T=T)
    check_logits(host(g_lg), r_lg, g_ids.cpu().numpy(), r_ids, 2e-2, "chunk")
    for t in range(2):
        ids = syn.make_token_ids(5, 1 + t, s.batch, s.vocab)
        r_ids, r_lg = ref.forward(ids)
        g_ids, g_lg = gpu.forward(torch.from_numpy(ids).cuda())
        check_logits(host(g_lg), r_lg, g_ids.cpu().numpy(), r_ids, 2e-2, f"decode {t}")


def test_stack_long_chunk_through_the_many_rows_kernels(M):
    """A chunk of 3 x 70 = 210 rows: every projection runs in the matrix-core kernel (row-major W_o input
    re-tiled first), the attention in bct_prefill; logits of all rows, then of the last token only on a second
    stack (same weights, same chunk), then a decode step on the state the chunk left."""
    import torch
    s = M.StackShape(n_layers=2, dim=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=704, vocab=512,
                     capacity_M=128, batch=3)
    T = 70
    ref, gpu = stack_pair(M, s, seed=6, max_prefill_T=T)
    _, gpu2 = stack_pair(M, s, seed=6, max_prefill_T=T)
    ids = syn.make_token_ids(6, 0, s.batch * T, s.vocab)
    r_ids, r_lg = ref.forward(ids, T=T)
    g_ids, g_lg = gpu.forward(torch.from_numpy(ids).cuda(), T=T)
    check_logits(host(g_lg), r_lg, g_ids.cpu().numpy(), r_ids, 2e-2, "chunk, all rows")
    l_ids, l_lg = gpu2.forward(torch.from_numpy(ids).cuda(), T=T, head="last")
    last = np.arange(s.batch) * T + T - 1
    assert l_lg.shape == (s.batch, s.vocab) and l_ids.shape == (s.batch,)
    assert np.array_equal(host(l_lg), host(g_lg)[last])          # the same kernels on the same rows
    assert np.array_equal(l_ids.cpu().numpy(), g_ids.cpu().numpy()[last])
    ids1 = syn.make_token_ids(6, 1, s.batch, s.vocab)
    r_ids, r_lg = ref.forward(ids1)
    for g in (gpu, gpu2):
        g_ids, g_lg = g.forward(torch.from_numpy(ids1).cuda())
        check_logits(host(g_lg), r_lg, g_ids.cpu().numpy(), r_ids, 2e-2, "decode after the chunk")


def test_stack_one_layer_at_the_7b_shape(M):
    """One layer at the full Llama-7B widths of the third workload (d_model 4096, ffn 11008, vocab 32000,
    32 heads of 128, M = 4096, batch 32): an 8-token chunk (256 rows: every projection, the 12288-, 11008-
    and 32000-wide ones included, in the many-rows kernel) and a decode step (the streaming kernels) against
    the oracle.  The oracle needs about 40 s for this."""
    import torch
    s = M.StackShape(n_layers=1, dim=4096, n_q_heads=32, n_kv_heads=32, head_dim=128, ffn=11008, vocab=32000,
                     capacity_M=4096, batch=32)
    T = 8
    ref, gpu = stack_pair(M, s, seed=9, max_prefill_T=T)
    ids = syn.make_token_ids(9, 1, s.batch * T, s.vocab)
    r_ids, r_lg = ref.forward(ids, T=T)
    g_ids, g_lg = gpu.forward(torch.from_numpy(ids).cuda(), T=T)
    n_clear = check_logits(host(g_lg), r_lg, g_ids.cpu().numpy(), r_ids, 2e-2, "chunk at the 7B shape")
    ids = syn.make_token_ids(9, 0, s.batch, s.vocab)
    r_ids, r_lg = ref.forward(ids)
    g_ids, g_lg = gpu.forward(torch.from_numpy(ids).cuda())
    n_clear += check_logits(host(g_lg), r_lg, g_ids.cpu().numpy(), r_ids, 2e-2, "decode step at the 7B shape")
    assert n_clear >= 32


@pytest.mark.parametrize("case", range(12))
def test_projection_shapes_drawn_at_random(M, case):
    """Seeded sweep over row counts on both sides of the 128- and 1024-row dispatch borders, K of one to 40
    steps, feature counts that select the streaming kernel, the 128 x 128 or the 256 x 256 workgroups."""
    rng = np.random.default_rng(1000 + case)
    rows = [int(rng.integers(1, 128)), int(rng.integers(128, 1024)), int(rng.integers(1024, 1600))][case % 3]
    K = 32 * int(rng.integers(1, 41))
    N = [64, 256, 128, 256][case % 4] * int(rng.integers(1, 5)) if case % 5 else 16 * int(rng.integers(1, 20))
    tiled, with_res = bool(rng.integers(2)), bool(rng.integers(2))
    x, w = draw(30 + case, (rows, K)), draw(50 + case, (N, K), K ** -0.5)
    res = draw(70 + case, (rows, N)) if with_res else None
    xin = M.bctm_pack_rows(dev(x)) if tiled else dev(x)
    out = M.bctm_linear(xin, M.bctm_pack_weight(dev(w)), dev(res) if with_res else None)
    mass = np.abs(R.bf16_to_f64(x)) @ np.abs(R.bf16_to_f64(w)).T
    check_close(host(out), R.linear(x, w, res), 2.0 ** -20 * mass, f"linear {rows}x{K}x{N} tiled={tiled} res={with_res}")
    if N % 2 == 0 and (N // 2) % 16 == 0:
        # the same weights as gate | up halves of a SwiGLU
        wg, wu = w[: N // 2], w[N // 2:]
        o2 = M.bctm_swiglu(xin, M.bctm_pack_weight(dev(wg)), M.bctm_pack_weight(dev(wu)))
        xa = np.abs(R.bf16_to_f64(x))
        g, u = R.linear_f64(x, wg), R.linear_f64(x, wu)
        mg, mu = xa @ np.abs(R.bf16_to_f64(wg)).T, xa @ np.abs(R.bf16_to_f64(wu)).T
        slack = 2.0 ** -20 * (1.1 * mg * np.abs(u) + (np.abs(g) + 1.0) * mu + np.abs(g * u))
        check_close(host(o2), R.swiglu(x, wg, wu), slack, f"swiglu {rows}x{K}x{N // 2}")
