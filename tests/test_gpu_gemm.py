"""GPU parity of the projection GEMM on its own (hs_debug_gemm) against its plain definition, C = A . W^T in fp64 on
the same bf16 operands: every epilogue (store, add to the residual, SwiGLU -> bf16, split-K partial sums + ordered
reduce), row counts that end inside a 32-row tile, on a tile edge and beyond one row pass, a SwiGLU width whose last
weight group is ragged; rows beyond the live count stay untouched, and the row hint -- which selects launch shapes
and row passes -- never changes a bit of the result."""
import numpy as np
import pytest
import torch

from hs_inputs import ModelShape, make_weights, rope_table
from gpu_common import np_of

pytestmark = pytest.mark.gpu

M_MAX = 1100
ROWS = [1, 31, 32, 33, 100, 220, 256, 257, 385, 1054]


def bf16_to_f64(t):
    return (np_of(t).view(np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


@pytest.fixture(scope="module")
def rig():
    from paper_2508_18588_amd.runtime import Engine
    # d_ffn = 704: 44 SwiGLU units of 16 columns, not a multiple of the 4 or 5 units a workgroup takes
    shape = ModelShape(n_layers=1, d_model=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ffn=704, vocab=16448)
    w = make_weights(shape, 51)
    eng = Engine(shape, w, rope_table(64, shape.head_dim), max_batch=64, k_max=16, c_max=1, max_len=32,
                 max_rows=M_MAX)
    g = torch.Generator(device="cuda:0").manual_seed(5)
    a_d = torch.randn(M_MAX, shape.d_model, device="cuda:0", generator=g).to(torch.bfloat16).view(torch.int16)
    a_f = torch.randn(M_MAX, shape.d_ffn, device="cuda:0", generator=g).to(torch.bfloat16).view(torch.int16)
    yield shape, eng, a_d, a_f
    eng.close()


def run(eng, epi, a, w, w2, m, hint, init=None):
    n = int(w.shape[0])
    c = torch.full((M_MAX, n), 7.0 if init is None else init, dtype=torch.float32, device="cuda:0")
    if epi == 2:
        c = torch.full((M_MAX, n), 0x4170, dtype=torch.int16, device="cuda:0")      # bf16 15.0
    m_dev = torch.full((1,), m, dtype=torch.int32, device="cuda:0")
    eng.gemm(epi, a, w, w2, c, m_dev, M_MAX, hint)
    torch.cuda.synchronize()
    assert eng.poll_error() == 0
    return c


@pytest.mark.parametrize("name", ["qkv", "o", "down", "lm_head", "gate_up"])
def test_projection_equals_its_definition_for_every_row_count_and_hint(rig, name):
    shape, eng, a_d, a_f = rig
    W = eng.w
    qh = shape.n_q_heads * shape.head_dim
    a, w, w2, epi = {"qkv": (a_d, W["wqkv"][0], None, 0), "o": (a_d[:, :qh].contiguous(), W["wo"][0], None, 1),
                     "down": (a_f, W["wdown"][0], None, 1), "lm_head": (a_d, W["lm_head"], None, 0),
                     "gate_up": (a_d, W["wgate"][0], W["wup"][0], 2)}[name]
    af, wf = bf16_to_f64(a), bf16_to_f64(w)
    for m in ROWS:
        want = af[:m] @ wf.T
        if epi == 2:
            up = af[:m] @ bf16_to_f64(w2).T
            want = want / (1.0 + np.exp(-want)) * up
        elif epi == 1:
            want = want + 7.0                                   # added to what the output held
        outs = []
        for hint in (m, 1, 5000):
            c = run(eng, epi, a, w, w2, m, hint)
            got = bf16_to_f64(c) if epi == 2 else np_of(c).astype(np.float64)
            scale = np.abs(want).max() + 1.0
            # fp32 accumulation over k <= 1024 (store/add); one bf16 rounding of the result (SwiGLU)
            tol = 2.0 ** -8 * scale if epi == 2 else 2e-5 * scale
            assert np.abs(got[:m] - want).max() <= tol, (name, m, hint)
            rest = np_of(c)[m:]
            assert (rest == (0x4170 if epi == 2 else 7.0)).all(), (name, m, hint, "rows beyond M were written")
            outs.append(np_of(c)[:m].copy())
        assert (outs[0] == outs[1]).all() and (outs[0] == outs[2]).all(), (name, m, "row hint changed the bits")


@pytest.mark.parametrize("vocab", [4160, 4097])
def test_lm_head_of_a_small_vocabulary_splits_k_and_has_room_for_its_partial_sums(vocab):
    """vocab 4160 with d_model 1024: the LM head runs in 3 K chunks whose partial sums (3 x 4160 columns) are wider
    than those of any layer projection; the workspace must hold them.  One projection against its definition, then a
    few decode steps end to end (the LM head inside hs_verify) against the oracle.  vocab 4097: rows of the partial
    sums and of the logits are not 16-byte aligned (the ordered reduce and the argmax take their scalar paths)."""
    import oracle
    from paper_2508_18588_amd.runtime import Engine, Policy
    from gpu_common import OracleBatch
    from test_gpu_decode import lockstep
    shape = ModelShape(n_layers=1, d_model=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ffn=1024, vocab=vocab)
    w = make_weights(shape, 53)
    rope = rope_table(128, shape.head_dim)
    eng = Engine(shape, w, rope, max_batch=4, k_max=4, c_max=1, max_len=64, max_rows=300)
    g = torch.Generator(device="cuda:0").manual_seed(6)
    a = torch.randn(300, shape.d_model, device="cuda:0", generator=g).to(torch.bfloat16).view(torch.int16)
    want = bf16_to_f64(a) @ bf16_to_f64(eng.w["lm_head"]).T
    for m in (3, 300):
        c = torch.zeros(300, shape.vocab, dtype=torch.float32, device="cuda:0")
        m_dev = torch.full((1,), m, dtype=torch.int32, device="cuda:0")
        eng.gemm(0, a, eng.w["lm_head"], None, c, m_dev, 300, m)
        torch.cuda.synchronize()
        assert np.abs(np_of(c)[:m] - want[:m]).max() <= 2e-5 * (np.abs(want).max() + 1.0)
        assert not np_of(c)[m:].any()
    rng = np.random.default_rng(9)
    prompts = [rng.integers(0, shape.vocab, 20).astype(np.int32) for _ in range(4)]
    eng.load_sequences(prompts, budgets=[6] * 4)
    eng.set_history([[np.zeros(0, np.int32)] for _ in prompts])
    eng.prefill(prompts)
    ob = OracleBatch(oracle.Model(shape, w, rope), prompts, [6] * 4, 64)
    stats = lockstep(eng, ob, [[np.zeros(0, np.int32)] for _ in prompts], Policy(window=8, m_min=3, k_fixed=0, k_max=4),
                     max_steps=6)
    assert stats["emitted"] == 24
    eng.close()


REAL_SHAPES = {
    # the layer projections of the 7B shape (configurations 3 and 4) and of the 14B shape (configuration 5)
    "7b": ModelShape(n_layers=1, d_model=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, d_ffn=18944, vocab=16448),
    "14b": ModelShape(n_layers=1, d_model=5120, n_q_heads=40, n_kv_heads=8, head_dim=128, d_ffn=13824, vocab=16448),
}


@pytest.mark.parametrize("which", ["7b", "14b"])
def test_projections_at_the_real_layer_shapes(which):
    """Each layer projection at its real (N, K) -- 7B: QKV 4608 x 3584, O 3584 x 3584, gate/up 2 x 18944 x 3584, down
    3584 x 18944 (nine K chunks); 14B: 7168 x 5120, 5120 x 5120, 2 x 13824 x 5120, 5120 x 13824 -- at 220, 385, 1054
    and 2176 rows (one short pass, two passes, three, six), against C = A . W^T: every element against an fp64 matrix
    product (library routine on the device), sampled rows and columns against fp64 dot products on the host; rows
    beyond M untouched; bits independent of the row hint."""
    from hs_inputs.device import make_weights_device
    from paper_2508_18588_amd.runtime import Engine
    shape = REAL_SHAPES[which]
    m_max = 2176
    w = make_weights_device(shape, 61, 1)
    eng = Engine(shape, w, rope_table(64, shape.head_dim), max_batch=128, k_max=16, c_max=1, max_len=32,
                 max_rows=m_max, keep_logits=False)
    g = torch.Generator(device="cuda:0").manual_seed(8)
    qh = shape.n_q_heads * shape.head_dim
    a_d = torch.randn(m_max, shape.d_model, device="cuda:0", generator=g).to(torch.bfloat16)
    a_q = torch.randn(m_max, qh, device="cuda:0", generator=g).to(torch.bfloat16)
    a_f = torch.randn(m_max, shape.d_ffn, device="cuda:0", generator=g).to(torch.bfloat16)
    W = eng.w
    rng = np.random.default_rng(12)
    cases = {"qkv": (a_d, W["wqkv"][0], None, 0), "o": (a_q, W["wo"][0], None, 1),
             "gate_up": (a_d, W["wgate"][0], W["wup"][0], 2), "down": (a_f, W["wdown"][0], None, 1)}
    for name, (a, wt, w2, epi) in cases.items():
        n, k = int(wt.shape[0]), int(wt.shape[1])
        ref = a.double() @ wt.double().T                       # [m_max, n] fp64 on the device
        if epi == 2:
            ref = ref / (1.0 + torch.exp(-ref)) * (a.double() @ w2.double().T)
        elif epi == 1:
            ref = ref + 7.0
        scale = float(ref.abs().max()) + 1.0
        for m in (220, 385, 1054, 2176):
            outs = []
            for hint in (m, 1, 5000):
                fill = 0x4170 if epi == 2 else 7.0
                c = torch.full((m_max, n), fill, dtype=torch.int16 if epi == 2 else torch.float32, device="cuda:0")
                m_dev = torch.full((1,), m, dtype=torch.int32, device="cuda:0")
                eng.gemm(epi, a.view(torch.int16), wt, w2, c, m_dev, m_max, hint)
                torch.cuda.synchronize()
                assert eng.poll_error() == 0
                got = c.view(torch.bfloat16).double() if epi == 2 else c.double()
                err = (got[:m] - ref[:m]).abs()
                if epi == 2:   # one bf16 rounding of the result (+ the epilogue's hardware exponential / reciprocal)
                    ok = bool((err <= 1.5 * 2.0 ** -8 * ref[:m].abs() + 4e-5 * scale).all())
                else:          # fp32 accumulation over K in the shape's chunk order
                    ok = float(err.max()) <= 2e-5 * scale
                assert ok, (which, name, m, hint, float(err.max()))
                assert bool((c[m:] == fill).all()), (which, name, m, hint, "rows beyond M were written")
                outs.append(c[:m].clone())
            assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2]), (name, m, "row hint changed bits")
            # sampled outputs against fp64 dot products computed on the host
            rs = np.unique(np.concatenate([rng.integers(0, m, 6), [0, m - 1, min(m - 1, 383), min(m - 1, 384)]]))
            cs = np.unique(np.concatenate([rng.integers(0, n, 12), [0, n - 1, 63, 64, 159, 160]]))
            ah = bf16_to_f64(a.view(torch.int16)[torch.as_tensor(rs, device="cuda:0")])
            want = ah @ bf16_to_f64(wt.view(torch.int16)[torch.as_tensor(cs, device="cuda:0")]).T
            if epi == 2:
                up = ah @ bf16_to_f64(w2.view(torch.int16)[torch.as_tensor(cs, device="cuda:0")]).T
                want = want / (1.0 + np.exp(-want)) * up
            elif epi == 1:
                want = want + 7.0
            sub = outs[0][torch.as_tensor(rs, device="cuda:0")][:, torch.as_tensor(cs, device="cuda:0")]
            sub = bf16_to_f64(sub) if epi == 2 else np_of(sub).astype(np.float64)
            tol = 1.5 * 2.0 ** -8 * np.abs(want) + 4e-5 * scale if epi == 2 else 2e-5 * scale
            assert (np.abs(sub - want) <= tol).all(), (which, name, m, "host dot products")
        del ref
    eng.close()
