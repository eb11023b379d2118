"""Pins of the CPU oracle against things other than itself: public parameter
counts, closed forms, the paper's printed memory formulas, invariants, brute
force, and numpy's Philox.  CPU only."""
import itertools
import os

import numpy as np
import pytest

from paper_2412_04788_amd import workloads as wl
from tests import bridge

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    vals = {}
    with open(os.path.join(GOLD, name)) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split()
                vals[k] = int(v)
    return vals


# ------------------------------------------------------------------ parameters

def test_param_counts_of_public_shapes(ora):
    """Stored parameters of the 7B shape plus its (2L+1)*d norm weights equal the
    publicly stated 6 738 415 616; the other shapes are fixed by hand arithmetic."""
    gold = _gold("param_counts.txt")
    for m in wl.MODELS_FULL:
        assert ora.params_total(bridge.ora_model(m)) == gold[m.name]
    m = wl.DENSE_7B
    assert ora.params_total(bridge.ora_model(m)) + (2 * m.L + 1) * m.d == gold["dense-7b-with-norms"]


def test_param_count_formula_by_hand(ora):
    for m in wl.MODELS_FULL:
        dh = m.d // m.n_h
        attn = m.d * m.n_h * dh * 2 + 2 * m.d * m.n_kv * dh
        ffn = 3 * m.d * m.d_ff * m.E
        router = m.d * m.E if m.E > 1 else 0
        assert ora.params_total(bridge.ora_model(m)) == m.L * (attn + ffn + router) + 2 * m.V * m.d
        assert ora.params_layer_active(bridge.ora_model(m)) == attn + 3 * m.d * m.d_ff * m.k + router


# ----------------------------------------------------------------------- FLOPs

@pytest.mark.parametrize("m", wl.MODELS_FULL, ids=lambda m: m.name)
@pytest.mark.parametrize("p", [1, 2, 8])
def test_linear_flops_are_two_params_tokens(ora, m, p):
    """Sum of the matmul FLOPs of a pass (all ops but attention), times p GPUs,
    is 2 * active parameters * tokens + 2 * LM-head rows * V * d."""
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    T, n_lm = 777.0, 5.0
    r = ora.pass_detail(om, oh, p, 16, T, T * 100, T * 3, n_lm)
    lin = r["F"][[0, 2, 3, 4, 5]].sum() * p
    if m.E > 1:  # router is replicated, not split
        lin -= r["F"][5] * (p - 1)
    assert lin == 2.0 * ora.params_layer_active(om) * T
    assert r["F"][7] * p == 2.0 * n_lm * m.V * m.d
    assert r["F"][6] == 0.0
    # the LM head reads its d x V slice and moves n_lm rows (not T) in and out
    assert r["B"][7] == 2 * m.d * m.V / p + 2 * n_lm * m.d + 2 * n_lm * m.V / p
    assert r["B"][6] == 8 * T * m.d


def test_attention_flops_and_kv_bytes(ora):
    """Attention: 4 * d_h * n_h FLOPs per (query, context) pair (QK^T and PV, 2
    FLOPs per MAC); KV read: K and V, 2 bytes each, g_kv elements per token."""
    m = wl.DENSE_34B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    r = ora.pass_detail(om, oh, 1, 16, 1.0, 1000.0, 1000.0, 1.0)
    assert r["F"][1] == 4 * m.d * 1000
    dh = m.d // m.n_h
    assert r["B"][1] == 2 * 2 * 1 * m.d + 2 * 2 * m.n_kv * dh * 1000
    # TP 16 > 8 KV heads: each GPU still holds one full KV head
    r = ora.pass_detail(om, oh, 16, 16, 1.0, 1000.0, 1000.0, 1.0)
    assert r["B"][1] == 2 * 2 * m.d / 16 + 2 * 2 * dh * 1000


# ------------------------------------------------------------ batch-1 decode

def test_batch1_decode_step_is_weight_bytes_over_bandwidth(ora):
    """Tiny profile (ridge 200 FLOP/B): every op of a batch-1 decode step is
    memory bound, so step time * BW = weight bytes read + KV bytes + activation
    bytes exactly; weight bytes of the 7B shape in fp16 = 13 214 154 752 (all
    layers + LM head, embedding table not read)."""
    gold = _gold("decode_bytes.txt")
    m = wl.DENSE_7B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    ctx = 128.0
    r = ora.pass_detail(om, oh, 1, 16, 1.0, ctx, ctx, 1.0)
    w_read = 2 * (ora.params_total(om) - m.V * m.d)
    assert w_read == gold["w_read_7b_fp16"]
    kv = 2 * 2 * m.n_kv * (m.d // m.n_h) * m.L * ctx
    assert kv == gold["kv_bytes_ctx128"]
    act_layer = (2 * m.d + 2 * 3 * m.d) + (2 * 2 * m.d) + (2 * m.d + 2 * m.d) + (2 * m.d + 2 * 2 * m.d_ff) \
        + (2 * m.d_ff + 2 * m.d) + 4 * 2 * m.d
    act = m.L * act_layer + 2 * m.d + 2 * m.V
    assert r["t_pass"] * wl.HW_TINY.hbm_bw == pytest.approx(w_read + kv + act, rel=1e-14)
    # all ops memory bound
    assert np.all(r["F"] / wl.HW_TINY.peak_flops <= r["B"] / wl.HW_TINY.hbm_bw)
    assert abs(r["t_pass"] - w_read / wl.HW_TINY.hbm_bw) / r["t_pass"] < 0.01
    assert w_read / wl.HW_TINY.hbm_bw == pytest.approx(2.6428309504e-3, rel=1e-12)


def test_decode_sum_closed_form_when_memory_bound(ora):
    """All-memory-bound decode: t_decode * BW = (s_out-1) * C0 + 4 g_kv L b * sum_{j}(s_in + j)."""
    m = wl.DENSE_7B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    b, s_in, s_out = 2, 256, 300
    r = ora.evaluate(om, oh, ora.knobs(b, s_in, s_out))
    c0 = ora.pass_detail(om, oh, 1, 16, float(b), 0.0, 0.0, float(b))["t_pass"] * wl.HW_TINY.hbm_bw
    n = s_out - 1
    series = n * s_in + n * (n + 1) // 2
    expect = n * c0 + 4 * m.d * m.L * b * series
    assert r.t_decode * wl.HW_TINY.hbm_bw == pytest.approx(expect, rel=1e-12)
    assert r.tpot == pytest.approx(r.t_decode / n, rel=1e-15)
    assert r.decode_tok_s == pytest.approx(b * n / r.t_decode, rel=1e-15)
    assert r.t_batch == r.t_prefill + r.t_decode
    assert r.cost == pytest.approx(1 * r.t_batch / 3600 * 1e6 / (b * s_out), rel=1e-15)


def test_compute_bound_prefill(ora):
    """Large prefill on the tiny profile: matmul ops take F / P."""
    m = wl.DENSE_7B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    T = 4096.0
    r = ora.pass_detail(om, oh, 1, 16, T, T * T, T, 1.0)
    for i in (0, 2, 3, 4):
        assert r["t"][i] == r["F"][i] / wl.HW_TINY.peak_flops
    assert r["t"][6] == r["B"][6] / wl.HW_TINY.hbm_bw     # norms are always bandwidth bound
    # additive variant is the sum of both terms
    ra = ora.pass_detail(om, oh, 1, 16, T, T * T, T, 1.0, time_model=ora.ADDITIVE)
    np.testing.assert_allclose(ra["t"], r["F"] / wl.HW_TINY.peak_flops + r["B"] / wl.HW_TINY.hbm_bw, rtol=1e-15)


def test_s_out_one_has_no_decode(ora):
    om, oh = bridge.ora_model(wl.DENSE_7B), bridge.ora_hw(wl.HW_TINY)
    r = ora.evaluate(om, oh, ora.knobs(4, 128, 1))
    assert r.t_decode == 0.0 and r.tpot == 0.0 and r.decode_tok_s == 0.0 and r.t_batch == r.t_prefill


# ---------------------------------------------------------------------- memory

def test_kv_formula_reduces_to_the_papers(ora):
    """MHA, p = 1, block 1: kv per request = 2 * N * H * S * kv (Dynamic Batch Size
    Adjustment) and B_max = floor(C_available / that)."""
    m = wl.DENSE_13B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    kn = ora.knobs(3, 700, 55, blk=1)
    r = ora.memory(om, oh, kn)
    assert r["kv_req"] == 2 * m.L * m.d * (700 + 55) * 2
    c_avail = wl.HW_TINY.cap_bytes - 2 * ora.params_total(om)
    assert r["c_avail"] == c_avail
    assert r["b_max"] == int(c_avail // r["kv_req"])


def test_kv_block_rounding_and_gqa_tp(ora):
    m = wl.DENSE_70B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    r = ora.memory(om, oh, ora.knobs(1, 100, 29, p=4, blk=32))
    dh = m.d // m.n_h
    assert r["kv_req"] == 160 * 2 * m.L * (m.n_kv // 4) * dh * 2
    assert ora.kv_bytes_token(om, 16) == 2 * m.L * dh * 2   # replicated head


@pytest.mark.parametrize("p,wbits", [(1, 16), (2, 8), (8, 4)])
def test_feasibility_boundary(ora, p, wbits):
    m = wl.DENSE_34B
    om = bridge.ora_model(m)
    b, kn = 37, ora.knobs(37, 1000, 200, p=p, wbits=wbits, blk=16)
    kv_req = ora.memory(om, bridge.ora_hw(wl.HW_TINY), kn)["kv_req"]
    w_gpu = ora.weight_bytes_gpu(om, p, wbits)
    assert w_gpu == wbits / 8 * ora.params_total(om) / p
    cap = w_gpu + b * kv_req
    h = wl.Hardware(1e15, 5e12, cap, 4e11)
    r = ora.memory(om, bridge.ora_hw(h), kn)
    assert r["feasible"] == 1 and r["b_max"] == b
    h = wl.Hardware(1e15, 5e12, cap - 1.0, 4e11)
    r = ora.memory(om, bridge.ora_hw(h), kn)
    assert r["feasible"] == 0 and r["b_max"] == b - 1
    h = wl.Hardware(1e15, 5e12, w_gpu, 4e11)           # nothing left for KV
    r = ora.memory(om, bridge.ora_hw(h), kn)
    assert r["feasible"] == 0 and r["b_max"] == 0


# ---------------------------------------------------------- prefill structure

def test_prefill_sub_batches_and_segments(ora):
    m = wl.DENSE_7B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)

    def one(R, s):
        return ora.pass_detail(om, oh, 1, 16, R * s, R * s * s, R * s, R)["t_pass"]

    # 10 prompts of 1000 tokens under 4096 tokens per pass: 4 + 4 + 2
    t = ora.prefill(om, oh, ora.knobs(10, 1000, 8, mbt=4096))
    assert t == (one(4, 1000) + one(4, 1000)) + one(2, 1000)
    # prompt longer than the budget: 3 segments of 2048, 2048, 904, per request
    t = ora.prefill(om, oh, ora.knobs(2, 5000, 8, mbt=2048))
    segs = [(2048, 2048, 0), (2048, 4096, 0), (904, 5000, 1)]
    tot = 0.0
    for _ in range(2):
        for c, ctx, lm in segs:
            tot += ora.pass_detail(om, oh, 1, 16, c, c * ctx, ctx, lm)["t_pass"]
    assert t == tot
    # everything fits one pass
    assert ora.prefill(om, oh, ora.knobs(4, 512, 8, mbt=8192)) == one(4, 512)


def test_monotone_in_lengths_and_batch(ora):
    g = wl.grid_tiny()
    r = ora.eval_grid(bridge.ora_grid(g))
    shape = g.radices
    for col in ("t_prefill", "t_batch"):
        a = r[col].reshape(shape)
        for ax in (2, 3, 4):          # batch, s_in, s_out
            assert np.all(np.diff(a, axis=ax) >= 0), (col, ax)
    assert np.all(np.diff(r["t_decode"].reshape(shape), axis=4) > 0)


# ---------------------------------------------------------------- TP and comm

def test_tp_scaling_and_comm_term(ora):
    m = wl.DENSE_7B
    om = bridge.ora_model(m)
    h_inf = bridge.ora_hw(wl.Hardware(1e15, 5e12, 192 * wl.GIB, float("inf"), 0.0))
    T, Q, K = 512.0, 512.0 * 512, 512.0
    r1 = ora.pass_detail(om, h_inf, 1, 16, T, Q, K, 1.0)
    assert r1["t_ar"] == 0.0
    for p in (2, 4, 8):
        rp = ora.pass_detail(om, h_inf, p, 16, T, Q, K, 1.0)
        np.testing.assert_array_equal(rp["F"] * p, r1["F"])
        assert rp["t_ar"] == 0.0
        # weight and KV bytes scale 1/p: compare at zero tokens / pure KV
        w1 = ora.pass_detail(om, h_inf, 1, 16, 0.0, 0.0, 0.0, 0.0)["B"]
        wp = ora.pass_detail(om, h_inf, p, 16, 0.0, 0.0, 0.0, 0.0)["B"]
        np.testing.assert_array_equal(wp * p, w1)
    # ring all-reduce: 2(p-1)/p * bytes / link + 2(p-1) * latency
    h = wl.Hardware(1e15, 5e12, 192 * wl.GIB, 4e11, 3e-6)
    r = ora.pass_detail(om, bridge.ora_hw(h), 4, 16, T, Q, K, 1.0)
    assert r["t_ar"] == pytest.approx(2 * 3 / 4 * (2 * T * m.d) / 4e11 + 2 * 3 * 3e-6, rel=1e-15)
    assert r["t_pass"] == pytest.approx(m.L * (r["t"][:7].sum() + 2 * r["t_ar"]) + r["t"][7], rel=1e-15)


# ------------------------------------- MoE expert loading, router, GQA, head split

@pytest.mark.parametrize("T", [1, 3, 8])
def test_moe_expert_and_router_bytes(ora, T):
    """A pass over T tokens reads min(E, k*T) experts' FFN weights (2, 6, 8 of the 8 top-2 experts for
    T = 1, 3, 8); the router reads its d x E matrix, the T x d input and writes T x E scores."""
    gold = _gold("op_bytes.txt")
    m = wl.MOE_8X
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    r = ora.pass_detail(om, oh, 1, 16, float(T), 100.0 * T, 100.0 * T, float(T))
    assert r["B"][3] == gold[f"moe_up_bytes_T{T}"]
    assert r["B"][4] == gold[f"moe_down_bytes_T{T}"]
    assert r["B"][5] == gold[f"moe_router_bytes_T{T}"]
    assert r["F"][5] == 2 * T * m.d * m.E
    if T in (1, 8):
        assert r["F"][5] == gold[f"moe_router_flops_T{T}"]
    n_exp = min(m.E, m.k * T)
    assert r["B"][3] == 2 * n_exp * 2 * m.d * m.d_ff + 2 * T * m.d + 4 * T * m.k * m.d_ff
    assert r["B"][5] == 2 * m.d * m.E + 2 * T * m.d + 2 * T * m.E


def test_moe_bytes_quantised_and_split(ora):
    """int4 weights on 2 GPUs: expert weights are split, the router is replicated."""
    gold = _gold("op_bytes.txt")
    om, oh = bridge.ora_model(wl.MOE_8X), bridge.ora_hw(wl.HW_TINY)
    r = ora.pass_detail(om, oh, 2, 4, 1.0, 100.0, 100.0, 1.0)
    assert r["B"][3] == gold["moe_up_bytes_T1_int4_tp2"]
    assert r["B"][4] == gold["moe_down_bytes_T1_int4_tp2"]
    assert r["B"][5] == gold["moe_router_bytes_T1_int4_tp2"]


@pytest.mark.parametrize("T", [1, 8])
def test_moe_decode_step_is_bytes_over_bandwidth(ora, T):
    """Decode step of the MoE shape with batch T on the tiny profile: every op is memory bound (ridge 200 FLOP/B),
    so step time * BW is every byte the step moves -- 2 (T = 1) or all 8 (T = 8) experts per layer."""
    gold = _gold("op_bytes.txt")
    m = wl.MOE_8X
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    ctx = 256.0
    r = ora.pass_detail(om, oh, 1, 16, float(T), T * ctx, T * ctx, float(T))
    assert np.all(r["F"] / wl.HW_TINY.peak_flops <= r["B"] / wl.HW_TINY.hbm_bw)
    assert r["t_pass"] * wl.HW_TINY.hbm_bw == pytest.approx(gold[f"moe_step_bytes_T{T}_ctx256"], rel=1e-14)
    # the same through the candidate evaluator: two decode passes at contexts 255 + 1 and 255 + 2
    e = ora.evaluate(om, oh, ora.knobs(T, 255, 3))
    r2 = ora.pass_detail(om, oh, 1, 16, float(T), T * 257.0, T * 257.0, float(T))
    assert e.t_decode == r["t_pass"] + r2["t_pass"]


@pytest.mark.parametrize("m", [wl.DENSE_34B, wl.DENSE_70B], ids=lambda m: m.name)
def test_gqa_qkv_projection(ora, m):
    """With 8 KV heads of 128 the qkv projection has dq + 2 dkv = 10 240 output columns."""
    gold = _gold("op_bytes.txt")
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    for p, wbits, T, tag in ((1, 16, 1, "fp16_tp1_T1"), (4, 8, 512, "int8_tp4_T512"), (8, 4, 64, "int4_tp8_T64")):
        r = ora.pass_detail(om, oh, p, wbits, float(T), 7.0 * T, 7.0 * T, 1.0)
        assert r["F"][0] == gold[f"gqa_qkv_flops_{tag}"]
        assert r["B"][0] == gold[f"gqa_qkv_bytes_{tag}"]
    # MHA for contrast: 3 d columns
    r = ora.pass_detail(bridge.ora_model(wl.DENSE_7B), oh, 1, 16, 1.0, 7.0, 7.0, 1.0)
    assert r["B"][0] == 2 * 4096 * 3 * 4096 + 2 * 4096 + 2 * 3 * 4096


def test_kv_heads_per_gpu_when_tp_does_not_divide(ora):
    """ceil(n_kv / p) whole KV heads per GPU: 8 heads over 3, 5, 6 GPUs leave 3, 2, 2."""
    gold = _gold("op_bytes.txt")
    o70, o34 = bridge.ora_model(wl.DENSE_70B), bridge.ora_model(wl.DENSE_34B)
    oh = bridge.ora_hw(wl.HW_TINY)
    for p in (1, 2, 3, 4, 5, 6, 8, 16):
        assert ora.kv_bytes_token(o70, p) == gold[f"kv_token_bytes_70b_tp{p}"]
    assert ora.kv_bytes_token(o34, 3) == gold["kv_token_bytes_34b_tp3"]
    assert ora.kv_bytes_token(o34, 6) == gold["kv_token_bytes_34b_tp6"]
    # the attention op reads that many bytes per cached token and layer: 2 (K, V) * heads * 128 * 2 B
    for p, heads in ((3, 3), (5, 2), (6, 2), (16, 1)):
        r = ora.pass_detail(o70, oh, p, 16, 1.0, 1000.0, 1000.0, 1.0)
        assert r["B"][1] == pytest.approx(4 * 8192 / p + 4 * heads * 128 * 1000, rel=1e-15)
    # and the memory check sizes a request with it
    r = ora.memory(o70, oh, ora.knobs(1, 100, 28, p=3, blk=16))
    assert r["kv_req"] == 128 * gold["kv_token_bytes_70b_tp3"]
    r = ora.memory(o70, oh, ora.knobs(1, 100, 28, p=6, blk=16))
    assert r["kv_req"] == 128 * gold["kv_token_bytes_70b_tp6"]


def test_efficiency_does_not_scale_the_link(ora):
    """Efficiency factors scale peak and memory bandwidth only: at p = 4 with a finite link, e_c = e_b = 1/2
    doubles every op time and leaves the all-reduce time as it was."""
    m = wl.DENSE_13B
    om = bridge.ora_model(m)
    h = wl.Hardware(1e15, 5e12, 192 * wl.GIB, 4e11, 3e-6)
    oh = bridge.ora_hw(h)
    T, Q, K = 640.0, 640.0 * 640, 640.0
    base = ora.pass_detail(om, oh, 4, 16, T, Q, K, 1.0)
    half = ora.pass_detail(om, oh, 4, 16, T, Q, K, 1.0, 0.5, 0.5)
    t_ar = 2 * 3 / 4 * (2 * T * m.d) / 4e11 + 2 * 3 * 3e-6
    assert base["t_ar"] == pytest.approx(t_ar, rel=1e-15) and half["t_ar"] == base["t_ar"]
    np.testing.assert_allclose(half["t"], 2 * base["t"], rtol=1e-15)
    assert half["t_pass"] == pytest.approx(m.L * (2 * base["t"][:7].sum() + 2 * t_ar) + 2 * base["t"][7], rel=1e-14)
    assert half["t_pass"] < 2 * base["t_pass"] * (1 - 1e-3)      # the comm share is visible at this size
    # only bandwidth scaled: memory-bound ops double, compute-bound ones stay, comm stays
    bw_half = ora.pass_detail(om, oh, 4, 16, T, Q, K, 1.0, 1.0, 0.5)
    assert bw_half["t_ar"] == base["t_ar"]
    assert bw_half["t"][6] == pytest.approx(2 * base["t"][6], rel=1e-15)
    # through the candidate evaluator as well
    kn = ora.knobs(8, 512, 64, p=4)
    e1, e2 = ora.evaluate(om, oh, kn), ora.evaluate(om, oh, kn, 0.5, 0.5)
    comm_prefill = m.L * 2 * (2 * 3 / 4 * (2 * 8 * 512 * m.d) / 4e11 + 6 * 3e-6)
    assert e2.t_prefill - comm_prefill == pytest.approx(2 * (e1.t_prefill - comm_prefill), rel=1e-12)


# --------------------------------------------------------- uncertainty sweep

def test_efficiency_scaling_and_percentiles(ora):
    m = wl.DENSE_13B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    kn = ora.knobs(8, 512, 64)
    base = ora.evaluate(om, oh, kn)
    half = ora.evaluate(om, oh, kn, 0.5, 0.5)
    assert half.t_prefill == pytest.approx(2 * base.t_prefill, rel=1e-14)
    assert half.t_decode == pytest.approx(2 * base.t_decode, rel=1e-14)
    g = bridge.ora_grid(wl.make_grid([m], [wl.HW_TINY], wl.Axis.table([8]), wl.Axis.table([512]), wl.Axis.table([64]),
                                     wl.Axis.table([1]), wl.Axis.table([16]), wl.Axis.table([16]),
                                     wl.Axis.table([8192])))
    ones = np.ones(64)
    s = ora.eval_sweep_grid(g, ones, ones)
    assert s["ttft_p10"][0] == s["ttft_p90"][0] == base.t_prefill
    assert s["ttft_mean"][0] == pytest.approx(base.t_prefill, rel=1e-15)
    # distinct samples: e = 1/(i+1) scales every time by (i+1) -> sorted order known
    e = 1.0 / np.arange(1, 65)
    s = ora.eval_sweep_grid(g, e, e)
    xs = np.array([ora.evaluate(om, oh, kn, ei, ei).t_batch for ei in e])
    assert s["t_batch_p10"][0] == np.sort(xs)[6] and s["t_batch_p90"][0] == np.sort(xs)[57]
    assert s["t_batch_mean"][0] == pytest.approx(xs.mean(), rel=1e-14)
    assert s["t_batch_p10"][0] <= s["t_batch_mean"][0] <= s["t_batch_p90"][0]
    assert s["cost"][0] == pytest.approx(s["t_batch_mean"][0] / 3600 * 1e6 / (8 * 64), rel=1e-15)
    # nearest rank for n = 10: ceil(1) - 1 = 0 and ceil(9) - 1 = 8
    e10 = 1.0 / np.arange(1, 11)
    s = ora.eval_sweep_grid(g, e10, e10)
    xs = np.sort([ora.evaluate(om, oh, kn, ei, ei).t_prefill for ei in e10])
    assert s["ttft_p10"][0] == xs[0] and s["ttft_p90"][0] == xs[8]


# ------------------------------------------------------------------ grid order

def test_flat_index_order(ora):
    g = wl.grid_full()
    og = bridge.ora_grid(g)
    assert og.size == 1900800 == g.size
    rng = np.random.default_rng(3)
    for idx in rng.integers(0, g.size, 20):
        mi, hi, b, s_in, s_out, p, wb, blk, mbt = g.values_at(int(idx))
        r = ora.eval_grid(og, int(idx), 1)
        e = ora.evaluate(bridge.ora_model(g.models[mi]), bridge.ora_hw(g.hws[hi]),
                         ora.knobs(b, s_in, s_out, p, wb, blk, mbt))
        assert r["t_batch"][0] == e.t_batch and r["b_max"][0] == e.b_max
    # fastest axis is max-batched-tokens, slowest the model
    assert g.values_at(1)[8] == 4096 and g.values_at(0)[8] == 2048
    assert g.values_at(g.size // 5)[0] == 1
    with pytest.raises(ValueError):
        ora.eval_grid(og, g.size - 1, 2)


# ------------------------------------------------------------------ simulation

def _one_req(n_in, n_out):
    return np.array([0.0]), np.array([n_in], dtype=np.uint32), np.array([n_out], dtype=np.uint32)


@pytest.mark.parametrize("n_in,n_out,mbt", [(700, 40, 2048), (5000, 17, 2048), (2048, 1, 2048), (16, 300, 8192)])
def test_single_request_simulation_equals_analytic(ora, n_in, n_out, mbt):
    m = wl.DENSE_34B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    arr, ins, outs = _one_req(n_in, n_out)
    s = ora.simulate(om, oh, 2, 8, 16, mbt, 4, 1.0, arr, ins, outs, detail=True)
    e = ora.evaluate(om, oh, ora.knobs(1, n_in, n_out, p=2, wbits=8, blk=16, mbt=mbt))
    assert s["status"] == ora.SIM_OK
    assert s["ttft"][0] == e.t_prefill
    assert s["fin"][0] == pytest.approx(e.t_batch, rel=1e-13)
    n_chunks = -(-n_in // mbt)
    assert s["n_steps"] == n_chunks + n_out - 1 == s["n_request_steps"]
    assert s["ttft_p50"] == s["ttft_p99"] == e.t_prefill
    if n_out > 1:
        assert s["mean_tpot"] == pytest.approx(e.tpot, rel=1e-13)
    assert s["tokens_s"] == pytest.approx(n_out / s["fin"][0], rel=1e-15)


def test_simulation_invariants(ora):
    m = wl.DENSE_7B
    om = bridge.ora_model(m)
    h = wl.Hardware(1e15, 5e12, 40 * wl.GIB, 4e11)          # tight KV pool
    oh = bridge.ora_hw(h)
    tr = wl.request_trace(n=200)
    for max_seqs, rate, mbt in [(1, 4.0, 2048), (8, 16.0, 2048), (64, 64.0, 8192), (256, 64.0, 4096)]:
        s = ora.simulate(om, oh, 1, 16, 16, mbt, max_seqs, rate, tr.arrival_unit, tr.n_in, tr.n_out, detail=True)
        assert s["status"] == ora.SIM_OK
        assert s["min_free"] >= 0
        arr = tr.arrival_unit / rate
        assert np.all(s["first"] > arr) and np.all(s["fin"] >= s["first"])
        assert np.all(np.diff(s["first"]) >= 0)            # FCFS: first tokens in arrival order
        # every request emits out tokens: out-1 decode steps + its prompt chunks
        assert s["n_request_steps"] >= int(tr.n_out.sum() - len(arr) + len(arr))
        assert s["n_request_steps"] <= int((tr.n_out.astype(np.int64) - 1).sum() +
                                           (-(-tr.n_in.astype(np.int64) // 1)).sum())
        np.testing.assert_array_equal(s["ttft"], s["first"] - arr)
        assert s["ttft_p50"] == np.sort(s["ttft"])[99] and s["ttft_p99"] == np.sort(s["ttft"])[197]
        assert s["tokens_s"] == pytest.approx(tr.n_out.sum() / (s["fin"].max() - arr.min()), rel=1e-15)
        if max_seqs == 1:
            assert s["n_steps"] == s["n_request_steps"]


def test_simulation_request_steps_exact_count(ora):
    """max_seqs = 1 and prompts under the budget: each request takes exactly one
    chunk and out-1 decode steps."""
    om, oh = bridge.ora_model(wl.DENSE_7B), bridge.ora_hw(wl.HW_TINY)
    tr = wl.request_trace(n=64)
    s = ora.simulate(om, oh, 1, 16, 16, 8192, 1, 1.0, tr.arrival_unit, tr.n_in, tr.n_out)
    assert s["n_request_steps"] == int(tr.n_out.sum()) == s["n_steps"]


def test_simulation_spaced_and_serial_requests(ora):
    m = wl.DENSE_7B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    ins = np.array([300, 5000, 64], dtype=np.uint32); outs = np.array([20, 5, 60], dtype=np.uint32)
    singles = [ora.evaluate(om, oh, ora.knobs(1, int(i), int(o), mbt=2048)) for i, o in zip(ins, outs)]
    # far apart: each request sees an empty engine
    arr = np.array([0.0, 100.0, 200.0])
    s = ora.simulate(om, oh, 1, 16, 16, 2048, 8, 1.0, arr, ins, outs, detail=True)
    for i, e in enumerate(singles):
        assert s["ttft"][i] == pytest.approx(e.t_prefill, rel=1e-12)
        assert s["fin"][i] - arr[i] == pytest.approx(e.t_batch, rel=1e-12)
    # all at time 0, one at a time: finish times are running sums
    s = ora.simulate(om, oh, 1, 16, 16, 2048, 1, 1.0, np.zeros(3), ins, outs, detail=True)
    run = np.cumsum([e.t_batch for e in singles])
    np.testing.assert_allclose(s["fin"], run, rtol=1e-13)


def test_simulation_batched_decode_by_hand(ora):
    """Two identical requests at t=0, both admitted: one prefill pass with both
    prompts, then out-1 decode steps with two tokens each."""
    m = wl.DENSE_7B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    n_in, n_out = 100, 4
    s = ora.simulate(om, oh, 1, 16, 16, 2048, 2, 1.0, np.zeros(2), np.array([n_in] * 2, dtype=np.uint32),
                     np.array([n_out] * 2, dtype=np.uint32), detail=True)
    t = ora.pass_detail(om, oh, 1, 16, 2 * n_in, 2 * n_in * n_in, 2 * n_in, 2)["t_pass"]
    assert s["ttft"][0] == s["ttft"][1] == t
    for j in range(1, n_out):
        ctx = n_in + j
        t += ora.pass_detail(om, oh, 1, 16, 2, 2 * ctx, 2 * ctx, 2)["t_pass"]
    assert s["fin"][0] == s["fin"][1] == t
    assert s["n_steps"] == n_out and s["n_request_steps"] == 2 * n_out
    # chunked: budget 150 -> step 1 gives 100 + 50, step 2: decode of req 0 + 50 of req 1
    s = ora.simulate(om, oh, 1, 16, 16, 150, 2, 1.0, np.zeros(2), np.array([n_in] * 2, dtype=np.uint32),
                     np.array([n_out] * 2, dtype=np.uint32), detail=True)
    t1 = ora.pass_detail(om, oh, 1, 16, 150, 100 * 100 + 50 * 50, 100 + 50, 1)["t_pass"]
    assert s["ttft"][0] == t1
    t2 = t1 + ora.pass_detail(om, oh, 1, 16, 1 + 50, 101 + 50 * 100, 101 + 100, 2)["t_pass"]
    assert s["ttft"][1] == t2
    assert s["n_request_steps"] == 2 + 2 + (n_out - 2) * 2 + 1


def test_simulation_infeasible_and_blocking(ora):
    m = wl.DENSE_7B
    om = bridge.ora_model(m)
    w = ora.weight_bytes_gpu(om, 1, 16)
    kv_tok = ora.kv_bytes_token(om, 1)
    ins = np.array([100, 100], dtype=np.uint32); outs = np.array([28, 28], dtype=np.uint32)
    # pool of exactly 8 blocks: each request needs 8 -> strictly serial even with max_seqs 2
    h = wl.Hardware(1e15, 5e12, w + 8 * 16 * kv_tok, 4e11)
    s = ora.simulate(om, bridge.ora_hw(h), 1, 16, 16, 2048, 2, 1.0, np.zeros(2), ins, outs, detail=True)
    assert s["status"] == ora.SIM_OK and s["min_free"] == 0
    assert s["first"][1] > s["fin"][0]
    # one block short: a request can never fit
    h = wl.Hardware(1e15, 5e12, w + 8 * 16 * kv_tok - 1, 4e11)
    s = ora.simulate(om, bridge.ora_hw(h), 1, 16, 16, 2048, 2, 1.0, np.zeros(2), ins, outs)
    assert s["status"] == ora.SIM_INFEASIBLE and np.isinf(s["ttft_p50"]) and s["n_steps"] == 0
    s = ora.simulate(om, bridge.ora_hw(h), 1, 16, 16, 2048, 2, 1.0, np.zeros(2), ins, outs, detail=True)
    assert np.all(np.isinf(s["ttft"])) and np.all(np.isinf(s["first"])) and np.all(np.isinf(s["fin"]))
    # weights do not fit
    h = wl.Hardware(1e15, 5e12, w, 4e11)
    assert ora.simulate(om, bridge.ora_hw(h), 1, 16, 16, 2048, 2, 1.0, np.zeros(2), ins, outs)["status"] == 1


# ------------------------------------------------------------------- selection

def _brute_topk(obj, ok, k):
    cand = sorted((float(v), i) for i, v in enumerate(obj) if ok[i])
    return cand[:k]


def test_select_topk_against_full_sort(ora):
    rng = np.random.default_rng(11)
    n = 1500
    obj = rng.integers(0, 40, n).astype(np.float64)      # many exact ties
    obj[rng.integers(0, n, 30)] = np.nan
    fe = (rng.random(n) < 0.7).astype(np.uint8)
    c1 = rng.random(n); c2 = rng.random(n)
    grp = rng.integers(0, 5, n).astype(np.uint32)
    ok = (fe == 1) & (c1 <= 0.6) & (c2 <= 0.9) & ~np.isnan(obj)
    idx, val, cnt = ora.select_topk(obj, fe, [(c1, 0.6), (c2, 0.9)], k=8)
    exp = _brute_topk(obj, ok, 8)
    assert [(v, i) for v, i in zip(val[0], idx[0])] == exp and cnt[0] == ok.sum()
    idx, val, cnt = ora.select_topk(obj, fe, [(c1, 0.6), (c2, 0.9)], group=grp, n_groups=6, k=3)
    for gi in range(6):
        exp = _brute_topk(obj, ok & (grp == gi), 3)
        got = [(v, i) for v, i in zip(val[gi], idx[gi]) if i != ora.NO_INDEX]
        assert got == exp and cnt[gi] == (ok & (grp == gi)).sum()
    assert np.all(idx[5] == ora.NO_INDEX) and np.all(np.isinf(val[5])) and cnt[5] == 0
    # constraint boundary is inclusive; nothing passes -> sentinel
    idx, val, cnt = ora.select_topk(np.array([3.0, 1.0, 2.0]), None, [(np.array([0.5, 0.7, 0.2]), 0.5)], k=2)
    assert list(idx[0]) == [2, 0] and cnt[0] == 2
    idx, val, cnt = ora.select_topk(np.array([3.0, 1.0]), np.zeros(2, dtype=np.uint8), k=1)
    assert idx[0, 0] == ora.NO_INDEX and val[0, 0] == np.inf and cnt[0] == 0


def test_tiny_grid_argmin_by_numpy(ora):
    g = wl.grid_tiny()
    r = ora.eval_grid(bridge.ora_grid(g))
    ok = (r["feasible"] == 1) & (r["t_prefill"] <= wl.TTFT_CAP_S)
    masked = np.where(ok, r["t_batch"], np.inf)
    idx, val, cnt = ora.select_topk(r["t_batch"], r["feasible"], [(r["t_prefill"], wl.TTFT_CAP_S)])
    assert idx[0, 0] == np.argmin(masked) and val[0, 0] == masked.min() and cnt[0] == ok.sum()


def _pareto_def(x, y, ok):
    keep = []
    for i in range(len(x)):
        if not ok[i]:
            continue
        dom = False
        for j in range(len(x)):
            if ok[j] and j != i and x[j] <= x[i] and y[j] <= y[i] and (x[j] < x[i] or y[j] < y[i]):
                dom = True
                break
        if not dom:
            keep.append(i)
    return sorted(keep, key=lambda i: (x[i], y[i], i))


def test_pareto_brute_and_sweep(ora):
    rng = np.random.default_rng(5)
    for trial in range(6):
        n = 400
        x = rng.integers(0, 25, n).astype(np.float64)
        y = rng.integers(0, 25, n).astype(np.float64)
        if trial == 1:
            x[:] = 3.0                                       # one column constant
        if trial == 2:
            y = 30.0 - x                                     # everything on the front, duplicates kept
        mask = (rng.random(n) < 0.8).astype(np.uint8)
        if trial == 3:
            x[5] = np.nan; y[9] = np.nan
        ok = (mask == 1) & ~np.isnan(x) & ~np.isnan(y)
        exp = _pareto_def(x, y, ok)
        assert list(ora.pareto_brute(x, y, mask)) == exp
        assert list(ora.pareto_sweep(x, y, mask)) == exp
    assert len(ora.pareto_sweep(np.array([1.0]), np.array([1.0]), np.array([0], dtype=np.uint8))) == 0
    x = rng.random(3000); y = rng.random(3000)
    assert list(ora.pareto_sweep(x, y)) == list(ora.pareto_brute(x, y))


# --------------------------------------------------------- sampled space / RNG

def test_philox_against_numpy(ora):
    """numpy's Philox is Philox4x64-10; it bumps the counter before producing a
    block, so the block for counter c is what numpy emits from counter c - 1."""
    rng = np.random.default_rng(7)
    for _ in range(20):
        key = rng.integers(0, 2 ** 63, 2, dtype=np.uint64)
        ctr = rng.integers(1, 2 ** 63, 4, dtype=np.uint64)
        prev = ctr.copy(); prev[0] -= np.uint64(1)
        ref = np.random.Philox(key=key, counter=prev).random_raw(4)
        np.testing.assert_array_equal(ora.philox4x64_10(ctr, key), ref)
    ref = np.random.Philox(key=[wl.SEED, 0], counter=[41, 0, 0, 0]).random_raw(4)
    np.testing.assert_array_equal(ora.philox4x64_10([42, 0, 0, 0], [wl.SEED, 0]), ref)


def test_sampled_config_draws(ora):
    sp = wl.sample_space()
    osp = bridge.ora_space(sp)
    seen_L, seen_kv = set(), set()
    for idx in range(3000):
        m, h, kn = ora.sample_config(osp, wl.SEED, idx)
        raw = np.random.Philox(key=[wl.SEED, 0], counter=[idx - 1 if idx else 2 ** 64 - 1,
                                                           0 if idx else 2 ** 64 - 1,
                                                           0 if idx else 2 ** 64 - 1,
                                                           0 if idx else 2 ** 64 - 1]).random_raw(4)
        u = [int((int(raw[j >> 2]) >> (16 * (j & 3))) & 0xFFFF) for j in range(14)]
        assert m.L == 16 + (u[0] * 81 >> 16)
        n_h = int(sp.heads[u[1] >> 6])
        assert (m.n_h, m.d) == (n_h, 128 * n_h)
        kvc = [1, 4, 8, n_h][u[2] >> 14]
        assert m.n_kv == kvc
        ratio = 2.5 + 1.5 * u[3] / 65536.0
        assert m.d_ff == 128 * int(np.floor(ratio * n_h + 0.5))
        assert 2.5 * n_h - 0.5 <= m.d_ff / 128 <= 4.0 * n_h + 0.5
        assert h.peak == sp.peak[u[4] >> 6] and h.bw == sp.bw[u[5] >> 6] and h.cap == sp.cap[u[6] * 6 >> 16]
        assert h.link_bw == h.bw / 12.5 and h.link_lat == 0.0
        assert (kn.b, kn.s_in, kn.s_out) == (sp.batch[u[7] >> 6], sp.s_in[u[8] >> 6], sp.s_out[u[9] >> 6])
        assert (kn.p, kn.wbits, kn.blk, kn.mbt) == (sp.tp[u[10] >> 14], sp.wbits[u[11] * 3 >> 16],
                                                    sp.kv_block[u[12] >> 15], sp.mbt[u[13] * 3 >> 16])
        assert (m.V, m.E, m.k) == (32000, 1, 1)
        seen_L.add(m.L); seen_kv.add(m.n_kv if m.n_kv in (1, 4, 8) else 0)
    assert min(seen_L) == 16 and max(seen_L) == 96 and seen_kv == {0, 1, 4, 8}
    # lattice end points
    assert sp.heads[0] == 16 and sp.heads[-1] == 128 and sp.batch[0] == 1 and sp.batch[-1] == 1024
    assert sp.s_in[0] == 64 and sp.s_in[-1] == 32768 and sp.s_out[-1] == 8192
    assert sp.peak[0] == 1e14 and sp.peak[-1] == pytest.approx(2.5e15) and sp.bw[-1] == pytest.approx(8e12)


def test_bucket_and_histogram_bins(ora):
    edges = wl.BUCKET_EDGES
    assert ora.bucket(0.99e9, edges) == 0 and ora.bucket(1e9, edges) == 1 and ora.bucket(6.7e9, edges) == 3
    assert ora.bucket(2.56e11, edges) == 9 and ora.bucket(1e13, edges) == 9
    assert ora.hist_bin(2.0 ** -12) == 0 and ora.hist_bin(1e-9) == 0
    assert ora.hist_bin(np.nextafter(2.0 ** -11, 0)) == 7 and ora.hist_bin(2.0 ** -11) == 8
    assert ora.hist_bin(1.0) == 96 and ora.hist_bin(1.125) == 97 and ora.hist_bin(1.9999) == 103
    assert ora.hist_bin(2.0 ** 20) == 255 and ora.hist_bin(np.nextafter(2.0 ** 20, 0)) == 255
    assert ora.hist_bin(2.0 ** 19) == 248


def test_sampled_reductions_against_columns(ora):
    sp = bridge.ora_space(wl.sample_space())
    n = 4000
    r = ora.eval_sampled(sp, wl.SEED, 100, n, wl.BUCKET_EDGES, wl.TTFT_CAP_S, columns=True)
    fe = r["feasible"] == 1
    assert r["feasible_count"] == fe.sum() == r["hist"].sum()
    assert 0 < fe.sum() < n
    bins = np.array([ora.hist_bin(t) for t in r["t_batch"][fe]])
    np.testing.assert_array_equal(np.bincount(bins, minlength=256), r["hist"])
    for b in range(wl.N_BUCKETS):
        ok = fe & (r["bucket"] == b) & (r["t_prefill"] <= wl.TTFT_CAP_S)
        if ok.any():
            masked = np.where(ok, r["cost"], np.inf)
            assert r["win_idx"][b] == 100 + np.argmin(masked) and r["win_val"][b] == masked.min()
        else:
            assert r["win_idx"][b] == ora.NO_INDEX and np.isinf(r["win_val"][b])
    # per-candidate columns are the plain evaluator on the drawn candidate
    for i in (0, 17, 3999):
        m, h, kn = ora.sample_config(sp, wl.SEED, 100 + i)
        e = ora.evaluate(m, h, kn)
        assert (e.t_prefill, e.t_batch, e.cost, e.b_max) == (r["t_prefill"][i], r["t_batch"][i], r["cost"][i],
                                                             r["b_max"][i])
        assert r["bucket"][i] == ora.bucket(ora.params_total(m), wl.BUCKET_EDGES)
    # two half ranges combine to the full range
    a = ora.eval_sampled(sp, wl.SEED, 100, n // 2, wl.BUCKET_EDGES, wl.TTFT_CAP_S)
    b = ora.eval_sampled(sp, wl.SEED, 100 + n // 2, n // 2, wl.BUCKET_EDGES, wl.TTFT_CAP_S)
    np.testing.assert_array_equal(a["hist"] + b["hist"], r["hist"])
    assert a["feasible_count"] + b["feasible_count"] == r["feasible_count"]


# ------------------------------------------------ prefill-first scheduler variant

@pytest.mark.parametrize("n_in,n_out,mbt", [(700, 40, 2048), (5000, 17, 2048), (2048, 1, 2048)])
def test_prefill_first_single_request(ora, n_in, n_out, mbt):
    """One request: the whole prompt runs in one pass (no chunking even beyond the budget), then
    out - 1 decode passes."""
    m = wl.DENSE_34B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    arr, ins, outs = _one_req(n_in, n_out)
    s = ora.simulate(om, oh, 2, 8, 16, mbt, 4, 1.0, arr, ins, outs, detail=True, scheduler=ora.SCHED_PREFILL_FIRST)
    t = ora.pass_detail(om, oh, 2, 8, n_in, n_in * n_in, n_in, 1)["t_pass"]
    assert s["ttft"][0] == t
    for j in range(1, n_out):
        t += ora.pass_detail(om, oh, 2, 8, 1, n_in + j, n_in + j, 1)["t_pass"]
    assert s["fin"][0] == pytest.approx(t, rel=1e-14)
    assert s["n_steps"] == n_out == s["n_request_steps"]


def test_prefill_first_two_requests_by_hand(ora):
    m = wl.DENSE_7B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    ins = np.array([100, 100], dtype=np.uint32); outs = np.array([3, 3], dtype=np.uint32)
    one = ora.pass_detail(om, oh, 1, 16, 100, 100 * 100, 100, 1)["t_pass"]
    # budget 150: the prompts run in two prefill-only steps; the first request's decoding waits for the second
    s = ora.simulate(om, oh, 1, 16, 16, 150, 2, 1.0, np.zeros(2), ins, outs, detail=True,
                     scheduler=ora.SCHED_PREFILL_FIRST)
    assert s["ttft"][0] == one and s["ttft"][1] == one + one
    t = one + one
    for ctx in (101, 102):
        t += ora.pass_detail(om, oh, 1, 16, 2, 2 * ctx, 2 * ctx, 2)["t_pass"]
    assert s["fin"][0] == s["fin"][1] == t
    assert s["n_steps"] == 4 and s["n_request_steps"] == 6
    # budget 250: both prompts share one pass
    s = ora.simulate(om, oh, 1, 16, 16, 250, 2, 1.0, np.zeros(2), ins, outs, detail=True,
                     scheduler=ora.SCHED_PREFILL_FIRST)
    both = ora.pass_detail(om, oh, 1, 16, 200, 2 * 100 * 100, 200, 2)["t_pass"]
    assert s["ttft"][0] == s["ttft"][1] == both and s["n_steps"] == 3
    # an arrival during decoding interrupts it with a prefill-only step
    s = ora.simulate(om, oh, 1, 16, 16, 250, 2, 1.0, np.array([0.0, 1.5 * one]), ins, outs, detail=True,
                     scheduler=ora.SCHED_PREFILL_FIRST)
    d1 = ora.pass_detail(om, oh, 1, 16, 1, 101, 101, 1)["t_pass"]
    assert s["ttft"][0] == one
    assert s["first"][1] == pytest.approx(one + d1 + one, rel=1e-15)      # decode step, then the second prompt
    assert s["n_request_steps"] == 6


def test_prefill_first_invariants_and_relation_to_split_fuse(ora):
    m = wl.DENSE_7B
    om = bridge.ora_model(m)
    oh = bridge.ora_hw(wl.Hardware(1e15, 5e12, 40 * wl.GIB, 4e11))
    tr = wl.request_trace(n=200)
    for max_seqs, rate, mbt in [(1, 4.0, 8192), (8, 16.0, 2048), (64, 64.0, 8192), (256, 64.0, 512)]:
        a = ora.simulate(om, oh, 1, 16, 16, mbt, max_seqs, rate, tr.arrival_unit, tr.n_in, tr.n_out, detail=True,
                         scheduler=ora.SCHED_PREFILL_FIRST)
        assert a["status"] == ora.SIM_OK and a["min_free"] >= 0
        assert a["n_request_steps"] == int(tr.n_out.sum())      # one prompt pass + out - 1 decode tokens each
        assert np.all(np.diff(a["first"]) >= 0)
        b = ora.simulate(om, oh, 1, 16, 16, mbt, max_seqs, rate, tr.arrival_unit, tr.n_in, tr.n_out, detail=True)
        if max_seqs == 1:       # one request at a time, prompts within the budget: the two schedulers coincide
            np.testing.assert_array_equal(a["fin"], b["fin"])
            np.testing.assert_array_equal(a["ttft"], b["ttft"])
        else:
            assert not np.array_equal(a["fin"], b["fin"])


# ------------------------------------------------------------ cluster-level extras

def test_extras_by_hand(ora):
    """S_max is the paper's floor(C_available / (2 N H B kv)) for MHA on one GPU; the boundary is exact;
    maximum parallelism = DP x B_max; the multi-GPU heuristic is N T_single / (1 + log2 P_TP)."""
    m = wl.DENSE_13B
    om = bridge.ora_model(m)
    b, tp = 6, 1
    w = 2 * ora.params_total(om)
    s_fit = 3000
    cap = w + b * (2 * m.L * m.d * 2) * s_fit            # exactly s_fit tokens per sequence fit
    for delta, s_exp in ((0.0, s_fit), (-1.0, s_fit - 1)):
        h = wl.Hardware(1e15, 5e12, cap + delta, 4e11)
        g = bridge.ora_grid(wl.make_grid([m], [h], wl.Axis.table([b]), wl.Axis.table([512]), wl.Axis.table([64]),
                                         wl.Axis.table([tp]), wl.Axis.table([16]), wl.Axis.table([16]),
                                         wl.Axis.table([8192])))
        e = ora.eval_extras_grid(g, 8)
        assert e["s_max"][0] == s_exp
    h = wl.HW_TINY
    g = wl.make_grid([m], [h], wl.Axis.table([b]), wl.Axis.table([512]), wl.Axis.table([64]),
                     wl.Axis.table([1, 2, 3, 8, 16]), wl.Axis.table([16]), wl.Axis.table([16]), wl.Axis.table([8192]))
    og = bridge.ora_grid(g)
    e = ora.eval_extras_grid(og, 8)
    r = ora.eval_grid(og)
    t_single = r["decode_tok_s"][0]
    for i, p in enumerate([1, 2, 3, 8, 16]):
        dp = 8 // p
        assert e["dp_max"][i] == dp
        assert e["max_parallelism"][i] == dp * int(r["b_max"][i])
        assert e["cluster_tok_s"][i] == dp * r["decode_tok_s"][i]
        assert e["paper_tok_s"][i] == pytest.approx(dp * p * t_single / (1 + np.log2(p)), rel=1e-15)
    assert e["paper_tok_s"][0] == 8 * t_single and e["paper_tok_s"][1] == pytest.approx(8 * t_single / 2, rel=1e-15)
    assert e["dp_max"][4] == 0 and e["cluster_tok_s"][4] == 0.0
    # weights do not fit: nothing fits
    g0 = bridge.ora_grid(wl.make_grid([wl.DENSE_70B], [wl.Hardware(1e15, 5e12, 24 * wl.GIB, 4e11)], wl.Axis.table([1]),
                                      wl.Axis.table([64]), wl.Axis.table([64]), wl.Axis.table([1]), wl.Axis.table([16]),
                                      wl.Axis.table([16]), wl.Axis.table([2048])))
    e = ora.eval_extras_grid(g0, 4)
    assert e["s_max"][0] == 0 and e["max_parallelism"][0] == 0


# ------------------------------------------------- closed-form decode runs (simulation)

def test_decode_run_closed_form_against_stepping(ora):
    """The closed form of a run of decode-only steps against the step-by-step sum of passes on 2^16 random runs:
    all five shapes, TP 1..8, three precisions, hardware from compute-starved to bandwidth-starved (so that
    attention is read bound, compute bound, or crosses over inside the run), both time models."""
    rng = np.random.default_rng(2024)
    models = [bridge.ora_model(m) for m in wl.MODELS_FULL]
    worst, crossed = 0.0, 0
    for case in range(1 << 16):
        m = models[case % 5]
        # ridge points from 2 to 2000 FLOP/B: the attention crossover context gamma / (alpha - beta) lands anywhere
        peak = 10.0 ** rng.uniform(13.0, 15.5)
        bw = peak / 10.0 ** rng.uniform(0.3, 3.3)
        h = bridge.ora_hw(wl.Hardware(peak, bw, 192 * wl.GIB, bw / 12.5, 1e-6 * (case % 3)))
        p, wbits, tm = int(rng.choice([1, 2, 4, 8])), int(rng.choice([16, 8, 4])), (case // 5) % 2
        T = float(rng.integers(1, 1025))
        C0 = T * float(rng.integers(2, 9000))
        r = int(rng.integers(1, 600))
        mw = wl.MODELS_FULL[case % 5]
        if case % 4 == 0 and mw.n_kv < mw.n_h:
            # aim at the crossover: with fewer KV heads than heads, attention turns compute bound at the mean
            # context rho / (1 - rho * n_kv / n_h) for a ridge rho = peak / bw below n_h / n_kv
            p = int(rng.choice([1, 2, 4, 8]))
            share = -(-mw.n_kv // p) * p / mw.n_h
            rho = rng.uniform(0.5, 0.999) / share
            bw = peak / rho
            h = bridge.ora_hw(wl.Hardware(peak, bw, 192 * wl.GIB, bw / 12.5, 0.0))
            star = rho / (1.0 - rho * share)
            C0 = T * float(max(2, int(star - r * rng.uniform(0.0, 1.0))))
            wbits, tm = 16, 0
        a = ora.decode_run_time(m, h, p, wbits, T, C0, r, time_model=tm)
        b = ora.decode_run_steps(m, h, p, wbits, T, C0, r, time_model=tm)
        worst = max(worst, abs(a - b) / b)
        if tm == 0:
            first = ora.pass_detail(m, h, p, wbits, T, C0, C0, T)
            last = ora.pass_detail(m, h, p, wbits, T, C0 + (r - 1) * T, C0 + (r - 1) * T, T)
            rd0 = first["B"][1] / h.bw >= first["F"][1] / h.peak
            rd1 = last["B"][1] / h.bw >= last["F"][1] / h.peak
            crossed += int(rd0 != rd1)
    assert worst <= 1e-12, worst
    assert crossed > 200                     # the crossover inside a run is exercised
    m, h = models[0], bridge.ora_hw(wl.HW_TINY)
    assert ora.decode_run_time(m, h, 1, 16, 3.0, 900.0, 0) == 0.0
    one = ora.pass_detail(m, h, 1, 16, 3.0, 900.0, 900.0, 3.0)["t_pass"]
    assert ora.decode_run_time(m, h, 1, 16, 3.0, 900.0, 1) == pytest.approx(one, rel=1e-15)


@pytest.mark.parametrize("scheduler", [0, 1])
def test_closed_form_runs_simulation_against_stepping(ora, scheduler):
    """Whole simulations with closed-form runs against the step-by-step simulation: engine steps and
    request-steps are the same integers, times agree to rounding (a TTFT is a difference of two nearby times,
    hence the looser bound on it)."""
    g = wl.grid_full()
    og = bridge.ora_grid(g)
    tr = wl.request_trace(n=256)
    idx, rate = wl.sim_configs(g, 96, seed=wl.SEED + 3)
    a = ora.simulate_grid(og, idx, rate, tr.arrival_unit, tr.n_in, tr.n_out, scheduler=scheduler)
    b = ora.simulate_grid(og, idx, rate, tr.arrival_unit, tr.n_in, tr.n_out,
                          scheduler=scheduler | ora.SIM_CLOSED_FORM_RUNS)
    np.testing.assert_array_equal(a["status"], b["status"])
    ok = a["status"] == 0
    assert ok.sum() > 60
    # an admission decided within rounding may differ between the two; such a configuration shows a tiny margin
    same = (a["n_steps"] == b["n_steps"]) & (a["n_request_steps"] == b["n_request_steps"])
    assert np.all(same | (np.minimum(a["min_admit_margin"], b["min_admit_margin"]) < 1e-9))
    assert same.sum() >= len(idx) - 1
    for k, tol in (("ttft_p50", 1e-9), ("ttft_p99", 1e-9), ("mean_tpot", 1e-11), ("tokens_s", 1e-12)):
        assert bridge.rel_err(b[k][ok & same], a[k][ok & same]).max() <= tol, k
    # single request: one prefill step, then one closed-form run of out - 2 steps and the last step
    arr, ins, outs = np.array([0.0]), np.array([700], dtype=np.uint32), np.array([40], dtype=np.uint32)
    om, oh = bridge.ora_model(wl.DENSE_34B), bridge.ora_hw(wl.HW_TINY)
    s0 = ora.simulate(om, oh, 2, 8, 16, 2048, 4, 1.0, arr, ins, outs, detail=True, scheduler=scheduler)
    s1 = ora.simulate(om, oh, 2, 8, 16, 2048, 4, 1.0, arr, ins, outs, detail=True,
                      scheduler=scheduler | ora.SIM_CLOSED_FORM_RUNS)
    assert s1["n_steps"] == s0["n_steps"] == 40 and s1["ttft"][0] == s0["ttft"][0]
    assert s1["fin"][0] == pytest.approx(s0["fin"][0], rel=1e-13)
    # a request that arrives exactly when a step ends is admitted before the next step, run or no run
    t1 = ora.pass_detail(om, oh, 2, 8, 700, 700 * 700, 700, 1)["t_pass"]
    arr2, ins2, outs2 = np.array([0.0, t1]), np.array([700, 300], dtype=np.uint32), np.array([40, 5], dtype=np.uint32)
    s0 = ora.simulate(om, oh, 2, 8, 16, 2048, 4, 1.0, arr2, ins2, outs2, detail=True, scheduler=scheduler)
    s1 = ora.simulate(om, oh, 2, 8, 16, 2048, 4, 1.0, arr2, ins2, outs2, detail=True,
                      scheduler=scheduler | ora.SIM_CLOSED_FORM_RUNS)
    second = ora.pass_detail(om, oh, 2, 8, 300 + (1 - scheduler), 300 * 300 + (1 - scheduler) * 701,
                             300 + (1 - scheduler) * 701, 1 + (1 - scheduler))["t_pass"]
    assert s0["ttft"][1] == pytest.approx(second, rel=1e-13) and s1["ttft"][1] == s0["ttft"][1]
    assert s1["n_steps"] == s0["n_steps"] and s1["n_request_steps"] == s0["n_request_steps"]


def test_adjustment_columns_by_hand(ora):
    """Adjusted batch and length, sub-batch and segment counts (Dynamic Batch Size / Sequence Length Adjustment)."""
    m = wl.DENSE_13B
    om = bridge.ora_model(m)
    w = 2 * ora.params_total(om)
    kv_tok = 2 * m.L * m.d * 2
    # capacity for exactly 5 requests of 1000 + 24 tokens; a batch of 8 is adjusted to 5, a batch of 4 stays
    h = wl.Hardware(1e15, 5e12, w + 5 * 1024 * kv_tok, 4e11)
    g = wl.make_grid([m], [h], wl.Axis.table([4, 8, 10]), wl.Axis.table([1000, 5000]), wl.Axis.table([24]),
                     wl.Axis.table([1]), wl.Axis.table([16]), wl.Axis.table([16]), wl.Axis.table([2048, 4096]))
    e = ora.eval_extras_grid(bridge.ora_grid(g), 8)

    def at(b, s_in, mbt):
        return g.flat((0, 0, (4, 8, 10).index(b), (1000, 5000).index(s_in), 0, 0, 0, 0, (2048, 4096).index(mbt)))

    assert [e["b_adj"][at(b, 1000, 2048)] for b in (4, 8, 10)] == [4, 5, 5]
    # 10 prompts of 1000 under 4096 tokens per pass: 4 + 4 + 2; under 2048: five pairs; a batch of 4 under 4096: one pass
    assert e["n_sub_batches"][at(10, 1000, 4096)] == 3 and e["n_sub_batches"][at(10, 1000, 2048)] == 5
    assert e["n_sub_batches"][at(4, 1000, 4096)] == 1 and e["n_segments"][at(10, 1000, 4096)] == 1
    # a 5000-token prompt: 3 segments of 2048 (2048 + 2048 + 904), 2 of 4096; every request runs alone
    assert e["n_segments"][at(8, 5000, 2048)] == 3 and e["n_segments"][at(8, 5000, 4096)] == 2
    assert e["n_sub_batches"][at(8, 5000, 2048)] == 8
    # S_max = floor(5 * 1024 / b) tokens per sequence: 1280 for b = 4 (1024 needed: unchanged), 512 for b = 10
    assert e["s_max"][at(4, 1000, 2048)] == 1280 and e["s_adj"][at(4, 1000, 2048)] == 1024
    assert e["s_max"][at(10, 1000, 2048)] == 512 and e["s_adj"][at(10, 1000, 2048)] == 512
    # the prefill evaluator runs exactly that many passes
    oh = bridge.ora_hw(h)
    one = ora.pass_detail(om, oh, 1, 16, 2000, 2 * 1000 * 1000, 2000, 2)["t_pass"]
    assert ora.prefill(om, oh, ora.knobs(10, 1000, 24, mbt=2048)) == pytest.approx(5 * one, rel=1e-15)


# ------------------------------------------- pins added after operator-level mutation of the oracle
#
# Each test below fails for at least one one-token change of oracle/guide_oracle.c (an operator, a comparison, a
# constant) that every earlier pin let through.

def test_output_projection_split_over_gpus(ora):
    gold = _gold("op_bytes.txt")
    om, oh = bridge.ora_model(wl.DENSE_7B), bridge.ora_hw(wl.HW_TINY)
    for p in (2, 4):
        r = ora.pass_detail(om, oh, p, 16, 3.0, 9.0, 3.0, 1.0)
        assert r["F"][2] == gold[f"oproj_flops_7b_tp{p}_T3"]
        assert r["B"][2] == gold[f"oproj_bytes_7b_tp{p}_T3"]


def test_lm_head_only_with_lm_rows(ora):
    """A pass without LM-head rows (a prompt segment that is not the last) pays nothing for the LM head, not even
    its weights; with one row it is the weight-bound closed form."""
    gold = _gold("op_bytes.txt")
    m = wl.DENSE_7B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)
    r0 = ora.pass_detail(om, oh, 1, 16, 64.0, 64.0 * 64, 64.0, 0.0)
    assert r0["t"][7] == 0.0
    assert r0["t_pass"] == pytest.approx(m.L * (r0["t"][:7].sum() + 2 * r0["t_ar"]), rel=1e-15)
    r1 = ora.pass_detail(om, oh, 1, 16, 64.0, 64.0 * 64, 64.0, 1.0)
    assert r1["B"][7] == gold["lm_head_bytes_7b_tp1_rows1"]
    assert r1["t"][7] == gold["lm_head_bytes_7b_tp1_rows1"] / wl.HW_TINY.hbm_bw
    assert r1["t_pass"] - r0["t_pass"] == pytest.approx(r1["t"][7], rel=1e-9)


@pytest.mark.parametrize("time_model", [0, 1])
def test_prefill_and_decode_pass_arguments_under_both_time_models(ora, time_model):
    """The passes of a prefill and of a decode, written out with their token, query-context and KV-token counts:
    under the additive model every one of those counts moves the time, whichever side of the roofline it is on."""
    m = wl.DENSE_7B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)

    def one(T, Q, K, n_lm, p=1):
        return ora.pass_detail(om, oh, p, 16, T, Q, K, n_lm, time_model=time_model)["t_pass"]

    # sub-batches: 10 prompts of 1000 tokens under 4096 tokens per pass: 4 + 4 + 2
    t = ora.prefill(om, oh, ora.knobs(10, 1000, 8, mbt=4096), time_model=time_model)
    assert t == (one(4000, 4 * 1000 * 1000, 4000, 4) + one(4000, 4 * 1000 * 1000, 4000, 4)) + one(2000, 2 * 1000 * 1000, 2000, 2)
    # a prompt of exactly two, and of exactly three budgets: two and three full segments, the LM head on the last
    for k in (2, 3):
        t = ora.prefill(om, oh, ora.knobs(1, k * 2048, 8, mbt=2048), time_model=time_model)
        tot = 0.0
        for j in range(k):
            tot += one(2048, 2048 * (j + 1) * 2048, (j + 1) * 2048, 1 if j == k - 1 else 0)
        assert t == tot
    # one token more: a further segment of one token
    t = ora.prefill(om, oh, ora.knobs(1, 4097, 8, mbt=2048), time_model=time_model)
    assert t == (one(2048, 2048 * 2048, 2048, 0) + one(2048, 2048 * 4096, 4096, 0)) + one(1, 4097, 4097, 1)
    # decode: s_out - 1 steps of b tokens at context s_in + j
    b, s_in, s_out = 3, 100, 6
    e = ora.evaluate(om, oh, ora.knobs(b, s_in, s_out, p=2), time_model=time_model)
    td = 0.0
    for j in range(1, s_out):
        td += one(b, b * (s_in + j), b * (s_in + j), b, p=2)
    assert e.t_decode == td


def test_grid_wrappers_cover_every_row_of_their_range(ora):
    """The range forms used by the GPU parity tests (sweep over a grid range, simulation of a list of grid rows)
    against the single-row calls, for ranges that start inside the grid and hold several rows."""
    g = wl.grid_tiny()
    og = bridge.ora_grid(g)
    e_c, e_b = wl.efficiency_pairs(n=64)
    first, count = 37, 6
    s = ora.eval_sweep_grid(og, e_c, e_b, first, count)
    per = [ora.eval_grid(og, first, count, e_c=float(a), e_b=float(b)) for a, b in zip(e_c, e_b)]
    tp = np.array([r["t_prefill"] for r in per]); tb = np.array([r["t_batch"] for r in per])      # [sample, row]
    for i in range(count):
        assert s["ttft_p10"][i] == np.sort(tp[:, i])[6] and s["ttft_p90"][i] == np.sort(tp[:, i])[57]
        assert s["t_batch_p10"][i] == np.sort(tb[:, i])[6] and s["t_batch_p90"][i] == np.sort(tb[:, i])[57]
        assert s["ttft_mean"][i] == pytest.approx(tp[:, i].mean(), rel=1e-14)
        assert s["t_batch_mean"][i] == pytest.approx(tb[:, i].mean(), rel=1e-14)
    assert len(set(s["t_batch_p90"].tolist())) == count          # six different rows
    # simulation of grid rows: the row's model, hardware, TP, precision, block and budget, its batch as the sequence cap
    tr = wl.request_trace(n=48)
    rows = np.array([5, 611, 1079], dtype=np.uint32)
    rates = np.array([2.0, 16.0, 64.0])
    sg = ora.simulate_grid(og, rows, rates, tr.arrival_unit, tr.n_in, tr.n_out)
    for j, (row, rate) in enumerate(zip(rows, rates)):
        mi, hi, b, _, _, p, wbits, blk, mbt = g.values_at(int(row))
        one = ora.simulate(bridge.ora_model(g.models[mi]), bridge.ora_hw(g.hws[hi]), p, wbits, blk, mbt, b, float(rate),
                           tr.arrival_unit, tr.n_in, tr.n_out)
        for k in ("ttft_p50", "ttft_p99", "mean_tpot", "tokens_s", "n_steps", "n_request_steps", "status"):
            assert sg[k][j] == one[k], (k, j)
    assert len(set(sg["n_steps"].tolist())) == 3
    # a model or hardware number equal to the table's length is outside it
    bad = wl.make_grid([wl.DENSE_7B], [wl.HW_TINY], *g.axes[2:])
    for axis in (0, 1):
        axes = list(bad.axes)
        axes[axis] = wl.Axis.table([1])
        with pytest.raises(ValueError):
            ora.eval_grid(bridge.ora_grid(wl.Grid(bad.models, bad.hws, tuple(axes))), 0, 1)


def test_scheduler_boundaries_by_hand(ora):
    m = wl.DENSE_7B
    om, oh = bridge.ora_model(m), bridge.ora_hw(wl.HW_TINY)

    def one(T, Q, K, n_lm):
        return ora.pass_detail(om, oh, 1, 16, T, Q, K, n_lm)["t_pass"]

    u32 = lambda *v: np.array(v, dtype=np.uint32)
    # prefill-first: two prompts that fill the budget exactly share one pass
    s = ora.simulate(om, oh, 1, 16, 16, 256, 4, 1.0, np.zeros(2), u32(100, 156), u32(2, 2), detail=True,
                     scheduler=ora.SCHED_PREFILL_FIRST)
    t1 = one(256, 100 * 100 + 156 * 156, 256, 2)
    assert s["ttft"][0] == s["ttft"][1] == t1
    assert s["n_steps"] == 2 and s["n_request_steps"] == 4
    assert s["fin"][0] == s["fin"][1] == t1 + one(2, 101 + 157, 101 + 157, 2)
    # one token more and the second prompt waits for the next pass
    s = ora.simulate(om, oh, 1, 16, 16, 256, 4, 1.0, np.zeros(2), u32(100, 157), u32(2, 2), detail=True,
                     scheduler=ora.SCHED_PREFILL_FIRST)
    assert s["ttft"][0] == one(100, 100 * 100, 100, 1) and s["n_steps"] == 3
    # split-fuse: a running decoder takes one token of the budget, so a prompt of 127 tokens under a budget of 64
    # goes in chunks of 63, 63 and 1 (request 0 has finished its prompt and decodes throughout)
    s = ora.simulate(om, oh, 1, 16, 16, 64, 4, 1.0, np.array([0.0, 1e-9]), u32(10, 127), u32(50, 2), detail=True)
    t = one(10, 10 * 10, 10, 1)                                   # request 0 alone: its whole prompt
    assert s["ttft"][0] == t
    ctx0 = 11
    for c, done in ((63, 63), (63, 126), (1, 127)):
        t += one(1 + c, ctx0 + c * done, ctx0 + done, 1 + (1 if done == 127 else 0))
        ctx0 += 1
    assert s["first"][1] == t
    # a budget that the decoders use up leaves nothing for a prompt: no chunk is scheduled, and none is counted
    s = ora.simulate(om, oh, 1, 16, 16, 2, 4, 1.0, np.array([0.0, 0.0, 1e-9]), u32(1, 1, 1), u32(4, 4, 2), detail=True)
    # step 1: both one-token prompts; steps 2-4: two decoders fill the budget of 2, request 2 waits; then it runs alone
    assert s["n_steps"] == 1 + 3 + 1 + 1
    assert s["n_request_steps"] == 2 + 3 * 2 + 1 + 1
    assert s["first"][2] > s["fin"][0] == s["fin"][1]


def test_mean_tpot_over_requests_with_more_than_one_token(ora):
    om, oh = bridge.ora_model(wl.DENSE_7B), bridge.ora_hw(wl.HW_TINY)
    ins = np.array([300, 64, 700], dtype=np.uint32); outs = np.array([5, 1, 9], dtype=np.uint32)
    arr = np.array([0.0, 100.0, 200.0])                           # far apart: each request has the engine to itself
    s = ora.simulate(om, oh, 1, 16, 16, 2048, 8, 1.0, arr, ins, outs, detail=True)
    tpot = [ora.evaluate(om, oh, ora.knobs(1, int(i), int(o), mbt=2048)).tpot for i, o in zip(ins, outs)]
    assert s["mean_tpot"] == pytest.approx((tpot[0] + tpot[2]) / 2.0, rel=1e-12)      # the one-token request is left out
    assert np.isfinite(s["mean_tpot"]) and tpot[0] != tpot[2]


def test_kv_cache_reduction_columns(ora):
    """Inference Engine Step 1 with a KV-cache reduction that keeps a fraction of every request's entries: the whole
    cache (fraction 1) is the plain analysis; a quarter of 1000 entries is 250, stored in 16 blocks of 16, worked by hand
    for the 7B shape (524 288 B per entry, 13 476 298 752 B of fp16 weights) on an 80 GiB GPU."""
    g = wl.grid_tiny()
    og = bridge.ora_grid(g)
    base, e1 = ora.eval_grid(og), ora.eval_extras_grid(og, 8, kv_keep=1.0)
    np.testing.assert_array_equal(e1["b_max_kept"], base["b_max"])
    np.testing.assert_array_equal(e1["feasible_kept"], base["feasible"])
    np.testing.assert_array_equal(e1["s_max_kept"], e1["s_max"])
    h = wl.Hardware(1e15, 5e12, 80 * wl.GIB, 4e11)
    g1 = wl.make_grid([wl.DENSE_7B], [h], wl.Axis.table([4, 600]), wl.Axis.table([900, 901]), wl.Axis.table([100]),
                      wl.Axis.table([1]), wl.Axis.table([16]), wl.Axis.table([16, 1]), wl.Axis.table([8192]))
    e = ora.eval_extras_grid(bridge.ora_grid(g1), 8, kv_keep=0.25)
    at = lambda b, s_in, blk: g1.flat((0, 0, (4, 600).index(b), (900, 901).index(s_in), 0, 0, 0, (16, 1).index(blk), 0))
    c_avail = 80 * 2 ** 30 - 13476298752
    assert c_avail == 72423047168
    # 250 kept entries -> 256 in blocks of 16: floor(72 423 047 168 / (256 * 524 288)) = 539 requests
    assert e["b_max_kept"][at(4, 900, 16)] == 539 and e["feasible_kept"][at(4, 900, 16)] == 1
    assert e["feasible_kept"][at(600, 900, 16)] == 0                      # 600 > 539
    # blocks of one entry: 250 entries -> floor(c / (250 * 524 288)) = 552; 1001 tokens keep ceil(250.25) = 251 -> 550
    assert e["b_max_kept"][at(4, 900, 1)] == 552 and e["b_max_kept"][at(4, 901, 1)] == 550
    assert e["feasible_kept"][at(600, 900, 1)] == 0 and e["b_max_kept"][at(600, 900, 1)] == 552
    # S_max = floor(c / (4 * 524 288)) = 34 534 entries per request; a quarter kept: sequences of up to 138 136 tokens
    assert e["s_max"][at(4, 900, 16)] == 34534 and e["s_max_kept"][at(4, 900, 16)] == 138136
    # the boundary is inclusive: capacity for exactly 6 requests' kept entries admits a batch of 6, one byte less does not
    kv_req = 256 * 524288
    for cap, ok in ((13476298752 + 6 * kv_req, 1), (13476298752 + 6 * kv_req - 1, 0)):
        gb = wl.make_grid([wl.DENSE_7B], [wl.Hardware(1e15, 5e12, float(cap), 4e11)], wl.Axis.table([6]), wl.Axis.table([900]),
                          wl.Axis.table([100]), wl.Axis.table([1]), wl.Axis.table([16]), wl.Axis.table([16]),
                          wl.Axis.table([8192]))
        eb = ora.eval_extras_grid(bridge.ora_grid(gb), 8, kv_keep=0.25)
        assert eb["feasible_kept"][0] == ok and eb["b_max_kept"][0] == 5 + ok
    # keeping less never admits fewer
    for keep in (0.9, 0.5, 0.1):
        k = ora.eval_extras_grid(og, 8, kv_keep=keep)
        assert np.all(k["b_max_kept"] >= base["b_max"]) and np.all(k["feasible_kept"] >= base["feasible"])
        assert np.all(k["s_max_kept"] >= e1["s_max"])
