"""The planner and the projection together: a multi-turn exchange in which an aLoRA request reuses
the cache blocks a base-model request filled (Sec. 3, Fig. 2's pipelines in miniature).  After the
turns, the K/V the aLoRA request sees through its block table -- partly written by the base
request, partly by its own prefill and decode steps -- must equal what the fp64 oracle computes
for the whole conversation from scratch."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_17910_amd import binding as ab
from paper_2512_17910_amd import planner as pl
from paper_2512_17910_amd import workloads as wl
from gpu_util import TOL, maxnorm_rel, to_dev, to_f64

pytestmark = pytest.mark.gpu

HIDDEN, NQH, NKVH, HD, L, RANK, BS, N_BLOCKS, VOCAB = 256, 4, 2, 128, 3, 16, 16, 40, 97
NQ, NKV = NQH * HD, NKVH * HD
NEVER = 1 << 30


class TinyModel:
    """Seeded weights and a token embedding; x of a row is a function of its token id only, so equal
    prefixes give equal layer inputs whichever request they belong to."""

    def __init__(self, dtype="bf16"):
        self.dtype = dtype
        ref = wl.small_mixed(dtype, hidden=HIDDEN, n_q_heads=NQH, n_kv_heads=NKVH, head_dim=HD, n_adapters=L,
                             rank=RANK, block_size=BS, seq_lens=(VOCAB,), seed=31)
        self.emb_host = ref.x[:VOCAB]                      # storage-rounded values
        self.W_host, self.A_host, self.B_host = ref.W, ref.A, ref.B
        self.W = to_dev(ref.W, dtype)
        self.A = [to_dev(a, dtype) for a in ref.A]
        self.B = [to_dev(b, dtype) for b in ref.B]
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.kc = torch.zeros((N_BLOCKS * BS, NKV), dtype=tdt, device="cuda")
        self.vc = torch.zeros((N_BLOCKS * BS, NKV), dtype=tdt, device="cuda")

    def forward(self, batch: pl.Batch, tokens_of_row):
        """Project the planned rows; tokens_of_row[i] = token id of row i."""
        pos, seg, aid, slot, starts = batch.rows()
        T = len(pos)
        x = to_dev(self.emb_host[np.asarray(tokens_of_row)], self.dtype)
        d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda")
        seg_d, pos_d = d(seg), d(pos)
        dims = ab.make_dims(ab.ALORA_BF16 if self.dtype == "bf16" else ab.ALORA_F32, T, HIDDEN, NQH, NKVH, HD, L,
                            RANK, len(starts), N_BLOCKS * BS, seg_d, pos_d)
        ws = ab.alloc_workspace(dims)
        q = torch.zeros((T, NQ), dtype=x.dtype, device="cuda")
        aid_d, start_d, slot_d = d(aid), d(starts), d(slot)
        assert ab.alora_qkv_validate(aid_d, start_d, slot_d, BS, dims) == ab.ALORA_OK
        ab.alora_qkv_forward(x, aid_d, start_d, self.W, self.A, self.B, q, self.kc, self.vc, slot_d, BS, dims, ws)
        torch.cuda.synchronize()
        return q

    def oracle_kv(self, tokens, adapter, start):
        """K and V rows of a whole request computed from scratch in fp64."""
        n = len(tokens)
        x = wl.widen_f64(self.emb_host[np.asarray(tokens)], self.dtype)
        W = wl.widen_f64(self.W_host, self.dtype)
        A = [wl.widen_f64(a, self.dtype) for a in self.A_host]
        B = [wl.widen_f64(b, self.dtype) for b in self.B_host]
        aid = np.full(n, adapter, np.int32)
        seg = np.zeros(n, np.int32)
        pos = np.arange(n, dtype=np.int32)
        _, act = oracle.classify(aid, seg, pos, np.asarray([start], np.int32))
        y = oracle.alora_rows(x, W, A, B, aid, act, np.arange(n, dtype=np.int32))
        return y[:, NQ:NQ + NKV], y[:, NQ + NKV:], act

    def cache_rows(self, table, n):
        slots = np.asarray([table[p // BS] * BS + p % BS for p in range(n)])
        idx = torch.from_numpy(slots).to("cuda")
        return to_f64(self.kc[idx]), to_f64(self.vc[idx])


def _check_request(m: TinyModel, planner, rid, tokens, adapter, start):
    k_ref, v_ref, act = m.oracle_kv(tokens, adapter, start)
    k, v = m.cache_rows(planner.block_table(rid), len(tokens))
    tol = TOL[m.dtype]
    assert maxnorm_rel(k, k_ref) <= tol and maxnorm_rel(v, v_ref) <= tol
    return act


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_alora_turn_reuses_base_blocks_and_the_cache_matches_a_from_scratch_oracle(dtype):
    rng = np.random.default_rng(5)
    m = TinyModel(dtype)
    planner = pl.Planner(BS, N_BLOCKS)
    prompt = [int(t) for t in rng.integers(0, VOCAB, 75)]
    invocation = [int(t) for t in rng.integers(0, VOCAB, 5)]

    # turn 1: the base model prefills the prompt and finishes
    b = pl.Batch(256, 4)
    assert planner.admit(1, prompt, -1, NEVER, b) == 0
    m.forward(b, prompt)
    planner.commit(1)
    _check_request(m, planner, 1, prompt, -1, NEVER)
    base_table = list(planner.block_table(1))
    planner.finish(1)

    # turn 2: an aLoRA is invoked on prompt + invocation tokens; only the uncached suffix is projected
    conv = prompt + invocation
    start = len(prompt)
    b = pl.Batch(256, 4)
    cached = planner.admit(2, conv, 1, start, b)
    assert cached == 64 and b.n_rows == len(conv) - 64
    assert list(planner.block_table(2))[:4] == base_table[:4]
    m.forward(b, conv[cached:])
    planner.commit(2)
    act = _check_request(m, planner, 2, conv, 1, start)
    assert act[:start].sum() == 0 and act[start:].all()

    # the adapter generates three tokens, one decode step each
    for step in range(3):
        tok = int(rng.integers(0, VOCAB))
        b = pl.Batch(8, 1)
        planner.append(2, [tok], b)
        conv = conv + [tok]
        assert list(b.rows()[0]) == [len(conv) - 1]
        m.forward(b, [tok])
        planner.commit(2)
    _check_request(m, planner, 2, conv, 1, start)

    # turn 3, the other direction: the base model continues the same conversation while request 2 is
    # still alive; it shares the four pre-activation blocks and recomputes the rest with base weights
    b = pl.Batch(256, 4)
    cached3 = planner.admit(3, conv, -1, NEVER, b)
    assert cached3 == 64
    m.forward(b, conv[cached3:])
    planner.commit(3)
    _check_request(m, planner, 3, conv, -1, NEVER)
    _check_request(m, planner, 2, conv, 1, start)      # request 2's own blocks were not disturbed
    t2, t3 = list(planner.block_table(2)), list(planner.block_table(3))
    assert t2[:4] == t3[:4] and not set(t2[4:]) & set(t3[4:])

    # a second invocation of the same aLoRA on the same conversation reuses the adapter's own blocks too
    b = pl.Batch(256, 4)
    assert planner.admit(4, conv, 1, start, b) == (len(conv) - 1) // BS * BS
    # a standard LoRA (activation at 0) shares nothing
    b = pl.Batch(256, 4)
    assert planner.admit(5, conv, 2, 0, b) == 0


def _attend(m: TinyModel, planner, rid, q, positions):
    """The reader over request rid's block table for rows at `positions` (their q from the projection)."""
    table = np.asarray(planner.block_table(rid), np.int32)[None, :]
    bt = torch.from_numpy(table).to("cuda")
    seq = torch.zeros(len(positions), dtype=torch.int32, device="cuda")
    pos = torch.from_numpy(np.asarray(positions, np.int32)).to("cuda")
    out = torch.empty_like(q)
    dims = ab.make_attn_dims(q, m.kc, bt, NQH, NKVH, HD, BS)
    assert ab.alora_paged_attention_validate(bt, seq, pos, dims) == ab.ALORA_OK
    ab.alora_paged_attention(q, m.kc, m.vc, bt, seq, pos, out, dims)
    torch.cuda.synchronize()
    got = to_f64(out)
    if m.dtype == "bf16":
        # the same rows through the row-block reader of projected suffixes (consecutive positions of one sequence)
        out2 = torch.full_like(q, float("nan"))
        ab.alora_paged_attention_suffix(q, m.kc, m.vc, bt, seq, pos, out2, dims)
        torch.cuda.synchronize()
        assert maxnorm_rel(to_f64(out2), got) <= TOL["bf16"]
    return got


def _dense_attention(m: TinyModel, tokens, adapter, start, positions):
    """The whole conversation from scratch in fp64: projection of every token (adapter applied from the
    activation point on), then causal attention over the dense K and V."""
    from oracle import attention as oatt
    n = len(tokens)
    x = wl.widen_f64(m.emb_host[np.asarray(tokens)], m.dtype)
    W = wl.widen_f64(m.W_host, m.dtype)
    A = [wl.widen_f64(a, m.dtype) for a in m.A_host]
    B = [wl.widen_f64(b, m.dtype) for b in m.B_host]
    aid = np.full(n, adapter, np.int32)
    _, act = oracle.classify(aid, np.zeros(n, np.int32), np.arange(n, dtype=np.int32), np.asarray([start], np.int32))
    y = oracle.alora_rows(x, W, A, B, aid, act, np.arange(n, dtype=np.int32))
    q, k, v = y[:, :NQ], y[:, NQ:NQ + NKV], y[:, NQ + NKV:]
    nb = (n + BS - 1) // BS
    pad = lambda a: np.vstack([a, np.zeros((nb * BS - n, a.shape[1]))])
    return oatt.paged_attention(q, pad(k), pad(v), np.arange(nb, dtype=np.int32)[None, :], np.zeros(n, np.int32),
                                np.arange(n, dtype=np.int32), BS, NQH, NKVH, HD, rows=np.asarray(positions))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention_over_reused_blocks_matches_a_dense_from_scratch_computation(dtype):
    """Sec. 2.3's claim in numbers: an aLoRA request whose first 64 positions were written by a base-model
    request's projection, the rest by its own (adapted from the activation point on), attends over both
    and gets what a dense computation of its whole sequence gives; the same for a base request that
    continues the conversation over the shared blocks."""
    rng = np.random.default_rng(6)
    m = TinyModel(dtype)
    planner = pl.Planner(BS, N_BLOCKS)
    prompt = [int(t) for t in rng.integers(0, VOCAB, 75)]
    invocation = [int(t) for t in rng.integers(0, VOCAB, 5)]
    # two chained steps (projection, then attention), each within the single-step gate
    tol = 2 * TOL[dtype]

    b = pl.Batch(256, 4)
    assert planner.admit(1, prompt, -1, NEVER, b) == 0
    q1 = m.forward(b, prompt)
    planner.commit(1)
    got = _attend(m, planner, 1, q1, list(range(75)))
    assert maxnorm_rel(got, _dense_attention(m, prompt, -1, NEVER, list(range(75)))) <= tol
    planner.finish(1)

    conv = prompt + invocation
    start = len(prompt)
    b = pl.Batch(256, 4)
    cached = planner.admit(2, conv, 1, start, b)
    assert cached == 64
    q2 = m.forward(b, conv[cached:])                       # rows for positions 64..79 only
    planner.commit(2)
    positions = list(range(cached, len(conv)))
    got = _attend(m, planner, 2, q2, positions)
    ref = _dense_attention(m, conv, 1, start, positions)
    assert maxnorm_rel(got, ref) <= tol
    # the adapter matters: the same rows computed as a base request differ by far more than the gate
    assert maxnorm_rel(_dense_attention(m, conv, -1, NEVER, positions)[start - cached:], ref[start - cached:]) > 10 * tol

    # the base model continues over the same conversation and shares the four pre-activation blocks
    b = pl.Batch(256, 4)
    assert planner.admit(3, conv, -1, NEVER, b) == 64
    q3 = m.forward(b, conv[64:])
    planner.commit(3)
    got = _attend(m, planner, 3, q3, positions)
    assert maxnorm_rel(got, _dense_attention(m, conv, -1, NEVER, positions)) <= tol
    # and request 2's view is unchanged by request 3's writes
    assert maxnorm_rel(_attend(m, planner, 2, q2, positions), ref) <= tol
