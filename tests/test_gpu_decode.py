"""GPU parity of the decode-time pieces: block scores from stored unit keys (Eq. 1-2, Section 4.2) and the
overlap-aware KV swap (Algorithm 1, Section 4.3), each through the C ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import slim_oracle as so
from paper_2508_06447_amd import inputs
from tests.helpers import errs, f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def slim():
    import paper_2508_06447_amd as slim
    slim.load_library()
    return slim


def rand(shape, dtype, seed, scale=1.0):
    g = np.random.default_rng(seed)
    return torch.from_numpy((scale * g.standard_normal(shape)).astype(np.float32)).to(dtype)


# ------------------------------------------------------------------------------- scores from stored unit keys
SCORE_SHAPES = [
    # N, window, Hq, Hkv, d, block, unit, dtype
    (512, 16, 4, 2, 64, 16, 4, torch.float32),
    (4096, 64, 32, 8, 128, 64, 8, torch.bfloat16),
    (1000, 4, 32, 8, 128, 64, 8, torch.bfloat16),        # ragged last block (40 tokens = 5 units)
    (1003, 4, 8, 2, 128, 64, 8, torch.bfloat16),         # ragged last unit as well (43 tokens)
    (45, 2, 4, 2, 32, 8, 3, torch.float32),              # unit does not divide block
    (700, 4, 28, 4, 128, 64, 8, torch.bfloat16),         # 7 query heads per kv head
    (64, 4, 2, 1, 8, 64, 64, torch.float32),             # one block, one unit
]


@pytest.mark.parametrize("N,w,Hq,Hkv,d,block,unit,dtype", SCORE_SHAPES)
def test_unit_keys_and_their_scores_match_oracle(slim, N, w, Hq, Hkv, d, block, unit, dtype):
    print(f"unit-key scores N={N} w={w} Hq={Hq} Hkv={Hkv} d={d} block={block} unit={unit} {dtype}", flush=True)
    k = rand((N, Hkv, d), dtype, seed=N + d)
    q = rand((w, Hq, d), dtype, seed=N + d + 1)
    k_rep = slim.slim_unit_keys(k.cuda(), block, unit)
    want_rep = so.all_unit_keys(f64(k), block, unit)                     # [nb, M, Hkv, d], NaN where no unit
    nb, M = want_rep.shape[:2]
    assert tuple(k_rep.shape) == (nb, M, Hkv * d)
    got_rep = f64(k_rep).reshape(nb, M, Hkv, d)
    present = ~np.isnan(want_rep)
    # float sums of at most `unit` inputs that are exact in float: a few ulp of the unit's magnitude
    assert np.abs(got_rep[present] - want_rep[present]).max() < 1e-5
    assert (got_rep[~present] == 0).all()
    scores = slim.slim_score_blocks_from_unit_keys(q.cuda(), k_rep, N, Hkv, block, unit)
    want = so.block_scores_from_unit_keys(f64(q), want_rep)
    scale = max(1.0, float(np.abs(want).max()))
    assert np.abs(f64(scores) - want).max() < 2e-5 * scale
    # the prefill form on the keys themselves gives the same numbers up to the order of the float additions
    direct = slim.slim_score_blocks(q.cuda(), k.cuda(), block, unit)
    assert (scores - direct).abs().max().item() < 2e-5 * scale


def test_a_decode_step_scores_stored_keys_with_a_new_window(slim):
    """The stored unit keys are computed once; later windows (the most recent decoded tokens) reuse them."""
    N, Hq, Hkv, d, block, unit = 2048, 32, 8, 128, 64, 8
    k = rand((N, Hkv, d), torch.bfloat16, seed=11)
    k_rep = slim.slim_unit_keys(k.cuda(), block, unit)
    want_rep = so.all_unit_keys(f64(k), block, unit)
    for step in range(3):
        q = rand((4, Hq, d), torch.bfloat16, seed=100 + step)
        got = slim.slim_score_blocks_from_unit_keys(q.cuda(), k_rep, N, Hkv, block, unit)
        want = so.block_scores_from_unit_keys(f64(q), want_rep)
        assert np.abs(f64(got) - want).max() < 2e-5 * max(1.0, float(np.abs(want).max()))


# ------------------------------------------------------------------------------------------------ KV swap
class SwapState:
    """Device state of the swap plus the payloads every block must carry wherever it lives."""

    def __init__(self, n_blocks, n_slots, payload_words, active, seed):
        g = np.random.default_rng(seed)
        self.nb, self.ns = n_blocks, n_slots
        self.data = torch.from_numpy(g.integers(-2**31, 2**31 - 1, (n_blocks, payload_words), dtype=np.int64)
                                     .astype(np.int32))
        slots = g.permutation(n_slots)[:len(active)]
        sob = np.full(n_blocks, -1, np.int32)
        bos = np.full(n_slots, -1, np.int32)
        for b, s in zip(sorted(active), slots):
            sob[b], bos[s] = s, b
        mem = np.ones(n_blocks, np.int32)
        mem[sorted(active)] = 0                          # what is on the GPU has not been written to the CPU pool
        self.host_pool = torch.full((n_blocks, payload_words), -1, dtype=torch.int32).pin_memory()
        in_pool = torch.from_numpy(mem == 1)
        self.host_pool[in_pool] = self.data[in_pool]
        gpu = torch.full((n_slots, payload_words), -2, dtype=torch.int32)
        for b in active:
            gpu[sob[b]] = self.data[b]
        self.gpu_pool = gpu.cuda()
        self.slot_of_block = torch.from_numpy(sob).cuda()
        self.block_of_slot = torch.from_numpy(bos).cuda()
        self.in_memory = torch.from_numpy(mem).cuda()

    def sets(self):
        sob = self.slot_of_block.cpu().numpy()
        mem = self.in_memory.cpu().numpy()
        return set(np.nonzero(sob >= 0)[0].tolist()), set(np.nonzero(mem)[0].tolist())

    def check_consistent(self):
        sob, bos = self.slot_of_block.cpu().numpy(), self.block_of_slot.cpu().numpy()
        torch.cuda.synchronize()
        gpu, host, mem = self.gpu_pool.cpu(), self.host_pool, self.in_memory.cpu().numpy()
        for b in range(self.nb):                         # the two maps are inverse to each other
            if sob[b] >= 0:
                assert 0 <= sob[b] < self.ns and bos[sob[b]] == b
                assert torch.equal(gpu[sob[b]], self.data[b]), f"GPU slot of block {b} holds other bytes"
            else:
                assert mem[b] == 1, f"block {b} is neither on the GPU nor in the CPU pool"
            if mem[b]:
                assert torch.equal(host[b], self.data[b]), f"CPU pool entry of block {b} holds other bytes"
        for s in range(self.ns):
            assert bos[s] == -1 or sob[bos[s]] == s


def run_step(slim, st, cand_list, gamma):
    active_prev, memory = st.sets()
    want = so.kv_swap_step(active_prev, cand_list, memory, gamma)
    info = slim.slim_kv_swap(torch.tensor(cand_list, dtype=torch.int32).cuda(), gamma, st.slot_of_block,
                             st.block_of_slot, st.in_memory, st.gpu_pool, st.host_pool)
    torch.cuda.synchronize()
    info = info.cpu().numpy()
    active, mem = st.sets()
    assert info[5] == 0
    assert info[0] == len(set(cand_list)) and info[1] == len(set(cand_list) & active_prev)
    assert bool(info[2]) == want["swapped"]
    assert active == want["active"] and mem == want["memory"]
    assert info[3] == len(want["offload"]) and info[4] == len(want["load"])
    assert info[6] == (len(active_prev - want["active"]) if want["swapped"] else 0)
    st.check_consistent()
    return want


@pytest.mark.parametrize("n_blocks,n_slots,n_active,words,seed", [
    (40, 12, 10, 20, 0),            # payload smaller than one thread's share
    (512, 128, 128, 4096, 1),       # every slot in use
    (333, 90, 50, 1028, 2),         # spare slots, payload not a multiple of the copy tile
    (2100, 1100, 1000, 8, 3),       # more blocks and slots than one pass of the planning workgroup
])
def test_kv_swap_random_walk_matches_algorithm_1(slim, n_blocks, n_slots, n_active, words, seed):
    print(f"kv swap walk nb={n_blocks} slots={n_slots} active={n_active} words={words}", flush=True)
    g = np.random.default_rng(seed)
    active0 = set(g.choice(n_blocks, n_active, replace=False).tolist())
    st = SwapState(n_blocks, n_slots, words, active0, seed)
    st.check_consistent()
    n_swaps = 0
    for step in range(14):
        active, _ = st.sets()
        gamma = [0.9, 0.5, 1.0, 0.0, 0.99, 0.9, 0.75][step % 7]
        # candidate: the active set with a random share replaced, its size drifting within the slots
        size = int(np.clip(len(active) + g.integers(-3, 4), 1, n_slots))
        stay = g.permutation(sorted(active))[:int(round(size * g.choice([1.0, 0.95, 0.9, 0.8, 0.4, 0.0])))]
        others = g.permutation(sorted(set(range(n_blocks)) - active))[:size - len(stay)]
        cand = [int(c) for c in np.concatenate([stay, others]).astype(np.int64)]
        if step % 3 == 0 and cand:
            cand = cand + cand[:2]                       # repeated indices count once
        cand = [cand[i] for i in g.permutation(len(cand))]
        want = run_step(slim, st, cand, gamma)
        n_swaps += want["swapped"]
    assert 0 < n_swaps < 14                              # both branches were taken


def test_kv_swap_edges_of_the_threshold(slim):
    st = SwapState(20, 10, 16, set(range(10)), seed=5)
    # 9 of 10 candidates already active: overlap 0.9 is not < 0.9 -> reuse; it is < 0.91 -> swap
    cand = list(range(9)) + [15]
    assert not run_step(slim, st, cand, 0.9)["swapped"]
    assert not run_step(slim, st, cand, 0.0)["swapped"]
    assert run_step(slim, st, cand, 0.91)["swapped"]
    # identical sets: overlap 1.0 never swaps, even at gamma = 1
    assert not run_step(slim, st, cand, 1.0)["swapped"]
    # disjoint candidate: swaps at any gamma > 0; the 10 leaving blocks are copied out only if not in the pool
    w = run_step(slim, st, list(range(10, 15)) + [16, 17], 0.5)
    assert w["swapped"] and w["offload"] == {0, 1, 2, 3, 4, 5, 6, 7, 8}      # block 15 was in the pool already
    # a single candidate
    assert run_step(slim, st, [3], 0.9)["swapped"]
    assert st.sets()[0] == {3}


def test_kv_swap_reports_errors_and_leaves_the_state_alone(slim):
    st = SwapState(20, 6, 16, {0, 1, 2, 3}, seed=6)

    def snapshot():
        return [t.clone() for t in (st.slot_of_block, st.block_of_slot, st.in_memory, st.gpu_pool)] + \
               [st.host_pool.clone()]

    def same(a, b):
        return all(torch.equal(x.cpu(), y.cpu()) for x, y in zip(a, b))

    def call(cand, gamma=0.9):
        info = slim.slim_kv_swap(torch.tensor(cand, dtype=torch.int32).cuda(), gamma, st.slot_of_block,
                                 st.block_of_slot, st.in_memory, st.gpu_pool, st.host_pool)
        torch.cuda.synchronize()
        return info.cpu().numpy()

    before = snapshot()
    assert call([0, 1, 25])[5] & 1                       # candidate outside [0, n_blocks)
    assert call([0, -1])[5] & 1
    assert call([5, 6, 7, 8, 9, 10, 11])[5] & 4          # seven candidates, six slots
    assert same(before, snapshot())
    st.in_memory[7] = 0                                  # block 7 is nowhere: it cannot be loaded
    before = snapshot()
    assert call([0, 7])[5] & 2
    assert same(before, snapshot())
    st.in_memory[7] = 1
    st.block_of_slot[int(st.slot_of_block[2])] = 3       # maps no longer inverse
    before = snapshot()
    assert call([0, 9])[5] & 8
    assert same(before, snapshot())
    # host-side argument errors
    with pytest.raises(slim.SlimError):
        call([0, 1], gamma=1.5)
    with pytest.raises(slim.SlimError):
        call([0, 1], gamma=float("nan"))


def test_kv_swap_on_a_second_stream_beside_compute(slim):
    """The swap is enqueued on its own stream while a projection runs on the current one (Section 4.3:
    the transfer overlaps the FFN and the next QKV generation); both results are intact."""
    n_blocks, n_slots, words = 512, 128, 65536           # 256 KiB per block: 64 tokens of K and V of one layer
    st = SwapState(n_blocks, n_slots, words, set(range(0, 256, 2)), seed=9)
    a = rand((2048, 4096), torch.bfloat16, 1).cuda()
    w = rand((4096, 4096), torch.bfloat16, 2, scale=0.02).cuda()
    ref = slim.slim_linear(a, w)
    torch.cuda.synchronize()
    active_prev, memory = st.sets()
    cand = sorted(active_prev)[:96] + list(range(257, 289))          # 32 of 128 replaced
    want = so.kv_swap_step(active_prev, cand, memory, 0.9)
    side = torch.cuda.Stream()
    cand_t = torch.tensor(cand, dtype=torch.int32).cuda()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        info = slim.slim_kv_swap(cand_t, 0.9, st.slot_of_block, st.block_of_slot, st.in_memory, st.gpu_pool,
                                 st.host_pool)
    outs = [slim.slim_linear(a, w) for _ in range(4)]
    torch.cuda.synchronize()
    assert info.cpu().numpy()[2] == 1 and st.sets()[0] == want["active"] and st.sets()[1] == want["memory"]
    st.check_consistent()
    for o in outs:
        assert torch.equal(o, ref)


# --------------------------------------------------------------------------------------- decode-step attention
def build_pool(k, v, active, n_slots, block, dtype, seed, layers=1, layer=0):
    """GPU slot pool holding K then V of the active blocks at random slots (NaN everywhere else), and its map."""
    g = np.random.default_rng(seed)
    n, Hkv, d = k.shape
    pool = torch.full((n_slots, layers, 2, block, Hkv, d), float("nan"), dtype=dtype)
    bos = np.full(n_slots, -1, np.int32)
    slots = g.permutation(n_slots)[:len(active)]
    for b, s in zip(sorted(active), slots):
        rows = min(block, n - b * block)
        pool[s, layer, 0, :rows] = k[b * block:b * block + rows]
        pool[s, layer, 1, :rows] = v[b * block:b * block + rows]
        bos[s] = b
    return pool, torch.from_numpy(bos)


@pytest.mark.parametrize("n_prompt,block,n_slots,n_active,n_resp,Hq,Hkv,dtype", [
    (1000, 64, 12, 9, 5, 32, 8, torch.bfloat16),         # ragged last prompt block, free slots, a few response tokens
    (2048, 128, 8, 8, 130, 8, 2, torch.bfloat16),        # two 64-key chunks per slot, three response chunks
    (333, 16, 21, 21, 0, 28, 4, torch.bfloat16),         # 7 query heads per kv head, no response tokens yet
    (512, 64, 8, 3, 64, 4, 4, torch.float32),            # one query head per kv head, fp32
    (64, 64, 0, 0, 77, 16, 2, torch.bfloat16),           # nothing in the pool: response tokens only
    (4096, 64, 64, 64, 1, 32, 8, torch.bfloat16),
])
def test_decode_attention_over_active_slots_matches_oracle(slim, n_prompt, block, n_slots, n_active, n_resp, Hq, Hkv, dtype):
    print(f"decode attn n={n_prompt} block={block} slots={n_slots} active={n_active} resp={n_resp} Hq={Hq} Hkv={Hkv} {dtype}",
          flush=True)
    d = 128
    g = np.random.default_rng(n_prompt + n_resp)
    k, v = rand((n_prompt, Hkv, d), dtype, 1), rand((n_prompt, Hkv, d), dtype, 2)
    kr, vr = rand((max(n_resp, 1), Hkv, d), dtype, 3)[:n_resp], rand((max(n_resp, 1), Hkv, d), dtype, 4)[:n_resp]
    q = rand((Hq, d), dtype, 5, 2.0)
    nb = (n_prompt + block - 1) // block
    active = set(g.choice(nb, n_active, replace=False).tolist()) if n_active else set()
    if n_active and n_prompt % block:
        active = set(list(active)[:-1]) | {nb - 1}        # the short last block among them
    layers, layer = (3, 1) if n_slots == 12 else (1, 0)
    pool, bos = build_pool(k, v, active, max(n_slots, 1), block, dtype, seed=7, layers=layers, layer=layer)
    pool, bos = pool[:n_slots], bos[:n_slots]
    T = so.active_token_index(active, block, n_prompt)
    k_all = np.concatenate([f64(k)[T], f64(kr)]) if n_resp else f64(k)[T]
    v_all = np.concatenate([f64(v)[T], f64(vr)]) if n_resp else f64(v)[T]
    want = so.decode_attention(f64(q), k_all, v_all)
    off = layer * 2 * block * Hkv * d * pool.element_size()
    got = slim.slim_decode_attn(q.cuda(), pool.cuda(), bos.cuda(), block, n_prompt, Hkv,
                                kr.cuda() if n_resp else None, vr.cuda() if n_resp else None, layer_offset=off)
    tol = 2.0 ** -8 if dtype == torch.bfloat16 else 2e-5
    np.testing.assert_allclose(f64(got), want, rtol=tol, atol=tol * np.abs(want).max())
    assert torch.isfinite(got.float()).all()              # nothing outside the active rows was read (it is NaN)


def test_a_decode_step_scores_selects_swaps_and_attends(slim):
    """One decode step of a layer through the C ABI: scores from stored unit keys and the window of recent Query
    states, top-k candidate set, overlap-aware swap of the K/V payloads, attention of the new token over what is
    then active -- each stage against the oracle's."""
    n_prompt, block, unit, Hq, Hkv, d, n_slots, n_keep = 2048 + 40, 64, 8, 32, 8, 128, 12, 10
    bf = torch.bfloat16
    nb = (n_prompt + block - 1) // block
    k, v = rand((n_prompt, Hkv, d), bf, 11), rand((n_prompt, Hkv, d), bf, 12)
    words = 2 * block * Hkv * d // 2                      # K then V rows of a block as int32 words
    payload = torch.zeros(nb, 2, block, Hkv, d, dtype=bf)
    for b in range(nb):
        rows = min(block, n_prompt - b * block)
        payload[b, 0, :rows], payload[b, 1, :rows] = k[b * block:b * block + rows], v[b * block:b * block + rows]
    payload_words = payload.view(torch.int32).reshape(nb, words)
    active0 = {0, 3, 4, 9, 10, 17, 20, 25, 30, nb - 1}
    st = SwapState(nb, n_slots, words, active0, seed=13)
    st.data = payload_words                               # the payloads are the real K/V rows
    st.host_pool.copy_(payload_words)
    gpu = torch.zeros(n_slots, words, dtype=torch.int32)
    sob = st.slot_of_block.cpu().numpy()
    for b in active0:
        gpu[sob[b]] = payload_words[b]
    st.gpu_pool = gpu.cuda()
    st.in_memory.fill_(1)
    k_rep = slim.slim_unit_keys(k.cuda(), block, unit)
    want_rep = so.all_unit_keys(f64(k), block, unit)
    kr, vr = rand((6, Hkv, d), bf, 14), rand((6, Hkv, d), bf, 15)
    n_swaps = 0
    for step, gamma in enumerate((0.9, 0.9, 0.3)):
        q_win = rand((4, Hq, d), bf, 20 + step, 1.5)      # Query states of the most recent tokens
        q_new = q_win[-1]
        scores = slim.slim_score_blocks_from_unit_keys(q_win.cuda(), k_rep, n_prompt, Hkv, block, unit)
        sc_ref = so.block_scores_from_unit_keys(f64(q_win), want_rep)
        assert np.abs(f64(scores) - sc_ref).max() < 2e-5 * max(1.0, np.abs(sc_ref).max())
        cand = slim.slim_select_topk_blocks(scores, n_keep)
        cand_ref = so.select_blocks(sc_ref, n_keep)
        np.testing.assert_array_equal(cand.cpu().numpy(), cand_ref)
        active_prev, memory = st.sets()
        want = so.kv_swap_step(active_prev, cand_ref.tolist(), memory, gamma)
        info = slim.slim_kv_swap(cand, gamma, st.slot_of_block, st.block_of_slot, st.in_memory, st.gpu_pool, st.host_pool)
        out = slim.slim_decode_attn(q_new.cuda(), st.gpu_pool.view(torch.bfloat16).view(n_slots, 2, block, Hkv, d),
                                    st.block_of_slot, block, n_prompt, Hkv, kr.cuda(), vr.cuda())
        torch.cuda.synchronize()
        assert bool(info.cpu()[2]) == want["swapped"] and st.sets()[0] == want["active"]
        st.check_consistent()
        T = so.active_token_index(want["active"], block, n_prompt)
        ref = so.decode_attention(f64(q_new), np.concatenate([f64(k)[T], f64(kr)]), np.concatenate([f64(v)[T], f64(vr)]))
        np.testing.assert_allclose(f64(out), ref, rtol=2.0 ** -8, atol=2.0 ** -8 * np.abs(ref).max())
        n_swaps += want["swapped"]
    assert n_swaps >= 1


def test_decode_step_at_the_full_size_of_the_32k_workload(slim):
    """The decode-time kernels in the configuration bench.py --workload decode times: 32768 prompt tokens = 512
    blocks of 64, 8 kv heads of 128, 128 GPU slots, K+V payloads of 256 KiB per block, 32 of the 128 active blocks
    replaced by one swap.  Scores and candidate set in full, swap sets and every payload byte, attention output."""
    n_prompt, block, unit, Hq, Hkv, d, n_slots = 32768, 64, 8, 32, 8, 128, 128
    bf = torch.bfloat16
    nb = n_prompt // block
    g = np.random.default_rng(41)
    k, v = rand((n_prompt, Hkv, d), bf, 31), rand((n_prompt, Hkv, d), bf, 32)
    words = 2 * block * Hkv * d // 2
    payload_words = torch.stack([k.view(nb, block, Hkv, d), v.view(nb, block, Hkv, d)], dim=1).contiguous() \
        .view(torch.int32).reshape(nb, words)
    # scores from stored unit keys with a window of 4 recent tokens; candidates = top 128 blocks (first and last forced)
    q_win = rand((4, Hq, d), bf, 33, 1.5)
    k_rep = slim.slim_unit_keys(k.cuda(), block, unit)
    scores = slim.slim_score_blocks_from_unit_keys(q_win.cuda(), k_rep, n_prompt, Hkv, block, unit)
    sc_ref = so.block_scores_from_unit_keys(f64(q_win), so.all_unit_keys(f64(k), block, unit))
    assert np.abs(f64(scores) - sc_ref).max() < 2e-5 * max(1.0, np.abs(sc_ref).max())
    cand = slim.slim_select_topk_blocks(scores, n_slots)
    cand_ref = so.select_blocks(sc_ref, n_slots)
    np.testing.assert_array_equal(cand.cpu().numpy(), cand_ref)
    # previous active set: 96 of the candidates + 32 other blocks -> overlap 0.75 < 0.9: a swap of 32 blocks
    others = [b for b in range(nb) if b not in set(cand_ref.tolist())]
    active0 = set(g.permutation(cand_ref)[:96].tolist()) | set(g.permutation(others)[:32].tolist())
    st = SwapState(nb, n_slots, words, active0, seed=43)
    st.data = payload_words
    in_pool = st.in_memory.cpu().bool()
    st.host_pool.fill_(-1)
    st.host_pool[in_pool] = payload_words[in_pool]        # what is on the GPU has not been written to the CPU pool
    gpu = torch.zeros(n_slots, words, dtype=torch.int32)
    sob = st.slot_of_block.cpu().numpy()
    for b in active0:
        gpu[sob[b]] = payload_words[b]
    st.gpu_pool = gpu.cuda()
    active_prev, memory = st.sets()
    want = so.kv_swap_step(active_prev, cand_ref.tolist(), memory, 0.9)
    assert want["swapped"] and len(want["load"]) == 32 and len(want["offload"]) == 32
    info = slim.slim_kv_swap(cand, 0.9, st.slot_of_block, st.block_of_slot, st.in_memory, st.gpu_pool, st.host_pool)
    kr, vr = rand((16, Hkv, d), bf, 34), rand((16, Hkv, d), bf, 35)
    out = slim.slim_decode_attn(q_win[-1].cuda(), st.gpu_pool.view(torch.bfloat16).view(n_slots, 2, block, Hkv, d),
                                st.block_of_slot, block, n_prompt, Hkv, kr.cuda(), vr.cuda())
    torch.cuda.synchronize()
    inf = info.cpu().numpy()
    assert inf[2] == 1 and inf[3] == 32 and inf[4] == 32 and inf[5] == 0
    assert st.sets() == (want["active"], want["memory"])
    st.check_consistent()
    T = so.active_token_index(want["active"], block, n_prompt)
    ref = so.decode_attention(f64(q_win[-1]), np.concatenate([f64(k)[T], f64(kr)]), np.concatenate([f64(v)[T], f64(vr)]))
    np.testing.assert_allclose(f64(out), ref, rtol=2.0 ** -8, atol=2.0 ** -8 * np.abs(ref).max())


# ------------------------------------------------------------------------------ single-token projections and layer
@pytest.mark.parametrize("n,k,dtype", [(4096, 4096, torch.bfloat16), (1024, 4096, torch.bfloat16), (70, 256, torch.bfloat16),
                                       (13, 64, torch.float32), (3584, 18944, torch.bfloat16)])
def test_gemv_all_epilogues(slim, n, k, dtype):
    print(f"gemv n={n} k={k} {dtype}", flush=True)
    if k > 16384:
        with pytest.raises(slim.SlimError):
            slim.slim_gemv(rand((8, k), dtype, 1).cuda(), rand((k,), dtype, 2).cuda())
        return
    w, w2, x = rand((n, k), dtype, 1, 0.05), rand((n, k), dtype, 2, 0.05), rand((k,), dtype, 3)
    b, r = rand((n,), dtype, 4), rand((n,), dtype, 5)
    sc = torch.tensor([0.37], dtype=torch.float32)
    W, W2, X = f64(w), f64(w2), f64(x)
    rel = 2.0 ** -8 if dtype == torch.bfloat16 else 1e-5
    def close(got, want):
        np.testing.assert_allclose(f64(got), want, rtol=rel, atol=rel * max(1e-6, np.abs(want).max()))
    close(slim.slim_gemv(w.cuda(), x.cuda()), W @ X)
    close(slim.slim_gemv(w.cuda(), x.cuda(), scale=sc.cuda(), bias=b.cuda()), 0.37 * (W @ X) + f64(b))
    rd = r.cuda().clone()
    slim.slim_gemv(w.cuda(), x.cuda(), residual=rd, out=rd)                 # in place
    close(rd, W @ X + f64(r))
    close(slim.slim_gemv(w.cuda(), x.cuda(), w_up=w2.cuda(), scale=sc.cuda()), so.silu(0.37 * (W @ X)) * (0.37 * (W2 @ X)))


def decode_case(slim, wl, n_slots, n_active, n_resp, fold, seed, np_dtype=np.float64):
    """One decoded token through slim_decode_layer against the oracle's decode_layer on the gathered context."""
    bf = torch.bfloat16
    Hq, Hkv, d, block, n_prompt = wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.block, wl.seq
    g = np.random.default_rng(seed)
    w = inputs.layer_weights(wl)
    k, v = rand((n_prompt, Hkv, d), bf, seed + 1), rand((n_prompt, Hkv, d), bf, seed + 2)
    nb = (n_prompt + block - 1) // block
    active = set(g.choice(nb - 1, n_active - 1, replace=False).tolist()) | {nb - 1}
    pool, bos = build_pool(k, v, active, n_slots, block, bf, seed=seed + 3)
    kr = torch.zeros(n_resp + 1, Hkv, d, dtype=bf)
    vr = torch.zeros(n_resp + 1, Hkv, d, dtype=bf)
    kr[:n_resp], vr[:n_resp] = rand((n_resp, Hkv, d), bf, seed + 4), rand((n_resp, Hkv, d), bf, seed + 5)
    x_new = rand((wl.hidden,), bf, seed + 6, 1.5)
    position = n_prompt + n_resp
    shape = slim.make_shape(wl.hidden, Hq, Hkv, d, wl.ffn, block, wl.unit, wl.window, bf, wl.rope_theta, wl.rms_eps)
    wd = {kk: vv.cuda() for kk, vv in w.items() if not (fold and kk in ("g_attn", "g_ffn"))}
    krd, vrd = kr.cuda(), vr.cuda()
    z, q = slim.slim_decode_layer(shape, wd, x_new.cuda(), position, pool.cuda(), bos.cuda(), n_prompt, krd, vrd, n_resp)
    torch.cuda.synchronize()
    s = so.LayerShape(wl.hidden, Hq, Hkv, d, wl.ffn, block, wl.unit, wl.window, wl.rope_theta, wl.rms_eps)
    ow = so.LayerWeights(**{kk: vv.to(torch.float32).numpy().astype(np_dtype) for kk, vv in w.items()})
    T = so.active_token_index(active, block, n_prompt)
    k_ctx = np.concatenate([f64(k)[T], f64(kr[:n_resp])]).astype(np_dtype)
    v_ctx = np.concatenate([f64(v)[T], f64(vr[:n_resp])]).astype(np_dtype)
    xs = f64(x_new).astype(np_dtype)
    z_ref, k_ref, v_ref = so.decode_layer(s, ow, xs, position, k_ctx, v_ctx)
    z_b, _, _ = so.decode_layer(s, ow, xs, position, k_ctx, v_ctx, rounding="bf16")
    fl_max, fl_mean = np.abs(z_b - z_ref).max(), np.abs(z_b - z_ref).mean()
    rel = 2.0 ** -8
    np.testing.assert_allclose(f64(krd[n_resp]), k_ref, rtol=rel, atol=rel * np.abs(k_ref).max())
    np.testing.assert_allclose(f64(vrd[n_resp]), v_ref, rtol=rel, atol=rel * np.abs(v_ref).max())
    assert torch.equal(krd[:n_resp].cpu(), kr[:n_resp]) and torch.equal(vrd[:n_resp].cpu(), vr[:n_resp])
    h = so.rmsnorm(xs[None], ow.g_attn, s.rms_eps)
    q_ref = so.project_heads(h, ow.wq, Hq, d, np.asarray([position]), s.rope_theta, True, None, ow.bq)[0]
    np.testing.assert_allclose(f64(q), q_ref, rtol=rel, atol=rel * np.abs(q_ref).max())
    mx, mean = errs(z, z_ref.astype(np.float64))
    print(f"decode layer {wl.family} hidden {wl.hidden} slots {n_slots} active {n_active} resp {n_resp} fold {fold}: z max-abs "
          f"{mx:.3e} mean-abs {mean:.3e} (bf16-rounding oracle {fl_max:.3e} / {fl_mean:.3e}); |z| max {np.abs(z_ref).max():.2f}",
          flush=True)
    assert mx <= max(2e-2, 1.5 * fl_max) and mean <= max(2e-3, 1.5 * fl_mean)


@pytest.mark.parametrize("fold", [False, True])
def test_decode_layer_reduced_shapes(slim, fold):
    llama = inputs.scaled(inputs.WORKLOADS["cfg2"], seq=1000, hidden=512, n_q_heads=8, n_kv_heads=2, ffn=1024)
    decode_case(slim, llama, n_slots=12, n_active=9, n_resp=5, fold=fold, seed=50)
    decode_case(slim, llama, n_slots=4, n_active=4, n_resp=0, fold=fold, seed=60)          # first decoded token
    qwen = inputs.scaled(inputs.WORKLOADS["cfg6"], seq=777, hidden=448, n_q_heads=14, n_kv_heads=2, ffn=1184, x_kind="normal")
    decode_case(slim, qwen, n_slots=10, n_active=7, n_resp=70, fold=fold, seed=70)         # biases, 7 heads per kv head


def test_decode_layer_full_llama_shape(slim):
    """LLaMA-3.1-8B-shaped layer, 32768-token prompt, 128 active blocks (8192 tokens), 16 response tokens, folded gains."""
    decode_case(slim, inputs.WORKLOADS["cfg3"], n_slots=128, n_active=128, n_resp=16, fold=True, seed=80, np_dtype=np.float32)


def test_decode_layer_replayed_from_a_hip_graph(slim):
    """The layer only enqueues kernels on the caller's stream (no allocation, no memset, no host synchronisation), so
    a caller can capture it into a HIP graph.  Every replay, with eager work and synchronisation in between and a new
    input each time, must equal the eager call bit for bit."""
    bf = torch.bfloat16
    wl = inputs.scaled(inputs.WORKLOADS["cfg2"], seq=1000, hidden=512, n_q_heads=8, n_kv_heads=2, ffn=1024)
    Hq, Hkv, d, block = wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.block
    w = {kk: vv.cuda() for kk, vv in inputs.layer_weights(wl).items() if kk not in ("g_attn", "g_ffn")}
    k, v = rand((wl.seq, Hkv, d), bf, 1), rand((wl.seq, Hkv, d), bf, 2)
    pool, bos = build_pool(k, v, {0, 2, 5, 7, 11, 15}, 8, block, bf, seed=3)
    pool, bos = pool.cuda(), bos.cuda()
    n_resp = 3
    kr, vr = torch.zeros(n_resp + 1, Hkv, d, dtype=bf).cuda(), torch.zeros(n_resp + 1, Hkv, d, dtype=bf).cuda()
    kr[:n_resp], vr[:n_resp] = rand((n_resp, Hkv, d), bf, 4).cuda(), rand((n_resp, Hkv, d), bf, 5).cuda()
    shape = slim.make_shape(wl.hidden, Hq, Hkv, d, wl.ffn, block, wl.unit, wl.window, bf, wl.rope_theta, wl.rms_eps)
    import ctypes
    ws = torch.empty(slim.load_library().slim_decode_layer_workspace_bytes(ctypes.byref(shape), 8, n_resp), dtype=torch.uint8,
                     device="cuda")
    x_in = rand((wl.hidden,), bf, 6).cuda()
    slim.slim_decode_layer(shape, w, x_in, wl.seq + n_resp, pool, bos, wl.seq, kr, vr, n_resp, workspace=ws)   # warm-up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        z_g, q_g = slim.slim_decode_layer(shape, w, x_in, wl.seq + n_resp, pool, bos, wl.seq, kr, vr, n_resp, workspace=ws)
    a, wt = rand((300, 512), bf, 7).cuda(), rand((256, 512), bf, 8, 0.05).cuda()
    for step in range(4):
        x_in.copy_(rand((wl.hidden,), bf, 10 + step).cuda())
        graph.replay()
        torch.cuda.synchronize()
        z_r, q_r, k_r = z_g.clone(), q_g.clone(), kr[n_resp].clone()
        slim.slim_linear(a, wt)                          # eager work between the replays
        z_e, q_e = slim.slim_decode_layer(shape, w, x_in, wl.seq + n_resp, pool, bos, wl.seq, kr, vr, n_resp, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(z_r, z_e) and torch.equal(q_r, q_e) and torch.equal(k_r, kr[n_resp]), f"replay {step} differs"
        assert torch.isfinite(z_r.float()).all()
