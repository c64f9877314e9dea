"""CPU-only check of the copy/compute chain of streaming attention (Sec. 4.3, Alg. 1 "AsyncPrefetch": the transfer
of block i + 1 runs while block i is attended).  ttkv_staged_schedule records the stream operations that
ttkv_decode_attn would issue (the same issuing code, a recorder in place of HIP).  From them this test builds the
happens-before graph that HIP's semantics give -- operations of one stream in issue order; a wait is ordered after
the latest record of its event issued before it -- and checks what makes staging-slot reuse safe:
  - the kernel that attends fetch i starts after copy i has finished;
  - the copy that overwrites a slot starts after the kernel that read the slot's previous contents has finished;
  - the first copy starts after everything issued earlier on the compute stream (an earlier call may still read
    the slots); the merge comes after every attention launch;
and that nothing else serialises the two streams: copy i + 1 is NOT ordered after kernel i while slots are free."""
import numpy as np
import pytest

from paper_2604_19769_amd import binding as B

N_EVENTS = 1 + 2 * B.TTKV_MAX_SLOTS


def offload_cache(n_host_tokens, bt=1024, batch=1, Hkv=8, paged=False, seed=0):
    """bf16 + int8 device tiers, int4 host tier holding n_host_tokens[b] tokens; pointers are never dereferenced."""
    c = B.ttkv_cache()
    c.batch, c.n_q_heads, c.n_kv_heads, c.head_dim, c.n_tiers = batch, 4 * Hkv, Hkv, 128, 3
    c.softmax_scale = 0.088
    keep = []
    spec = [("bf16", "bf16", 128, 4096, [300] * batch), ("i8", "i8", 128, 28672, [2000] * batch), ("i4", "i4", bt, 10**9, n_host_tokens)]
    for t, (kf, vf, b_, cap, lens) in enumerate(spec):
        T = c.tier[t]
        T.k_fmt, T.v_fmt, T.block_tokens, T.capacity_tokens = B.FMT_NAMES[kf], B.FMT_NAMES[vf], b_, cap
        T.mem = B.MEM_HOST_PINNED if t == 2 else B.MEM_DEVICE
        T.ring_blocks = max(lens) // b_ + 3
        T.pool_blocks = T.ring_blocks * batch
        buf = np.zeros(16, np.uint8)
        s, l = np.zeros(batch, np.int64), np.array(lens, np.int64)
        T.data, T.start, T.len = buf.ctypes.data, s.ctypes.data, l.ctypes.data
        keep += [buf, s, l]
        if paged and t == 2:
            tab = np.random.default_rng(seed).permutation(T.pool_blocks).astype(np.int32)
            T.block_table, T.block_table_dev = tab.ctypes.data, buf.ctypes.data
            keep.append(tab)
    c._keep = keep
    return c


def happens_before(ops):
    """Adjacency lists of the happens-before graph over op indices (edges point forward in time)."""
    succ = [[] for _ in ops]
    last_on_stream = {}
    last_record = {}
    for i, op in enumerate(ops):
        s = op["stream"]
        if s in last_on_stream:
            succ[last_on_stream[s]].append(i)
        last_on_stream[s] = i
        if op["kind"] == B.OP_RECORD:
            last_record[op["event"]] = i
        elif op["kind"] == B.OP_WAIT:
            assert 0 <= op["event"] < N_EVENTS
            if op["event"] in last_record:           # an event never recorded is complete: the wait is a no-op
                succ[last_record[op["event"]]].append(i)
    return succ


def reaches(succ, a, b):
    seen, stack = {a}, [a]
    while stack:
        x = stack.pop()
        if x == b:
            return True
        for y in succ[x]:
            if y not in seen:
                seen.add(y)
                stack.append(y)
    return False


def check_chain(ops, n_slots, same_stream):
    copies = {op["fetch"]: i for i, op in enumerate(ops) if op["kind"] == B.OP_COPY}
    kernels = {op["fetch"]: i for i, op in enumerate(ops) if op["kind"] == B.OP_ATTEND and op["fetch"] >= 0}
    merges = [i for i, op in enumerate(ops) if op["kind"] == B.OP_MERGE]
    n = len(copies)
    assert sorted(copies) == sorted(kernels) == list(range(n)) and len(merges) == 1
    succ = happens_before(ops)
    for f in range(n):
        assert ops[copies[f]]["slot"] == ops[kernels[f]]["slot"] == f % n_slots
        assert reaches(succ, copies[f], kernels[f]), f"kernel {f} may start before its copy has landed"
        if f >= n_slots:
            assert reaches(succ, kernels[f - n_slots], copies[f]), f"copy {f} may overwrite slot {f % n_slots} while kernel {f - n_slots} reads it"
        assert reaches(succ, kernels[f], merges[0])
        if not same_stream and f + 1 < n and n_slots >= 2:
            assert not reaches(succ, kernels[f], copies[f + 1]), f"copy {f + 1} waits for kernel {f}: no overlap"
    if n and not same_stream:
        # the in-place launch (issued first on compute) and all earlier compute work precede the first copy through the fence
        first_compute = next(i for i, op in enumerate(ops) if op["stream"] == 0)
        assert ops[first_compute]["kind"] == B.OP_RECORD and ops[first_compute]["event"] == 0
        assert reaches(succ, first_compute, copies[0])
    if same_stream:
        assert all(op["stream"] == 0 for op in ops) and not any(op["kind"] in (B.OP_RECORD, B.OP_WAIT) for op in ops)
    return n


@pytest.mark.parametrize("n_slots", [1, 2, 3, 16])
@pytest.mark.parametrize("same_stream", [False, True])
def test_slot_reuse_is_ordered_after_the_kernel_that_read_the_slot(n_slots, same_stream):
    h = B.ttkv_create()
    try:
        # 128K offload shape: 96 records of 1,179,648 B, 27 per copy (32 MiB) -> 4 copies
        c = offload_cache([98304])
        ops = B.ttkv_staged_schedule(h, c, n_slots=n_slots, same_stream=same_stream)
        assert check_chain(ops, n_slots, same_stream) == 4
        assert sum(op["bytes"] for op in ops if op["kind"] == B.OP_COPY) == 113246208
        # paged host tier (records scattered over the pool: hardly any merge) and a ragged batch: many copies, slots reused often
        c = offload_cache([5000, 300, 0, 12000], bt=256, batch=4, paged=True, seed=3)
        ops = B.ttkv_staged_schedule(h, c, n_slots=n_slots, same_stream=same_stream)
        n = check_chain(ops, n_slots, same_stream)
        assert 30 <= n <= 20 + 2 + 47
    finally:
        B.ttkv_destroy(h)


def test_selected_blocks_are_the_only_ones_copied():
    h = B.ttkv_create()
    try:
        c = offload_cache([98304 - 500])
        sel = np.array([[3, 4, 5, 40, 95]], np.int32)
        cnt = np.array([5], np.int32)
        ops = B.ttkv_staged_schedule(h, c, sel.ctypes.data, cnt.ctypes.data, 5, n_slots=2)
        check_chain(ops, 2, False)
        copies = [op for op in ops if op["kind"] == B.OP_COPY]
        # adjacent records 3, 4, 5 travel as one copy; the partly filled newest record is copied whole
        assert [op["bytes"] for op in copies] == [3 * 1179648, 1179648, 1179648]
    finally:
        B.ttkv_destroy(h)


def test_in_place_mode_issues_one_launch_and_no_copies():
    h = B.ttkv_create()
    try:
        c = offload_cache([98304])
        ops = B.ttkv_staged_schedule(h, c, n_slots=0)
        assert [op["kind"] for op in ops] == [B.OP_ATTEND, B.OP_MERGE] and ops[0]["fetch"] == -1
    finally:
        B.ttkv_destroy(h)


def test_a_planted_missing_wait_is_caught():
    """The checker itself: drop the wait on freed[slot] from a recorded schedule and the reuse check must fail."""
    h = B.ttkv_create()
    try:
        c = offload_cache([98304])
        ops = B.ttkv_staged_schedule(h, c, n_slots=2)
        check_chain(ops, 2, False)
        freed0 = 1 + B.TTKV_MAX_SLOTS
        broken = [op for op in ops if not (op["kind"] == B.OP_WAIT and op["event"] >= freed0)]
        assert len(broken) < len(ops)
        with pytest.raises(AssertionError, match="may overwrite"):
            check_chain(broken, 2, False)
    finally:
        B.ttkv_destroy(h)
