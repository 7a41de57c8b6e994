"""CPU-only checks: the shared library loads, exports every symbol the headers
declare, and its host-side logic (KV allocator, pass planner, configuration
checks) behaves.  No GPU call is made."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2505_24298_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    return binding.lib()


@pytest.fixture(scope="module")
def HL():
    """Host-only entry points: from the main library, or from the sanitizer build when
    AREAL_HOST_LIB names it (test_host_logic_under_sanitizers runs this file that way)."""
    return binding.host_lib()


def _declared():
    names = set()
    for h in ("areal.h", "areal_host.h", "areal_ops.h"):
        src = open(os.path.join(ROOT, "include", h)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(areal_[a-z0-9_]+)\s*\(", src))
    return names


def test_every_declared_symbol_is_exported_and_bound(L):
    decl = _declared()
    assert {"areal_load_weights", "areal_prefill", "areal_decode_step",
            "areal_update_weights_interrupt", "areal_sample_logprob"} <= decl
    for n in decl:
        assert hasattr(L, n), n
    assert decl == set(binding._SIGNATURES)


def test_cfg_struct_matches_header_layout():
    # field order and widths as in areal_model_cfg
    assert [f[0] for f in binding.ModelCfg._fields_][:7] == [
        "n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab"]
    assert C.sizeof(binding.ModelCfg) == 13 * 4 + 4 + 5 * 8     # 13 words, pad, 5 x 8 bytes


def test_workspace_and_block_bytes(L):
    cfg = binding.make_cfg(synth.shape("qwen2-1.5b"), 256, 8704, 8192, convert_weights=False)
    assert L.areal_kv_block_bytes(C.byref(cfg)) == 16 * 28672
    ws = L.areal_workspace_bytes(C.byref(cfg))
    assert 2 ** 20 < ws < 2 ** 31
    # space for a converted half-precision copy of a bf16 / float32 parameter set
    cfg_c = binding.make_cfg(synth.shape("qwen2-1.5b"), 256, 8704, 8192, convert_weights=True)
    extra = L.areal_workspace_bytes(C.byref(cfg_c)) - ws
    n_params = 1_543_656_960 + 151936 * 1536 + 28 * 1536      # + embedding, + second norm gain
    assert 2 * n_params <= extra <= 2 * n_params + 2 ** 20
    cfg7 = binding.make_cfg(synth.shape("qwen2-7b"), 64, 33792 + 16, 4096)
    assert L.areal_kv_block_bytes(C.byref(cfg7)) == 16 * 57344
    bad = binding.make_cfg(synth.shape("tiny", head_dim=48), 8, 128, 64)
    assert L.areal_workspace_bytes(C.byref(bad)) == 0
    bad = binding.make_cfg(synth.shape("tiny"), 8, 128, 4)        # fewer rows than sequences
    assert L.areal_workspace_bytes(C.byref(bad)) == 0


def test_create_rejects_bad_buffers_without_touching_the_gpu(L):
    cfg = binding.make_cfg(synth.shape("tiny"), 8, 128, 64)
    ctx = C.c_void_p()
    assert L.areal_create(C.byref(cfg), C.byref(ctx)) == binding.E_NOMEM     # no workspace
    assert b"workspace" in L.areal_last_error(None)
    assert L.areal_create(None, C.byref(ctx)) == binding.E_INVAL


# ------------------------------------------------------------- KV allocator
def _table(L, a, seq):
    buf = np.zeros(64, dtype=np.int32)
    n = L.areal_kvalloc_table(a, seq, buf.ctypes.data_as(binding._I32P), 64)
    return buf[:n].tolist()


def test_allocator_grows_on_block_boundaries_and_reuses(HL):
    L = HL
    a = L.areal_kvalloc_create(10, 4, 8)
    assert L.areal_kvalloc_free_blocks(a) == 10
    assert L.areal_kvalloc_reserve(a, 0, 16) == 0 and _table(L, a, 0) == [0]
    assert L.areal_kvalloc_reserve(a, 0, 16) == 0 and _table(L, a, 0) == [0]       # no growth
    assert L.areal_kvalloc_reserve(a, 0, 17) == 0 and _table(L, a, 0) == [0, 1]
    assert L.areal_kvalloc_reserve(a, 1, 40) == 0 and _table(L, a, 1) == [2, 3, 4]
    assert L.areal_kvalloc_free_blocks(a) == 5
    L.areal_kvalloc_release(a, 0)
    assert L.areal_kvalloc_free_blocks(a) == 7 and _table(L, a, 0) == []
    assert L.areal_kvalloc_reserve(a, 2, 33) == 0
    t2 = _table(L, a, 2)
    assert len(t2) == 3 and not set(t2) & set(_table(L, a, 1))
    L.areal_kvalloc_destroy(a)


def test_allocator_exhaustion_is_all_or_nothing(HL):
    L = HL
    a = L.areal_kvalloc_create(4, 2, 3)
    assert L.areal_kvalloc_reserve(a, 0, 3 * 16) == 0
    assert L.areal_kvalloc_reserve(a, 1, 2 * 16) == binding.E_NOMEM      # pool: 1 left, 2 needed
    assert _table(L, a, 1) == [] and L.areal_kvalloc_free_blocks(a) == 1
    assert L.areal_kvalloc_reserve(a, 0, 3 * 16 + 1) == binding.E_NOMEM  # per-sequence limit
    assert len(_table(L, a, 0)) == 3
    L.areal_kvalloc_destroy(a)


def test_allocator_never_leaks_or_double_books(HL):
    L = HL
    rng = np.random.default_rng(0)
    a = L.areal_kvalloc_create(200, 16, 40)
    L.areal_kvalloc_shuffle(a, 7)
    lens = [0] * 16
    for step in range(3000):
        s = int(rng.integers(0, 16))
        if lens[s] and rng.random() < 0.05:
            L.areal_kvalloc_release(a, s)
            lens[s] = 0
        else:
            want = lens[s] + int(rng.integers(1, 40))
            if L.areal_kvalloc_reserve(a, s, want) == 0:
                lens[s] = want
        tabs = [_table(L, a, q) for q in range(16)]
        flat = [b for t in tabs for b in t]
        assert len(flat) == len(set(flat))
        assert all(len(t) == -(-n // 16) for t, n in zip(tabs, lens))
        assert L.areal_kvalloc_free_blocks(a) == 200 - len(flat)
    for s in range(16):
        L.areal_kvalloc_release(a, s)
    assert L.areal_kvalloc_free_blocks(a) == 200
    L.areal_kvalloc_destroy(a)


# ------------------------------------------------------------- pass planner
def _plan(L, lens, max_rows):
    lens = np.asarray(lens, dtype=np.int32)
    out = np.zeros((1024, 6), dtype=np.int32)
    n = L.areal_plan_passes(len(lens), lens.ctypes.data_as(binding._I32P), max_rows,
                            out.ctypes.data_as(binding._I32P), 1024)
    return out[:n]

def test_planner_covers_every_position_once_in_order(HL):
    L = HL
    rng = np.random.default_rng(1)
    for trial in range(20):
        lens = rng.integers(1, 90, size=int(rng.integers(1, 12)))
        max_rows = int(rng.integers(8, 64))
        rec = _plan(L, lens, max_rows)
        rows_in_pass = {}
        nxt = [0] * len(lens)
        for p, span, pos0, ln, row0, out_index in rec:
            assert pos0 == nxt[span] and ln > 0
            nxt[span] += ln
            assert row0 == rows_in_pass.get(p, 0)
            rows_in_pass[p] = row0 + ln
            assert out_index == (span if nxt[span] == lens[span] else -1)
        assert nxt == lens.tolist()
        assert all(v <= max_rows for v in rows_in_pass.values())
        assert all(v == max_rows for k, v in rows_in_pass.items() if k != max(rows_in_pass))
        assert list(rec[:, 0]) == sorted(rec[:, 0]) and list(rec[:, 1]) == sorted(rec[:, 1])


def test_bench_refuses_more_than_one_gpu():
    """Every box has one GPU: bench.py --gpus N with N > 1 exits with a message
    before it touches the device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one MI355X" in r.stderr and r.stdout.strip() == ""


def test_host_logic_under_sanitizers():
    """The allocator, planner, gate and batching tests of this file once more, in a child
    process, against csrc/host_api.cpp built with -fsanitize=address,undefined (any report
    aborts the child)."""
    import subprocess
    import sys
    from paper_2505_24298_amd import build as b
    if os.environ.get("AREAL_HOST_LIB"):
        pytest.skip("already inside the sanitizer run")
    lib, runtimes = b.build_host_sanitized()
    assert runtimes, "sanitizer runtimes not found next to the host compiler"
    env = dict(os.environ, AREAL_HOST_LIB=lib, LD_PRELOAD=":".join(runtimes),
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.abspath(__file__), "-q", "-x", "-p", "no:cacheprovider",
                        "-k", "allocator or planner or gate or kvalloc or dynamic_batching or stream"],
                       capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert " passed" in r.stdout and "failed" not in r.stdout


def test_staleness_gate_matches_oracle_request_by_request():
    """The library's gate (budget form) against the oracle that applies the
    paper's inequality one request at a time, over random interleavings of
    submissions and version bumps, for every small (B, eta)."""
    from oracle import staleness
    L = binding.host_lib()
    rng = np.random.default_rng(3)
    for B in (1, 2, 5, 16):
        for eta in (0, 1, 4):
            g = L.areal_gate_create(B, eta)
            o = staleness.StalenessGate(B, eta)
            v = 0
            for _ in range(200):
                if rng.random() < 0.3:
                    v += int(rng.integers(0, 3))
                    assert L.areal_gate_set_version(g, v) == 0
                    o.set_version(v)
                n = int(rng.integers(0, 3 * B))
                assert L.areal_gate_budget(g) == _budget(o)
                assert L.areal_gate_submit(g, n) == o.submit(n)
                assert L.areal_gate_submitted(g) == o.submitted
            assert L.areal_gate_set_version(g, v - 1) == binding.E_STATE if v > 0 else True
            L.areal_gate_destroy(g)
    assert not L.areal_gate_create(0, 1) and not L.areal_gate_create(4, -1)


def _budget(o):
    """How many requests the oracle gate would admit now (on a copy)."""
    from oracle import staleness
    c = staleness.StalenessGate(o.B, o.eta, o.version)
    c.submitted = o.submitted
    return c.submit(10 ** 6)


def test_kvalloc_shared_prefix_refcounts():
    L = binding.host_lib()
    a = L.areal_kvalloc_create(10, 4, 8)
    assert L.areal_kvalloc_reserve(a, 0, 40) == 0 and _table(L, a, 0) == [0, 1, 2]
    assert L.areal_kvalloc_share(a, 1, 0, 2) == 0 and _table(L, a, 1) == [0, 1]
    assert L.areal_kvalloc_share(a, 2, 0, 2) == 0
    assert L.areal_kvalloc_share(a, 1, 0, 1) == binding.E_INVAL          # holder is not empty
    assert L.areal_kvalloc_share(a, 3, 0, 4) == binding.E_INVAL          # more than the source holds
    assert L.areal_kvalloc_reserve(a, 1, 40) == 0 and _table(L, a, 1) == [0, 1, 3]   # own third block
    assert L.areal_kvalloc_free_blocks(a) == 6
    L.areal_kvalloc_release(a, 0)                                        # the first holder leaves:
    assert L.areal_kvalloc_free_blocks(a) == 7                           # only its own block 2 returns
    L.areal_kvalloc_release(a, 1)
    assert L.areal_kvalloc_free_blocks(a) == 8                           # block 3; 0 and 1 still held by 2
    L.areal_kvalloc_release(a, 2)
    assert L.areal_kvalloc_free_blocks(a) == 10
    assert L.areal_kvalloc_reserve(a, 3, 160) == binding.E_NOMEM         # per-sequence limit 8 blocks
    assert L.areal_kvalloc_reserve(a, 3, 128) == 0 and len(set(_table(L, a, 3))) == 8
    L.areal_kvalloc_destroy(a)


def test_dynamic_batching_matches_oracle():
    """Algorithm 1 in the library against the oracle on random length sets
    (ties in length and in sequence count included) and on the edge cases."""
    from oracle import trainer_side
    L = binding.host_lib()
    rng = np.random.default_rng(11)
    for _ in range(200):
        n = int(rng.integers(0, 60))
        lens = rng.integers(1, 30, size=n).astype(np.int32)
        cap, k = int(rng.integers(10, 90)), int(rng.integers(1, 7))
        out = np.full(n, -1, dtype=np.int32)
        nb = L.areal_dynamic_batching(n, lens.ctypes.data_as(binding._I32P), cap, k,
                                      out.ctypes.data_as(binding._I32P))
        want = trainer_side.dynamic_batching(lens, cap, k)
        assert nb == len(want)
        for b, members in enumerate(want):
            assert sorted(np.nonzero(out == b)[0].tolist()) == sorted(members)
    bad = np.array([3, 0], dtype=np.int32)
    o = np.zeros(2, dtype=np.int32)
    assert L.areal_dynamic_batching(2, bad.ctypes.data_as(binding._I32P), 10, 1,
                                    o.ctypes.data_as(binding._I32P)) == binding.E_INVAL
    assert L.areal_dynamic_batching(2, bad.ctypes.data_as(binding._I32P), 0, 1,
                                    o.ctypes.data_as(binding._I32P)) == binding.E_INVAL


# ------------------------------------------------- streaming controller (host logic)
class _FakeTensor:
    def __getitem__(self, k):
        return self

    def contiguous(self):
        return self

    def to(self, d):
        return self


class _FakeTorch:
    """Just enough of torch for harness.streaming_rollout to run without a GPU."""
    float32, int32 = "f32", "i32"

    class cuda:
        class Event:
            def __init__(self, enable_timing=True):
                pass

            def record(self):
                pass

            def elapsed_time(self, other):
                return 1.0

        @staticmethod
        def synchronize():
            pass

    @staticmethod
    def empty(shape, dtype=None, device=None):
        return _FakeTensor()

    @staticmethod
    def empty_like(a):
        return a

    @staticmethod
    def from_numpy(a):
        return _FakeTensor()


class _FakeEngine:
    device = "cpu"

    def __init__(self):
        self.live = set()

    def prefill(self, ids, prompts, logits_out=None):
        assert not self.live & set(int(i) for i in ids)
        self.live.update(int(i) for i in ids)

    def sample_logprob(self, *a, **k):
        pass

    def decode_step(self, ids, *a, **k):
        assert set(int(i) for i in ids) <= self.live

    def free_seq(self, i):
        self.live.remove(int(i))

    def update_weights_interrupt(self, w, version, logits_out=None):
        return np.array(sorted(self.live), dtype=np.int32), None, 0


@pytest.mark.parametrize("eta", [0, 1, 2, 3, 5])
def test_streaming_controller_follows_the_oracle_event_loop(eta):
    """The refill loop of the streaming regime (slots, staleness gate through the C entry
    points, one weight update per finished training batch) with the GPU calls stubbed out:
    the same number of ticks as the oracle's plain event loop and every request submitted and
    completed under the versions that loop gives it (Section 5.1)."""
    from oracle import staleness
    from paper_2505_24298_amd import harness
    n_total, slots, B = 48, 8, 8
    for seed in range(6):
        outs = synth.output_lengths(n_total, 12, 1.0, 60, seed=seed)
        prompts = [np.zeros(3, dtype=np.int32)] * n_total
        eng = _FakeEngine()
        r = harness.streaming_rollout(eng, _FakeTorch, dict(vocab=16), binding.host_lib(), prompts, outs, slots, B,
                                      eta, [0, 1], 1.0, 1.0, 0)
        ticks, done = staleness.simulate_stream(n_total, B, eta, slots, outs)
        assert r["ticks"] == ticks and sorted(r["records"]) == sorted(done)
        assert r["gen_tokens"] == int(outs.sum()) and not eng.live


def test_tile_choice_for_the_decoder_shapes(L):
    """areal_op_gemm_choose (host only): the tile configuration and K split the library takes for
    the products of the 1.5B and 7B shapes, at the row counts where the rules change.  Pins the
    rules that were read off sweeps on the MI355X, so that an edit of one does not silently
    move another: configuration numbers as in gemm.hip's dispatch."""
    import ctypes as C

    def choose(M, N, K, mode):
        c, s = C.c_int32(), C.c_int32()
        assert L.areal_op_gemm_choose(M, N, K, mode, C.byref(c), C.byref(s)) == 0
        return c.value, s.value

    STORE, ADD, SWIGLU = 0, 1, 2
    H, F, V = 1536, 8960, 151936
    # prefill passes of 8,192 rows: 256 x 256 tiles; the down projection with its last round evened out
    assert choose(8192, 2048, H, STORE) == (19, 1)
    assert choose(8192, F, H, SWIGLU) == (19, 1)
    assert choose(8192, H, F, ADD) == (24, 1)
    assert choose(8192, 3584, 18944, ADD) == (24, 1)
    assert choose(8192, H, H, ADD)[0] == 20
    # decode steps: gate/up by row count, no K split (the SwiGLU epilogue needs whole sums)
    assert [choose(M, F, H, SWIGLU) for M in (24, 48, 100, 200)] == [(12, 1), (10, 1), (21, 1), (20, 1)]
    # narrow products split K; the down projection at few rows takes 64-column tiles
    assert choose(24, H, F, ADD) == (25, 8)
    assert choose(100, H, F, ADD) == (23, 8)
    for M in (8, 64, 256):
        cfg, splits = choose(M, 2048, H, STORE)
        assert cfg in (21, 22, 23) and 1 < splits <= 12
    # output projection: one work-group per column panel, never split
    assert [choose(M, V, H, STORE)[1] for M in (1, 100, 256)] == [1, 1, 1]
    # a ragged K (not a multiple of 64) falls back to the register-staged tiles
    assert choose(100, 1000, 344, STORE)[0] in (0, 2, 4)
    # invalid shapes are refused
    c, s = C.c_int32(), C.c_int32()
    assert L.areal_op_gemm_choose(0, 8, 8, 0, C.byref(c), C.byref(s)) != 0
    assert L.areal_op_gemm_choose(8, 8, 8, 3, C.byref(c), C.byref(s)) != 0
