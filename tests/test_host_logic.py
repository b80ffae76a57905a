"""CPU tests of the library's host side: exported symbols of the C boundary and the page allocator."""
import ctypes as C
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_17891_amd", "csrc")


def test_library_exports_every_declared_symbol():
    from paper_2510_17891_amd import binding
    L = binding.lib()                       # loads without a GPU; no compute call is made here
    header = open(os.path.join(ROOT, "include", "rl.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(rl_[a-z_0-9]+)\s*\(", header)))
    assert len(declared) >= 18
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(binding.EXPORTS) == declared
    assert L.rl_last_error() is not None


def test_config_validation_needs_no_gpu():
    from paper_2510_17891_amd import binding as B
    import rollout_inputs as ri
    L = B.lib()
    need = C.c_uint64()
    cfg = B.make_config(ri.SHAPES["full8b"], B.RL_BF16, 256, 16384, 256)
    assert L.rl_query_workspace(C.byref(cfg), C.byref(need)) == B.RL_OK
    assert 100e6 < need.value < 2e9
    assert L.rl_kv_page_bytes(C.byref(cfg)) == 36 * 2 * 8 * 16 * 128 * 2      # 147456 B per token
    bad = B.make_config(dict(ri.SHAPES["full8b"], head_dim=64), B.RL_BF16, 4, 64, 4)
    assert L.rl_query_workspace(C.byref(bad), C.byref(need)) == B.RL_ERR_UNSUPPORTED
    assert b"head_dim" in L.rl_last_error()
    bad = B.make_config(ri.SHAPES["tiny"], B.RL_F32, 4, 60, 4)                 # max_ctx not a multiple of 16
    assert L.rl_query_workspace(C.byref(bad), C.byref(need)) == B.RL_ERR_INVALID_ARG
    bad = B.make_config(ri.SHAPES["tiny"], B.RL_F32, 4, 64, 1025)              # max_rows beyond 1024
    assert L.rl_query_workspace(C.byref(bad), C.byref(need)) == B.RL_ERR_INVALID_ARG
    cfg = B.make_config(ri.SHAPES["tiny"], B.RL_F32, 4, 64, 4)
    cfg.struct_size = 8
    assert L.rl_query_workspace(C.byref(cfg), C.byref(need)) == B.RL_ERR_INVALID_ARG
    assert L.rl_init_model(None, None, None) == B.RL_ERR_INVALID_ARG


@pytest.fixture(scope="module")
def st(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("st") / "libseqtable.so")
    subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-fsanitize=undefined", "-fno-sanitize-recover",
                    "-o", out, os.path.join(CSRC, "seq_table_capi.cpp")], check=True)
    L = C.CDLL(out)
    L.st_create.restype = C.c_void_p
    L.st_create.argtypes = [C.c_int, C.c_int, C.c_longlong]
    L.st_free_pages.restype = C.c_longlong
    for f in ("st_destroy", "st_free_pages"):
        getattr(L, f).argtypes = [C.c_void_p]
    for f in ("st_active", "st_len", "st_activate", "st_release", "st_n_seq_pages"):
        getattr(L, f).argtypes = [C.c_void_p, C.c_int]
    for f in ("st_pages_missing", "st_set_len", "st_seq_page"):
        getattr(L, f).argtypes = [C.c_void_p, C.c_int, C.c_int]
    L.st_share_prefix.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int]
    L.st_refcount.argtypes = [C.c_void_p, C.c_int]
    L.st_shuffle.argtypes = [C.c_void_p, C.c_ulonglong]
    L.st_reserve.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_int), C.c_int]
    L.st_prefix_id.restype = C.c_longlong
    L.st_prefix_id.argtypes = [C.c_void_p, C.c_int]
    L.st_prefix_blocks.argtypes = [C.c_void_p, C.c_int]
    L.st_plan_shared.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.c_int,
                                 C.POINTER(C.c_int), C.POINTER(C.c_int), C.c_int]
    return L


def _reserve(L, t, s, tokens):
    buf = (C.c_int * 3000)()
    n = L.st_reserve(t, s, tokens, buf, 1000)
    return [(buf[3 * i], buf[3 * i + 1], buf[3 * i + 2]) for i in range(n)]


def test_page_allocator_growth_free_reuse(st):
    t = st.st_create(4, 64, 6)
    assert st.st_free_pages(t) == 6 and not st.st_active(t, 0)
    assert st.st_pages_missing(t, 0, 17) == 2
    st.st_activate(t, 0)
    g = _reserve(st, t, 0, 17)
    assert [(s, b) for s, b, _ in g] == [(0, 0), (0, 1)] and st.st_free_pages(t) == 4
    st.st_set_len(t, 0, 17)
    assert st.st_pages_missing(t, 0, 32) == 0 and st.st_pages_missing(t, 0, 33) == 1
    assert _reserve(st, t, 0, 32) == []                       # ragged growth: no page until the boundary
    g2 = _reserve(st, t, 0, 33)
    assert len(g2) == 1 and g2[0][1] == 2
    st.st_activate(t, 1)
    g3 = _reserve(st, t, 1, 48)
    assert st.st_free_pages(t) == 0
    pages = [p for _, _, p in g + g2 + g3]
    assert sorted(pages) == list(range(6))                    # every page handed out exactly once
    assert st.st_pages_missing(t, 2, 1) == 1                  # an inactive sequence needs all its pages
    st.st_release(t, 0)
    assert st.st_free_pages(t) == 3 and not st.st_active(t, 0) and st.st_len(t, 0) == -1
    st.st_activate(t, 2)
    g4 = _reserve(st, t, 2, 40)
    assert sorted(p for _, _, p in g4) == sorted(p for _, _, p in g + g2)   # freed pages are reused
    assert st.st_n_seq_pages(t, 2) == 3 and st.st_seq_page(t, 2, 0) == g4[0][2]
    st.st_destroy(t)


def test_page_allocator_shuffle_is_a_permutation(st):
    t = st.st_create(2, 16 * 100, 100)
    st.st_shuffle(t, 42)
    st.st_activate(t, 0)
    g = _reserve(st, t, 0, 1600)
    pages = [p for _, _, p in g]
    assert sorted(pages) == list(range(100)) and pages != list(range(100))
    st.st_destroy(t)


def test_page_sharing_reference_counts(st):
    t = st.st_create(4, 64, 8)
    st.st_activate(t, 0)
    g = _reserve(st, t, 0, 40)                                # 3 pages, the last one partial
    pages = [p for _, _, p in g]
    for s in (1, 2):
        st.st_activate(t, s)
        st.st_share_prefix(t, s, 0, 2)                        # share the two full pages
        own = _reserve(st, t, s, 40)                          # private copy target for the partial page
        assert len(own) == 1 and own[0][1] == 2 and own[0][2] not in pages
        assert [st.st_seq_page(t, s, i) for i in range(2)] == pages[:2]
    assert st.st_refcount(t, pages[0]) == 3 and st.st_refcount(t, pages[2]) == 1
    assert st.st_free_pages(t) == 8 - 5
    st.st_release(t, 0)                                       # shared pages survive their first holder
    assert st.st_free_pages(t) == 8 - 4 and st.st_refcount(t, pages[0]) == 2
    st.st_release(t, 1)
    assert st.st_free_pages(t) == 8 - 3
    st.st_release(t, 2)
    assert st.st_free_pages(t) == 8 and st.st_refcount(t, pages[0]) == 0
    st.st_destroy(t)


def test_lockstep_growth_keeps_sequences_physically_contiguous(st):
    """Eight sequences growing one page at a time in turn: each still gets consecutive pages inside its own run,
    the pool is used completely before anything fails, and frees/reuse keep the accounting exact."""
    n_pages, n_seq = 8 * 32 + 5, 8
    t = st.st_create(n_seq, 16 * 64, n_pages)
    for s in range(n_seq):
        st.st_activate(t, s)
    for blk in range(1, 33):
        for s in range(n_seq):
            g = _reserve(st, t, s, 16 * blk)
            assert len(g) == 1
    for s in range(n_seq):
        pages = [st.st_seq_page(t, s, i) for i in range(32)]
        assert pages == list(range(pages[0], pages[0] + 32)) and pages[0] % 32 == 0
    assert st.st_free_pages(t) == 5
    got = _reserve(st, t, 0, 16 * 37)                        # the odd pages at the end are still usable
    assert sorted(p for _, _, p in got) == list(range(256, 261)) and st.st_free_pages(t) == 0
    st.st_release(t, 3)
    assert st.st_free_pages(t) == 32
    st.st_activate(t, 3)
    g = _reserve(st, t, 3, 16 * 32)
    assert len({p for _, _, p in g}) == 32 and st.st_free_pages(t) == 0
    all_pages = [st.st_seq_page(t, s, i) for s in range(n_seq) for i in range(st.st_n_seq_pages(t, s))]
    assert sorted(all_pages) == list(range(n_pages))         # nothing handed out twice
    for _ in range(6):                                       # churn: stale stack entries never surface
        st.st_release(t, 3)
        st.st_activate(t, 3)
        g = _reserve(st, t, 3, 16 * 32)
        assert len({p for _, _, p in g}) == 32 and st.st_free_pages(t) == 0
    st.st_destroy(t)


def _plan(L, t, seqs, pos, rows_per_set):
    n = len(seqs)
    skip = (C.c_int * n)()
    sets = (C.c_int * (10 * n))()                  # per set: rows[8], n_rows, n_segs
    k = L.st_plan_shared(t, n, (C.c_int * n)(*seqs), (C.c_int * n)(*pos), rows_per_set, skip, sets, n)
    for i in range(k):                             # the unused row slots repeat the first row
        assert all(sets[10 * i + e] == sets[10 * i] for e in range(sets[10 * i + 8], 8))
    return list(skip), [(list(sets[10 * i:10 * i + sets[10 * i + 8]]), sets[10 * i + 9]) for i in range(k)]


def test_attention_segments_partition_every_context(st):
    """The segment bounds are monotone, start at 0, end at the number of 32-key steps, and there are
    4*ceil(ctx/1024) of them: every key of a context belongs to exactly one segment."""
    for ctx in list(range(1, 200)) + [1023, 1024, 1025, 4095, 4096, 4097, 16383, 16384, 65536]:
        n = st.st_attn_num_segments(ctx)
        assert n == 4 * ((ctx + 1023) // 1024)
        b = [st.st_attn_seg_begin(c, ctx) for c in range(n + 1)]
        assert b[0] == 0 and b[-1] == (ctx + 31) // 32 and all(x <= y for x, y in zip(b, b[1:]))


def test_shared_attention_plan(st):
    """Sets hold rows of one sharing family at one position; the covered segments end inside the common pages;
    a left-over single row, rows at other positions and sequences that share nothing stay on their own."""
    t = st.st_create(16, 4096, 2000)
    for s in range(12):
        st.st_activate(t, s)
    _reserve(st, t, 0, 1100)                       # leader of family A: 68 full pages
    for s in range(1, 7):
        st.st_share_prefix(t, s, 0, 68)
    _reserve(st, t, 7, 300)                        # family B: 18 full pages
    st.st_share_prefix(t, 8, 7, 18)
    _reserve(st, t, 9, 1100)                       # shares nothing
    assert st.st_prefix_id(t, 0) == st.st_prefix_id(t, 6) != 0 and st.st_prefix_blocks(t, 3) == 68
    assert st.st_prefix_id(t, 7) == st.st_prefix_id(t, 8) not in (0, st.st_prefix_id(t, 0))
    assert st.st_prefix_id(t, 9) == 0

    def covered(ctx, shared_keys):                # brute force over the printed bounds
        n = st.st_attn_num_segments(ctx)
        k = 0
        while k < n and st.st_attn_seg_begin(k + 1, ctx) * 32 <= shared_keys:
            k += 1
        return k

    seqs = [0, 9, 1, 2, 7, 3, 8, 4, 5, 6]
    pos = [1150, 1150, 1150, 1150, 320, 1150, 320, 1151, 1150, 1150]
    skip, sets = _plan(st, t, seqs, pos, 4)
    sA, sB = covered(1151, 68 * 16), covered(321, 18 * 16)
    assert sA >= 6 and sB >= 2
    # family A at position 1150: rows 0,2,3,5,8,9 -> a set of four and a set of two; row 7 stands elsewhere
    assert sets == [([0, 2, 3, 5], sA), ([8, 9], sA), ([4, 6], sB)]
    assert skip == [sA, 0, sA, sA, sB, sA, sB, 0, sA, sA]
    # five rows with sets of four: the fifth computes everything itself
    skip, sets = _plan(st, t, [0, 1, 2, 3, 4], [1150] * 5, 4)
    assert sets == [([0, 1, 2, 3], sA)] and skip == [sA] * 4 + [0]
    # sets of eight (two 16-column operands at four query heads per kv head): all seven rows of the family in one set
    skip, sets = _plan(st, t, [0, 1, 2, 3, 4, 5, 6], [1150] * 7, 8)
    assert sets == [([0, 1, 2, 3, 4, 5, 6], sA)] and skip == [sA] * 7
    # ... which the model asks for only with bf16 pages and at least 1024 (row, kv head) pairs in the call
    assert [st.st_attn_rows_per_set(g, 0, 128, 8) for g in (1, 2, 4, 8)] == [8, 8, 8, 4]
    assert [st.st_attn_rows_per_set(g, 1, 128, 8) for g in (1, 2, 4, 8)] == [4, 4, 4, 2]
    assert [st.st_attn_rows_per_set(4, 0, n, 8) for n in (1, 32, 64, 127, 128, 256)] == [4, 4, 4, 4, 8, 8]
    # right after the prompt the last shared page may hold the row's own position: never shared
    skip, sets = _plan(st, t, [0, 1], [1088, 1088], 2)
    assert sets and sets[0][1] == covered(1089, 1088) and st.st_attn_seg_begin(sets[0][1], 1089) * 32 <= 1088
    # a sequence that is freed and reused forgets its family
    st.st_release(t, 8)
    st.st_activate(t, 8)
    assert st.st_prefix_id(t, 8) == 0
    st.st_destroy(t)


def test_window_sets_of_prefill_rows(st):
    """Rows of one sequence at neighbouring positions form sets only inside one aligned window of 32 positions (same
    step count and segments), up to the given size, never across sequences or gaps; a set lists its highest position
    first and covers every segment of its rows; single rows stay on their own."""
    st.st_plan_windows.argtypes = [C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.c_int, C.POINTER(C.c_int),
                                   C.POINTER(C.c_int), C.c_int]

    def plan(seq, pos, per_set):
        n = len(seq)
        skip = (C.c_int * n)()
        sets = (C.c_int * (10 * n))()
        k = st.st_plan_windows(n, (C.c_int * n)(*seq), (C.c_int * n)(*pos), per_set, skip, sets, n)
        # per set: rows[8], n_rows, n_segs; returned as (the four first rows, n_rows, n_segs, all eight rows)
        return list(skip), [tuple(sets[10 * i:10 * i + 4]) + (sets[10 * i + 8], sets[10 * i + 9], tuple(sets[10 * i:10 * i + 8]))
                            for i in range(k)]

    # one sequence, positions 28..37: the window boundary at 32 cuts the sets; sets of four
    seq, pos = [5] * 10, list(range(28, 38))
    skip, sets = plan(seq, pos, 4)
    members = [sorted(set(s[:4])) for s in sets]
    assert members == [[0, 1, 2, 3], [4, 5, 6, 7], [8, 9]]
    assert all(s[0] == max(s[:4]) for s in sets)                       # the longest context leads
    assert [s[4] for s in sets] == [4, 4, 2]
    for s in sets:
        ctx = pos[s[0]] + 1
        assert s[5] == st.st_attn_num_segments(ctx) and all(skip[r] == s[5] for r in set(s[:4]))
        assert len({(pos[r] >> 5) for r in set(s[:4])}) == 1
    # two sequences back to back, a position gap, a single left-over row, sets of two
    seq = [1, 1, 1, 2, 2, 2, 2, 2]
    pos = [0, 1, 2, 40, 41, 50, 51, 52]
    skip, sets = plan(seq, pos, 2)
    assert [sorted(set(s[:4])) for s in sets] == [[0, 1], [3, 4], [5, 6]]
    assert skip[2] == 0 and skip[7] == 0
    # a context just past 1024 keys has more segments than the one before it, but they are in different windows
    seq, pos = [0] * 4, [1022, 1023, 1024, 1025]
    skip, sets = plan(seq, pos, 4)
    assert [sorted(set(s[:4])) for s in sets] == [[0, 1], [2, 3]] and [s[5] for s in sets] == [4, 8]
    # sets of eight: a whole window of 32 positions gives four sets, each led by its highest position
    seq, pos = [3] * 32, list(range(64, 96))
    skip, sets = plan(seq, pos, 8)
    assert [s[4] for s in sets] == [8, 8, 8, 8]
    assert [list(s[6]) for s in sets] == [list(range(b + 7, b - 1, -1)) for b in (0, 8, 16, 24)]


def test_weight_k_block_order_is_a_permutation_that_interleaves_four_segments(st):
    """Order of the k blocks of a packed weight row block: for every (number of k blocks, segment length) the 8B shape
    uses and a few others, the slots are a permutation, the four segments of a K split are interleaved block by
    block (what four waves read at the same moment is adjacent), and splits follow one another."""
    for n_kb, seg in [(64, 4), (64, 16), (192, 12), (192, 48), (8, 1), (8, 2), (16, 4), (48, 3)]:
        assert n_kb % (4 * seg) == 0
        slots = [st.st_weight_kb_slot(kb, seg) for kb in range(n_kb)]
        assert sorted(slots) == list(range(n_kb)), (n_kb, seg)
        for kb in range(n_kb):
            s, i = divmod(kb, seg)                 # segment (wave range) and block inside it
            split, wave = divmod(s, 4)
            assert slots[kb] == (split * seg + i) * 4 + wave
        # the blocks that the four waves of a split read at step i are one run of four slots
        for split in range(n_kb // (4 * seg)):
            for i in range(seg):
                run = [slots[(4 * split + w) * seg + i] for w in range(4)]
                assert run == list(range(run[0], run[0] + 4)) and run[0] % 4 == 0


def test_group_page_need_matches_the_allocator(st):
    """The rollout loop admits a group when the pool can hold it up to its length limits; its estimate must equal what
    the allocator really hands out when the group is prefilled (shared full pages, one partial-page copy per member)
    and every member is decoded to its limit."""
    from paper_2510_17891_amd.rollout_loop import group_page_need
    for P, limits in [(37, [1, 5, 30]), (32, [1, 1, 1]), (5, [12, 11, 28, 1]), (48, [17, 16, 1, 33]), (1, [16, 17])]:
        G = len(limits)
        t = st.st_create(G, 4096, 1000)
        st.st_activate(t, 0)
        _reserve(st, t, 0, P)
        st.st_set_len(t, 0, P)
        for j in range(1, G):
            st.st_activate(t, j)
            st.st_share_prefix(t, j, 0, P // 16)
            if P % 16:
                _reserve(st, t, j, P)
            st.st_set_len(t, j, P)
        peak = 1000 - st.st_free_pages(t)
        # a member that has sampled `new` tokens has been fed new - 1 of them
        for j, new in enumerate(limits):
            for k in range(new - 1):
                _reserve(st, t, j, P + k + 1)
                st.st_set_len(t, j, P + k + 1)
        peak = max(peak, 1000 - st.st_free_pages(t))
        assert peak == group_page_need(P, limits), (P, limits)
        for j in range(G):
            st.st_release(t, j)
        assert st.st_free_pages(t) == 1000
        st.st_destroy(t)


def test_bench_refuses_more_than_one_gpu():
    """The measurement script covers one GPU; any other count ends with a message and a non-zero status before
    anything touches a device."""
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for extra_env, argv in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "2"}, [])):
        env = dict(os.environ, **extra_env)
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), *argv], capture_output=True, text=True,
                           env=env, timeout=120)
        assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_binding_fails_loudly_without_the_library():
    """No fallback: when the shared library is not there, the first call through the binding raises and names the
    build command."""
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import paper_2510_17891_amd.binding as b\n"
            "b.LIB_PATH = '/nonexistent/librl_rollout.so'\n"
            "b._lib = None\n"
            "try:\n"
            "    b.lib()\n"
            "except RuntimeError as e:\n"
            "    print('raised:', e)\n")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=root, timeout=120)
    assert r.returncode == 0 and "raised:" in r.stdout and "paper_2510_17891_amd.build" in r.stdout
