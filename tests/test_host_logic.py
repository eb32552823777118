"""CPU tests of the host-side logic behind the C ABI: the library loads without a
GPU and exports every declared symbol; argument validation; the caching allocator
over a fake backing store; the tape's reverse replay."""
import ctypes as C
import os
import re

import pytest

from paper_2201_12465_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(hdr):
    text = open(os.path.join(ROOT, "include", hdr)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(fl_[a-z0-9_]+)\s*\(", text))
    return {n for n in names if not n.endswith("_fn")}


def _exported(path):
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
    return {ln.split()[-1] for ln in out.splitlines() if ln.split()[-1].startswith("fl_")}


def test_library_exports_every_declared_symbol():
    """The product library exports exactly what include/fl_layer.h declares -- no test entry point, no
    kernel-selection override; the test build adds exactly what include/fl_test.h declares."""
    product, test = _declared("fl_layer.h"), _declared("fl_test.h")
    assert len(product) >= 19 and len(test) >= 25 and not (product & test)
    for n in sorted(product):
        assert hasattr(b.lib(), n), f"{n} is declared in include/fl_layer.h but not exported"
    for n in sorted(product | test):
        assert hasattr(b.test_lib(), n), f"{n} is declared in include/ but not exported by the test build"
    assert _exported(b.LIB_PATH) == product
    assert _exported(b.TEST_LIB_PATH) == product | test


def test_create_validates_arguments():
    def status(*a, **kw):
        try:
            b.Layer(*a, **kw).destroy()
            return b.FL_OK
        except b.FlError as e:
            assert str(e)
            return e.status
    assert status(2, 16, 64, 4, 256) == b.FL_OK
    assert status(0, 16, 64, 4, 256) == b.FL_ERR_INVALID_ARG
    assert status(2, 16, 64, 3, 256) == b.FL_ERR_INVALID_ARG       # D % heads
    assert status(2, 16, 60, 4, 256) == b.FL_ERR_UNSUPPORTED       # D % 8
    assert status(2, 16, 64, 8, 256) == b.FL_ERR_UNSUPPORTED       # head size 8
    assert status(2, 16, 64, 4, 250) == b.FL_ERR_UNSUPPORTED       # F % 8
    assert status(2, 16, 8192, 32, 256) == b.FL_ERR_UNSUPPORTED    # D too large
    lib = b.lib()
    assert lib.fl_layer_create(None, None) == b.FL_ERR_INVALID_ARG
    assert b"null" in lib.fl_last_error()
    assert lib.fl_layer_destroy(None) == b.FL_OK
    assert lib.fl_layer_forward(None, None, None, None, 1, 1, None, None) == b.FL_ERR_INVALID_ARG
    assert lib.fl_layer_backward(None, None, None, None, None, None) == b.FL_ERR_INVALID_ARG
    assert lib.fl_alloc_get_stats(None) == b.FL_ERR_INVALID_ARG


def test_forward_rejects_bad_arguments_before_touching_the_device():
    layer = b.Layer(2, 16, 64, 4, 256)
    fake = {n: 0x1000 for n in b.PARAM_FIELDS}
    with pytest.raises(b.FlError) as e:
        layer.forward(fake, 0x1000, None, 3, 16, 0x2000)            # B > max_B
    assert e.value.status == b.FL_ERR_INVALID_ARG
    with pytest.raises(b.FlError) as e:
        layer.forward(fake, 0x1004, None, 2, 16, 0x2000)            # misaligned X
    assert e.value.status == b.FL_ERR_UNSUPPORTED
    with pytest.raises(b.FlError) as e:
        layer.backward(fake, 0x1000, 0x2000, fake)                  # nothing recorded
    assert e.value.status == b.FL_ERR_STATE
    layer.destroy()


class FakeStore:
    """Stands in for the device allocator: hands out distinct fake addresses, can run dry."""

    def __init__(self, capacity=1 << 40):
        self.next, self.live, self.mallocs, self.frees, self.capacity = 1 << 32, {}, 0, 0, capacity

        def m(pp, n):
            if sum(self.live.values()) + n > self.capacity:
                return 1
            self.mallocs += 1
            pp[0] = self.next
            self.live[self.next] = n
            self.next += (n + 4095) // 4096 * 4096 + 4096
            return 0

        def f(p):
            self.frees += 1
            del self.live[p]
            return 0
        self.m, self.f = b.BACKING_MALLOC(m), b.BACKING_FREE(f)


@pytest.fixture
def alloc():
    lib = b.test_lib()
    store = FakeStore()
    a = lib.fl_test_alloc_create(store.m, store.f)

    def stats():
        s = b.fl_alloc_stats_t()
        lib.fl_test_alloc_stats(a, C.byref(s))
        return s.as_dict()
    yield lib, a, store, stats
    lib.fl_test_alloc_destroy(a)


MB = 1 << 20


def test_allocator_reuses_cached_blocks(alloc):
    lib, a, store, stats = alloc
    p1 = lib.fl_test_alloc_alloc(a, 5 * MB, None)
    p2 = lib.fl_test_alloc_alloc(a, 5 * MB, None)
    assert p1 and p2 and p1 != p2 and store.mallocs == 2
    assert stats()["live_bytes"] == 2 * 5 * MB
    assert lib.fl_test_alloc_release(a, p1) == 0
    assert lib.fl_test_alloc_release(a, p1) == 1               # double release is reported
    assert lib.fl_test_alloc_release(a, 12345) == 1            # unknown pointer
    p3 = lib.fl_test_alloc_alloc(a, 5 * MB, None)
    assert p3 == p1 and store.mallocs == 2                     # served from the cache
    s = stats()
    assert s["cache_hits"] == 1 and s["cache_misses"] == 2 and s["backing_mallocs"] == 2
    assert s["peak_bytes"] == 2 * 5 * MB
    for p in (p2, p3):
        lib.fl_test_alloc_release(a, p)
    # steady state: the same request sequence again needs no backing allocation
    for _ in range(3):
        ps = [lib.fl_test_alloc_alloc(a, n, None) for n in (5 * MB, 3 * MB, 5 * MB - 7)]
        for p in ps:
            lib.fl_test_alloc_release(a, p)
    assert store.mallocs == 3 and stats()["live_bytes"] == 0


def test_allocator_splits_and_merges(alloc):
    lib, a, store, stats = alloc
    big = lib.fl_test_alloc_alloc(a, 64 * MB, None)
    lib.fl_test_alloc_release(a, big)
    p1 = lib.fl_test_alloc_alloc(a, 10 * MB, None)              # split off the front of the cached 64 MiB
    p2 = lib.fl_test_alloc_alloc(a, 20 * MB, None)
    assert store.mallocs == 1 and p1 == big and p2 == big + 10 * MB
    assert stats()["split_count"] >= 2 and stats()["cached_bytes"] == 34 * MB
    lib.fl_test_alloc_release(a, p1)
    lib.fl_test_alloc_release(a, p2)                            # neighbours merge back into one block
    p3 = lib.fl_test_alloc_alloc(a, 64 * MB, None)
    assert p3 == big and store.mallocs == 1
    lib.fl_test_alloc_release(a, p3)
    # small requests share a 2 MiB slab; sizes are rounded to 512 bytes
    s1 = lib.fl_test_alloc_alloc(a, 100, None)
    s2 = lib.fl_test_alloc_alloc(a, 100, None)
    assert s2 - s1 == 512
    lib.fl_test_alloc_release(a, s1)
    lib.fl_test_alloc_release(a, s2)


def test_allocator_split_limit(alloc):
    lib, a, store, stats = alloc
    big = lib.fl_test_alloc_alloc(a, 64 * MB, None)
    lib.fl_test_alloc_release(a, big)
    lib.fl_test_alloc_set_split_limit(a, 32 * MB)               # cached 64 MiB block may no longer be split
    p = lib.fl_test_alloc_alloc(a, 10 * MB, None)
    assert p != big and store.mallocs == 2                      # a fresh slab instead of carving the big block
    q = lib.fl_test_alloc_alloc(a, 40 * MB, None)               # wastes < half: takes the big block whole
    assert q == big and stats()["live_bytes"] == 10 * MB + 64 * MB
    lib.fl_test_alloc_release(a, p)
    lib.fl_test_alloc_release(a, q)
    lib.fl_test_alloc_set_split_limit(a, 0)
    r = lib.fl_test_alloc_alloc(a, 1 * MB + 512, None)
    assert store.mallocs == 2                                   # splitting allowed again
    lib.fl_test_alloc_release(a, r)


def test_allocator_streams_do_not_share_cached_blocks(alloc):
    lib, a, store, stats = alloc
    p = lib.fl_test_alloc_alloc(a, 8 * MB, 0x10)
    lib.fl_test_alloc_release(a, p)
    q = lib.fl_test_alloc_alloc(a, 8 * MB, 0x20)                # other stream: kernels on 0x10 may still use p
    assert q != p and store.mallocs == 2
    r = lib.fl_test_alloc_alloc(a, 8 * MB, 0x10)
    assert r == p and store.mallocs == 2
    lib.fl_test_alloc_release(a, q)
    lib.fl_test_alloc_release(a, r)


def test_allocator_trim_and_out_of_memory():
    lib = b.test_lib()
    store = FakeStore(capacity=100 * MB)
    a = lib.fl_test_alloc_create(store.m, store.f)
    p = lib.fl_test_alloc_alloc(a, 60 * MB, None)
    assert p
    assert not lib.fl_test_alloc_alloc(a, 60 * MB, None)        # store exhausted -> NULL, allocator stays usable
    lib.fl_test_alloc_release(a, p)
    q = lib.fl_test_alloc_alloc(a, 70 * MB, None)               # cached 60 MiB slab is given back, then retried
    assert q and store.frees == 1
    lib.fl_test_alloc_release(a, q)
    lib.fl_test_alloc_trim(a)
    assert store.live == {} and store.frees == 2
    s = b.fl_alloc_stats_t()
    lib.fl_test_alloc_stats(a, C.byref(s))
    assert s.backing_bytes == 0 and s.cached_bytes == 0 and s.live_bytes == 0
    lib.fl_test_alloc_destroy(a)


def test_allocator_fragmentation_figures(alloc):
    lib, a, store, stats = alloc
    p = lib.fl_test_alloc_alloc(a, 5 * MB + 1, None)            # rounded up to 512 bytes, slab to 2 MiB
    s = stats()
    assert s["requested_bytes"] == 5 * MB + 1 and s["live_bytes"] == 5 * MB + 512
    assert s["free_blocks"] == 1 and s["largest_free_block"] == MB - 512 == s["cached_bytes"]
    q = lib.fl_test_alloc_alloc(a, 3 * MB, None)                # does not fit the rest: a 4 MiB slab of its own
    lib.fl_test_alloc_release(a, p)                             # merges with the rest of its slab
    s = stats()
    assert s["requested_bytes"] == 3 * MB and s["live_bytes"] == 3 * MB
    assert s["free_blocks"] == 2 and s["largest_free_block"] == 6 * MB and s["cached_bytes"] == 7 * MB
    lib.fl_test_alloc_release(a, q)
    s = stats()
    assert s["requested_bytes"] == 0 and s["free_blocks"] == 2 and s["largest_free_block"] == 6 * MB
    assert s["cached_bytes"] == 10 * MB == s["backing_bytes"]


def test_allocator_trace_ties_operators_to_allocations(alloc):
    lib, a, store, stats = alloc

    def read(cap=64):
        ev = (b.fl_alloc_event_t * cap)()
        return b.events_as_dicts(ev, lib.fl_test_alloc_trace_read(a, ev, cap))

    x = lib.fl_test_alloc_alloc_tagged(a, 4 * MB, None, (3 << 8) | 1)
    assert read() == []                                          # nothing is recorded while the trace is off
    lib.fl_test_alloc_trace_enable(a, 8)
    y = lib.fl_test_alloc_alloc_tagged(a, 6 * MB - 100, None, (5 << 8) | 4)
    lib.fl_test_alloc_release(a, x)
    z = lib.fl_test_alloc_alloc_tagged(a, 4 * MB, None, (7 << 8) | 6)
    ev = read()
    assert [e["kind"] for e in ev] == ["from_device", "release", "from_cache"]
    assert [(e["op"], e["node"]) for e in ev] == [("linear_bwd", 5), ("linear_fwd", 3), ("layernorm_bwd", 7)]
    assert ev[0]["ptr"] == y and ev[0]["requested"] == 6 * MB - 100 and ev[0]["granted"] == 6 * MB
    assert ev[1]["ptr"] == x and ev[1]["requested"] == 0 and ev[1]["granted"] == 4 * MB
    assert ev[2]["ptr"] == z == x                                # the released block serves the next operator
    assert [e["seq"] for e in ev] == [0, 1, 2]
    assert read() == []                                          # reading drains the ring
    # the ring keeps the newest `capacity` events
    ps = [lib.fl_test_alloc_alloc_tagged(a, 1 * MB, None, i << 8) for i in range(12)]
    ev = read()
    assert len(ev) == 8 and [e["node"] for e in ev] == list(range(4, 12))
    assert [e["seq"] for e in ev] == list(range(7, 15))
    lib.fl_test_alloc_trace_enable(a, 0)
    for p in ps + [y, z]:
        lib.fl_test_alloc_release(a, p)
    assert read() == []


def _replay_requests(lib, a, store, requests):
    """requests: ('a', key, bytes) / ('r', key).  Returns bytes obtained from the backing store."""
    live = {}
    for r in requests:
        if r[0] == "a":
            live[r[1]] = lib.fl_test_alloc_alloc(a, r[2], None)
            assert live[r[1]]
        else:
            assert lib.fl_test_alloc_release(a, live.pop(r[1])) == 0
    for p in live.values():
        lib.fl_test_alloc_release(a, p)
    return sum(store.live.values())


def test_split_limit_reduces_fragmentation_on_mixed_sizes():
    """Section 5.2.2's finding on a request stream with its cause in it: a large activation buffer is
    freed, long-lived small buffers are then carved out of it, and the next iteration's large request
    no longer fits the carved block, so the device is asked for more memory.  With a split limit the
    large block stays whole and the total taken from the device is smaller."""
    lib = b.test_lib()
    seq = []
    for it in range(4):
        seq.append(("a", ("big", it), 96 * MB))
        seq.append(("r", ("big", it)))
        for j in range(3):                                        # small buffers that outlive the iteration
            seq.append(("a", ("small", it, j), 3 * MB))
    taken = {}
    for limit in (0, 32 * MB):
        store = FakeStore()
        a = lib.fl_test_alloc_create(store.m, store.f)
        lib.fl_test_alloc_set_split_limit(a, limit)
        taken[limit] = _replay_requests(lib, a, store, seq)
        s = b.fl_alloc_stats_t()
        lib.fl_test_alloc_stats(a, C.byref(s))
        assert s.live_bytes == 0 and s.cached_bytes == taken[limit]
        lib.fl_test_alloc_destroy(a)
    assert taken[0] == 2 * 96 * MB                               # the carved slab forces a second large one
    assert taken[32 * MB] == 96 * MB + 12 * 4 * MB               # one large slab, a 4 MiB slab per small buffer


def _replay(in0, in1, n_inputs, fail_at=-1):
    lib = b.test_lib()
    n = len(in0)
    arr = lambda v: (C.c_int32 * len(v))(*v)
    order, ran = (C.c_int32 * n)(), C.c_int32(0)
    nslots = n_inputs + n
    fc = (C.c_int32 * nslots)()
    rc = lib.fl_test_tape_replay(n, arr(in0), arr(in1), n_inputs, fail_at, order, C.byref(ran), fc, nslots)
    return rc, list(order)[:ran.value], list(fc)


def test_tape_replays_in_reverse_and_tracks_first_consumers():
    # the post-LN layer's graph: slot 0 = X; nodes: qkv(0) attn(1) out-proj(2; residual X) ln1(3)
    # ffn1(4) ffn2(5; residual = ln1's output) ln2(6); node i writes slot 1+i
    in0 = [0, 1, 2, 3, 4, 5, 6]
    in1 = [-1, -1, 0, -1, -1, 4, -1]
    rc, order, fc = _replay(in0, in1, 1)
    assert rc == 0 and order == [6, 5, 4, 3, 2, 1, 0]
    assert fc[0] == 0          # X: first consumed by the QKV projection, which therefore finishes dX
    assert fc[4] == 4          # ln1's output: first consumed by ffn1, not by ffn2's residual
    assert fc[7] == -1         # the layer output has no consumer


def test_tape_stops_at_a_failing_gradient_function():
    rc, order, _ = _replay([0, 1, 2, 3], [-1, -1, -1, -1], 1, fail_at=1)
    assert rc == 77 and order == [3, 2]
    rc, order, _ = _replay([], [], 1)
    assert rc == 0 and order == []
    rc, _, _ = _replay([5], [-1], 1)       # reads a slot that does not exist
    assert rc == -1


def test_profile_summary_classifies_kernel_names():
    from paper_2201_12465_amd.profile_summary import classify
    cases = {
        "_ZN2fl12_GLOBAL__N_111gemm_kernelIDF16bLb0ELb0ELi2EEEvNS_7GemmDevE": "gemm_tn",
        "_ZN2fl12_GLOBAL__N_111gemm_kernelIDF16bLb1ELb0ELi1EEEvNS_7GemmDevE": "gemm_nn",
        "_ZN2fl12_GLOBAL__N_111gemm_kernelIfLb1ELb1ELi2EEEvNS_7GemmDevE": "gemm_nt",
        "void fl::(anonymous namespace)::gemm_kernel<bool _Accum, bool, E, false, 1>(fl::GemmDev)": "gemm_nn",
        "void fl::(anonymous namespace)::gemm_kernel<float, false, false, 2>(fl::GemmDev)": "gemm_tn",
        "void fl::(anonymous namespace)::gemm_kernel<bool _Accum, bool, E, false, 1, false>(fl::GemmDev)": "gemm_nn",
        "void fl::(anonymous namespace)::gemm_kernel<float, true, true, 2, true>(fl::GemmDev)": "gemm_nt",
        "_ZN2fl12_GLOBAL__N_111gemm_kernelIDF16bLb1ELb0ELi1ELb0EEEvNS_7GemmDevE": "gemm_nn",
        "_ZN2fl12_GLOBAL__N_111gemm_kernelIDF16bLb0ELb0ELi2ELb0EEEvNS_7GemmDevE": "gemm_tn",
        "void fl::(anonymous namespace)::gemm_bf16_pipe<true, true, 256, 192, 2, 4, 2, false, 1>(fl::GemmDev)": "gemm_nt",
        "void fl::(anonymous namespace)::gemm_bf16_pipe<true, true, 128, 128, 2>(fl::GemmDev)": "gemm_nt",
        "_ZN2fl12_GLOBAL__N_122reduce_partials_kernelIDF16bEEvPKfimmPT_S5_S5_": "splitk_reduce",
        "_ZN2fl12_GLOBAL__N_127reduce_partials_tall_kernelIDF16bEEvPKfimmPT_S5_S5_": "splitk_reduce",
        "_ZN2fl12_GLOBAL__N_117attn_bwd_dkv_mfmaILi64EEEvPKDF16bS3_PKfS5_PKiiifPDF16b": "attn_bwd",
        "void fl::(anonymous namespace)::attn_fwd_mfma<64>(bool _Accum const*, int const, int)": "attn_fwd",
        "_ZN2fl12_GLOBAL__N_113ln_bwd_kernelIDF16bLi2EEEvPKT_S4_PKfS6_S4_S4_iiiPS2_Pf": "ln_bwd",
        "_ZN2fl12_GLOBAL__N_113ln_fwd_kernelIDF16bLi2EEEvPKT_S4_S4_fiiPS2_PfS6_": "ln_fwd",
        "_ZN2fl12_GLOBAL__N_120colsum_stage1_kernelIDF16bEEvPKT_iiPf": "colsum",
        "fl::(anonymous namespace)::copy_kernel(HIP_vector_type<unsigned int, 4u> const*, ...)": "copy",
        "void fl::(anonymous namespace)::gemm_f32_small<true, false, false>(fl::GemmDev)": "gemm_nn",
        "void fl::(anonymous namespace)::gemm_f32_small<false, false, true>(fl::GemmDev)": "gemm_tn",
        "_ZN2fl12_GLOBAL__N_114gemm_f32_smallILb1ELb1ELb0EEEvNS_7GemmDevE": "gemm_nt",
        "void fl::(anonymous namespace)::attn_bwd_dq_mfma_f32<64, false, false>(float const*, float const*)": "attn_bwd",
        "fl::(anonymous namespace)::transpose_tiles_kernel(fl::(anonymous namespace)::TransposeJobs)": "wt_transpose",
        "_ZN2fl12_GLOBAL__N_115attn_delta_rowsIDF16bEEvPKT_S4_iiiiPf": "attn_bwd",
    }
    for name, cls in cases.items():
        assert classify(name) == cls, name


def test_kernel_selection_rules():
    """The host-side rules that pick a kernel for a problem, on the shapes they were measured on: a change
    of a rule shows up here before it shows up as a slower benchmark."""
    from paper_2201_12465_amd import binding as b
    lib = b.test_lib()
    D, F = 768, 3072
    nt = lambda M, N, K: lib.fl_test_gemm_variant(1, 1, M, N, K)
    # BERT-base-shaped layer (M = 4096): the widest output fills the chip in one round of 256x192 tiles; the
    # fused projection (576 tiles of 128x128 for 512 places) runs 468 tiles of 160x128 in one round; narrow
    # outputs (at most one 128x128 tile per CU) run three stages and two k-groups of wavefronts per tile
    assert [nt(4096, 3 * D, D), nt(4096, D, D), nt(4096, F, D), nt(4096, D, F), nt(4096, D, 3 * D)] == [10, 9, 7, 9, 9]
    # ViT-shaped stack (M = 12608): 3.1 rounds of 256x192 tiles are not worth it; N = 768 has 594 tiles of
    # 128x128 for 512 places and runs 474 tiles of 160x128 in one round
    assert [nt(12608, 3 * D, D), nt(12608, D, D), nt(12608, F, D), nt(12608, D, F)] == [0, 10, 0, 10]
    # speech-shaped layer (M = 8000): two full rounds are; the 378 tiles of an N = 768 output become 504 tiles of
    # 96x128 in the forward pass, where nothing else would use the places they leave empty
    assert nt(8000, F, D) == 7 and nt(8000, D, F) == 0
    fwd = lib.fl_test_gemm_variant_forward
    assert [fwd(8000, D, F), fwd(8000, D, D), fwd(8000, F, D), fwd(8000, 3 * D, D)] == [11, 11, 7, 0]
    assert [fwd(4096, 3 * D, D), fwd(4096, D, D), fwd(4096, F, D), fwd(12608, D, F)] == [10, 9, 7, 10]
    # operands that are not contiguous along k (dy W without transposed weights, dy^T x): 128x128 tiles, 2 stages,
    # or the 160x128 tiles where they turn one round and a bit into one
    assert lib.fl_test_gemm_variant(1, 0, 12608, F, D) == 0 and lib.fl_test_gemm_variant(0, 0, D, F, 4096) == 0
    assert [lib.fl_test_gemm_variant(1, 0, 12608, D, k) for k in (F, D, 3 * D)] == [10, 10, 10]
    assert lib.fl_test_gemm_variant(1, 0, 8000, D, F) == 0 and lib.fl_test_gemm_variant(0, 0, D, 12608, 4096) == 0
    # weight gradients of the BERT-base layer: about 430 workgroups
    splits = lambda M, N, K: lib.fl_test_gemm_splits(b.FL_BF16, M, N, K)
    assert [splits(D, F, 4096), splits(F, D, 4096), splits(D, D, 4096), splits(3 * D, D, 4096)] == [3, 3, 6, 4]
    # fp32: few-tile outputs run on 32x32 tiles and do not split k below 4096
    assert lib.fl_test_gemm_f32_small(1024, 1024) == 1 and lib.fl_test_gemm_f32_small(4096, 3072) == 0
    assert lib.fl_test_gemm_splits(b.FL_F32, 256, 1024, 1024) == 1 and lib.fl_test_gemm_splits(b.FL_F32, 256, 1024, 8192) == 2
    # attention: every head size the layer accepts has matrix-core kernels, except fp32 above 128
    for dh in range(16, 257, 16):
        assert lib.fl_test_attention_path(b.FL_BF16, dh) == 1
        assert lib.fl_test_attention_path(b.FL_F32, dh) == (2 if dh <= 128 else 0)
    assert lib.fl_test_attention_path(b.FL_BF16, 24) == 0 and lib.fl_test_attention_path(b.FL_F32, 8) == 0

