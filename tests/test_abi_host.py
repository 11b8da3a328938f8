"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header declares,
its integer helpers are exact, and argument validation rejects bad calls before anything is launched."""
import ctypes
import os
import re

import pytest

from oracle import layer_oracle as O
from paper_1909_08053_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "mlm_shard.h")).read()
    return sorted(set(re.findall(r"MLM_API\s+(?:int|const char\*)\s+(mlm_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 15 and set(names) == set(B.EXPORTS)
    L = B.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_shard_range_bit_exact_against_brute_force():
    for n, p in ((32, 8), (3072, 8), (12288, 8), (51200, 8), (30592, 4), (40, 4), (7, 1), (0, 3)):
        covered = []
        for r in range(p):
            b, e = B.mlm_shard_range(n, p, r)
            assert (b, e) == O.shard_range(n, p, r) if n else (b, e) == (0, 0)
            covered.extend(range(b, e))
        assert covered == list(range(n))
    for bad in ((10, 3, 0), (8, 2, 2), (8, 0, 0), (8, 2, -1), (-8, 2, 0)):
        with pytest.raises(B.MlmError) as ei:
            B.mlm_shard_range(*bad)
        assert ei.value.code == -2


def test_deferred_sums_list_is_per_thread_and_opens_and_closes_without_a_gpu():
    """begin / flush keep host-side state only: an empty list opens and closes without any launch."""
    import threading
    L = B.lib()
    fake = ctypes.c_void_p(0x10000)                      # never dereferenced on the host
    assert L.mlm_deferred_sums_flush(ctypes.c_void_p(0)) == -7          # nothing open
    assert L.mlm_deferred_sums_begin(ctypes.c_void_p(0), ctypes.c_size_t(1024)) == -1
    assert L.mlm_deferred_sums_begin(ctypes.c_void_p(0x10010), ctypes.c_size_t(1024)) == -5
    assert L.mlm_deferred_sums_begin(fake, ctypes.c_size_t(1024)) == 0
    assert L.mlm_deferred_sums_begin(fake, ctypes.c_size_t(1024)) == -7  # already open on this thread
    other = []
    t = threading.Thread(target=lambda: other.append((L.mlm_deferred_sums_begin(fake, ctypes.c_size_t(0)),
                                                      L.mlm_deferred_sums_flush(ctypes.c_void_p(0)))))
    t.start(); t.join()
    assert other == [(0, 0)]                             # another thread has its own list
    assert L.mlm_deferred_sums_flush(ctypes.c_void_p(0)) == 0
    assert L.mlm_deferred_sums_flush(ctypes.c_void_p(0)) == -7
    n = ctypes.c_size_t(0)
    d = B.make_dims(b=2, s=128, H=256, h=4, F=1024, V=1024, p=2, r=0, dtype=B.MLM_BF16)
    assert L.mlm_deferred_sums_bytes(ctypes.byref(d), ctypes.byref(n)) == 0
    ln = ((256 + 31) // 32) * 3 * 256 * 4
    assert n.value >= 4 * ln and n.value % 256 == 0
    assert L.mlm_deferred_sums_bytes(ctypes.byref(d), None) == -1


def _dims(**kw):
    base = dict(b=2, s=128, H=256, h=4, F=1024, V=1024, p=2, r=0, dtype=B.MLM_F32)
    base.update(kw)
    return B.make_dims(**base)


def test_validation_error_codes():
    L = B.lib()
    n = ctypes.c_size_t(0)
    call = lambda d, which=0: L.mlm_workspace_bytes(ctypes.byref(d), which, ctypes.byref(n))
    assert call(_dims()) == 0
    assert call(_dims(h=3)) == -2            # H % h
    assert call(_dims(p=3)) == -2            # h % p
    assert call(_dims(r=2)) == -2            # r outside [0,p)
    assert call(_dims(V=1023)) == -2         # V % p
    assert call(_dims(b=0)) == -2
    assert call(_dims(dtype=7)) == -3
    assert call(_dims(V=1028)) == -5         # V/p = 514 not a multiple of 8
    assert call(_dims(), 99) == -2
    assert L.mlm_workspace_bytes(None, 0, ctypes.byref(n)) == -1
    d = _dims()
    # NULL pointers are rejected before any launch
    assert L.mlm_layernorm_fwd(ctypes.byref(d), None, None, None, None, None, None, None) == -1
    assert L.mlm_gemm(1, 1, 1, ctypes.c_int64(64), ctypes.c_int64(64), ctypes.c_int64(64), ctypes.c_void_p(256),
                      ctypes.c_void_p(256), ctypes.c_void_p(256), None, None) == -7
    assert L.mlm_gemm(1, 0, 0, ctypes.c_int64(64), ctypes.c_int64(60), ctypes.c_int64(64), ctypes.c_void_p(256),
                      ctypes.c_void_p(256), ctypes.c_void_p(256), None, None) == -5
    assert L.mlm_gemm(1, 0, 0, ctypes.c_int64(64), ctypes.c_int64(64), ctypes.c_int64(64), ctypes.c_void_p(8),
                      ctypes.c_void_p(256), ctypes.c_void_p(256), None, None) == -5
    for code in range(0, -9, -1):
        assert B.status_string(code).startswith("MLM_")


def test_workspace_sizes_are_positive_and_aligned():
    d = _dims(b=8, s=1024, H=3072, h=32, F=12288, V=51200, p=8, dtype=B.MLM_BF16)
    for which in range(8):
        nbytes = B.mlm_workspace_bytes(d, which)
        assert nbytes % 256 == 0
    assert B.mlm_workspace_bytes(d, B.WS_VOCAB_CE_BWD) == 8192 * 6400 * 2 + 64 * 2 ** 20


def test_validation_of_fused_and_optimizer_entry_points():
    """Bad arguments of the fused layer-norm calls and of the optimizer calls are refused on the host, before any
    launch (no GPU is touched: the pointers below are never dereferenced)."""
    L = B.lib()
    d = _dims()
    P = ctypes.c_void_p
    ok = P(4096)                                   # an aligned, non-NULL address that is never used
    one = (P * 1)(4096)
    f = ctypes.c_float
    # fused combine + layer norm: NULL partial list, n out of range, NULL / misaligned partial
    assert L.mlm_combine_layernorm_fwd(ctypes.byref(d), None, 1, None, None, ok, ok, ok, ok, ok, ok, None) == -1
    assert L.mlm_combine_layernorm_fwd(ctypes.byref(d), one, 0, None, None, ok, ok, ok, ok, ok, ok, None) == -2
    assert L.mlm_combine_layernorm_fwd(ctypes.byref(d), one, 17, None, None, ok, ok, ok, ok, ok, ok, None) == -2
    assert L.mlm_combine_layernorm_fwd(ctypes.byref(d), (P * 1)(None), 1, None, None, ok, ok, ok, ok, ok, ok, None) == -1
    assert L.mlm_combine_layernorm_fwd(ctypes.byref(d), (P * 1)(4100), 1, None, None, ok, ok, ok, ok, ok, ok, None) == -5
    assert L.mlm_combine_layernorm_fwd(ctypes.byref(d), one, 1, None, None, None, ok, ok, ok, ok, ok, None) == -1
    # backward: a workspace that is too small
    assert L.mlm_combine_layernorm_bwd(ctypes.byref(d), one, 1, ok, ok, ok, ok, None, None, ok, ok, ok, None, ok,
                                       ctypes.c_size_t(16), None) == -4
    assert L.mlm_combine_layernorm_bwd(ctypes.byref(d), one, 1, ok, ok, ok, ok, None, None, None, ok, ok, None, ok,
                                       ctypes.c_size_t(1 << 30), None) == -1
    # optimizer
    cnt = (ctypes.c_int64 * 1)(64)
    assert L.mlm_grad_sqnorm(7, one, cnt, 1, None, ok, ok, ctypes.c_size_t(4096), None) == -3
    assert L.mlm_grad_sqnorm(0, one, cnt, 0, None, ok, ok, ctypes.c_size_t(4096), None) == -2
    assert L.mlm_grad_sqnorm(0, one, cnt, 1, None, ok, ok, ctypes.c_size_t(100), None) == -4
    assert L.mlm_grad_sqnorm(1, one, (ctypes.c_int64 * 1)(60), 1, None, ok, ok, ctypes.c_size_t(4096), None) == -5
    step = lambda count, st, clip, sq: L.mlm_adamw_step(0, ctypes.c_int64(count), ok, ok, ok, ok, None, sq, f(clip),
                                                        f(1e-3), f(0.9), f(0.999), f(1e-8), f(0.0), st, None)
    assert step(6, 1, 0.0, None) == -5             # count not a multiple of 4 (fp32)
    assert step(64, 0, 0.0, None) == -2            # step is 1-based
    assert step(64, 1, 1.0, None) == -1            # clipping asked for without a norm
    assert L.mlm_adamw_step(0, ctypes.c_int64(64), ok, ok, ok, ok, None, None, f(0.0), f(1e-3), f(1.0), f(0.999),
                            f(1e-8), f(0.0), 1, None) == -2          # beta1 must be < 1


def test_rng_stream_seeds_and_keep_words_are_exact():
    """Integer host helpers of the dropout entry points against the oracle's rule and a direct count."""
    from oracle import rng_embed_oracle as R
    for base in (0, 1, 7, 2 ** 32 - 1, 2 ** 32, 2 ** 63, 2 ** 64 - 9, 2 ** 64 - 1):
        for r in (0, 1, 7, 8, 511):
            assert B.mlm_rng_stream_seed(base, B.STREAM_REPLICATED, r) == R.stream_seed(base, R.STREAM_REPLICATED, r)
            assert B.mlm_rng_stream_seed(base, B.STREAM_MODEL_PARALLEL, r) == R.stream_seed(base, R.STREAM_MODEL_PARALLEL, r)
    for bad in ((5, 2, 0), (5, 1, -1)):
        with pytest.raises(B.MlmError) as ei:
            B.mlm_rng_stream_seed(*bad)
        assert ei.value.code == -2
    for b, s, h, p in ((2, 128, 4, 2), (3, 200, 4, 4), (1, 40, 2, 1), (8, 1024, 32, 8)):
        d = _dims(b=b, s=s, H=64 * h, h=h, F=256 * h, V=1024, p=p)
        pitch = 4 * -(-s // 128)                    # whole 16-byte groups of 32-key words per query row
        assert pitch * 32 >= s
        assert B.mlm_attn_keep_words(d) == b * (h // p) * s * pitch


def test_validation_of_dropout_embedding_and_row_entry_points():
    """Bad arguments are refused on the host before any launch (the addresses below are never dereferenced)."""
    L = B.lib()
    d = _dims()                                    # b=2, s=128: T = 256
    P = ctypes.c_void_p
    ok, odd = P(4096), P(4100)
    one = (P * 1)(4096)
    drop = lambda p: ctypes.byref(B.make_dropout(p, 1, 2))
    ref = ctypes.byref
    # probability outside [0, 1)
    assert L.mlm_combine_dropout(ref(d), one, 1, None, 1, drop(1.0), None, ok, None) == -2
    assert L.mlm_combine_dropout(ref(d), one, 1, None, 1, drop(-0.5), None, ok, None) == -2
    assert L.mlm_combine_dropout(ref(d), one, 1, ok, 0, None, None, ok, None) == -2          # bias rows < 1
    assert L.mlm_combine_dropout(ref(d), one, 1, ok, 257, None, None, ok, None) == -2        # more bias rows than tokens
    assert L.mlm_combine_dropout(ref(d), one, 1, None, 1, None, None, None, None) == -1
    assert L.mlm_combine_dropout(ref(d), one, 1, None, 1, None, None, odd, None) == -5
    # layer-norm backward with dropout needs somewhere to put dz, and not on top of dx
    big = ctypes.c_size_t(1 << 30)
    assert L.mlm_combine_layernorm_bwd_dropout(ref(d), one, 1, ok, ok, ok, ok, None, drop(0.1), None, ok, None, ok, ok,
                                               None, ok, big, None) == -1
    assert L.mlm_combine_layernorm_bwd_dropout(ref(d), one, 1, ok, ok, ok, ok, None, drop(0.1), None, ok, ok, ok, ok,
                                               None, ok, big, None) == -1
    # attention dropout: keep-bit buffer required, sequence length a multiple of 4
    args = lambda dd, dr, kb: L.mlm_attn_shard_fwd_dropout(ref(dd), ok, ok, None, ok, None, dr, ok, ok, ok, kb, ok, ok,
                                                           big, None)
    assert args(d, drop(0.1), None) == -1
    assert args(d, drop(0.1), odd) == -5
    assert args(_dims(s=126), drop(0.1), ok) == -5
    assert args(d, drop(1.5), ok) == -2
    # embedding and row gather / scatter
    assert L.mlm_embed_shard_fwd(ref(d), None, ok, ok, ok, None) == -1
    assert L.mlm_embed_shard_fwd(ref(d), ok, odd, ok, ok, None) == -5
    assert L.mlm_embed_bwd_replicated(ref(d), ok, None, None, None, None) == -1
    assert L.mlm_embed_bwd_replicated(ref(d), ok, drop(0.1), None, ok, None) == -1            # dropout needs dz0
    assert L.mlm_embed_shard_bwd(ref(d), ok, ok, ok, None, None) == -1
    assert L.mlm_rows_gather(ref(d), ok, ok, 300, 304, ok, None) == -2                        # more rows than tokens
    assert L.mlm_rows_gather(ref(d), ok, ok, 10, 8, ok, None) == -2                           # n_out < n
    assert L.mlm_rows_gather(ref(d), ok, None, 10, 16, ok, None) == -1
    assert L.mlm_rows_scatter(ref(d), ok, ok, -1, ok, None) == -2
    assert L.mlm_rows_scatter(ref(d), odd, ok, 4, ok, None) == -5


def test_bench_refuses_more_than_one_gpu():
    """This build has no collectives: bench.py must say so and exit non-zero for --gpus > 1 (before touching the GPU)."""
    import subprocess
    import sys as _sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([_sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)


def test_attention_tile_walk_stays_inside_the_buffers_for_any_key_length():
    """Host-side model of the streamed attention kernels' index arithmetic (forward / dQ: key tiles of 64 through a ring
    kept full by re-reading the last tile; dK/dV: query tiles): with the kernels' clamp max(1, min(key_len, s)) every
    tile index and every row index that a copy is issued for lies inside [0, s) -- for key_len = 0, negative, 1, s and
    beyond s alike.  (Without the lower clamp key_len = 0 gives nt = 0 and a first tile index of -1.)"""
    ATILE, BQ = 64, 128
    for s in (8, 64, 136, 200, 1024):
        for causal in (False, True):
            for given in (-3, 0, 1, s - 1, s, s + 1, 10 * s):
                klen = max(1, min(given, s))
                assert 1 <= klen <= s
                nqb = (s + BQ - 1) // BQ
                for qb in range(nqb):
                    q0 = qb * BQ
                    kv_end = min(klen, q0 + BQ) if causal else klen
                    nt = (kv_end + ATILE - 1) // ATILE
                    assert nt >= 1
                    for ng, nst in ((2, 3), (2, 2), (1, 3)):
                        njt = (nt + ng - 1) // ng
                        for grp in range(ng):
                            tiles = [min(ng * t + grp, nt - 1) for t in range(nst - 1)]
                            tiles += [min(ng * j + grp + ng * (nst - 1), nt - 1) for j in range(njt)]
                            for t in tiles:
                                assert 0 <= t < nt
                                for row in (0, ATILE - 1):
                                    r = min(t * ATILE + row, s - 1)
                                    assert 0 <= r < s
                # dK/dV: key blocks of 128, query tiles from the block's first tile (causal) or 0
                nqt = (s + ATILE - 1) // ATILE
                for kb in range((s + 127) // 128):
                    kb0 = kb * 128
                    qt0 = kb0 // ATILE if causal else 0
                    if kb0 >= klen:
                        qt0 = nqt
                    nt = nqt - qt0
                    assert nt >= 0
                    for t in range(nt + 2):
                        if nt > 0:
                            r0 = (qt0 + min(t, nt - 1)) * ATILE
                            assert 0 <= r0 < s and 0 <= min(r0 + 63, s - 1) < s


def test_gemm_lds_swizzles_are_permutations_and_conflict_free_for_both_mfma_shapes():
    """Host-side model of the bf16 GEMM's [k][rows] LDS layout (operands contiguous along m / n, read with the
    transposing 8-byte LDS read): the position function is a permutation of a k-row's 16-byte units with the chunk
    function as its inverse (so the copies, which permute on the global-address side, and the reads agree), every
    position stays inside the k-row, and a 32-lane pass of the fragment read touches no LDS bank twice -- for the
    16 x 16 x 32 MFMA's operand (lane group g holds k = 8 g .. 8 g + 7) and for the 32 x 32 x 16 one (half wave h
    holds k = 8 h .. of a 16-deep step), 256-row and 192-row tiles."""
    def swz256(k):
        return ((k & 3) << 2) | (((k >> 3) & 1) << 1)

    def rot192(k):
        return (((k >> 1) & 1) << 2) + (((k >> 3) & 1) << 1)

    def pos(rows, u, k):
        if rows == 256:
            return u ^ swz256(k)
        t = u + rot192(k)
        return t - rows // 8 if t >= rows // 8 else t

    def chunk(rows, p, k):
        if rows == 256:
            return p ^ swz256(k)
        t = p - rot192(k)
        return t + rows // 8 if t < 0 else t

    def worst(lanes):                              # lanes: (byte address, bytes); 64 banks of 4 bytes
        cnt = {}
        for addr, n in lanes:
            for i in range(n // 4):
                b = ((addr + 4 * i) // 4) % 64
                cnt[b] = cnt.get(b, 0) + 1
        return max(cnt.values())

    for rows in (256, 192):
        units = rows // 8
        for k in range(32):
            assert sorted(pos(rows, u, k) for u in range(units)) == list(range(units))
            assert all(chunk(rows, pos(rows, u, k), k) == u for u in range(units))
        # 16 x 16 x 32 operand: two reads r = 0, 1 per fragment
        for r0 in range(0, rows, 16):
            for r in (0, 1):
                for p in (0, 1):
                    lanes = []
                    for lane in range(32 * p, 32 * p + 32):
                        g, i16 = lane >> 4, lane & 15
                        u = (r0 >> 3) + ((i16 & 3) >> 1)
                        k = 8 * g + 4 * r + (i16 >> 2)
                        lanes.append((k * rows * 2 + pos(rows, u, k) * 16 + (i16 & 1) * 8, 8))
                    assert worst(lanes) == 1, (rows, r0, r, p)
        # 32 x 32 x 16 operand: 16-deep step ks, two reads per fragment
        for r0 in range(0, rows, 32):
            for ks in (0, 1):
                for r in (0, 1):
                    for p in (0, 1):
                        lanes = []
                        for lane in range(32 * p, 32 * p + 32):
                            g, i16 = lane >> 4, lane & 15
                            u = (r0 >> 3) + 2 * (g & 1) + ((i16 & 3) >> 1)
                            k = ks * 16 + 8 * (g >> 1) + 4 * r + (i16 >> 2)
                            lanes.append((k * rows * 2 + pos(rows, u, k) * 16 + (i16 & 1) * 8, 8))
                        assert worst(lanes) == 1, (rows, r0, ks, r, p)
