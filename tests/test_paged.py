"""Paged and strided tensors: splitzip_compress_paged / splitzip_decompress_paged against the oracle on the
gathered tensor (GPU), and the argument rules of the page description (CPU)."""
import ctypes as C

import numpy as np
import pytest
import torch

import kv_synth
import oracle
import paper_2605_01708_amd as sz
from paper_2605_01708_amd.binding import _CPaged

DT = {sz.BF16: oracle.BF16, sz.FP8_E5M2: oracle.E5M2}
GEN = {sz.BF16: kv_synth.kv_bf16, sz.FP8_E5M2: kv_synth.kv_e5m2}


def test_page_descriptions_are_checked():
    L = sz.lib()
    cb = sz.calibrate(kv_synth.kv_bf16(8, 1), sz.BF16)
    buf = 1 << 12

    def desc(**k):
        return _CPaged(k.get("pool", buf), k.get("table", buf), k.get("n_blocks", 4), k.get("n_pool", 8),
                       k.get("block_elems", 2048), 0, k.get("stride", 8192), k.get("offset", 0))

    def comp(d, n=5000):
        return L.splitzip_compress_paged(C.byref(d), n, sz.BF16, C.byref(cb.c), buf, 1 << 20, buf, 1 << 20, buf, None)

    def decomp(d, n=5000):
        return L.splitzip_decompress_paged(buf, 1 << 20, n, sz.BF16, C.byref(cb.c), C.byref(d), None, None)

    for f in (comp, decomp):
        assert f(desc(pool=None)) == -1
        assert f(desc(table=None)) == -1
        assert f(desc(pool=buf + 8)) == -1                  # pool not 16-byte aligned
        assert f(desc(table=buf + 2)) == -1
        assert f(desc(block_elems=1000)) == -1              # not a power of two
        assert f(desc(block_elems=512)) == -1               # below the chunk
        assert f(desc(stride=4096 + 8)) == -1               # not a multiple of 16
        assert f(desc(offset=8)) == -1
        assert f(desc(stride=4080)) == -1                   # a page does not hold block_elems words
        assert f(desc(offset=4112)) == -1                   # ... behind the offset
        assert f(desc(n_blocks=2)) == -1                    # the table does not cover the tensor
        assert f(desc(n_pool=0)) == -1
        assert f(desc(), n=1 << 32) == -1                   # (the table cannot cover it)
    # the batch forms: the same geometry rules (the pool of the description is not looked at), every item must fit the table
    from paper_2605_01708_amd.binding import _CItem, _CDItem
    items = (_CItem * 2)(_CItem(buf, 5000, buf, 1 << 20, C.pointer(cb.c)), _CItem(buf, 9000, buf, 1 << 20, C.pointer(cb.c)))
    ditems = (_CDItem * 1)(_CDItem(buf, 1 << 20, 9000, buf, C.pointer(cb.c)))
    for bad in (desc(table=None), desc(block_elems=1000), desc(stride=4080), desc(n_pool=0), desc()):   # desc(): 4 x 2048 < 9000
        assert L.splitzip_compress_batch_paged(items, 2, sz.BF16, C.byref(bad), buf, 1 << 24, buf, None) == -1
        assert L.splitzip_decompress_batch_paged(ditems, 1, sz.BF16, C.byref(bad), None, None) == -1
    assert L.splitzip_compress_batch_paged(items, 2, sz.BF16, None, buf, 1 << 24, buf, None) == -1
    assert L.splitzip_compress_batch_paged(items, 0, sz.BF16, C.byref(desc(pool=None)), buf, 1 << 24, buf, None) == 0
    assert L.splitzip_compress_paged(None, 10, sz.BF16, C.byref(cb.c), buf, 1 << 20, buf, 1 << 20, buf, None) == -1
    assert L.splitzip_decompress_paged(buf, 1 << 20, 10, 7, C.byref(cb.c), C.byref(desc()), None, None) == -1


def paged_case(dtype, n, block_elems, stride_extra, offset, seed):
    """a pool of shuffled pages holding an n-element tensor; returns (pool tensor, table tensor, logical words, page stride)"""
    es = 2 if dtype == sz.BF16 else 1
    tokens = -(-n // 1024)
    x = kv_synth.to_numpy_words(GEN[dtype](tokens, seed))[:n].copy()
    n_blocks = max(1, -(-n // block_elems))
    n_pool = n_blocks + 5
    stride = offset + block_elems * es + stride_extra
    rng = np.random.default_rng(seed)
    table = rng.permutation(n_pool)[:n_blocks].astype(np.int32)
    pool = np.full(n_pool * stride, 0xEE, np.uint8)
    xb = x.view(np.uint8)
    for b in range(n_blocks):
        chunk = xb[b * block_elems * es:(b + 1) * block_elems * es]
        at = int(table[b]) * stride + offset
        pool[at:at + chunk.size] = chunk
    return pool, table, x, stride, n_pool


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [sz.BF16, sz.FP8_E5M2])
def test_paged_pool_round_trip_matches_the_oracle_on_the_gathered_tensor(dtype):
    assert torch.cuda.is_available()
    es = 2 if dtype == sz.BF16 else 1
    cb_or = oracle.calibrate(kv_synth.to_numpy_words(GEN[dtype](1024, 1)), DT[dtype])
    cb = sz.codebook_from_dec(cb_or.dec.tolist(), dtype)
    cases = [(16 * 16384, 16384, 0, 0), (300_000, 16384, 4096, 32768),      # whole pages; a ragged last page, offset, gap
             (5 * 1024 + 77, 1024, 512, 0), (1, 2048, 0, 16), (0, 1024, 0, 0),  # one token per page: a strided tensor
             (2_500_000, 65536, 0, 131072)]
    for k, (n, be, extra, off) in enumerate(cases):
        print(f"case paged: dtype={dtype} n={n} block_elems={be} stride_extra={extra} offset={off}", flush=True)
        pool_np, table_np, x, stride, n_pool = paged_case(dtype, n, be, extra, off, 20 + k)
        pool = torch.from_numpy(pool_np).cuda()
        table = torch.from_numpy(table_np).cuda()
        src = sz.Paged(pool, table, be, stride, off, n_pool)
        ref, m_ref = oracle.compress(x, cb_or)
        out = torch.full((sz.compress_bound(max(n, 1), dtype) + 4096,), 0xA5, dtype=torch.uint8, device="cuda")
        ws = sz.Workspace(max(n, 1), dtype)
        sizes = sz.new_sizes()
        sz.compress_paged(src, n, cb, out, ws, sizes)
        torch.cuda.synchronize()
        assert sz.read_sizes(sizes) == (ref.size, m_ref, 0)
        assert np.array_equal(out[:ref.size].cpu().numpy(), ref), "paged stream differs from the oracle's"
        assert (out[ref.size:ref.size + 4096].cpu().numpy() == 0xA5).all()
        assert np.array_equal(pool.cpu().numpy(), pool_np), "compress wrote into the pool"
        # decompress into a fresh pool with another page order: the tensor's words land, nothing else changes
        rng = np.random.default_rng(99 + k)
        table2_np = rng.permutation(n_pool)[:table_np.size].astype(np.int32)
        pool2 = torch.full((pool_np.size,), 0x77, dtype=torch.uint8, device="cuda")
        dst = sz.Paged(pool2, torch.from_numpy(table2_np).cuda(), be, stride, off, n_pool)
        st = sz.new_sizes()
        sz.decompress_paged(out, ref.size, n, cb, dst, st)
        torch.cuda.synchronize()
        assert sz.read_sizes(st) == (ref.size, m_ref, 0)
        want = np.full(pool_np.size, 0x77, np.uint8)
        xb = x.view(np.uint8)
        for b in range(table2_np.size):
            piece = xb[b * be * es:(b + 1) * be * es]
            at = int(table2_np[b]) * stride + off
            want[at:at + piece.size] = piece
        got = pool2.cpu().numpy()
        assert np.array_equal(got, want), f"paged decompress: {np.flatnonzero(got != want)[:8]}"


@pytest.mark.gpu
def test_table_entries_outside_the_pool_are_clamped():
    """a bad page index reads the last page instead of memory outside the pool (the stream is then that of the clamped table)"""
    n, be = 4 * 2048, 2048
    pool_np, table_np, x, stride, n_pool = paged_case(sz.BF16, n, be, 0, 0, 31)
    bad = table_np.copy()
    bad[2] = 1_000_000
    cb_or = oracle.calibrate(kv_synth.to_numpy_words(kv_synth.kv_bf16(1024, 1)), oracle.BF16)
    cb = sz.codebook_from_dec(cb_or.dec.tolist(), sz.BF16)
    pool = torch.from_numpy(pool_np).cuda()
    src = sz.Paged(pool, torch.from_numpy(bad).cuda(), be, stride, 0, n_pool)
    out = torch.empty(sz.compress_bound(n, sz.BF16), dtype=torch.uint8, device="cuda")
    sizes = sz.new_sizes()
    sz.compress_paged(src, n, cb, out, sz.Workspace(n, sz.BF16), sizes)
    torch.cuda.synchronize()
    total, m, status = sz.read_sizes(sizes)
    last = pool_np[(n_pool - 1) * stride:(n_pool - 1) * stride + be * 2].view(np.uint16)
    x2 = x.copy()
    x2[2 * be:3 * be] = last
    ref, m_ref = oracle.compress(x2, cb_or)
    assert (total, m, status) == (ref.size, m_ref, 0) and np.array_equal(out[:total].cpu().numpy(), ref)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [sz.BF16, sz.FP8_E5M2])
def test_batch_of_tensors_behind_one_block_table(dtype):
    """K and V of several layers in one pool per layer ([pages, 2, block, 8, 128]: V behind K inside every page), one block
    table for the sequence; one launch each way; streams are those of the gathered tensors"""
    es = 2 if dtype == sz.BF16 else 1
    layers, be, n = 3, 4096, 37 * 1024 + 500               # a ragged last page
    n_blocks = -(-n // be)
    n_pool = n_blocks + 3
    stride = 2 * be * es                                     # K part, then V part
    rng = np.random.default_rng(5)
    table_np = rng.permutation(n_pool)[:n_blocks].astype(np.int32)
    cbs_or = {k: oracle.calibrate(kv_synth.to_numpy_words(GEN[dtype](1024, 1, 0, k)), DT[dtype]) for k in "KV"}
    cbs = {k: sz.codebook_from_dec(cbs_or[k].dec.tolist(), dtype) for k in "KV"}
    pools_np, words = [], []
    for layer in range(layers):
        pool = np.full(n_pool * stride, 0xEE, np.uint8)
        for half, kind in enumerate("KV"):
            x = kv_synth.to_numpy_words(GEN[dtype](-(-n // 1024), 3, layer, kind))[:n].copy()
            words.append((layer, half, kind, x))
            xb = x.view(np.uint8)
            for b in range(n_blocks):
                piece = xb[b * be * es:(b + 1) * be * es]
                at = int(table_np[b]) * stride + half * be * es
                pool[at:at + piece.size] = piece
        pools_np.append(pool)
    pools = [torch.from_numpy(p).cuda() for p in pools_np]
    table = torch.from_numpy(table_np).cuda()
    paging = sz.Paged(pools[0], table, be, stride, 0, n_pool)    # the pool of this description is ignored by the batch calls
    views = [pools[layer][half * be * es:] for layer, half, _, _ in words]
    books = [cbs[kind] for _, _, kind, _ in words]
    k = len(words)
    outs = [torch.full((sz.compress_bound(n, dtype) + 256,), 0xA5, dtype=torch.uint8, device="cuda") for _ in range(k)]
    rec = sz.new_sizes_array(k)
    ws = sz.Workspace(n, dtype)
    sz.CompressBatchPaged(views, [n] * k, books, outs, paging, capacities=[o.numel() - 256 for o in outs]).launch(ws, rec)
    torch.cuda.synchronize()
    got = sz.read_sizes_array(rec)
    for i, (layer, half, kind, x) in enumerate(words):
        ref, m = oracle.compress(x, cbs_or[kind])
        assert got[i] == (ref.size, m, 0), (i, got[i], ref.size, m)
        assert np.array_equal(outs[i][:ref.size].cpu().numpy(), ref), f"item {i} differs"
        assert (outs[i][ref.size:ref.size + 256].cpu().numpy() == 0xA5).all()
    # back into fresh pools
    pools2 = [torch.full_like(p, 0x77) for p in pools]
    views2 = [pools2[layer][half * be * es:] for layer, half, _, _ in words]
    st = sz.new_sizes()
    sz.DecompressBatchPaged(outs, [g[0] for g in got], [n] * k, books, views2, paging).launch(st)
    torch.cuda.synchronize()
    assert sz.read_sizes(st)[2] == 0
    for layer in range(layers):
        want = np.full(pools_np[layer].size, 0x77, np.uint8)
        for (ly, half, kind, x) in words:
            if ly != layer:
                continue
            xb = x.view(np.uint8)
            for b in range(n_blocks):
                piece = xb[b * be * es:(b + 1) * be * es]
                at = int(table_np[b]) * stride + half * be * es
                want[at:at + piece.size] = piece
        assert np.array_equal(pools2[layer].cpu().numpy(), want), f"layer {layer}"
    # a table too short for a tensor is refused
    short = sz.Paged(pools[0], table[:2].contiguous(), be, stride, 0, n_pool)
    with pytest.raises(sz.SplitZipError):
        sz.CompressBatchPaged(views, [n] * k, books, outs, short).launch(ws, rec)
