"""GPU parity of harli_decode_step against the CPU oracle (through the C ABI).

Bar: page-table / block indexing bit-exact (the set of slab elements the step changes is
exactly the oracle's); fp outputs max-abs error <= 2e-2 * max|ref| and relative Frobenius
error <= 5e-3 for bf16 storage with fp32 accumulation.
"""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from tests.gpu_util import DecodeCase, assert_close

pytestmark = pytest.mark.gpu


def variant(idx, **kw):
    w = wl.workload(idx)
    return w, dataclasses.replace(w.model, **kw)


# fp32 storage and arithmetic: unit round-off 6e-8, dot products of up to ~700 terms summed lane-wise then by a
# butterfly (error ~ sqrt(K) u), seven chained steps and an fp32 exp -- 1e-4 of the largest output and 2e-5 in
# relative Frobenius norm leave a factor ~10 of slack.
F32_BAR = dict(max_ratio=1e-4, fro=2e-5)


def run_case(w, m, lengths, **kw):
    case = DecodeCase(w, m, np.asarray(lengths, np.int32), **kw)
    y = case.run_gpu()
    ref = case.run_oracle()
    bar = F32_BAR if m.dtype == "f32" else {}
    stats = assert_close(y, ref, "decode output", **bar)
    n = case.check_cache(*((1e-4, 2e-5) if m.dtype == "f32" else ()))
    assert n == len(lengths) * m.n_layers * 2 * m.n_kv * m.head_dim
    return case, stats


def test_tiny_bf16_config0_shapes():
    """Config 0's shapes (hidden 256, 4 x 64 heads, ffn 688 = 43 tiles, ragged) stored as bf16."""
    w, m = variant(0, dtype="bf16")
    run_case(w, m, wl.draw_lengths(w), block_bytes=64 << 10)


@pytest.mark.parametrize("lengths", [
    [0], [0, 1, 15, 16, 17], [255, 256, 257, 511, 512], [700, 3, 1300], [31] * 16, [40] * 17, list(range(5, 105, 3)),
])
def test_tiny_edge_lengths_and_batches(lengths):
    """Empty cache, page boundaries (15/16/17), chunk boundaries (255/256/257), ragged mixes,
    batch 16/17 (one and two MFMA column tiles) and 34 (three)."""
    w, m = variant(0, dtype="bf16")
    run_case(w, m, lengths, block_bytes=64 << 10)


def test_batch_above_64_runs_in_passes():
    w, m = variant(0, dtype="bf16")
    run_case(w, m, [7 + (i * 5) % 90 for i in range(100)], block_bytes=64 << 10)


def test_three_layers_at_batch_250_with_embedding_and_logits():
    """Above 32 sequences the layer GEMMs take the tiled path: here one batch tile of 256 rows with 250 real ones (the
    last 16-row group ragged), a ragged last weight tile (ffn 688 of 768), three layers chained through the row norms
    and the output layer after them."""
    w, m = variant(0, dtype="bf16", n_layers=3, vocab=1000)
    lengths = np.asarray([(i * 29) % 150 for i in range(250)], np.int32)
    case = DecodeCase(w, m, lengths, full_model=True, block_bytes=64 << 10)
    tok = wl.make_token_ids(dataclasses.replace(w, model=m), (250,))
    hid = case.run_gpu(token_ids=tok)
    ref_hid, ref_logits, _ = case.run_oracle(token_ids=tok)
    assert_close(hid, ref_hid, "hidden state")
    assert_close(case.logits_dev.cpu().numpy(), ref_logits, "logits")
    case.check_cache()
    first = (case.y_dev.clone(), case.logits_dev.clone(), case.slab.clone())
    case.slab.copy_(torch.from_numpy(case.img0.view(np.uint8)))
    case.run_gpu(token_ids=tok)                      # the partial tiles are added in a fixed order: the same bits again
    assert torch.equal(case.y_dev, first[0]) and torch.equal(case.logits_dev, first[1]) and torch.equal(case.slab, first[2])


def test_a_context_for_large_batches_serves_small_ones_on_the_streaming_kernels():
    """max_batch decides whether the workspace of the tiled path exists; the batch of the step decides the path: a step
    of 9 sequences gives the same bits in a context made for 200 as in one made for 9."""
    w, m = variant(0, dtype="bf16", n_layers=2)
    lengths = np.asarray([12, 200, 0, 77, 300, 33, 5, 129, 64], np.int32)
    small = DecodeCase(w, m, lengths, block_bytes=64 << 10)
    roomy = DecodeCase(w, m, lengths, block_bytes=64 << 10, max_batch=200)
    assert roomy.ctx.device_bytes().decode_workspace > small.ctx.device_bytes().decode_workspace
    assert np.array_equal(np.asarray(small.run_gpu()), np.asarray(roomy.run_gpu()))


def test_out_of_range_page_id_is_reported_at_large_batch():
    from paper_2511_11729_amd import binding as hb
    w, m = variant(0, dtype="bf16")
    case = DecodeCase(w, m, np.asarray([20 + i % 30 for i in range(80)], np.int32), block_bytes=64 << 10)
    case.table_dev[70, 1] = 10_000_000
    with pytest.raises(hb.HarliError) as e:
        case.run_gpu()
    assert "page id" in str(e.value)
    case.table_dev[70, 1] = int(case.table[70, 1])
    case.run_gpu()


@pytest.mark.parametrize("n_q,n_kv,d", [(8, 2, 64), (8, 8, 128), (8, 4, 128), (8, 2, 128), (8, 1, 128), (6, 2, 128), (5, 1, 128),
                                        (6, 1, 128), (7, 1, 128)])
def test_head_layouts(n_q, n_kv, d):
    """GQA ratios 1, 2, 4, 8 and both head sizes."""
    w, m = variant(0, dtype="bf16", hidden=n_q * d // 2, n_q=n_q, n_kv=n_kv, head_dim=d, ffn=320)
    run_case(w, m, [0, 37, 300, 16], block_bytes=256 << 10)


def test_non_dividing_page_size():
    """Pages that do not divide the block (3 per 64 KiB block with slack), several chunks."""
    w, m = variant(0, dtype="bf16", hidden=640, n_q=5, n_kv=5, head_dim=128, ffn=256)
    case, _ = run_case(w, m, [100, 33, 250], block_bytes=64 << 10)
    assert case.geom.pages_per_block == 3 and case.pool.stats().kv_chunks > 3


def test_three_layer_model_with_embedding_and_logits():
    w, m = variant(0, dtype="bf16", n_layers=3, vocab=1000)
    lengths = [12, 200, 0, 77]
    case = DecodeCase(w, m, np.asarray(lengths, np.int32), full_model=True, block_bytes=64 << 10)
    tok = wl.make_token_ids(dataclasses.replace(w, model=m), (4,))
    hid = case.run_gpu(token_ids=tok)
    ref_hid, ref_logits, ref_next = case.run_oracle(token_ids=tok)
    assert_close(hid, ref_hid, "hidden state")
    logits = case.logits_dev.cpu().numpy()
    assert_close(logits, ref_logits, "logits")
    case.check_cache()
    nxt = case.next_dev.cpu().numpy()
    # argmax is exact on the GPU's own logits (ties to the lowest index) ...
    assert np.array_equal(nxt, np.argmax(logits, axis=-1))
    # ... and equals the oracle's wherever the oracle's top-2 gap exceeds the tolerance
    srt = np.sort(ref_logits, axis=-1)
    clear = (srt[:, -1] - srt[:, -2]) > 4e-2 * np.max(np.abs(ref_logits))
    assert np.array_equal(nxt[clear], ref_next[clear])


def test_step_is_bit_reproducible():
    """The same step gives the same bits every time, on any stream and whatever ran in between (the row norms are
    summed across workgroups as integers, in which the order of arrival does not matter)."""
    w, m = variant(0, dtype="bf16", n_layers=3, vocab=1000)
    lengths = [12, 200, 0, 77, 300, 33, 5, 129, 64]
    case = DecodeCase(w, m, np.asarray(lengths, np.int32), full_model=True, block_bytes=64 << 10)
    tok = wl.make_token_ids(dataclasses.replace(w, model=m), (len(lengths),))
    case.run_gpu(token_ids=tok)
    first = (case.y_dev.clone(), case.logits_dev.clone(), case.next_dev.clone(), case.slab.clone())
    side = torch.cuda.Stream()
    busy = torch.randn(2048, 2048, device="cuda:0")
    for rep in range(6):
        case.slab.copy_(torch.from_numpy(case.img0.view(np.uint8)))
        if rep % 2:                                   # unrelated work on another stream while the step runs
            with torch.cuda.stream(side):
                for _ in range(4):
                    busy = busy @ busy * 1e-3
        case.run_gpu(token_ids=tok, stream=side if rep >= 3 else None)
        assert torch.equal(case.y_dev, first[0]) and torch.equal(case.logits_dev, first[1])
        assert torch.equal(case.next_dev, first[2]) and torch.equal(case.slab, first[3])


def test_argmax_ties_go_to_the_lowest_index():
    w, m = variant(0, dtype="bf16", n_layers=1, vocab=64)
    def same_rows(case):             # identical rows in the output layer give exactly equal logits
        case.extras_np["wlm"][5] = case.extras_np["wlm"][40]
    case = DecodeCase(w, m, np.asarray([3, 9], np.int32), full_model=True, block_bytes=64 << 10, tweak=same_rows)
    case.run_gpu(token_ids=[1, 2])
    logits = case.logits_dev.cpu().numpy()
    assert np.array_equal(logits[:, 5], logits[:, 40])
    assert np.array_equal(case.next_dev.cpu().numpy(), np.argmax(logits, axis=-1))


def test_out_of_range_page_id_is_reported_not_dereferenced():
    from paper_2511_11729_amd import binding as hb
    w, m = variant(0, dtype="bf16")
    case = DecodeCase(w, m, np.asarray([20, 40], np.int32), block_bytes=64 << 10)
    case.table_dev[1, 1] = 10_000_000
    with pytest.raises(hb.HarliError) as e:
        case.run_gpu()
    assert "page id" in str(e.value)
    case.table_dev[1, 1] = int(case.table[1, 1])
    case.run_gpu()                                   # the flag was cleared; a clean step passes


def test_config1_full_size_layer():
    """The 7B-class layer at its real shape: batch 8, lengths uniform in [256, 2048]."""
    w = wl.workload(1)
    case, stats = run_case(w, w.model, wl.draw_lengths(w))
    print("config 1 decode parity: max-abs ratio %.2e, rel-Fro %.2e" % stats)


def test_two_steps_in_a_row_use_the_appended_token():
    """Step t+1 attends to the K/V that step t appended (same context, same pages)."""
    w, m = variant(0, dtype="bf16")
    lengths = np.asarray([14, 30, 250], np.int32)
    case = DecodeCase(w, m, lengths, block_bytes=64 << 10)
    y1 = case.run_gpu()
    ref1 = case.run_oracle()
    assert_close(y1, ref1, "step 1")
    # second step: feed y1 back in as the next input on both sides
    case.x_dev.copy_(torch.from_numpy(ref1.astype(np.float32)))
    case.kv_len_dev += 1
    case.ctx.decode_step(batch=3, kv_len=case.kv_len_dev, page_table=case.table_dev, max_pages=case.max_pages,
                         max_kv_len=int(lengths.max()) + 2, x_in=case.x_dev, x_out=case.y_dev)
    torch.cuda.synchronize()
    case.ctx.check()
    from oracle import harli_oracle as O
    from tests.gpu_util import shapes_of
    ref2 = O.decode_model_paged(ref1.astype(np.float32), case.layers_np, None, shapes_of(m), case.okv, lengths + 1, case.table)
    assert_close(case.y_dev.cpu().numpy(), ref2, "step 2")


# ---- fp32 storage (config 0 as written): every tensor fp32, generic kernels without tile restrictions ----

def test_config0_fp32_as_written():
    w = wl.workload(0)
    assert w.model.dtype == "f32"
    case, stats = run_case(w, w.model, wl.draw_lengths(w), block_bytes=64 << 10)
    print("config 0 fp32 decode parity: max-abs ratio %.2e, rel-Fro %.2e" % stats)


@pytest.mark.parametrize("lengths", [[0], [0, 1, 15, 16, 17], [255, 256, 257], [31] * 17, list(range(5, 105, 9))])
def test_fp32_edge_lengths_and_batches(lengths):
    """Empty cache, page boundaries, a batch that spans three 8-row tiles."""
    w = wl.workload(0)
    run_case(w, w.model, lengths, block_bytes=128 << 10)


@pytest.mark.parametrize("hidden,n_q,n_kv,d,ffn", [(200, 6, 2, 20, 333), (96, 3, 1, 34, 70), (320, 2, 2, 160, 64)])
def test_fp32_arbitrary_shapes(hidden, n_q, n_kv, d, ffn):
    """Shapes that are multiples of nothing: grouped heads, head sizes above and below a wave, odd widths."""
    w, m = variant(0, hidden=hidden, n_q=n_q, n_kv=n_kv, head_dim=d, ffn=ffn)
    run_case(w, m, [0, 37, 130, 16], block_bytes=64 << 10)


def test_fp32_three_layer_model_with_embedding_and_logits():
    w, m = variant(0, n_layers=3, vocab=777)
    lengths = [12, 100, 0, 77]
    case = DecodeCase(w, m, np.asarray(lengths, np.int32), full_model=True, block_bytes=64 << 10)
    tok = wl.make_token_ids(dataclasses.replace(w, model=m), (4,))
    hid = case.run_gpu(token_ids=tok)
    ref_hid, ref_logits, ref_next = case.run_oracle(token_ids=tok)
    assert_close(hid, ref_hid, "hidden state", **F32_BAR)
    logits = case.logits_dev.cpu().numpy()
    assert_close(logits, ref_logits, "logits", **F32_BAR)
    case.check_cache(1e-4, 2e-5)
    nxt = case.next_dev.cpu().numpy()
    assert np.array_equal(nxt, np.argmax(logits, axis=-1))
    srt = np.sort(ref_logits, axis=-1)
    clear = (srt[:, -1] - srt[:, -2]) > 2e-4 * np.max(np.abs(ref_logits))
    assert np.array_equal(nxt[clear], ref_next[clear])


# ---- the other workloads at their real layer width (depth cut to what the oracle finishes in seconds) ----

def test_config2_width_two_layers_batch16_with_logits():
    """7B-class model, batch 16 at 1024 cached tokens, embedding + 2 of the 32 layers + output layer (V = 32000)."""
    w, m = variant(2, n_layers=2)
    lengths = wl.draw_lengths(w)
    assert len(lengths) == 16 and int(lengths[0]) == 1024
    case = DecodeCase(w, m, lengths, full_model=True)
    tok = wl.make_token_ids(dataclasses.replace(w, model=m), (16,))
    hid = case.run_gpu(token_ids=tok)
    ref_hid, ref_logits, ref_next = case.run_oracle(token_ids=tok)
    assert_close(hid, ref_hid, "hidden state")
    logits = case.logits_dev.cpu().numpy()
    assert_close(logits, ref_logits, "logits")
    case.check_cache()
    nxt = case.next_dev.cpu().numpy()
    assert np.array_equal(nxt, np.argmax(logits, axis=-1))
    srt = np.sort(ref_logits, axis=-1)
    clear = (srt[:, -1] - srt[:, -2]) > 4e-2 * np.max(np.abs(ref_logits))
    assert np.array_equal(nxt[clear], ref_next[clear])


def test_config2_width_batch256():
    """The largest decode batch (one tile of 256 batch rows, no idle row) on one 7B-class layer."""
    w, m = variant(2, n_layers=1)
    run_case(w, m, [100 + (i * 37) % 400 for i in range(256)])


@pytest.mark.parametrize("batch", [70, 150, 200])
def test_config4_width_batches_that_split_into_uneven_passes(batch):
    """Batches above 64 rows on the GQA layer: tiles of 128, 192 and 256 batch rows (70: 58 idle rows; 150: 42; 200: 56),
    every GEMM cut into ranges of K."""
    w, m = variant(4, n_layers=1)
    run_case(w, m, [60 + (i * 53) % 300 for i in range(batch)])


def test_config5_width_biases_at_batch_80():
    """The tiled path with q, k, v biases and groups of seven query heads per KV head (hidden 3584: 14 weight tiles of
    256 rows exactly; ffn 18944: 74)."""
    w, m = variant(5, n_layers=1)
    run_case(w, m, [40 + (i * 31) % 200 for i in range(80)])


def test_config3_width_layer_lognormal_lengths():
    """13B-class layer (hidden 5120, 40 heads, ffn 13824): 160 KiB pages do not divide the 2 MiB block (12 + slack),
    batch 32 with log-normal lengths capped at 4096."""
    w, m = variant(3, n_layers=1)
    lengths = wl.draw_lengths(w)
    case, stats = run_case(w, m, lengths)
    assert case.geom.pages_per_block == 12
    print("config 3 layer decode parity: max-abs ratio %.2e, rel-Fro %.2e, lengths %d..%d" % (stats + (lengths.min(), lengths.max())))


def test_config4_width_layer_gqa_long_context():
    """8B-class GQA layer (32 query / 8 KV heads, ffn 14336), batch 8, log-normal lengths capped at 8192."""
    w, m = variant(4, n_layers=1)
    lengths = wl.draw_lengths(w)
    case, stats = run_case(w, m, lengths)
    print("config 4 layer decode parity: max-abs ratio %.2e, rel-Fro %.2e, lengths %d..%d" % (stats + (lengths.min(), lengths.max())))


def test_config5_width_layer_biases_and_groups_of_seven():
    """Qwen2.5-7B-class layer (hidden 3584, 28 query / 4 KV heads, ffn 18944, RoPE base 1e6, biases on q, k, v), batch 8,
    log-normal lengths."""
    w, m = variant(5, n_layers=1)
    assert m.qkv_bias
    lengths = wl.draw_lengths(w)
    case, stats = run_case(w, m, lengths)
    assert "bq" in case.layers_np[0]
    print("config 5 layer decode parity: max-abs ratio %.2e, rel-Fro %.2e, lengths %d..%d" % (stats + (lengths.min(), lengths.max())))


def test_biases_small_shapes_bf16_and_fp32():
    """Biases with two layers, ragged lengths, both storage types (the fp32 path adds them in its rotary kernel)."""
    for dtype in ("bf16", "f32"):
        w, m = variant(0, dtype=dtype, n_layers=2, qkv_bias=True)
        run_case(w, m, [0, 5, 16, 31, 77])


def test_tiled_path_on_a_compute_unit_partition_and_in_a_replayed_graph():
    """The cut of the tiled GEMMs follows the compute units of the stream the step runs on (fewer ranges of K on a small
    partition): the result meets the oracle there too.  And the step is capturable: a replayed HIP graph gives the bits
    of the eager step on every replay, with eager work in between."""
    from paper_2511_11729_amd import colocate
    w, m = variant(0, dtype="bf16", n_layers=2, hidden=1024, n_q=8, n_kv=2, head_dim=128, ffn=2816, vocab=1000)
    lengths = np.asarray([5 + (i * 13) % 120 for i in range(100)], np.int32)
    case = DecodeCase(w, m, lengths, full_model=True, block_bytes=256 << 10)
    tok = wl.make_token_ids(dataclasses.replace(w, model=m), (100,))
    ref_hid, ref_logits, _ = case.run_oracle(token_ids=tok)
    img0 = torch.from_numpy(case.img0.view(np.uint8))
    hid = case.run_gpu(token_ids=tok)
    assert_close(hid, ref_hid, "hidden state, whole chip")
    eager = (case.y_dev.clone(), case.logits_dev.clone(), case.slab.clone())
    cs = colocate.CuStreams()
    part = cs.low(2)                                   # 20 % of the compute units: other cuts
    case.slab.copy_(img0)
    torch.cuda.synchronize()
    hid_p = case.run_gpu(token_ids=tok, stream=part)
    assert_close(hid_p, ref_hid, "hidden state on 2/10 of the compute units")
    assert_close(case.logits_dev.cpu().numpy(), ref_logits, "logits on 2/10 of the compute units")
    case.check_cache()
    torch.cuda.synchronize()
    cs.close()
    # graph: captured on an ordinary stream, replayed three times with eager steps between the replays
    st = torch.cuda.Stream()
    tok_dev = torch.from_numpy(np.asarray(tok, np.int32)).to("cuda:0")
    y_g, logits_g, next_g = torch.empty_like(eager[0]), torch.empty_like(eager[1]), torch.empty_like(case.next_dev)

    def step():
        case.ctx.decode_step(batch=case.B, kv_len=case.kv_len_dev, page_table=case.table_dev, max_pages=case.max_pages,
                             max_kv_len=int(case.kv_len.max()) + 1, token_ids=tok_dev, logits=logits_g,
                             next_token=next_g, x_out=y_g, stream=st)

    case.slab.copy_(img0)
    torch.cuda.synchronize()
    step()
    st.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st):
        step()
    for rep in range(3):
        case.slab.copy_(img0)
        y_g.zero_()
        logits_g.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            g.replay()
        st.synchronize()
        assert torch.equal(y_g, eager[0]) and torch.equal(logits_g, eager[1]) and torch.equal(case.slab, eager[2])
        case.slab.copy_(img0)                          # the program's own eager work between replays
        torch.cuda.synchronize()
        case.run_gpu(token_ids=tok)
        assert torch.equal(case.y_dev, eager[0])
    case.ctx.check()
    del g


@pytest.mark.parametrize("batch", [4, 40])
def test_vocabulary_that_is_not_a_multiple_of_four(batch):
    """Rows of the logits that are not 16-byte aligned (vocabulary 1003) on both kernel families: the streaming output
    layer at batch 4, the tiled one at batch 40."""
    w, m = variant(0, dtype="bf16", n_layers=1, vocab=1003)
    lengths = np.asarray([3 + (i * 11) % 90 for i in range(batch)], np.int32)
    case = DecodeCase(w, m, lengths, full_model=True, block_bytes=64 << 10)
    tok = wl.make_token_ids(dataclasses.replace(w, model=m), (batch,))
    hid = case.run_gpu(token_ids=tok)
    ref_hid, ref_logits, _ = case.run_oracle(token_ids=tok)
    assert_close(hid, ref_hid, "hidden state")
    logits = case.logits_dev.cpu().numpy()
    assert_close(logits, ref_logits, "logits")
    assert np.array_equal(case.next_dev.cpu().numpy(), np.argmax(logits, axis=-1))
