"""The decode entry point that allocates nothing (lkv_paged_decode_attention_static): same kernels as
lkv_paged_decode_attention, the split-K partial results in the library's fixed device array instead of the
context's workspace.  Its output must equal the ordinary entry point's bit for bit (same launch, same arithmetic),
which in turn is checked against the oracle; two calls in a row, the second with a smaller batch, so that whatever
the first call left in the array cannot leak into the second."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2410_00428_amd import binding as lkv  # noqa: E402
from paper_2410_00428_amd import workloads as wl  # noqa: E402
from tests import gpu_harness as H  # noqa: E402
from tests.test_gpu_parity import Scenario, ORC_THREADS  # noqa: E402

pytestmark = pytest.mark.gpu


def decode_inputs(sc, seqs, seed):
    shape = sc.shape
    q = wl.normal_tensor(np.random.default_rng(seed), (len(seqs), shape.num_q_heads, shape.head_dim), 1.0, "bf16")
    bt = sc.c.padded_block_table(seqs, 0)
    ctx = np.asarray([sc.lens[s] for s in seqs], dtype=np.int32)
    return q, bt, ctx


@pytest.mark.parametrize("shape", [wl.KVShape(1, 8, 8, 128, 16, "bf16"), wl.KVShape(1, 16, 2, 128, 16, "bf16")])
def test_static_scratch_decode_equals_the_ordinary_entry_point_twice_in_a_row(shape):
    lens = (3000, 1234, 2049, 700, 16, 1)
    sc = Scenario(41, shape, lens, sum((n + 15) // 16 for n in lens) + 4)
    sc.prefill_layer(0, check_attn=False)
    torch.cuda.synchronize()
    for seqs, seed in ((range(6), 1), ((1, 3, 5), 2)):     # the second call is the smaller one
        q, bt, ctx = decode_inputs(sc, list(seqs), seed)
        B = len(ctx)
        qd, btd, cd = H.to_dev(q), H.to_dev(bt), H.to_dev(ctx)
        O_ws = H.empty_like_storage(q.shape, "bf16")
        O_st = H.empty_like_storage(q.shape, "bf16")
        O_ws.fill_(0x7FC0)
        O_st.fill_(0x7FC0)
        sc.c.paged_decode_attention(0, qd, O_ws, btd, bt.shape[1], cd, B)
        sc.c.paged_decode_attention_static(0, qd, O_st, btd, bt.shape[1], cd, B)
        torch.cuda.synchronize()
        assert torch.equal(O_ws, O_st), "the two entry points differ"
        ref = sc.o.paged_decode_attention(q, bt, ctx, threads=ORC_THREADS)
        H.check_attention(H.to_host(O_st, "bf16"), ref, "bf16", 1.0, f"static-scratch decode, {B} sequences")
    sc.close()


def test_static_scratch_decode_is_really_split_and_rejects_what_does_not_fit():
    """The case above must go through the scratch (a launch that is not split would prove nothing), and a launch
    whose partial results exceed the fixed 8 MiB is refused before anything is enqueued."""
    shape = wl.KVShape(1, 64, 8, 128, 16, "bf16")
    sc = Scenario(42, shape, (100, 40), 16)
    sc.prefill_layer(0, check_attn=False)
    # a second context forced to 64-token partitions: every 100-token context has two partial results
    c2 = lkv.LKV(1, 64, 8, 128, 16, 16, "bf16", pool=sc.pool, decode_partition=64)
    q, bt, ctx = decode_inputs(sc, [0, 1], 3)
    O1 = H.empty_like_storage(q.shape, "bf16")
    c2.paged_decode_attention_static(0, H.to_dev(q), O1, H.to_dev(bt), bt.shape[1], H.to_dev(ctx), 2)
    torch.cuda.synchronize()
    ref = sc.o.paged_decode_attention(q, bt, ctx, threads=ORC_THREADS)
    H.check_attention(H.to_host(O1, "bf16"), ref, "bf16", 1.0, "64-token partitions through the fixed scratch")
    # 272 sequences (more than an evenly cut launch takes: partitions) x 64 heads x 512-block tables (2 partitions)
    # x 130 floats = 17 MiB > 8 MiB
    B, width = 272, 512
    wide = np.full((B, width), -1, dtype=np.int32)
    wide[:, :bt.shape[1]] = bt[0]
    qq = wl.normal_tensor(np.random.default_rng(4), (B, 64, 128), 1.0, "bf16")
    O2 = H.empty_like_storage(qq.shape, "bf16")
    O2.fill_(0x1234)
    with pytest.raises(lkv.LkvError) as e:
        sc.c.paged_decode_attention_static(0, H.to_dev(qq), O2, H.to_dev(wide), width,
                                           H.to_dev(np.full(B, 100, dtype=np.int32)), B)
    assert e.value.status == lkv.LKV_ERR_INVALID_ARG and "fixed scratch" in str(e.value)
    torch.cuda.synchronize()
    assert (O2 == 0x1234).all()     # nothing ran
    sc.c.paged_decode_attention(0, H.to_dev(qq), O2, H.to_dev(wide), width, H.to_dev(np.full(B, 100, dtype=np.int32)), B)
    torch.cuda.synchronize()        # the ordinary entry point takes the same launch (17 MiB < its 32 MiB workspace)
    c2.destroy()
    sc.close()
