"""Head sizes 64 and 256 through the whole path against the oracle (128 is what every other GPU
test runs): the pooling, score and fused kernels take the head size as a parameter, and the attention
kernel is one template over the block size and the head size, instantiated for all six combinations."""
import pytest

from paper_2603_06274_amd import workloads as wl

from test_gpu_parity import run_both

pytestmark = pytest.mark.gpu


def cases(d):
    return {
        # ragged single sequence, GQA 2:1, B = 64
        "ragged_b64": wl.small("ragged_b64_d%d" % d, seed=61, num_q_heads=4, num_kv_heads=2, seq_lens=(1000,),
                               block_size=64, k_start=(6,), n_sink=1, n_local=1, outliers=(2,), head_dim=d),
        # packed batch with an empty and a sub-block sequence, GQA 4:1, B = 128
        "packed_b128": wl.small("packed_b128_d%d" % d, seed=62, num_q_heads=8, num_kv_heads=2,
                                seq_lens=(700, 0, 1536, 130, 50), block_size=128, k_start=(3, 1, 5, 2, 1),
                                n_sink=1, n_local=2, outliers=(1, 0, 2, 1, 1), head_dim=d),
        # more than 64 blocks: several score tiles per row, B = 128, MHA
        "long_b128": wl.small("long_b128_d%d" % d, seed=63, num_q_heads=2, num_kv_heads=2, seq_lens=(9000,),
                              block_size=128, k_start=(12,), n_sink=2, n_local=2, outliers=(6,), head_dim=d),
        # a start budget of zero: every row keeps exactly its forced windows
        "forced_only_b64": wl.small("forced_only_b64_d%d" % d, seed=64, num_q_heads=2, num_kv_heads=1,
                                    seq_lens=(2000, 300), block_size=64, k_start=(0, 0), n_sink=2, n_local=3,
                                    outliers=(1, 1), head_dim=d),
    }


@pytest.mark.parametrize("name", ["ragged_b64", "packed_b128", "long_b128", "forced_only_b64"])
@pytest.mark.parametrize("d", [64, 256])
def test_head_size_whole_path(d, name):
    run_both(cases(d)[name])


@pytest.mark.parametrize("d,ad_stride", [(64, 1), (256, 2)])
def test_head_size_fused_above_1024_blocks(d, ad_stride):
    """The fused stage 1-2 with more than 1024 key blocks per row (its 4-row bands) at the other head
    sizes: dumped scores and lists against the oracle."""
    import torch
    import parity_util as pu
    w = wl.small("many_blocks_d%d" % d, seed=65, num_q_heads=2, num_kv_heads=1, seq_lens=(1100 * 64 + 5,),
                 block_size=64, k_start=(30,), n_sink=2, n_local=2, outliers=(8,), head_dim=d)
    data = wl.generate(w)
    qkv = pu.host_arrays(data)
    pf = pu.device_prefill(w, data, ad_stride=ad_stride)
    assert pf.nbmax > 1024
    dump = torch.full_like(pf.scores, float("nan"))
    pf.estimate_select(dump)
    torch.cuda.synchronize()
    scores = pu.oracle_estimate(w, qkv, ad_stride)[3]
    pu.check_scores(dump.cpu().numpy(), scores)
    _, counts, indices = pu.oracle_select(w, scores)
    same = pu.check_lists(w, pf.counts.cpu().numpy(), pf.indices.cpu().numpy(), counts, indices, scores, print)
    assert same.mean() > 0.99
