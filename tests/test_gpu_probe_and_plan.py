"""The two informational entry points on a GPU: tf_stream_read_probe (a plain streaming read used as
the measured bandwidth ceiling) and tf_decode_attn_plan (the launch shape an attention call takes)."""
import pytest
import torch

import paper_2404_11912_amd as tf

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_stream_read_probe_reads_whole_rounds_inside_the_buffer():
    print("case stream_read_probe", flush=True)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(cus * 256, dtype=torch.int32, device=DEV)
    round_bytes = cus * 256 * 8 * 16                       # one round: 8 loads of 16 bytes per thread, all workgroups
    for nbytes in (round_bytes, 3 * round_bytes + 4096, 64 << 20, (64 << 20) + 48):
        buf = torch.full((nbytes // 4,), 0x01010101, dtype=torch.int32, device=DEV)
        sink.fill_(-1)
        n = tf.tf_stream_read_probe(buf, sink)
        torch.cuda.synchronize()
        assert 0 < n <= buf.numel() * 4 and n % round_bytes == 0 and buf.numel() * 4 - n < round_bytes + cus * 16
        # every thread XORs 4 words per load, an even number of equal words: the stored word is 0
        assert int(sink.abs().max()) == 0
    with pytest.raises(tf.TfError):                        # too small to give every workgroup one round
        tf.tf_stream_read_probe(torch.zeros(round_bytes // 4 - 4, dtype=torch.int32, device=DEV), sink)
    with pytest.raises(tf.TfError):                        # sink too small
        tf.tf_stream_read_probe(torch.zeros(round_bytes // 4, dtype=torch.int32, device=DEV), sink[:64])


def test_plan_matches_the_partials_a_call_needs():
    """The plan query names the launch shape: a workspace of exactly batch x heads x splits x 4 waves x
    8 rows x 130 floats is accepted, one partial less is refused."""
    print("case attn_plan vs workspace", flush=True)
    B, H, N, G = 1, 4, 5000, 3
    K = torch.randn((B, H, N, 128), device=DEV).to(torch.bfloat16)
    Q = torch.randn((B, H, G, 128), device=DEV).to(torch.bfloat16)
    O = torch.empty((B, H, G, 128), dtype=torch.float32, device=DEV)
    for kind, fn in ((0, tf.tf_decode_attn_full), (1, tf.tf_decode_attn_retrieval)):
        nsplit, tps = tf.tf_decode_attn_plan(kind, B, H, N)
        assert nsplit * tps >= N and (nsplit - 1) * tps < N
        need = B * H * nsplit * 4 * 8 * 130 * 4
        fn(Q, K, K, O, ws=tf.workspace(need, DEV))
        with pytest.raises(tf.TfError) as e:
            fn(Q, K, K, O, ws=tf.workspace(need - 256, DEV))
        assert e.value.code == -3
    torch.cuda.synchronize()
