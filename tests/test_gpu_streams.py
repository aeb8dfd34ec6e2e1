"""Calls on two HIP streams at once, each with a workspace of its own (the header's rule: calls that
share a workspace must be ordered on one stream; calls that do not may overlap). Each stream runs a
small decode step on its own inputs; the results must equal, bit for bit, those of the same steps run
one after the other on one stream. Both streams have the default priority."""
import pytest
import torch

import paper_2404_11912_amd as tf
from paper_2404_11912_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda"


class _Step:
    def __init__(self, seed, B, H, N, G, c, k, V):
        x = synth.make_layer(B, H, N, G, c, 4, seed=seed)
        self.K, self.V, self.Q, self.q_r = (x[n].to(DEV) for n in ("K", "V", "Q", "q_r"))
        self.c, self.k, self.M = c, k, N // c
        self.Kmean = torch.empty((B, H, self.M, 128), dtype=torch.float32, device=DEV)
        self.idx = torch.empty((B, H, k), dtype=torch.int32, device=DEV)
        self.Kr = torch.zeros((B, H, k * c, 128), dtype=torch.bfloat16, device=DEV)
        self.Vr = torch.zeros_like(self.Kr)
        self.O = torch.empty((B, H, G, 128), dtype=torch.float32, device=DEV)
        self.L = torch.empty((B, H, G), dtype=torch.float32, device=DEV)
        self.O_d = torch.empty_like(self.O)
        self.a = synth.make_accept_inputs(B, G - 1, V, 0.6, seed + 1, correlated=True, device=DEV)
        self.n = torch.empty((B,), dtype=torch.int32, device=DEV)
        self.out = torch.empty((B, G), dtype=torch.int32, device=DEV)
        self.ws = tf.workspace(max(tf.tf_decode_attn_full_workspace_bytes(B, H, N, G),
                                   tf.tf_decode_attn_retrieval_workspace_bytes(B, H, k * c, G),
                                   tf.tf_chunk_topk_gather_workspace_bytes(B, H, self.M, k),
                                   tf.tf_spec_accept_workspace_bytes(B, G, V)), DEV)

    def outputs(self):
        return (self.Kmean, self.idx, self.Kr, self.Vr, self.O_d, self.O, self.L, self.n, self.out)

    def run(self, stream):
        a = self.a
        tf.tf_chunk_summarize(self.K, self.c, self.Kmean, 0, self.M, stream=stream)
        tf.tf_chunk_topk_gather(self.q_r, self.Kmean, self.K, self.V, self.c, self.k, self.idx, self.Kr, self.Vr,
                                ws=self.ws, stream=stream)
        tf.tf_decode_attn_retrieval(self.Q, self.Kr, self.Vr, self.O_d, causal=False, ws=self.ws, stream=stream)
        tf.tf_decode_attn_full(self.Q, self.K, self.V, self.O, self.L, ws=self.ws, stream=stream)
        tf.tf_spec_accept(a["target_logits"], a["draft_logits"], a["draft_tokens"], 0.6, a["u_accept"],
                          a["u_sample"], self.n, self.out, ws=self.ws, stream=stream)


def test_two_streams_with_their_own_workspaces_do_not_disturb_each_other():
    print("case two_streams seeds=170,172", flush=True)
    steps = [_Step(170, 2, 4, 6000, 5, 8, 64, 5000), _Step(172, 1, 8, 9000, 3, 4, 128, 33000)]
    torch.cuda.synchronize()
    main = torch.cuda.current_stream()
    for s in steps:                                   # one after the other on one stream
        s.run(main)
    torch.cuda.synchronize()
    want = [[t.clone() for t in s.outputs()] for s in steps]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(5):
        for s in steps:
            for t in s.outputs():
                t.zero_()
        torch.cuda.synchronize()
        for _ in range(3):                            # interleaved enqueue, both streams busy
            for s, st in zip(steps, streams):
                s.run(st)
        torch.cuda.synchronize()
        for s, w in zip(steps, want):
            for got, wnt in zip(s.outputs(), w):
                assert torch.equal(got, wnt), f"repetition {rep}: results differ from the one-stream run"


def test_two_host_threads_with_their_own_split_options():
    """Two host threads, each driving its own stream with its own workspace and its own split
    options (tf_set_thread_option: visible to the setting thread only). The results must equal, bit
    for bit, those of the same step run alone with the same options."""
    import threading
    print("case two_threads seeds=174,176", flush=True)
    steps = [_Step(174, 2, 4, 6000, 5, 8, 64, 5000), _Step(176, 1, 8, 9000, 3, 4, 128, 33000)]
    options = [{"attn_full_tokens_per_split": 1024, "attn_retr_tokens_per_split": 128, "score_steps_per_wave": 1},
               {"attn_full_tokens_per_split": 2048, "attn_retr_tokens_per_split": 256, "score_steps_per_wave": 3}]
    torch.cuda.synchronize()

    def with_options(opts, fn):
        for k, v in opts.items():
            tf.tf_set_thread_option(k, v)
        try:
            return fn()
        finally:
            for k in opts:
                tf.tf_set_thread_option(k, -1)

    def alloc_ws(s):            # sized under the options the step will run with
        B, H, N, _ = s.K.shape
        G, k, c = s.Q.shape[2], s.k, s.c
        s.ws = tf.workspace(max(tf.tf_decode_attn_full_workspace_bytes(B, H, N, G),
                                tf.tf_decode_attn_retrieval_workspace_bytes(B, H, k * c, G),
                                tf.tf_chunk_topk_gather_workspace_bytes(B, H, s.M, k),
                                tf.tf_spec_accept_workspace_bytes(B, G, s.a["target_logits"].shape[2])), DEV)

    main = torch.cuda.current_stream()
    want = []
    for s, o in zip(steps, options):
        with_options(o, lambda: (alloc_ws(s), s.run(main)))
        torch.cuda.synchronize()
        want.append([t.clone() for t in s.outputs()])
    plans = [with_options(o, lambda: tf.tf_decode_attn_plan(0, 1, 8, 9000)) for o in options]
    assert plans[0] != plans[1]                                  # the two threads really plan differently
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    errors = []

    def worker(s, o, st, gate):
        try:
            torch.cuda.set_device(0)
            def body():
                gate.wait(timeout=60)
                for _ in range(6):
                    s.run(st)
            with_options(o, body)
        except Exception as e:                                   # noqa: BLE001
            errors.append(e)

    for rep in range(3):
        for s in steps:
            for t in s.outputs():
                t.zero_()
        torch.cuda.synchronize()
        gate = threading.Barrier(2)
        ts = [threading.Thread(target=worker, args=(s, o, st, gate)) for s, o, st in zip(steps, options, streams)]
        for t in ts:
            t.start()
        for t in ts:
            t.join()
        torch.cuda.synchronize()
        assert not errors, errors
        for s, w in zip(steps, want):
            for got, wnt in zip(s.outputs(), w):
                assert torch.equal(got, wnt), f"repetition {rep}: results differ from the run alone"


def test_temporary_workspace_belongs_to_the_call_stream():
    """Calls without a caller workspace on a side stream: the binding's temporary scratch is dropped
    right after the kernels are enqueued, so its block must belong to the side stream; otherwise the
    current stream's next allocation of that size could take it while the kernels still run. The
    current stream allocates and fills same-sized buffers throughout; results must equal the
    reference run's."""
    print("case temp_workspace_side_stream seed=178", flush=True)
    x = synth.make_layer(1, 8, 20000, 5, 8, 4, seed=178)
    K, V, Q = (x[n].to(DEV) for n in ("K", "V", "Q"))
    O_ref = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L_ref = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_full(Q, K, V, O_ref, L_ref)
    torch.cuda.synchronize()
    nbytes = tf.tf_decode_attn_full_workspace_bytes(1, 8, 20000, 5)
    side = torch.cuda.Stream()
    O = torch.empty_like(O_ref)
    L = torch.empty_like(L_ref)
    for rep in range(20):
        O.zero_()
        torch.cuda.synchronize()
        tf.tf_decode_attn_full(Q, K, V, O, L, stream=side)         # ws=None: temporary scratch
        for _ in range(4):                                         # same-sized blocks on the current stream
            junk = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
            junk.fill_(0xff)
            del junk
        torch.cuda.synchronize()
        assert torch.equal(O, O_ref) and torch.equal(L, L_ref), f"repetition {rep}"
