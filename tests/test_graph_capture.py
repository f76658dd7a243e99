"""The library only enqueues kernels on the caller's stream (no allocation, no memset,
no synchronisation), so its calls can be recorded into a HIP graph.  Replays are checked
against the eager results, several times, with eager work and synchronisations between."""
import pytest
import torch

import paper_2505_18573_amd as e3
from paper_2505_18573_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("rows_per_prompt", [2, 80])       # 16 rows: small-batch path; 640 rows: row blocks
def test_replays_match_eager(rows_per_prompt):
    V = 20_000
    w = wl.decode_step(DEV, seed=5, prompts=8, rollouts=rows_per_prompt, V=V)
    rows = w.logits.shape[0]
    g = torch.Generator(device=DEV).manual_seed(3)
    rewards = (torch.rand(rows, generator=g, device=DEV) < 0.5).float()
    offsets = torch.arange(0, rows + 1, rows_per_prompt, dtype=torch.int32, device=DEV)
    ws = e3.new_workspace(rows, V, DEV)

    def alloc():
        return dict(tok=torch.empty(rows, dtype=torch.int32, device=DEV),
                    lp=torch.empty(rows, device=DEV), ent=torch.empty(rows, device=DEV),
                    lp2=torch.empty(rows, device=DEV), ent2=torch.empty(rows, device=DEV),
                    hsum=torch.empty(1, dtype=torch.float64, device=DEV),
                    hcnt=torch.empty(1, dtype=torch.int64, device=DEV),
                    adv=torch.empty(rows, device=DEV),
                    rtok=torch.empty(rows, dtype=torch.int32, device=DEV),
                    rlp=torch.empty(rows, device=DEV),
                    kept=torch.empty(rows, dtype=torch.int32, device=DEV))

    def run(o):
        e3.e3_grpo_advantages(rewards, offsets, 0, 0.0, adv_out=o["adv"])
        e3.e3_sample_entropy(w.logits, w.tau_rows, 1.0, seed=4, row_base=9, token_out=o["tok"],
                             logp_out=o["lp"], entropy_out=o["ent"], workspace=ws)
        e3.e3_logprob_entropy(w.logits, o["tok"], None, w.tau_rows, 1.0, logp_out=o["lp2"],
                              entropy_out=o["ent2"], entropy_sum_out=o["hsum"],
                              entropy_count_out=o["hcnt"], workspace=ws)
        e3.e3_sample_restricted(w.logits, w.tau_rows, 1.0, 40, 0.9, seed=4, row_base=9,
                                token_out=o["rtok"], logp_out=o["rlp"], kept_out=o["kept"])

    eager = alloc()
    run(eager)
    torch.cuda.synchronize()

    out = alloc()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(out)                                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(out)
    for replay in range(4):
        for t in out.values():
            t.zero_()                                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in eager:
            assert torch.equal(out[name], eager[name]), (replay, name)
