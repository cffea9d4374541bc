"""amla_decode under HIP graph capture: the entry point allocates nothing, synchronises nothing and
records no memset, so a caller may capture it once and replay it.  The graph is replayed several times
with eager work and synchronisations in between, and every replay is compared with the eager result."""
import numpy as np
import pytest

from test_gpu_parity import ADD, MUL, env, to_dev  # noqa: F401

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("variant,splits,flags", [(ADD, 1, 0), (MUL, 4, 0), (ADD, 3, 8), (ADD, 4, 128)])
def test_replays_of_a_captured_decode_match_the_eager_call(env, variant, splits, flags):
    torch, orc, amla, wl = env
    case = wl.make_case("graph", 71, batch=3, s_q=2, heads=128, seqlens=[700, 1300, 64])
    q, kv, tab, lens = to_dev(torch, case)
    out = torch.empty((case.batch, case.s_q, case.heads, 512), dtype=torch.bfloat16, device=q.device)
    lse = torch.empty((case.batch, case.s_q, case.heads), dtype=torch.float32, device=q.device)
    desc = amla.make_desc(case.batch, case.s_q, case.heads, case.num_blocks, case.max_blocks_per_seq, variant, splits, flags)
    ws = torch.empty(max(amla.amla_workspace_bytes(desc), 16), dtype=torch.uint8, device=q.device)

    def call():
        amla.amla_decode(q, kv, tab, lens, case.softmax_scale, out, lse, variant=variant, num_splits=splits,
                         flags=flags, workspace=ws)

    call()                                            # eager reference (also the warm-up torch asks for)
    torch.cuda.synchronize()
    want_out, want_lse = out.clone(), lse.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for replay in range(3):
        out.fill_(7.0)                                # eager work between the replays
        lse.fill_(-3.0)
        ws.random_(0, 255)                            # stale partials must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want_out), replay
        assert torch.equal(lse, want_lse), replay
