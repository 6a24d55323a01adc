"""Run as a script in a fresh process (tests/test_gpu_parity.py starts it): the
process's FIRST decode-attention call is recorded into a HIP graph, with no
eager call of it before, then replayed and compared with an eager call made
afterwards.  Prints OK and exits 0 when the replays match bit for bit."""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

from paper_2410_15651_amd import binding as rb          # noqa: E402
from paper_2410_15651_amd import workloads as wl        # noqa: E402
import gpu_util as gu                                   # noqa: E402


def main():
    cfg = wl.small_variant(wl.config(5), batch=24, n_q_heads=32, n_kv_heads=4, len_lo=0, len_hi=700)
    lens = wl.seq_lengths(cfg)
    lens[2] = 0
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)              # arena calls only: no attention kernel has run yet
    k, v, table, dl = A.views()
    params = rb.attn_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, A.mpps,
                            wl.DTYPE_CODE[cfg.kv_dtype], out_dtype=rb.RLHF_F32)
    ws = torch.full((rb.rlhf_decode_attention_workspace_bytes(params),), 0xFF, dtype=torch.uint8, device=gu.DEV)
    out = torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device=gu.DEV)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        rb.rlhf_decode_attention(params, q, k, v, table, dl, out, ws, stream=side)   # the first call of the process
    replays = []
    for _ in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        replays.append(out.clone())
    eager = torch.full_like(out, float("nan"))
    ws2 = torch.full_like(ws, 0xFF)
    rb.rlhf_decode_attention(params, q, k, v, table, dl, eager, ws2)
    torch.cuda.synchronize()
    assert torch.isfinite(eager).all() and (eager[lens == 0] == 0).all()
    for r in replays:
        assert int((r.view(torch.uint8) != eager.view(torch.uint8)).sum()) == 0
    A.close()
    print("OK", flush=True)


if __name__ == "__main__":
    main()
