"""Command line front end (host only, no GPU needed): inspect a reconfiguration plan.

    python -m paper_2312_05181_amd plan --layers 24 --hidden 2048 --heads 16 --ffn 8192 --vocab 50304 \\
        --src 4,2,1 --dst 2,4,1
    python -m paper_2312_05181_amd manifest --layers 2 --hidden 256 --heads 4 --ffn 1024 --vocab 1024 \\
        --src 2,1,1 --dst 4,2,1 --side dst --rank 3
"""
from __future__ import annotations

import argparse
import json
import sys

from . import binding as B
from . import tpx_param_name, tpx_plan


def _cfg(text: str, stages, qkv, transposed, shard_kinds) -> dict:
    t, p, d = (int(x) for x in text.split(","))
    out = dict(T=t, P=p, D=d, qkv_layout=qkv, w_transposed=transposed, shard_kinds=shard_kinds)
    if stages:
        out["stage_first_layer"] = tuple(int(x) for x in stages.split(","))
    return out


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(prog="python -m paper_2312_05181_amd")
    ap.add_argument("command", choices=["plan", "manifest"])
    ap.add_argument("--layers", type=int, required=True)
    ap.add_argument("--hidden", type=int, required=True)
    ap.add_argument("--heads", type=int, required=True)
    ap.add_argument("--ffn", type=int, required=True)
    ap.add_argument("--vocab", type=int, required=True)
    ap.add_argument("--max-pos", type=int, default=1024)
    ap.add_argument("--vocab-divisor", type=int, default=0)
    ap.add_argument("--state-bytes", default="2,4,4,4", help="element bytes of each state kind")
    ap.add_argument("--tied-head", action="store_true")
    ap.add_argument("--src", required=True, help="T,P,D")
    ap.add_argument("--dst", required=True, help="T,P,D")
    ap.add_argument("--src-stages", default=None, help="P+1 layer boundaries")
    ap.add_argument("--dst-stages", default=None)
    ap.add_argument("--src-qkv", type=int, default=0)
    ap.add_argument("--dst-qkv", type=int, default=0)
    ap.add_argument("--src-transposed", type=int, default=0)
    ap.add_argument("--dst-transposed", type=int, default=0)
    ap.add_argument("--src-shard-kinds", type=int, default=0, help="bit k: state kind k is sharded over the D replicas")
    ap.add_argument("--dst-shard-kinds", type=int, default=0)
    ap.add_argument("--side", choices=["src", "dst"], default="dst")
    ap.add_argument("--rank", type=int, default=0)
    a = ap.parse_args(argv)
    model = dict(n_layers=a.layers, hidden=a.hidden, n_heads=a.heads, ffn=a.ffn, vocab_true=a.vocab, max_pos=a.max_pos,
                 vocab_divisor=a.vocab_divisor, state_elem_bytes=tuple(int(x) for x in a.state_bytes.split(",")),
                 tied_head=a.tied_head)
    try:
        plan = tpx_plan(model, _cfg(a.src, a.src_stages, a.src_qkv, a.src_transposed, a.src_shard_kinds),
                        _cfg(a.dst, a.dst_stages, a.dst_qkv, a.dst_transposed, a.dst_shard_kinds))
    except B.TpxError as e:
        print(str(e), file=sys.stderr)
        return 1
    if a.command == "plan":
        out = dict(plan.stats())
        out["src_buffer_bytes"] = [plan.buffer_bytes(0, r) for r in range(plan.num_buffers(0))]
        out["dst_buffer_bytes"] = [plan.buffer_bytes(1, r) for r in range(plan.num_buffers(1))]
        out["workspace_bytes"] = plan.workspace_bytes()
        out["traffic_bytes_src_to_dst"] = plan.traffic()
        print(json.dumps(out))
    else:
        side = 0 if a.side == "src" else 1
        for e in plan.manifest(side, a.rank):
            nd = e.ndim
            print(f"/{a.rank}/{'layer%d/' % e.layer if e.layer >= 0 else ''}{tpx_param_name(e.name)}[kind {e.kind}] "
                  f"offset {e.offset} bytes {e.nbytes} box {list(zip(e.lo[:nd], e.hi[:nd]))} of {list(e.full_shape[:nd])} "
                  f"stored in axis order {list(e.perm[:nd])}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
