"""Times a whole speculative-sampling cycle of the hot path with the stop decision on the device.

One cycle = t_max = 8 draft-call expansions with the prediction model fused in (the root alone,
then k = 10 rows; V = 128256; the first call starts the cycle, no radar_cycle_begin), rerank to 60 nodes, one layer of tree attention
(2048-token prefix, 32/8 heads, D = 128) and the sampled verify walk.  It is enqueued either call
by call (argument marshalling done beforehand) or as one captured HIP graph, and the drafting is
scripted to stop after 2, 4 or all 8 draft calls.  Inputs rotate through several sets (one graph
per set).  Prints one JSON line per (mode, stop) with the microseconds per cycle.

    python -m benchmarks.cycle_bench [--cycles 300] [--sets 4] [--batch B]

--batch B > 1 runs the cycles of B sequences together: batched draft calls (radar_draft_expand_batch with
every sequence's own state and decision), one batched rerank, attention and the verify walk over the B
sequences; a scripted stop then applies to every second sequence only, so that the batch is ragged.
"""
import argparse
import json
import sys
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cycles", type=int, default=300)
    ap.add_argument("--sets", type=int, default=4)
    ap.add_argument("--batch", type=int, default=1)
    args = ap.parse_args()
    import numpy as np
    import torch
    from paper_2512_14069_amd import binding as b, synth

    if not torch.cuda.is_available():
        print("cycle_bench: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda"
    c2, c3 = synth.config(2), synth.config(3)
    A = c2.attn
    V, k, N, t_max = c3.vocab, c3.k, c3.N, c3.expand_steps
    T = N + 1
    cap = k + (t_max - 1) * k * k
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.seed_for(3, 77))
    rng = np.random.default_rng(synth.seed_for(3, 78))
    pol = b.policy_params({n: torch.from_numpy(v).to(dev) for n, v in synth.policy_params(rng, k).items()})
    par_np, _, _ = synth.make_tree(rng, A.n_nodes[0], A.depths[0], A.k, V)
    attn_parents = torch.from_numpy(par_np[None].copy()).to(dev)
    ctx = torch.tensor(A.ctx_lens, dtype=torch.int32, device=dev)
    nn_ = torch.tensor(A.n_nodes, dtype=torch.int32, device=dev)

    class Cycle:
        def __init__(self):
            self.logits = [torch.log_softmax(torch.randn((1 if s == 0 else k, V), generator=gen, device=dev) * c3.logit_std,
                                             dim=-1).contiguous() for s in range(t_max)]
            self.uni = torch.zeros(t_max, dtype=torch.float32, device=dev)
            self.target = torch.randn((1, T, V), generator=gen, device=dev)
            self.acc_uni = torch.rand((1, T + 1), generator=gen, device=dev)
            self.q = torch.randn((A.B, A.T, A.Hq, A.D), generator=gen, device=dev).to(torch.bfloat16)
            self.kc = torch.randn((A.B, A.Hkv, A.S, A.D), generator=gen, device=dev).to(torch.bfloat16)
            self.vc = torch.randn((A.B, A.Hkv, A.S, A.D), generator=gen, device=dev).to(torch.bfloat16)
            self.attn_out = torch.empty((A.B, A.T, A.Hq, A.D), dtype=torch.bfloat16, device=dev)
            self.pool = b.DraftPool(cap)
            self.state = b.new_cycle_state()
            self.ps0 = torch.zeros(1, dtype=torch.float32, device=dev)
            self.pi0 = torch.full((1,), -1, dtype=torch.int32, device=dev)
            self.eouts = [b.ExpandOut(1 if s == 0 else k, k, dev) for s in range(t_max)]
            self.pout = b.PolicyOut(1, synth.POLICY_H, dev)
            self.tree = b.TreeOut(N, dev)
            self.ws = b.new_workspace(b.radar_draft_expand_workspace_bytes(b.expand_desc(k, V, k, 0, cap)))
            self.acc_ws = b.new_workspace(b.radar_verify_accept_workspace_bytes(
                b.accept_desc(1, T, V, T - 1, b.RADAR_ACCEPT_SAMPLE, 1.0)))
            self.acc_out = (torch.empty(1, dtype=torch.int32, device=dev), torch.empty((1, T), dtype=torch.int32, device=dev),
                            torch.empty(1, dtype=torch.int32, device=dev))
            adesc = b.attn_desc(self.q, self.kc)
            self.attn_ws = b.new_workspace(b.radar_tree_attention_workspace_bytes(adesc))
            self.adesc = adesc
            self.calls = self.prepare()

        def prepare(self):
            calls = []                                    # no radar_cycle_begin: the first draft call starts the cycle itself
            ps, pi, count_max = self.ps0, self.pi0, 0
            for s in range(t_max):
                decide = s + 1 < t_max
                calls.append(b.radar_draft_expand_cycle(
                    self.logits[s], ps, pi, k, self.pool, count_max, self.state, params=pol if decide else None,
                    h=self.pout.h if decide and s > 0 else None, c=self.pout.c if decide and s > 0 else None,
                    uniform=self.uni[s:s + 1] if decide else None, out=self.eouts[s],
                    policy_out=self.pout if decide else None, workspace=self.ws, prepared=True))
                count_max += (1 if s == 0 else k) * k
                ps, pi = self.eouts[s].frontier_scores, self.eouts[s].frontier_pool_idx
            calls.append(b.radar_draft_rerank_cycle(self.pool, self.state, cap, N, 1, out=self.tree, prepared=True))
            calls.append(b.radar_tree_attention(self.q, self.kc, self.vc, attn_parents, ctx, nn_, out=self.attn_out,
                                                desc=self.adesc, workspace=self.attn_ws, prepared=True))
            calls.append(b.radar_verify_accept(self.target, self.tree.tokens.view(1, -1), self.tree.parents.view(1, -1),
                                               self.tree.n_nodes, self.acc_uni, mode=b.RADAR_ACCEPT_SAMPLE, D_max=T - 1,
                                               out=self.acc_out, workspace=self.acc_ws, prepared=True))
            return calls

        def enqueue(self, calls=None):
            for c in (calls or self.calls):
                c()

        def script_stop(self, stop_after):
            u = torch.zeros(t_max, dtype=torch.float32)
            if 1 <= stop_after < t_max:
                u[stop_after - 1] = 0.999999
            self.uni.copy_(u)

    B = args.batch

    class BatchCycle:
        """The same cycle for B sequences at once; every array has a leading B."""

        def __init__(self):
            self.logits = [torch.log_softmax(torch.randn((B, 1 if s == 0 else k, V), generator=gen, device=dev) * c3.logit_std,
                                             dim=-1).contiguous() for s in range(t_max)]
            self.uni = torch.zeros((t_max, B), dtype=torch.float32, device=dev)
            self.target = torch.randn((B, T, V), generator=gen, device=dev)
            self.acc_uni = torch.rand((B, T + 1), generator=gen, device=dev)
            self.q = torch.randn((B, A.T, A.Hq, A.D), generator=gen, device=dev).to(torch.bfloat16)
            self.kc = torch.randn((B, A.Hkv, A.S, A.D), generator=gen, device=dev).to(torch.bfloat16)
            self.vc = torch.randn((B, A.Hkv, A.S, A.D), generator=gen, device=dev).to(torch.bfloat16)
            self.attn_out = torch.empty((B, A.T, A.Hq, A.D), dtype=torch.bfloat16, device=dev)
            self.attn_parents = attn_parents.expand(B, -1).contiguous()
            self.ctx, self.nn = ctx.expand(B).contiguous(), nn_.expand(B).contiguous()
            self.pool = b.DraftPool(cap, B=B)
            self.state = torch.zeros((B, 4), dtype=torch.int32, device=dev)
            self.ps0 = torch.zeros((B, 1), dtype=torch.float32, device=dev)
            self.pi0 = torch.full((B, 1), -1, dtype=torch.int32, device=dev)
            self.roots = torch.ones(B, dtype=torch.int32, device=dev)
            self.eouts = [b.ExpandOut(1 if s == 0 else k, k, dev, B=B) for s in range(t_max)]
            self.pout = b.PolicyOut(B, synth.POLICY_H, dev)
            self.tree = b.TreeOut(N, dev, B=B)
            self.ws = b.new_workspace(b.radar_draft_expand_batch_workspace_bytes(b.expand_desc(k, V, k, 0, cap), B))
            self.acc_ws = b.new_workspace(b.radar_verify_accept_workspace_bytes(
                b.accept_desc(B, T, V, T - 1, b.RADAR_ACCEPT_SAMPLE, 1.0)))
            self.acc_out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty((B, T), dtype=torch.int32, device=dev),
                            torch.empty(B, dtype=torch.int32, device=dev))
            self.adesc = b.attn_desc(self.q, self.kc)
            self.attn_ws = b.new_workspace(b.radar_tree_attention_workspace_bytes(self.adesc))
            self.calls = self.prepare()

        def prepare(self):
            calls = []
            ps, pi, count_max = self.ps0, self.pi0, 0
            for s in range(t_max):
                decide = s + 1 < t_max
                calls.append(b.radar_draft_expand_batch(
                    self.logits[s], ps, pi, k, self.pool, states=self.state, pool_count_max=count_max,
                    params=pol if decide else None, h=self.pout.h if decide and s > 0 else None,
                    c=self.pout.c if decide and s > 0 else None, uniform=self.uni[s] if decide else None,
                    out=self.eouts[s], policy_out=self.pout if decide else None, workspace=self.ws, prepared=True))
                count_max += (1 if s == 0 else k) * k
                ps, pi = self.eouts[s].frontier_scores, self.eouts[s].frontier_pool_idx
            calls.append(b.radar_draft_rerank_batch(self.pool, N, self.roots, states=self.state, pool_count_max=cap,
                                                    out=self.tree, prepared=True))
            calls.append(b.radar_tree_attention(self.q, self.kc, self.vc, self.attn_parents, self.ctx, self.nn,
                                                out=self.attn_out, desc=self.adesc, workspace=self.attn_ws, prepared=True))
            calls.append(b.radar_verify_accept(self.target, self.tree.tokens, self.tree.parents, self.tree.n_nodes, self.acc_uni,
                                               mode=b.RADAR_ACCEPT_SAMPLE, D_max=T - 1, out=self.acc_out, workspace=self.acc_ws,
                                               prepared=True))
            return calls

        def enqueue(self, calls=None):
            for c in (calls or self.calls):
                c()

        def script_stop(self, stop_after):
            u = torch.zeros((t_max, B), dtype=torch.float32)
            if 1 <= stop_after < t_max:
                u[stop_after - 1, ::2] = 0.999999          # every second sequence stops there, the others run on
            self.uni.copy_(u)

    if B > 1:
        Cycle = BatchCycle
    cycles = [Cycle() for _ in range(args.sets)]
    graphs = []
    side = torch.cuda.Stream()
    for cy in cycles:
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            cy.enqueue(cy.prepare())                       # a prepared call keeps the stream it was made on
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            held = cy.prepare()                            # made on the capture stream
            cy.enqueue(held)
        graphs.append((g, held))

    n = args.cycles
    for stop_after in (t_max, 4, 2):
        for cy in cycles:
            cy.script_stop(stop_after)
        for mode in ("calls", "graph"):
            run = (lambda i: cycles[i % len(cycles)].enqueue()) if mode == "calls" else (lambda i: graphs[i % len(graphs)][0].replay())
            for i in range(20):
                run(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(n):
                run(i)
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) / n * 1e6
            st = cycles[0].state.cpu().tolist()
            extra = {}
            if B > 1:                                      # report the batch: sequence 0 stops, sequence 1 does not
                extra = {"batch": B, "us_per_cycle_and_sequence": round(us / B, 2),
                         "draft_calls_run_per_sequence": [r[2] for r in st][:8]}
                st = st[0]
            print(json.dumps({"mode": mode, **extra, "draft_calls_allowed": t_max, "stop_after": stop_after,
                              "draft_calls_run": st[2], "pool_count": st[1], "us_per_cycle": round(us, 2),
                              "launches_per_cycle": (2 * t_max - 1 if B > 1 else t_max) + 1 + 2 + 1, "cycles": n,
                              "workload": "c3 expand chain (V=%d, k=%d, fused prediction model) + rerank N=%d + one c2 attention layer + sampled accept" % (V, k, N)}),
                  flush=True)


if __name__ == "__main__":
    main()
