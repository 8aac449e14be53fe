"""Times the entry points that widen the hot path, at the 8B shape (V = 128256, k = 10, 61 tree rows):
acceptance-length distribution, prediction-model step (alone and fused into the expansion), the
expansion of 4, 16 and 64 sequences in one launch, and verification with draft distributions.  One JSON line per entry point with the per-kernel device
durations the library records (radar_profile_begin / radar_profile_end) and the algorithmic bytes.

    python -m benchmarks.rows_bench [--reps 100]
"""
import argparse
import json
import sys


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=100)
    args = ap.parse_args()
    import numpy as np
    import torch
    from paper_2512_14069_amd import binding as b, synth

    if not torch.cuda.is_available():
        print("rows_bench: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda"
    c3 = synth.config(3)
    V, k, N = c3.vocab, c3.k, c3.N
    T = N + 1
    rng = np.random.default_rng(synth.seed_for(3, 91))
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    def timed(name, calls, bytes_per_call, note):
        for _ in range(10):
            for c in calls:
                c()
        torch.cuda.synchronize()
        b.radar_profile_begin(args.reps * len(calls) * 4)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(args.reps):
            for c in calls:
                c()
        kern = b.radar_profile_end()
        e0.record()
        for _ in range(args.reps):
            for c in calls:
                c()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / args.reps
        print(json.dumps({"entry": name, "us_back_to_back": round(us, 2), "algorithmic_bytes": int(bytes_per_call),
                          "GBps_back_to_back": round(bytes_per_call / us / 1e3, 1),
                          "kernels_us": {n: round(v["mean_us"], 2) for n, v in kern.items()}, "note": note}), flush=True)

    # trees of the verify shape with sampled tokens
    par = [synth.make_tree(rng, T, 8, k, V)[0]]
    x = synth.sampled_draft_inputs(rng, par, V, T, std=2.0, noise=1.0, shared_rows=True)
    d = {n: to(v) for n, v in x.items()}

    desc = b.accept_desc(1, T, V, T - 1, b.RADAR_ACCEPT_SAMPLE, 1.0)
    ws = b.new_workspace(b.radar_verify_accept_workspace_bytes(desc))
    call = b.radar_accept_length_distribution(d["target_logits"], d["draft_tokens"], d["parents"], d["n_nodes"],
                                              workspace=ws, prepared=True)
    timed("radar_accept_length_distribution", [call], T * V * 4, "61 target rows read once")

    pw = synth.policy_params(rng, k)
    pp = b.policy_params({n: to(v) for n, v in pw.items()})
    pbytes = sum(v.nbytes for v in pw.values())
    conf = to(synth.policy_conf(rng, 1, k)[0])
    pout = b.PolicyOut(1, synth.POLICY_H, dev)
    call = b.radar_policy_step(conf, pp, pout.h, pout.c, out=pout, prepared=True)
    timed("radar_policy_step", [call], pbytes, "parameters read once (they stay in L2 between calls)")

    for F in (1, k):
        logits = to(synth.expand_logits(rng, F, V, c3.logit_std))
        ps, pi = torch.zeros(F, device=dev), torch.full((F,), -1, dtype=torch.int32, device=dev)
        pool = b.DraftPool(4096)
        ews = b.new_workspace(b.radar_draft_expand_workspace_bytes(b.expand_desc(F, V, k, 0, 4096)))
        eo = b.ExpandOut(F, k, dev)
        plain = b.radar_draft_expand(logits, ps, pi, k, pool, out=eo, workspace=ews, prepared=True)
        pool.count = 0
        fused = b.radar_draft_expand_policy(logits, ps, pi, k, pool, pp, pout.h, pout.c, out=eo, policy_out=pout,
                                            workspace=ews, prepared=True)
        pool.count = 0
        sep = b.radar_policy_step(eo.frontier_conf, pp, pout.h, pout.c, out=pout, prepared=True)
        timed("radar_draft_expand F=%d" % F, [plain], F * V * 4, "for comparison")
        timed("radar_draft_expand_policy F=%d" % F, [fused], F * V * 4 + pbytes, "expansion and decision in one launch")
        timed("radar_draft_expand + radar_policy_step F=%d" % F, [plain, sep], F * V * 4 + pbytes, "two launches")

    # one draft call for B sequences in one launch; inputs rotated through more memory than the caches hold
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.seed_for(3, 92))
    for B in (4, 16, 64):
        nsets = max(2, int(600e6 // (B * k * V * 4)) + 1)
        sets = [torch.log_softmax(torch.randn((B, k, V), generator=gen, device=dev) * c3.logit_std, dim=-1).contiguous()
                for _ in range(nsets)]
        ps = torch.zeros((B, k), device=dev)
        pi = torch.full((B, k), -1, dtype=torch.int32, device=dev)
        pool = b.DraftPool(k * k, B=B)
        bws = b.new_workspace(b.radar_draft_expand_batch_workspace_bytes(b.expand_desc(k, V, k, 0, k * k), B))
        eo = b.ExpandOut(k, k, dev, B=B)
        calls = []
        for lg in sets:
            pool.count = 0
            calls.append(b.radar_draft_expand_batch(lg, ps, pi, k, pool, out=eo, workspace=bws, prepared=True))
        # timed() runs the whole list per repetition: report per call
        args.reps, keep = max(1, args.reps // nsets), args.reps
        timed("radar_draft_expand_batch B=%d F=%d (%d calls)" % (B, k, nsets), calls, nsets * B * k * V * 4,
              "%d sequences per launch; time and bytes are for %d calls on different inputs" % (B, nsets))
        if B == 16:                                        # the same calls with the decision of every sequence in them
            poutB = b.PolicyOut(B, synth.POLICY_H, dev)
            poutB.h.zero_(); poutB.c.zero_()
            calls = []
            for lg in sets:
                pool.count = 0
                calls.append(b.radar_draft_expand_batch(lg, ps, pi, k, pool, params=pp, h=poutB.h, c=poutB.c, out=eo,
                                                        policy_out=poutB, workspace=bws, prepared=True))
            args.reps = max(1, keep // nsets)
            timed("radar_draft_expand_batch B=%d F=%d with the prediction model (%d calls)" % (B, k, nsets), calls,
                  nsets * (B * k * V * 4 + pbytes), "as above, with every sequence's continue / stop decision in the call")
        args.reps = keep
        del sets, calls
        torch.cuda.empty_cache()

    qd = b.accept_q_desc(1, T, T, V, T - 1)
    qws = b.new_workspace(b.radar_verify_accept_q_workspace_bytes(qd))
    for limit, label in ((0, "walk shared by 32 workgroups"), (-1, "walk by one workgroup")):
        call = b.radar_verify_accept_q(d["target_logits"], d["draft_logits"], d["draft_tokens"], d["parents"], d["n_nodes"],
                                       d["uniforms"], d["q_rows"], workspace=qws, prepared=True, walk_spin_limit=limit)
        used = len(set(x["q_rows"][0, 1:T].tolist()))
        timed("radar_verify_accept_q", [call], (T + used) * V * 4, label + "; %d target rows and %d draft rows read once by the statistics launch" % (T, used))


if __name__ == "__main__":
    main()
