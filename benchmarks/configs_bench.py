"""Times tree-verify attention and verify-accept at every full-size configuration (2: 8B verify,
4: 16 ragged sequences, 5: 70B-class, four sequences of 16384 cached rows), one JSON line per
(configuration, entry point, mode): time per call back to back on inputs rotated through more
memory than the caches hold, per-kernel device durations recorded by the library
(radar_profile_begin / radar_profile_end), algorithmic bytes and flops, and the fraction of the
roof that binds (HBM 8 TB/s; dense bf16 MFMA 2.5 PFLOP/s for attention at configuration 5).

    python -m benchmarks.configs_bench [--reps 30] [--configs 2,4,5] [--modes greedy,sampling]

Inputs are synthetic: the trees come from the seeded generators, tensors are drawn on the device
(timing does not depend on their values beyond the shape of the accepted path).
"""
import argparse
import json
import sys

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
COLD_BYTES = 600e6          # rotate each entry point's inputs through at least this much


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=30)
    ap.add_argument("--configs", default="2,4,5")
    ap.add_argument("--modes", default="greedy,sampling", help="verify-accept modes to time (none: attention only)")
    ap.add_argument("--attn-kps", type=int, default=0, help="cache rows per range of the attention call (0: the library's plan)")
    args = ap.parse_args()
    import numpy as np
    import torch
    from paper_2512_14069_amd import binding as b, synth

    if not torch.cuda.is_available():
        print("configs_bench: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda"
    gen = torch.Generator(device=dev)
    gen.manual_seed(20251214)

    def timed(calls):
        n = len(calls)
        for i in range(max(5, n)):
            calls[i % n]()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(args.reps):
            calls[i % n]()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / args.reps
        b.radar_profile_begin(args.reps * 4)
        for i in range(args.reps):
            calls[i % n]()
        torch.cuda.synchronize()
        kern = b.radar_profile_end()
        return us, {k: round(v["mean_us"], 2) for k, v in kern.items()}

    for cid in [int(x) for x in args.configs.split(",")]:
        cfg = synth.config(cid)
        A = cfg.attn
        B, T, V = A.B, A.T, cfg.vocab
        rng = np.random.default_rng(synth.seed_for(cid, 77))
        par = np.full((B, T), -1, np.int32)
        tok = np.zeros((B, T), np.int32)
        for i in range(B):
            nn = A.n_nodes[i]
            if nn > 1:
                p, t, _ = synth.make_tree(rng, nn, min(A.depths[i], nn - 1), A.k, V)
                par[i, :nn], tok[i, :nn] = p, t
        parents = torch.from_numpy(par).to(dev)
        tokens = torch.from_numpy(tok).to(dev)
        ctx = torch.tensor(A.ctx_lens, dtype=torch.int32, device=dev)
        n_nodes = torch.tensor(A.n_nodes, dtype=torch.int32, device=dev)
        rows = int(sum(A.n_nodes))

        # ---------------------------------------------------------------- attention
        kv_rows = sum(A.ctx_lens[i] + A.n_nodes[i] for i in range(B))
        kv_bytes = kv_rows * A.Hkv * A.D * 2 * 2
        qo_bytes = 2 * rows * A.Hq * A.D * 2
        flops = 4.0 * sum((A.ctx_lens[i] + A.n_nodes[i]) * A.n_nodes[i] for i in range(B)) * A.Hq * A.D
        set_bytes = 2 * B * A.Hkv * A.S * A.D * 2
        nsets = max(2, int(COLD_BYTES // set_bytes) + 1)
        out = torch.empty((B, T, A.Hq, A.D), dtype=torch.bfloat16, device=dev)
        sets = []
        for _ in range(nsets):
            q = torch.randn((B, T, A.Hq, A.D), generator=gen, device=dev).to(torch.bfloat16)
            kc = torch.randn((B, A.Hkv, A.S, A.D), generator=gen, device=dev).to(torch.bfloat16)
            vc = torch.randn((B, A.Hkv, A.S, A.D), generator=gen, device=dev).to(torch.bfloat16)
            sets.append((q, kc, vc))
        desc = b.attn_desc(sets[0][0], sets[0][1], keys_per_split=args.attn_kps)
        ws = b.new_workspace(b.radar_tree_attention_workspace_bytes(desc))
        calls = [b.radar_tree_attention(q, kc, vc, parents, ctx, n_nodes, out=out, desc=desc, workspace=ws, prepared=True)
                 for q, kc, vc in sets]
        us, kern = timed(calls)
        k_us = sum(kern.values())
        intensity = flops / (kv_bytes + qo_bytes)
        bound = "mfma" if intensity > MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBPS else "hbm"
        ach = flops / k_us / 1e6 if bound == "mfma" else (kv_bytes + qo_bytes) / k_us / 1e3
        peak = MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else HBM_PEAK_GBPS
        print(json.dumps({"config": cfg.name, "entry": "radar_tree_attention", "us_back_to_back": round(us, 1),
                          "kernels_us": kern, "algorithmic_bytes": int(kv_bytes + qo_bytes), "flops": int(flops),
                          "GBps": round((kv_bytes + qo_bytes) / k_us / 1e3, 1), "TFLOPps": round(flops / k_us / 1e6, 1),
                          "roofline": {"bound": bound, "achieved": round(ach, 1), "peak": peak,
                                       "unit": "TFLOP/s" if bound == "mfma" else "GB/s", "frac": round(ach / peak, 4)},
                          "keys_per_split": args.attn_kps, "sets": nsets}), flush=True)
        del sets, calls, out, ws
        torch.cuda.empty_cache()

        # ------------------------------------------------------------ verify-accept
        if not [m for m in args.modes.split(",") if m in ("greedy", "sampling")]:
            continue
        set_bytes = B * T * V * 4
        nsets = max(2, int(COLD_BYTES // set_bytes) + 1)
        logit_sets = []
        for _ in range(nsets):
            x = torch.randn((B, T, V), generator=gen, device=dev)
            u = torch.rand((B, T, V), generator=gen, device=dev).clamp_(1e-9, 1.0)
            x -= torch.log(-torch.log(u))                       # + Gumbel(0, 1)
            del u
            logit_sets.append(x)
        uniforms = torch.rand((B, T + 1), generator=gen, device=dev)
        alg = rows * V * 4
        for mode_name, mode in (("greedy", b.RADAR_ACCEPT_GREEDY), ("sampling", b.RADAR_ACCEPT_SAMPLE)):
            if mode_name not in args.modes.split(","):
                continue
            desc = b.accept_desc(B, T, V, T - 1, mode, 1.0)
            ws = b.new_workspace(b.radar_verify_accept_workspace_bytes(desc))
            outs = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty((B, T), dtype=torch.int32, device=dev),
                    torch.empty(B, dtype=torch.int32, device=dev))
            calls = [b.radar_verify_accept(x, tokens, parents, n_nodes, uniforms, mode=mode, temperature=1.0, out=outs,
                                           workspace=ws, prepared=True) for x in logit_sets]
            us, kern = timed(calls)
            k_us = sum(kern.values())
            print(json.dumps({"config": cfg.name, "entry": "radar_verify_accept", "mode": mode_name,
                              "us_back_to_back": round(us, 1), "kernels_us": kern, "rows_read": rows,
                              "algorithmic_bytes": int(alg), "GBps": round(alg / k_us / 1e3, 1),
                              "roofline": {"bound": "hbm", "achieved": round(alg / k_us / 1e3, 1), "peak": HBM_PEAK_GBPS,
                                           "unit": "GB/s", "frac": round(alg / k_us / 1e3 / HBM_PEAK_GBPS, 4)},
                              "sets": nsets}), flush=True)
            del calls, ws
        del logit_sets
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
