"""Timing of the ragged long-context sweep: 8 sequences (32/8 grouped-query heads, head_dim 128,
prefix lengths drawn once by seed from [512, 16384]), N = 5, G = W for W in {5, 10, 15, 20, 30},
once as one la_step_attention call per sequence and once as a single la_step_attention_batch
launch, each replayed as a HIP graph of four repetitions.

    python -m paper_2402_02057_amd.sweep

Prints, per W, both times, the algorithmic bytes and flops and the fraction of the roofline
(the larger of bytes / 8 TB/s and flops / 2.5 PFLOP/s over the measured time).
"""
import numpy as np
import torch

from . import binding, workloads as wl

HBM_PEAK = 8.0e12
MFMA_BF16_PEAK = 2.5e15


def main():
    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)

    def rb(*shape):
        return torch.randn(shape, device="cuda", generator=gen).bfloat16()
    print("prefix lengths", wl.ragged_prefix_lengths(), flush=True)
    for W in (5, 10, 15, 20, 30):
        seqs = []
        for i in range(wl.RAGGED_SEQS):
            s = wl.ragged_shape(i, W)
            T, H, KV, d, P = s.T, s.heads, s.kv_heads, s.head_dim, s.P
            seqs.append((s, rb(T, H, d), rb(KV, P, d), rb(KV, P, d), rb(T, KV, d), rb(T, KV, d),
                         torch.empty((T, H, d), device="cuda", dtype=torch.bfloat16)))

        descs = [dict(q=q, k_cache=k, v_cache=v, step_k=sk, step_v=sv, out=o, P=s.P) for s, q, k, v, sk, sv, o in seqs]
        s0 = seqs[0][0]

        def calls():
            for s, q, k, v, sk, sv, o in seqs:
                binding.la_step_attention(q, k, v, sk, sv, s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim, o)

        def batch():
            binding.la_step_attention_batch(descs, s0.W, s0.N, s0.G, s0.heads, s0.kv_heads, s0.head_dim)

        def measure(run, reps=4):
            run()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for _ in range(reps):
                    run()
            graph.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            times = []
            for _ in range(20):
                e0.record()
                graph.replay()
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1) * 1e-3 / reps)
            return float(np.median(times))
        t, tb = measure(calls), measure(batch)
        nbytes = sum(2 * s.P * s.kv_heads * s.head_dim * 2 + 2 * s.T * s.kv_heads * s.head_dim * 2 +
                     2 * s.T * s.heads * s.head_dim * 2 for s, *_ in seqs)
        flops = sum(4 * s.head_dim * s.heads * s.T * (s.P + s.T) for s, *_ in seqs)
        t_hbm, t_mfma = nbytes / HBM_PEAK, flops / MFMA_BF16_PEAK
        roof = max(t_hbm, t_mfma)
        print("W=%2d (T=%3d): 8 calls %6.1f us (%.1f %%), one launch %6.1f us (%.1f %%) | %.1f MB, %.1f GFLOP | "
              "roofline %.1f us (%s)" % (W, s0.T, t * 1e6, 100 * roof / t, tb * 1e6, 100 * roof / tb, nbytes / 1e6,
                                         flops / 1e9, roof * 1e6, "HBM" if t_hbm > t_mfma else "MFMA"), flush=True)


if __name__ == "__main__":
    main()
