#!/usr/bin/env python3
"""Benchmark: decode attention over a CommVQ-compressed KV cache on one MI355X.

One step = one commvq_decode_attn call (score, bins and output stages) over one batch of
synthetic input that is already resident in HBM.  Successive steps rotate through several
distinct copies of the codes and codebooks so that the rotated footprint exceeds the 256 MB
last-level cache and the code stream really comes from HBM.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X published HBM3E bandwidth
FP32_PEAK_TFLOPS = 157.3    # MI355X published fp32 peak (vector, and equally the fp32 matrix instructions)
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix peak
MFMA_I8_PEAK_TOPS = 5000.0      # MI355X published dense int8 matrix peak
LDS_PEAK_TBS = 157.3        # 256 CUs x 256 B/clk (ds_read_b128 without bank conflicts) x 2.4 GHz
COLD_FOOTPRINT = 640 << 20  # rotate through at least this many bytes of codes + codebooks


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--config", type=int, default=3,
                    help="workload 1..11 (3 = 8B-shaped layer, 128K context, 1-bit; 6, 7 = the same layer with keys in "
                         "the paper's paired format, R = 11 / 21; 8, 9 = the same layer with values in the paper's binary "
                         "form, N_c = 1024 / 2048; 10, 11 = both: the paper's 1-bit and 2-bit settings)")
    ap.add_argument("--context-tokens", type=int, default=None,
                    help="shrink every context of the workload to at most this many tokens (short-context plans: score "
                         "tiles cut along the codebook slices); the workload name then ends in _ctx<N>")
    ap.add_argument("--batch", type=int, default=None,
                    help="with --context-tokens N: a serving-like batch of this many sequences of the workload's layer, "
                         "lengths uniform on [N/2, N] (index-form configurations 2..5); the workload name then ends in _b<B>_ctx<N>")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--warm", action="store_true", help="do not rotate buffers (cache-resident numbers)")
    ap.add_argument("--no-stage-events", action="store_true", help="do not bracket the stages with HIP events")
    ap.add_argument("--stage-event-interval", type=int, default=8,
                    help="bracket the stages of every N-th timed call with HIP events (an event between two kernels "
                         "costs ~5 us of GPU time, 11 us per call with all four: N = 1 times every launch and "
                         "lowers the whole-call rate by 8 %%, N = 8 by 1 %%)")
    ap.add_argument("--no-prepack", action="store_true",
                    help="re-lay the key codebook inside every call instead of once before the timed region")
    ap.add_argument("--graph", action="store_true",
                    help="replay each call from a captured HIP graph (one graph per rotated buffer copy); stage "
                         "timings then come from an eager pass after the timed region")
    ap.add_argument("--position-free", action="store_true",
                    help="no RoPE between query and keys: scores through the scalar look-up table kernel (HBM-bound)")
    ap.add_argument("--what", choices=["decode_attn", "encode", "em"], default="decode_attn",
                    help="encode: time the key encoder (cache append) on --encode-tokens new tokens instead; "
                         "em: time one iteration of the EM codebook learner (64 sub-spaces, --em-points points each)")
    ap.add_argument("--em-points", type=int, default=8192)
    ap.add_argument("--em-shared", action="store_true",
                    help="with --what em: the 64 sub-spaces share one code per vector (the learner of the paired key table)")
    ap.add_argument("--encode-tokens", type=int, default=4096)
    return ap.parse_args()


def bench_em(args):
    """One step = one EM iteration (E step + M step) for the 64 sub-spaces of a head, N_c' = 64."""
    import numpy as np
    import torch

    from paper_2506_18879_amd import binding as B
    from paper_2506_18879_amd import synth

    torch.cuda.set_device(0)
    J, N, Nc, T = 64, args.em_points, 64, 0.2
    rng = np.random.default_rng(synth.BASE_SEED)
    data = rng.standard_normal((J, N, 2)).astype(np.float32)
    phi0 = (rng.standard_normal((J, Nc, 2)) * 0.5).astype(np.float32)
    d = torch.from_numpy(data).cuda()
    nb = B.commvq_em_workspace_bytes(J, N, Nc)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    sp = int(torch.cuda.current_stream().cuda_stream)
    p = torch.from_numpy(phi0).cuda()
    for _ in range(args.warmup):
        p.copy_(torch.from_numpy(phi0))
        B.commvq_em_step(d, J, N, Nc, T, p, ws, nb, sp)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    p.copy_(torch.from_numpy(phi0))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        B.commvq_em_step(d, J, N, Nc, T, p, ws, nb, sp)   # successive iterations of the same run
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / args.steps
    kernel_ms = e0.elapsed_time(e1) / args.steps
    # per (point, centre) pair: distance (5 flop + sqrt) and exp in both passes, 5 more to accumulate
    flop = J * N * Nc * Nc * (2 * 8 + 5)
    tf = flop / (kernel_ms * 1e-3) / 1e12
    result = {"metric": "EM codebook learner: calibration points/sec per head (one iteration, 64 sub-spaces)",
              "value": round(N / (ms * 1e-3), 1), "unit": "points/s per head", "n_gpus": 1, "steps": args.steps,
              "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": "f32", "data": "synthetic",
              "config": {"workload": f"em_64_subspaces_{N}_points_64_levels", "centres_per_subspace": Nc * Nc,
                         "temperature": T},
              "roofline": {"kernel": "k_em_norm + k_em_accum", "bound": "alu", "achieved": round(tf, 3),
                           "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / FP32_PEAK_TFLOPS, 4),
                           "traffic": None, "kernel_ms": round(kernel_ms, 5)}}
    if not args.no_cpu_baseline:
        import oracle
        m = min(N, 1024)
        c0 = time.perf_counter()
        oracle.em_step(data[0, :m], phi0[0], temperature=T)
        c1 = time.perf_counter()
        result["cpu_baseline"] = {"value": round(m / 64 / (c1 - c0), 1), "unit": "points/s per head", "cores": 1,
                                  "kind": "oracle", "sample": f"one sub-space, {m} points, {c1 - c0:.1f} s wall "
                                                              "(a head has 64 sub-spaces)"}
    print(json.dumps(result))


def bench_em_shared(args):
    """One step = one EM iteration for a head whose 64 sub-spaces share one code per vector, N_c' = 64."""
    import numpy as np
    import torch

    from paper_2506_18879_amd import binding as B
    from paper_2506_18879_amd import synth

    torch.cuda.set_device(0)
    J, N, Nc, T = 64, args.em_points, 64, 2.0
    rng = np.random.default_rng(synth.BASE_SEED)
    data = rng.standard_normal((N, J, 2)).astype(np.float32)
    phi0 = (rng.standard_normal((J, Nc, 2)) * 0.5).astype(np.float32)
    d = torch.from_numpy(data).cuda()
    nb = B.commvq_em_shared_workspace_bytes(J, N, Nc)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    sp = int(torch.cuda.current_stream().cuda_stream)
    p = torch.from_numpy(phi0).cuda()
    for _ in range(args.warmup):
        p.copy_(torch.from_numpy(phi0))
        B.commvq_em_step_shared(d, J, N, Nc, T, p, ws, nb, sp)
    p.copy_(torch.from_numpy(phi0))
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        B.commvq_em_step_shared(d, J, N, Nc, T, p, ws, nb, sp)   # successive iterations of the same run
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / args.steps
    kernel_ms = e0.elapsed_time(e1) / args.steps
    # per point: 2 x Nc dot products of length 2J, then four sweeps over the Nc^2 centres (4 adds + sqrt, and exp in three)
    flop = N * (2 * Nc * 2 * 2 * J + Nc * Nc * (4 * 6 + 3 * 3))
    tf = flop / (kernel_ms * 1e-3) / 1e12
    result = {"metric": "EM codebook learner, one code per vector: calibration vectors/sec per head (one iteration)",
              "value": round(N / (ms * 1e-3), 1), "unit": "vectors/s per head", "n_gpus": 1, "steps": args.steps,
              "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": "f32", "data": "synthetic",
              "config": {"workload": f"em_shared_group64_{N}_vectors_64_levels", "centres": Nc * Nc, "temperature": T},
              "roofline": {"kernel": "k_ems_assign", "bound": "alu", "achieved": round(tf, 3), "peak": FP32_PEAK_TFLOPS,
                           "unit": "TFLOP/s", "frac": round(tf / FP32_PEAK_TFLOPS, 4), "traffic": None,
                           "kernel_ms": round(kernel_ms, 5)}}
    if not args.no_cpu_baseline:
        import oracle
        m = min(N, 512)
        c0 = time.perf_counter()
        oracle.em_step_shared(data[:m], phi0, temperature=T)
        c1 = time.perf_counter()
        result["cpu_baseline"] = {"value": round(m / (c1 - c0), 1), "unit": "vectors/s per head", "cores": 1,
                                  "kind": "oracle", "sample": f"{m} vectors, {c1 - c0:.1f} s wall"}
    print(json.dumps(result))


def bench_encode(args):
    """One step = commvq_encode_keys over a chunk of new tokens (all KV heads) of the chosen workload's layer."""
    import numpy as np
    import torch

    from paper_2506_18879_amd import binding as B
    from paper_2506_18879_amd import synth
    from paper_2506_18879_amd.device import DecodeAttention, to_device

    torch.cuda.set_device(0)
    w = synth.config(args.config, max_len=64)
    assert w.dtype == "bf16", "the encoder benchmark uses the bf16 workloads"
    paired = w.key_format == "paired"
    levels = w.key_levels if paired else w.Mk
    K = 64 if paired else w.K
    rec = (12 * levels + 7) // 8 if paired else levels
    n = args.encode_tokens
    rng = np.random.default_rng(synth.BASE_SEED)
    keys = to_device(synth.f32_to_bf16_bits(rng.standard_normal((n, w.Hkv, w.d)).astype(np.float32)), True)
    kcb = to_device(w.key_codebooks, True)
    op = DecodeAttention(w)
    tables = torch.empty(B.commvq_encoder_table_bytes(op.handle), dtype=torch.uint8, device="cuda")
    cache = torch.zeros((w.Hkv, n, rec), dtype=torch.uint8, device="cuda")
    B.commvq_encoder_prepare(op.handle, kcb, tables)
    sp = op.stream_ptr()
    for _ in range(args.warmup):
        B.commvq_encode_keys(op.handle, keys, n, kcb, tables, cache, rec, n * rec, sp)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        B.commvq_encode_keys(op.handle, keys, n, kcb, tables, cache, rec, n * rec, sp)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / args.steps
    kernel_ms = e0.elapsed_time(e1) / args.steps
    # algorithmic work per (token, head, level): the dot products with the level's rows, the candidate scan
    flop = n * w.Hkv * levels * (2 * w.d * (2 * K if paired else K) + (5 * K * K if paired else 2 * K) + 2 * w.d)
    tf = flop / (kernel_ms * 1e-3) / 1e12
    roof = {"kernel": "k_encode_lds" if paired else "k_encode_dma", "bound": "alu", "achieved": round(tf, 3),
            "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / FP32_PEAK_TFLOPS, 4), "traffic": None,
            "kernel_ms": round(kernel_ms, 5)}
    if not paired and n >= 64:
        # 64 tokens per workgroup: the dot products run as bf16 MFMA on an exact three-way split of the fp32 residual
        mf = 3 * n * w.Hkv * levels * 2 * w.d * K / (kernel_ms * 1e-3) / 1e12
        roof = {"kernel": "k_encode_batch", "bound": "mfma", "achieved": round(mf, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(mf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                "kernel_ms": round(kernel_ms, 5)}
    if paired and n >= 64:
        # 64 tokens per workgroup: the 2 x 64 dot products of a level run as bf16 MFMA (three exact parts), the scan
        # of the 64 x 64 centres is one add and one minimum per centre on the vector ALU (peak counts fused,
        # packed operations: plain ones reach a quarter of it) and reads each cross term from LDS once per token
        ops = n * w.Hkv * levels * 2 * K * K / (kernel_ms * 1e-3) / 1e12
        lds = n * w.Hkv * levels * 4 * K * K / (kernel_ms * 1e-3) / 1e12
        roof = {"kernel": "k_encode_pair_batch", "bound": "alu", "achieved": round(ops, 2), "peak": FP32_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(ops / FP32_PEAK_TFLOPS, 4), "traffic": None,
                "kernel_ms": round(kernel_ms, 5),
                "lds_view": {"cross_term_TBs": round(lds, 1), "peak_TBs": LDS_PEAK_TBS, "frac": round(lds / LDS_PEAK_TBS, 3)}}
    result = {"metric": "key-encode new tokens/sec per layer (cache append)", "value": round(n / (ms * 1e-3), 1),
              "unit": "tokens/s per layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
              "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
              "dtype": "f32", "data": "synthetic",
              "config": {"workload": f"encode_{n}_tokens_of_{w.name}", "kv_heads": w.Hkv, "head_dim": w.d,
                         "key_format": w.key_format, "levels": levels, "centres_per_level": K * K if paired else K},
              "roofline": roof}
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        m = min(n, 16 if paired else 256)
        kf = synth.bf16_bits_to_f32(keys[:m, 0].view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
        c0 = time.perf_counter()
        oracle.encode_keys(kf, w.as_f64("key_codebooks")[0], paired=paired)
        c1 = time.perf_counter()
        result["cpu_baseline"] = {"value": round(m / w.Hkv / (c1 - c0), 1), "unit": "tokens/s per layer", "cores": 1,
                                  "kind": "oracle", "sample": f"{m} vectors of one KV head, {c1 - c0:.1f} s wall"}
    print(json.dumps(result))
    op.close()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the path shards by KV head or sequence without any exchange "
              "(each KV head or sequence is an independent unit), but no multi-GPU launch is provided. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if args.what == "encode":
        return bench_encode(args)
    if args.what == "em":
        return bench_em_shared(args) if args.em_shared else bench_em(args)
    import numpy as np
    import torch

    from paper_2506_18879_amd import binding as B
    from paper_2506_18879_amd import synth
    from paper_2506_18879_amd.device import DecodeAttention, DeviceWorkload

    torch.cuda.set_device(0)
    w = synth.config(args.config, max_len=args.context_tokens)
    if args.context_tokens is not None:
        w.name = f"{w.name}_ctx{args.context_tokens}"
    if args.batch is not None:
        assert args.context_tokens is not None and w.key_format == "indexed" and w.dtype == "bf16", "--batch: configurations 2..5 with --context-tokens"
        lens = np.random.Generator(np.random.PCG64(args.batch * 1000003 + args.context_tokens)).integers(
            max(1, args.context_tokens // 2), args.context_tokens, size=args.batch, endpoint=True)
        base = w.name.split("_ctx")[0]
        w = synth.make_workload(f"{base}_b{args.batch}_ctx{args.context_tokens}", B=args.batch, Hq=w.Hq, Hkv=w.Hkv, seqlens=lens,
                                Mk=w.Mk, Mv=w.Mv, dtype=w.dtype, seed=250618879 + 100 * args.config, code_dist=w.code_dist)
    T, G = w.total_tokens, w.Hq // w.Hkv
    esz = 2 if w.dtype == "bf16" else 4
    code_bytes = w.key_codes.nbytes + w.val_codes.nbytes
    cb_bytes = w.key_codebooks.nbytes + w.val_codebooks.nbytes
    per_copy = code_bytes + cb_bytes
    n_copies = 1 if args.warm else max(2, -(-COLD_FOOTPRINT // per_copy))

    base = DeviceWorkload(w)
    copies = [base]
    for _ in range(n_copies - 1):
        c = DeviceWorkload.__new__(DeviceWorkload)
        c.__dict__.update(base.__dict__)
        c.key_codes, c.val_codes = base.key_codes.clone(), base.val_codes.clone()
        c.key_codebooks, c.val_codebooks = base.key_codebooks.clone(), base.val_codebooks.clone()
        copies.append(c)
    op = DecodeAttention(w, position_free=args.position_free)
    stream = torch.cuda.current_stream()
    # the key codebooks are per-layer constants: their re-layout for the score kernel is done once, outside
    # the timed region (commvq_pack_key_codebooks); --no-prepack keeps it inside every call instead
    prepacked = w.dtype == "bf16" and not args.no_prepack and not args.position_free
    if prepacked:
        for c in copies:
            op.pack_key_codebooks(c)
            op.pack_value_codebooks(c)   # (used by the batched output kernel only: 16 or more output rows per KV head)
        torch.cuda.synchronize()

    for i in range(args.warmup):
        op(copies[i % n_copies])
    torch.cuda.synchronize()
    if args.graph:
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for c in copies:
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr, stream=side):
                    op(c)
                graphs.append(gr)
        torch.cuda.synchronize()
        for i in range(args.warmup):
            graphs[i % n_copies].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[i % n_copies].replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        B.commvq_profile_enable(op.handle, True)   # stage timings: eager calls outside the timed region
        for i in range(min(args.steps, 28)):
            op(copies[i % n_copies])
        torch.cuda.synchronize()
    else:
        B.commvq_profile_enable(op.handle, 0 if args.no_stage_events else args.stage_event_interval)
        t0 = time.perf_counter()
        for i in range(args.steps):
            op(copies[i % n_copies])
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    stage_ms, n_prof = B.commvq_profile_read(op.handle)
    B.commvq_profile_enable(op.handle, False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = T / (ms_per_step * 1e-3)
    assert torch.isfinite(op.out).all()

    # dominant kernel: the score kernel (k_score_mfma for bf16 codebooks; with the codebook packed ahead of
    # time it is the only kernel of the score stage, so the stage's HIP events time exactly its launches).
    # Algorithmic work per launch (per (token, KV head) unit): M_k*d additions of the gather-sum, 3d for the
    # rotation, 2dG for the G dot products.
    score_s = stage_ms[0] * 1e-3
    units = T * w.Hkv
    score_flops = units * w.d * (w.Mk + 3 + 2 * G)
    achieved_tflops = score_flops / score_s / 1e12 if score_s > 0 else 0.0
    paired = w.key_format == "paired"
    kname = "k_score_pair" if paired else ("k_score_mfma" if w.dtype == "bf16" else "k_score")
    if args.position_free:
        kname = "k_score_lut"
    # HBM bytes per launch from rocprofv3 counter passes (FETCH_SIZE, WRITE_SIZE) of this same command: counters
    # cannot be read from inside the process, so the figures are the stored ones of the committed passes
    traffic, stored = None, {}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            stored = json.load(open(tpath)).get(w.name, {})
            traffic = stored.get(kname)
        except Exception:
            traffic, stored = None, {}
    traffic_source = ("stored: profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE passes over this command)"
                      if traffic is not None else None)
    key_stream_gbs = w.key_codes.nbytes / score_s / 1e9 if score_s > 0 else 0.0
    # the pipes the kernel actually loads: codeword pieces gathered from LDS, and the matrix instructions that
    # sum them: 256 issued flop per 16-byte piece (mostly multiplications by zero), as one dense 16x16x32 bf16 MFMA
    # per 64 pieces (paired keys) or one structured-sparse 16x16x64 per 128 (index form; twice the dense rate)
    gather_bytes = units * w.Mk * w.d * esz
    gather_tbs = gather_bytes / score_s / 1e12 if score_s > 0 else 0.0
    mfma_tflops = (gather_bytes / 16 / 64 * 16384) / score_s / 1e12 if (score_s > 0 and w.dtype == "bf16") else 0.0
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if paired else 2.0 * MFMA_BF16_PEAK_TFLOPS
    roofline = {"kernel": kname, "bound": "alu", "achieved": round(achieved_tflops, 3), "peak": FP32_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved_tflops / FP32_PEAK_TFLOPS, 4), "traffic": traffic,
                "traffic_source": traffic_source,
                "kernel_ms": round(stage_ms[0], 5), "launches_averaged": n_prof,
                "launches_sampled": ("every call of a separate eager run" if args.graph else
                                     f"every {args.stage_event_interval}th call of the timed region"),
                "timed_region_includes": ("index unpacking (k_unpack_pairs) + k_score_pair" if paired else
                                          "k_score_mfma + k_score_combine" if prepacked and op.plan.score_slice_groups > 1 else
                                          "k_score_mfma only" if prepacked else "codebook re-layout (k_prep) + score kernel"),
                "lds_gather_view": {"codeword_bytes_TBs": round(gather_tbs, 2), "peak_TBs": LDS_PEAK_TBS,
                                    "frac": round(gather_tbs / LDS_PEAK_TBS, 4)},
                "mfma_view": {"issued_bf16_TFLOPs": round(mfma_tflops, 1), "peak_TFLOPs": mfma_peak,
                              "instruction": "v_mfma_f32_16x16x32_bf16" if paired else "v_smfmac_f32_16x16x64_bf16 (sparse first operand)",
                              "frac": round(mfma_tflops / mfma_peak, 4)},
                "hbm_view": {"key_code_stream_GBs": round(key_stream_gbs, 1),
                             "frac_of_hbm_peak": round(key_stream_gbs / HBM_PEAK_GBS, 4)}}

    if args.position_free:
        # scalar-LUT scores: the stage streams the key codes in and the logits out; judged against HBM
        lut_bytes = w.key_codes.nbytes + T * w.Hq * 4
        gbs = lut_bytes / score_s / 1e9 if score_s > 0 else 0.0
        roofline = {"kernel": kname, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None, "kernel_ms": round(stage_ms[0], 5),
                    "launches_averaged": n_prof, "timed_region_includes": "k_lut_build + k_score_lut"}
    # the two stages that can be judged against HBM: the value stage streams the value codes (and re-reads the
    # logits), the output stage reads the bins of every value split and the value codebook once per sequence
    bins_s, out_s = stage_ms[1] * 1e-3, stage_ms[2] * 1e-3
    val_gbs = w.val_codes.nbytes / bins_s / 1e9 if bins_s > 0 else 0.0
    bins_alg = w.val_codes.nbytes + T * w.Hq * 4
    vbin = w.val_format == "binary"
    val_rows = w.val_bits if vbin else w.Mv * w.K            # bins per query head
    out_alg = op.plan.value_splits * w.B * w.Hq * val_rows * 4 + w.B * w.val_codebooks.nbytes
    stage_views = {
        "value_stream_view": {"stage": "k_vbits" if vbin else "k_bins", "value_code_GBs": round(val_gbs, 1),
                              "frac_of_hbm_peak": round(val_gbs / HBM_PEAK_GBS, 4),
                              "with_logits_read_GBs": round(bins_alg / bins_s / 1e9, 1) if bins_s > 0 else 0.0,
                              "with_logits_read_and_bins_written_GBs": round((bins_alg + op.plan.value_splits * w.B * w.Hq * val_rows * 4) / bins_s / 1e9, 1) if bins_s > 0 else 0.0,
                              "counter_bytes": stored.get("k_vbits" if vbin else "k_bins"), "stage_ms": round(stage_ms[1], 5)},
        "output_view": {"stage": "k_out (k_out_mfma for batches) + k_out_final", "bins_and_codebook_GBs": round(out_alg / out_s / 1e9, 1) if out_s > 0 else 0.0,
                        "frac_of_hbm_peak": round(out_alg / out_s / 1e9 / HBM_PEAK_GBS, 4) if out_s > 0 else 0.0,
                        "counter_bytes": sum(v for k, v in stored.items() if k.startswith("k_out") and isinstance(v, (int, float))) or None,
                        "stage_ms": round(stage_ms[2], 5)}}
    if vbin and bins_s > 0:
        # Softmax(A) S_V as a dense product: heads (padded to 32 per workgroup) x N_c x tokens, four 8-bit digits
        heads = -(-w.Hq // 32) * 32
        i8_tops = 2.0 * 4 * heads * w.val_bits * T / bins_s / 1e12
        stage_views["value_stream_view"]["mfma_view"] = {
            "issued_int8_TOPs": round(i8_tops, 1), "peak_TOPs": MFMA_I8_PEAK_TOPS, "instruction": "v_mfma_i32_16x16x64_i8",
            "frac": round(i8_tops / MFMA_I8_PEAK_TOPS, 4),
            "algorithmic_TOPs": round(2.0 * w.Hq * w.val_bits * T / bins_s / 1e12, 1)}
    alg_bytes = per_copy + w.B * w.Hq * w.d * (esz + 4)
    call_counter = sum(v for k, v in stored.items() if isinstance(v, (int, float)) and (not k.startswith("k_prep") or not prepacked)) or None
    result = {
        "metric": "decode-attention context tokens/sec per layer at 128K; % of HBM roofline",
        "value": round(tokens_per_s, 1), "unit": "context tokens/s per layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32 arithmetic on bf16 storage" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.B, "q_heads": w.Hq, "kv_heads": w.Hkv, "head_dim": w.d,
                   "context_tokens": T, "m_key": w.Mk, "m_val": w.Mv, "codewords": w.K, "storage": w.dtype,
                   "key_format": w.key_format, "key_levels": w.key_levels, "value_format": w.val_format,
                   "value_bits": w.val_bits, "position_free": bool(args.position_free),
                   "codes": w.code_dist, "score_tile_tokens": op.plan.score_split_len,
                   "score_slice_groups": op.plan.score_slice_groups, "value_split_tokens": op.plan.value_split_len,
                   "buffer_copies_rotated": n_copies,
                   "key_codebooks_packed_before_timed_region": prepacked, "value_codebooks_packed_before_timed_region": prepacked, "hip_graph_replay": bool(args.graph),
                   "cache_state": "warm" if args.warm else "cold (rotating copies > 256 MB LLC)"},
        "whole_call": {"code_stream_GBs": round(code_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                       "algorithmic_GBs": round((per_copy + w.B * w.Hq * w.d * (esz + 4)) / (ms_per_step * 1e-3) / 1e9, 1),
                       "code_stream_frac_of_hbm_peak": round(code_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                       "algorithmic_bytes": alg_bytes, "counter_bytes": call_counter,
                       "counter_over_algorithmic": round(call_counter / alg_bytes, 2) if call_counter else None,
                       "counter_source": traffic_source,
                       "stage_ms": {"scores": round(stage_ms[0], 5), "bins": round(stage_ms[1], 5),
                                    "output": round(stage_ms[2], 5)}},
        "roofline": roofline,
    }
    result["roofline"].update(stage_views)
    # what the memory system of this machine delivers to a plain streaming kernel: a device-to-device copy of 1 GiB (torch's
    # copy kernel; every byte read once and written once), as a measured companion to the published 8 TB/s
    try:
        n = 1 << 30
        src, dst = torch.empty(n, dtype=torch.uint8, device="cuda"), torch.empty(n, dtype=torch.uint8, device="cuda")
        src.zero_()
        for _ in range(2):
            dst.copy_(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 5 * 2 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst
        result["whole_call"]["measured_copy_GBs"] = round(copy_gbs, 1)
        result["whole_call"]["code_stream_frac_of_measured_copy"] = round(result["whole_call"]["code_stream_GBs"] / copy_gbs, 4)
    except Exception:  # (a box without 2 GiB to spare: the figure is a companion, not part of the metric)
        result["whole_call"]["measured_copy_GBs"] = None

    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        # bounded sample: as many (sequence, KV head) units as threads, one unit per thread
        n_threads = min(16, os.cpu_count() or 1, w.B * w.Hkv)
        mask = np.zeros(w.B * w.Hkv, bool)
        mask[:n_threads] = True
        sample_tokens = sum(int(w.cu_seqlens[u // w.Hkv + 1] - w.cu_seqlens[u // w.Hkv]) for u in range(n_threads))
        if paired:  # the oracle reads the same records and table, as index form with 2R tied codebooks
            o_codes = oracle.paired_as_indexed(w.key_codes, w.key_levels, w.cu_seqlens, w.Hkv)
            o_kcb = oracle.tied_table_as_codebooks(w.as_f64("key_codebooks"), K=w.K)
        else:
            o_codes, o_kcb = w.key_codes, w.as_f64("key_codebooks")
        o_pos = w.key_pos
        if args.position_free:  # no rotation == every key at the query's position
            o_pos = np.concatenate([np.full(int(n), int(p), np.int32) for n, p in zip(np.diff(w.cu_seqlens), w.q_pos)])
        o_q, o_vcb = w.as_f64("q"), w.as_f64("val_codebooks")
        reps = 0
        c0 = time.perf_counter()
        while reps < 8 and (reps == 0 or time.perf_counter() - c0 < 2.0):  # about 10-30 core-seconds
            o_fn = oracle.decode_attn_binary_values if vbin else oracle.decode_attn
            o_fn(o_q, o_codes, w.val_codes, o_kcb, o_vcb, w.cu_seqlens, w.q_pos, key_pos=o_pos,
                 rope_base=w.rope_base, unit_mask=mask.reshape(w.B, w.Hkv), n_threads=n_threads)
            reps += 1
        c1 = time.perf_counter()
        sample_tokens *= reps
        # a layer's context token is processed once all Hkv heads have seen it
        cpu_tok_s = sample_tokens / w.Hkv / (c1 - c0)
        result["cpu_baseline"] = {"value": round(cpu_tok_s, 1), "unit": "context tokens/s per layer", "cores": n_threads,
                                  "kind": "oracle",
                                  "sample": f"{n_threads} of {w.B * w.Hkv} (sequence, KV head) units of {w.name}, {reps} times, "
                                            f"{sample_tokens} unit-tokens, one unit per thread, {c1 - c0:.1f} s wall"}
    print(json.dumps(result))
    op.close()


if __name__ == "__main__":
    main()
