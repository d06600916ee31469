#!/usr/bin/env python3
"""Benchmark of the Evoformer gated-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-others] [--no-cpu]

One step = one pass of the whole hot path (LayerNorm, merged projections, pair bias,
softmax(QK^T*scale + mask + bias) V, gate, output projection) over one synthetic input of the
workload: one ff_gated_attention call (ff_attention_chunked for the chunked workload).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

value = counted FLOP / time, counted FLOP = projections + bias projection + QK^T + PV +
output projection (2*M*N*K each).  The default workload is the AlphaFold initial-training
crop of the MSA row attention with pair bias (N_seq=128, N_res=256, c_m=256, H=8, d=32,
bf16); the N_res=256 triangle modules, the N_res=2048 chunked triangle attention and the
paper's fine-tuning shapes are timed as well and reported under "others".
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# published MI355X peaks used for the roofline fractions
PEAK_MFMA_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
# plain (unpacked) float32 vector instructions: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second
# (the published 157.3 TFLOP/s is this rate x 2 for the packed forms, which this build switches off, x 2 for FMA)
PEAK_VALU_GLANEOPS = 256 * 4 * 16 * 2.4
VALU_SIMDS = 256 * 4

# Peaks measured on an MI355X of this machine with the library's own probes (a bare loop of bf16
# 32x32x16 matrix instructions; a plain 256 MiB copy): bench.py measures both again in every run
# (the "calibration" object of the line) and quotes fractions against the published peaks and
# against what it has just measured.

# HBM bytes per launch come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file, whose
# summaries (profiles/traffic_<workload>_hbm_counters.txt) end in machine-readable lines
#   traffic_bytes_per_launch <kernel kind> = <bytes>
# (KiB per dispatch, each counter scaled by the factor that the same counter gives for a plain copy
# of known size in the same run).  Workloads without such a file, or a tree without profiles/,
# report null.
def traffic_bytes(workload):
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}_hbm_counters.txt")
    out = {}
    try:
        for ln in open(path):
            if ln.startswith("traffic_bytes_per_launch "):
                name, _, val = ln[len("traffic_bytes_per_launch "):].rpartition("=")
                out[name.strip()] = int(float(val))
    except OSError:
        pass
    return out


def counted_flop(sp):
    R, L = sp.batch_len
    hd = sp.heads * sp.head_dim
    f = {}
    f["proj"] = 2.0 * R * L * sp.c * 4 * hd
    if sp.mode == 0:
        f["bias"] = 2.0 * L * L * sp.c_z * sp.heads
    elif sp.mode in (2, 3):
        f["bias"] = 2.0 * R * L * sp.c * sp.heads
    else:
        f["bias"] = 0.0
    f["attn"] = 2 * 2.0 * R * sp.heads * L * L * sp.head_dim
    f["out"] = 2.0 * R * L * hd * sp.c
    f["total"] = sum(f.values())
    return f


def algorithmic_bytes(sp):
    """Each operand once: x in, z in (row mode), out, weights."""
    esz = 4 if sp.dtype == "f32" else 2
    n = sp.n_a * sp.n_b * sp.c * esz
    hd = sp.heads * sp.head_dim
    w = (4 * hd * sp.c + hd * sp.c) * esz
    z = sp.n_b * sp.n_b * sp.c_z * esz if sp.mode == 0 else 0
    return 2 * n + z + w


def time_workload(name, steps, warmup, copies=3, profile=True, residual=False):
    import torch
    import paper_2203_00854_amd as P
    from paper_2203_00854_amd import inputs as I

    case = I.make_case(name)
    sp = case.spec
    desc, w, x, z, mask = P.to_device(case, "cuda:0")
    chunk = sp.chunk_rows
    big = x.numel() * x.element_size() > (1 << 29)
    copies = 1 if big else copies
    xs = [x] + [x.clone() for _ in range(copies - 1)]
    zs = [z] + [z.clone() if z is not None else None for _ in range(copies - 1)]
    outs = [torch.empty_like(x) for _ in range(copies)]
    ws = torch.empty(P.ff_attention_workspace_bytes(desc, chunk), dtype=torch.uint8, device="cuda:0")

    def step(i):
        j = i % copies
        if residual:
            P.ff_gated_attention_residual(desc, w, xs[j], zs[j], mask, chunk_rows=chunk, out=outs[j], ws=ws)
        elif chunk:
            P.ff_attention_chunked(desc, w, xs[j], zs[j], mask, chunk_rows=chunk, out=outs[j], ws=ws)
        else:
            P.ff_gated_attention(desc, w, xs[j], zs[j], mask, out=outs[j], ws=ws)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps

    kernels = {}
    if profile:
        # the same steps again with the library's launch timer (HIP events on the launch stream)
        P.ff_profile_enable(True)
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        kernels = P.ff_profile_collect()
        P.ff_profile_enable(False)
    return case, desc, outs[(steps - 1) % copies], ms, kernels


def time_graph_replay(name, steps, warmup):
    """The same step recorded once into a HIP graph and replayed (the library only enqueues kernels,
    so a call can be captured); one resident copy of the inputs."""
    import torch
    import paper_2203_00854_amd as P
    from paper_2203_00854_amd import inputs as I
    case = I.make_case(name)
    desc, w, x, z, mask = P.to_device(case, "cuda:0")
    chunk = case.spec.chunk_rows
    out = torch.empty_like(x)
    ws = torch.empty(P.ff_attention_workspace_bytes(desc, chunk), dtype=torch.uint8, device="cuda:0")

    def step():
        if chunk:
            P.ff_attention_chunked(desc, w, x, z, mask, chunk_rows=chunk, out=out, ws=ws)
        else:
            P.ff_gated_attention(desc, w, x, z, mask, out=out, ws=ws)

    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def kernel_rooflines(sp, kernels, steps, measured=None):
    """Per kernel: counted flop and HBM bytes of one step, and the roofline that bounds it.

    A dense contraction (the two GEMMs) is priced against the bf16 matrix peak: frac = counted flop /
    duration / peak.  Its HBM figure is given beside it twice: with the operands the METHOD needs
    (x and weights in; for the output projection, out written) and with the intermediates this
    implementation moves through HBM as well (q, k, v, gate, context).  The attention kernel at
    head dims <= 32 is bound by the vector unit ("alu"), the pair-bias pass by HBM.
    measured: {"mfma_tflops": ..., "copy_gbs": ...} from this run's probes, for the second set of fractions."""
    fl = counted_flop(sp)
    R, L = sp.batch_len
    rows_per_launch = sp.chunk_rows if sp.chunk_rows else R
    hd = sp.heads * sp.head_dim
    tok = R * L                                    # tokens per step (all launches of a step together)
    tri_fused = sp.mode in (2, 3) and not sp.chunk_rows
    bias_out = sp.heads * L * L * 4
    w_main = (4 * hd + 32) * sp.c * 2
    per_step = {   # name -> (flop, bytes the method needs, bytes with this implementation's intermediates, natural bound)
        "k_prep": (0.0, 2.0 * ((4 * hd + sp.heads) * sp.c * 2), None, "hbm"),
        "k_gemm<PROJ>": (fl["proj"] + (fl["bias"] if tri_fused else 0.0),
                         tok * sp.c * 2 + w_main,
                         tok * (sp.c + 4 * hd) * 2 + w_main + (bias_out if tri_fused else 0), "mfma"),
        "k_attn": (fl["attn"], None,
                   tok * 5 * hd * 2 + (bias_out * (R // rows_per_launch) if sp.mode != 1 else 0), "alu"),
        # sequences of at most 256 positions at head dim 32: projections and attention in one kernel, which
        # reads x, the weights and the bias and writes the gated context only
        "k_proj_attn": (fl["proj"] + fl["attn"], tok * sp.c * 2 + w_main + (bias_out if sp.mode != 1 else 0),
                        tok * (sp.c + hd) * 2 + w_main + (bias_out * (R // rows_per_launch) if sp.mode != 1 else 0), "mfma"),
        "k_gemm<OUT>": (fl["out"], tok * sp.c * 2 + hd * sp.c * 2, tok * (hd + sp.c) * 2 + hd * sp.c * 2, "mfma"),
        # row mode: k_prep_bias (z once, the float32 bias, and the weight preparation in the same
        # launch); chunked triangle modes: the pair-bias pass over all of x
        "pair bias pass": (fl["bias"], (L * L * sp.c_z if sp.mode == 0 else tok * sp.c) * 2 + bias_out
                           + (2.0 * (4 * hd + sp.heads) * sp.c * 2 if sp.mode == 0 else 0.0), None, "hbm"),
    }
    # vector-unit work of the attention kernel that no design can avoid, in lane-operations per score
    # element: exp2 at half rate (2), half a pack (two elements per instruction) and half a
    # partial-denominator instruction (two elements per dot instruction); the maximum is taken for the
    # first key tile only
    alu_per_step = {"k_attn": R * sp.heads * L * L * 3.0}
    traffic = traffic_bytes(sp.name)
    rows = []
    for name, (ms, cnt) in kernels.items():
        r = {"kernel": name, "launches_per_step": cnt / steps, "avg_us": ms / cnt * 1e3, "ms_per_step": ms / steps}
        if name in per_step:
            flop, b_method, b_impl, bound = per_step[name]
            sec = ms / steps * 1e-3
            tf = flop / sec / 1e12
            r.update(flop_per_step=flop, achieved_tflops=tf, frac_mfma=tf / PEAK_MFMA_BF16_TFLOPS)
            if b_method is not None:
                r.update(method_bytes_per_step=b_method, method_gbs=b_method / sec / 1e9,
                         frac_hbm_method_bytes=b_method / sec / 1e9 / PEAK_HBM_GBS)
            if b_impl is not None:
                r.update(bytes_with_intermediates_per_step=b_impl, gbs_with_intermediates=b_impl / sec / 1e9,
                         frac_hbm_with_intermediates=b_impl / sec / 1e9 / PEAK_HBM_GBS)
            if name in alu_per_step:
                gl = alu_per_step[name] / sec / 1e9
                r.update(achieved_glaneops=gl, frac_alu=gl / PEAK_VALU_GLANEOPS, alu_laneops_per_step=alu_per_step[name])
            if bound == "alu":
                # (at head dims of 64 and more the matrix core would bind; the workloads here have d <= 32)
                r.update(bound="alu", achieved=r["achieved_glaneops"], peak=PEAK_VALU_GLANEOPS, unit="Glane-op/s",
                         frac=r["frac_alu"])
                if measured and measured.get("attention_elements_per_s_at_measured_rates"):
                    # the same elements against what the vector-instruction probes sustain for this kernel's mix
                    r["frac_of_measured_peak"] = (alu_per_step[name] / 3.0 / sec) / measured["attention_elements_per_s_at_measured_rates"]
            elif bound == "mfma":
                r.update(bound="mfma", achieved=tf, peak=PEAK_MFMA_BF16_TFLOPS, unit="TFLOP/s", frac=tf / PEAK_MFMA_BF16_TFLOPS)
                if measured and measured.get("mfma_tflops"):
                    r["frac_of_measured_peak"] = tf / measured["mfma_tflops"]
            else:
                gb = b_method / sec / 1e9
                r.update(bound="hbm", achieved=gb, peak=PEAK_HBM_GBS, unit="GB/s", frac=gb / PEAK_HBM_GBS)
                if measured and measured.get("copy_gbs"):
                    r["frac_of_measured_peak"] = gb / measured["copy_gbs"]
        r["traffic"] = traffic.get(name)
        rows.append(r)
    rows.sort(key=lambda r: -r["ms_per_step"])
    return rows


def calibrate():
    """What this GPU sustains on the library's two probes: a bare loop of bf16 32x32x16 matrix
    instructions and a plain 256 MiB copy (read + written bytes per second)."""
    import torch
    import paper_2203_00854_amd as P
    sink = torch.empty(P.lib().ff_probe_sink_bytes(), dtype=torch.uint8, device="cuda:0")
    src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    P.ff_probe_mfma(sink, 2000)
    P.ff_probe_copy(dst, src)
    torch.cuda.synchronize()
    P.ff_profile_enable(True)
    flop = 0.0
    for _ in range(5):
        flop = P.ff_probe_mfma(sink, 20000)
        P.ff_probe_copy(dst, src)
    torch.cuda.synchronize()
    k = P.ff_profile_collect()
    P.ff_profile_enable(False)
    ms_m, n_m = k["probe: mfma loop"]
    ms_c, n_c = k["probe: copy"]
    # loops of ONE vector instruction: nanoseconds a SIMD spends per wavefront-wide instruction (1024 SIMDs share the launch)
    valu_ns = {}
    for kind, name in enumerate(("fma_f32", "exp_f32", "cvt_pk_bf16_f32", "dot2_f32_bf16")):
        P.ff_probe_valu(sink, kind, 256)
        torch.cuda.synchronize()
        P.ff_profile_enable(True)
        for _ in range(3):
            insts = P.ff_probe_valu(sink, kind, 4096)
        torch.cuda.synchronize()
        kk = P.ff_profile_collect()
        P.ff_profile_enable(False)
        ms_v, n_v = kk["probe: vector loop"]
        valu_ns[name] = (ms_v / n_v * 1e6) / (insts / VALU_SIMDS)
    # rounds of four matrix instructions with vector instructions between them: do the two overlap?
    mix_ns = {}
    for kind, name in ((4, "4_mfma"), (5, "4_mfma_16_fma"), (6, "4_mfma_32_fma"), (7, "4_mfma_16_exp")):
        P.ff_probe_valu(sink, kind, 256)
        torch.cuda.synchronize()
        P.ff_profile_enable(True)
        for _ in range(3):
            rounds = P.ff_probe_valu(sink, kind, 2048)
        torch.cuda.synchronize()
        kk = P.ff_profile_collect()
        P.ff_profile_enable(False)
        ms_v, n_v = kk["probe: vector loop"]
        mix_ns[name] = (ms_v / n_v * 1e6) / (rounds / VALU_SIMDS)
    # per score element of the attention kernel: one fused multiply-add (scale and reference), one exponential,
    # half a pack and half a partial-denominator instruction, each per wavefront of 64 elements
    attn_ns = valu_ns["fma_f32"] + valu_ns["exp_f32"] + 0.5 * valu_ns["cvt_pk_bf16_f32"] + 0.5 * valu_ns["dot2_f32_bf16"]
    return {"mfma_tflops": flop / (ms_m / n_m * 1e-3) / 1e12, "copy_gbs": 2.0 * (256 << 20) / (ms_c / n_c * 1e-3) / 1e9,
            "valu_ns_per_wave_instruction": valu_ns,
            "ns_per_round_of_4_matrix_instructions_per_wavefront": mix_ns,
            "attention_elements_per_s_at_measured_rates": 64.0 * VALU_SIMDS / (attn_ns * 1e-9),
            "note": "library probes, HIP-event timed: 32x32x16 bf16 matrix-instruction loop, 256 MiB copy (read + written), "
                    "loops of one vector instruction (16 independent registers, 8 wavefronts per SIMD)"}


def trimul_flop(sp):
    n, cz, c = sp.n, sp.c_z, sp.c
    f = {"k_tm_proj": 2.0 * n * n * cz * 4 * c, "k_tm_mul": 2.0 * c * n ** 3, "k_tm_out": 2.0 * n * n * (c * cz + cz * cz)}
    f["total"] = sum(f.values())
    return f


def time_trimul(name, steps, warmup, measured):
    """Triangular multiplicative update (ff_triangle_multiplication): one module per step, three resident
    input copies; counted flop = left/right projections with gates + output gate + the N^3 contraction per
    channel + output projection.  Every kernel of it is a dense contraction, priced against the bf16 matrix peak."""
    import torch
    import paper_2203_00854_amd as P
    from paper_2203_00854_amd import inputs as I
    case = I.make_trimul_case(name)
    sp = case.spec
    desc, w, z, mask = P.trimul_to_device(case, "cuda:0")
    copies = 1 if z.numel() * 2 > (1 << 29) else 3
    zs = [z] + [z.clone() for _ in range(copies - 1)]
    outs = [torch.empty_like(z) for _ in range(copies)]
    ws = torch.empty(P.ff_triangle_multiplication_workspace_bytes(desc), dtype=torch.uint8, device="cuda:0")

    def step(i):
        P.ff_triangle_multiplication(desc, w, zs[i % copies], mask, out=outs[i % copies], ws=ws)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    P.ff_profile_enable(True)
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    kernels = P.ff_profile_collect()
    P.ff_profile_enable(False)
    fl = trimul_flop(sp)
    rows = []
    for kname, (kms, cnt) in kernels.items():
        r = {"kernel": kname, "avg_us": kms / cnt * 1e3}
        if kname in fl:
            tf = fl[kname] / (kms / cnt * 1e-3) / 1e12
            r.update(bound="mfma", achieved_tflops=tf, frac=tf / PEAK_MFMA_BF16_TFLOPS, frac_of_measured_peak=tf / measured["mfma_tflops"])
        rows.append(r)
    rows.sort(key=lambda r: -r["avg_us"])
    n_bytes = sp.n * sp.n * sp.c_z * 2
    return {"ms_per_module": ms, "tflops": fl["total"] / (ms * 1e-3) / 1e12, "frac_mfma_peak_whole_module":
            fl["total"] / (ms * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS, "steps": steps, "counted_flop_per_step": fl["total"],
            "algorithmic_bytes_per_step": 2 * n_bytes, "workspace_bytes": P.ff_triangle_multiplication_workspace_bytes(desc),
            "kernels": rows}


def time_global(name, steps, warmup, measured):
    """Extra-MSA global column attention (ff_global_column_attention).  The module is linear in the number of
    sequences and bound by HBM: the method reads m and writes out once each (algorithmic bytes); this
    implementation reads m twice (key/value/query pass, gate/output pass) and moves k, v (bfloat16) and one mask
    byte per token through HBM once each way."""
    import torch
    import paper_2203_00854_amd as P
    from paper_2203_00854_amd import inputs as I
    case = I.make_global_case(name)
    sp = case.spec
    desc, w, m, mask = P.global_to_device(case, "cuda:0")
    copies = 3 if m.numel() * 2 < (1 << 28) else 1
    ms_ = [m] + [m.clone() for _ in range(copies - 1)]
    outs = [torch.empty_like(m) for _ in range(copies)]
    ws = torch.empty(P.ff_global_column_attention_workspace_bytes(desc), dtype=torch.uint8, device="cuda:0")

    def step(i):
        P.ff_global_column_attention(desc, w, ms_[i % copies], mask, out=outs[i % copies], ws=ws)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    P.ff_profile_enable(True)
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    kernels = P.ff_profile_collect()
    P.ff_profile_enable(False)
    hd, tok = sp.heads * sp.head_dim, sp.n_seq * sp.n_res
    flop = 2.0 * tok * sp.c * (2 * hd + 2 * sp.head_dim) + 2.0 * tok * hd * sp.c + 2.0 * 2 * tok * hd
    n_bytes = tok * sp.c * 2
    kv_bytes = tok * 2 * sp.head_dim * 2 + (tok if mask is not None else 0)
    per_kernel = {"k_gca_kv": n_bytes + kv_bytes, "k_gca_softmax": kv_bytes, "k_gca_out": 2 * n_bytes}
    rows = []
    for kname, (kms, cnt) in kernels.items():
        r = {"kernel": kname, "avg_us": kms / cnt * 1e3}
        if kname in per_kernel:
            gb = per_kernel[kname] / (kms / cnt * 1e-3) / 1e9
            r.update(bound="hbm", bytes_per_launch=per_kernel[kname], achieved_gbs=gb, frac=gb / PEAK_HBM_GBS,
                     frac_of_measured_peak=gb / measured["copy_gbs"])
        rows.append(r)
    rows.sort(key=lambda r: -r["avg_us"])
    gbs = 2 * n_bytes / (ms * 1e-3) / 1e9
    return {"ms_per_module": ms, "tflops": flop / (ms * 1e-3) / 1e12, "steps": steps, "counted_flop_per_step": flop,
            "algorithmic_bytes_per_step": 2 * n_bytes, "bound": "hbm", "achieved_gbs_algorithmic": gbs,
            "frac_hbm_peak_whole_module": gbs / PEAK_HBM_GBS, "frac_of_measured_copy": gbs / measured["copy_gbs"],
            "workspace_bytes": P.ff_global_column_attention_workspace_bytes(desc), "kernels": rows}


def time_backward(name, steps, warmup, measured):
    """Backward pass of the fused attention core (ff_attention_core_backward): counted flop = the five
    contractions of the chain rule (dv, dP, dq, dk: 2 L^2 d each per (row, head); the recomputed S is not
    counted as useful work), i.e. twice the forward core's."""
    import torch
    import paper_2203_00854_amd as P
    from paper_2203_00854_amd import inputs as I
    case = I.make_core_case(name)
    sp = case.spec
    desc, t, mask = P.core_to_device(case, "cuda:0")
    ws = torch.empty(P.ff_attention_core_backward_workspace_bytes(desc), dtype=torch.uint8, device="cuda:0")

    def step():
        P.ff_attention_core_backward(desc, t["q"], t["k"], t["v"], t["g"], t.get("bias"), mask, t["do"], ws=ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    P.ff_profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    kernels = P.ff_profile_collect()
    P.ff_profile_enable(False)
    pair = 2.0 * sp.rows * sp.heads * sp.length * sp.length * sp.head_dim      # one L x L x d contraction over all (row, head)
    executed = {"k_bwd_stats": 2 * pair, "k_bwd_dq": 3 * pair, "k_bwd_dkv": 4 * pair, "k_bwd_dbias": 2 * pair}
    rows = []
    for kname, (kms, cnt) in kernels.items():
        r = {"kernel": kname, "avg_us": kms / cnt * 1e3}
        if kname in executed:
            tf = executed[kname] / (kms / cnt * 1e-3) / 1e12
            r.update(bound="mfma", executed_flop=executed[kname], achieved_tflops=tf, frac=tf / PEAK_MFMA_BF16_TFLOPS,
                     frac_of_measured_peak=tf / measured["mfma_tflops"])
        rows.append(r)
    rows.sort(key=lambda r: -r["avg_us"])
    flop = 4 * pair
    return {"ms_per_call": ms, "tflops": flop / (ms * 1e-3) / 1e12, "frac_mfma_peak": flop / (ms * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS,
            "counted_flop_per_step": flop, "steps": steps, "kernels": rows}


def time_layernorm(steps):
    """ff_layernorm alone (the stand-alone entry point; inside the attention the LayerNorm is
    part of the projection GEMM): rows x c as in the MSA and pair representations of the
    workloads, bf16, HBM bound with 2 * rows * c * 2 bytes per call."""
    import torch
    import paper_2203_00854_amd as P
    P.ff_profile_enable(True)
    res = {}
    for name, rows, c in (("msa 128x256 rows, c=256", 128 * 256, 256), ("pair 256x256 rows, c=128", 256 * 256, 128),
                          ("pair 2048x2048 rows, c=128", 2048 * 2048, 128)):
        x = torch.randn(rows, c, device="cuda:0").to(torch.bfloat16)
        g = torch.ones(c, device="cuda:0", dtype=torch.bfloat16)
        b = torch.zeros(c, device="cuda:0", dtype=torch.bfloat16)
        y = torch.empty_like(x)
        n = max(steps // 4, 5)
        for _ in range(3):
            P.ff_layernorm(x, g, b, out=y)
        torch.cuda.synchronize()
        P.ff_profile_collect()
        for _ in range(n):
            P.ff_layernorm(x, g, b, out=y)
        torch.cuda.synchronize()
        k = P.ff_profile_collect()
        ms, cnt = k.get("k_layernorm", next(iter(k.values())))
        us = ms / cnt * 1e3
        gbs = 2.0 * rows * c * 2 / (us * 1e-6) / 1e9
        res[name] = {"avg_us": us, "achieved_gbs": gbs, "frac_hbm": gbs / PEAK_HBM_GBS}
        del x, y
    P.ff_profile_enable(False)
    return res


def cpu_baseline(case, budget_s=12.0):
    """The float64 oracle as it stands, on the host cores, full module of the workload: repeated for about
    budget_s seconds of CPU work (3 to 25 runs), the median run reported."""
    import numpy as np
    from oracle import evoformer_attention as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    sp = case.spec
    x = case.widened("x").astype(np.float64)
    z = None if case.z is None else case.widened("z").astype(np.float64)
    w = {k: v.astype(np.float64) for k, v in case.widened_weights().items()}
    ts = []
    ref = None
    runs = 3
    while len(ts) < runs:
        t0 = time.perf_counter()
        ref = O.gated_attention(sp.mode, x, z, case.mask, w, sp.heads, sp.ln_eps)
        ts.append(time.perf_counter() - t0)
        if len(ts) == 1:
            runs = int(min(25, max(3, round(budget_s / max(ts[0], 1e-3)))))
    ts.sort()
    sec = ts[len(ts) // 2]
    return ref, {"value": counted_flop(sp)["total"] / sec / 1e12, "unit": "TFLOP/s", "cores": threads,
                 "kind": "oracle", "seconds_per_module": sec,
                 "sample": f"full {sp.name} module (all {sp.batch_len[0]} batch rows), float64 numpy, median of {runs} runs ({sum(ts):.1f} s of CPU work)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2_row_bf16_train")
    ap.add_argument("--no-others", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--calibration-only", action="store_true", help="run only the two calibration probes")
    ap.add_argument("--layernorm-only", action="store_true", help="time only ff_layernorm at the three bench shapes")
    ap.add_argument("--backward-only", action="store_true", help="time only the attention-core backward pass")
    ap.add_argument("--global-only", action="store_true", help="time only the extra-MSA global column attention shapes")
    ap.add_argument("--trimul-only", action="store_true", help="time only the triangular multiplicative update shapes")
    ap.add_argument("--shape", default=None, help="with --trimul-only / --global-only / --backward-only: this shape only")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy 5 times (reference for HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    import paper_2203_00854_amd as P
    P.lib()          # fails loudly if libff.so has not been built

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    measured = calibrate()
    if args.calibration_only:
        print(json.dumps({"calibration": measured}))
        return
    if args.layernorm_only:
        print(json.dumps({"calibration": measured, "layernorm": time_layernorm(args.steps)}))
        return
    wanted = lambda name: args.shape is None or args.shape == name      # (--shape: one shape of a --*-only run)
    if args.backward_only:
        print(json.dumps({name: time_backward(name, args.steps, 3, measured) for name in ("core_row_256", "core_tri_256")
                          if wanted(name)}))
        return
    if args.global_only:
        print(json.dumps({name: time_global(name, st, 3, measured) for name, st in
                          (("gca_bf16_1024x384", args.steps), ("gca_bf16_5120x384", max(args.steps // 5, 3))) if wanted(name)}))
        return
    if args.trimul_only:
        print(json.dumps({name: time_trimul(name, st, 3, measured) for name, st in
                          (("tm_out_bf16_256", args.steps), ("tm_in_bf16_256", args.steps), ("tm_out_bf16_384", args.steps),
                           ("tm_out_bf16_2048", 3)) if wanted(name)}))
        return
    case, desc, out, ms, kernels = time_workload(args.workload, args.steps, args.warmup)
    path_taken = P.ff_attention_last_path()
    sp = case.spec
    fl = counted_flop(sp)
    value = fl["total"] / (ms * 1e-3) / 1e12
    roof = kernel_rooflines(sp, kernels, args.steps, measured)

    line = {
        "metric": "evoformer_attention_tflops", "value": value, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if sp.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{sp.name}: gated attention mode {sp.mode}, x[{sp.n_a},{sp.n_b},{sp.c}], c_z={sp.c_z}, "
                               f"H={sp.heads}, d={sp.head_dim}, mask {sp.mask}, one module per step",
                   "path": path_taken, "counted_flop_per_step": fl["total"],
                   "algorithmic_bytes_per_step": algorithmic_bytes(sp)},
        "ms_per_module": ms,
        "frac_mfma_peak_whole_module": value / PEAK_MFMA_BF16_TFLOPS,
        "frac_hbm_peak_whole_module": algorithmic_bytes(sp) / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "calibration": measured,
        "frac_measured_mfma_whole_module": value / measured["mfma_tflops"],
    }
    if roof:
        d = roof[0]
        line["roofline"] = {"kernel": d["kernel"], "bound": d.get("bound"), "achieved": d.get("achieved"),
                            "peak": d.get("peak"), "unit": d.get("unit"), "frac": d.get("frac"),
                            "traffic": d.get("traffic"), "avg_us": d["avg_us"],
                            "frac_of_measured_peak": d.get("frac_of_measured_peak")}
        line["kernels"] = roof
        # HBM bytes the whole module moved (counter runs) over the bytes the method needs
        tr = [r.get("traffic") for r in roof]
        if tr and all(t is not None for t in tr):
            line["traffic_bytes_whole_module"] = sum(t * r["launches_per_step"] for t, r in zip(tr, roof))
            line["traffic_ratio"] = line["traffic_bytes_whole_module"] / algorithmic_bytes(sp)
        else:
            line["traffic_bytes_whole_module"] = None
            line["traffic_ratio"] = None

    if not args.no_cpu:
        ref, base = cpu_baseline(case)
        got = out.float().cpu().numpy().astype(np.float64)
        base["gpu_vs_oracle_max_abs"] = float(np.max(np.abs(got - ref)))
        base["gpu_vs_oracle_rel_l2"] = float(np.linalg.norm(got - ref) / np.linalg.norm(ref))
        line["cpu_baseline"] = base

    if not args.no_others:
        others = {}
        for name, st, wu in (("c1_row_f32_tiny", args.steps, args.warmup),
                             ("c3_tri_start_bf16_256", args.steps, args.warmup),
                             ("c3_tri_end_bf16_256", args.steps, args.warmup),
                             ("c4_col_bf16_extra", max(args.steps // 4, 5), 3),
                             ("c5_tri_start_bf16_2048", max(args.steps // 40, 3), 1),
                             # the paper's fine-tuning shapes (Table 1: N_res 384, N_seq 512, N_extra_seq 5120)
                             ("ft_row_bf16_512x384", max(args.steps // 10, 5), 3),
                             ("ft_col_bf16_512x384", max(args.steps // 10, 5), 3),
                             ("ft_tri_start_bf16_384", max(args.steps // 4, 5), 3),
                             ("ft_tri_end_bf16_384", max(args.steps // 4, 5), 3),
                             ("ft_col_bf16_extra_5120", max(args.steps // 40, 3), 1)):
            c2, d2, _, ms2, k2 = time_workload(name, st, wu)
            f2 = counted_flop(c2.spec)["total"]
            others[name] = {"ms_per_module": ms2, "tflops": f2 / (ms2 * 1e-3) / 1e12, "steps": st,
                            "chunk_rows": c2.spec.chunk_rows, "path": P.ff_attention_last_path(),
                            "workspace_bytes": P.ff_attention_workspace_bytes(d2, c2.spec.chunk_rows),
                            "kernels": [{k: r[k] for k in ("kernel", "avg_us", "launches_per_step", "frac", "bound")
                                         if k in r} for r in kernel_rooflines(c2.spec, k2, st, measured)]}
            del c2
            torch.cuda.empty_cache()
        # backward pass of the fused attention core at the initial-training shapes
        line["attention_core_backward"] = {name: time_backward(name, max(args.steps // 4, 5), 3, measured)
                                           for name in ("core_row_256", "core_tri_256")}
        torch.cuda.empty_cache()
        # the extra-MSA global column attention at the paper's two extra-MSA sizes
        line["global_column_attention"] = {
            name: time_global(name, st, wu, measured)
            for name, st, wu in (("gca_bf16_1024x384", max(args.steps // 4, 5), 3), ("gca_bf16_5120x384", max(args.steps // 20, 3), 1))}
        torch.cuda.empty_cache()
        line["others"] = others
        # the pair stack's triangular multiplicative update at the paper's shapes
        line["triangle_multiplication"] = {
            name: time_trimul(name, st, wu, measured)
            for name, st, wu in (("tm_out_bf16_256", args.steps, args.warmup), ("tm_in_bf16_256", args.steps, args.warmup),
                                 ("tm_out_bf16_384", max(args.steps // 4, 5), 3), ("tm_in_bf16_384", max(args.steps // 4, 5), 3),
                                 ("tm_out_bf16_2048", max(args.steps // 40, 3), 1))}
        torch.cuda.empty_cache()
        # the module with the residual add that closes it in the Evoformer block fused into the output
        # projection (ff_gated_attention_residual): x + module(x) in one pass
        upd = {}
        for name, st, wu in ((args.workload, args.steps, args.warmup),
                             ("c5_tri_start_bf16_2048", max(args.steps // 40, 3), 1)):
            c2, _, _, ms2, k2 = time_workload(name, st, wu, residual=True)
            og = k2.get("k_gemm<OUT>")
            upd[name] = {"ms_per_module": ms2, "k_gemm<OUT>_avg_us": og[0] / og[1] * 1e3 if og else None,
                         "extra_algorithmic_bytes": c2.spec.n_a * c2.spec.n_b * c2.spec.c * 2}
            del c2
            torch.cuda.empty_cache()
        line["residual_update"] = upd
        line["hip_graph_replay"] = {"workload": args.workload, "ms_per_step":
                                    time_graph_replay(args.workload, args.steps, args.warmup),
                                    "note": "one captured step replayed; one resident input copy"}
        line["layernorm"] = time_layernorm(args.steps)

    print(json.dumps(line))


if __name__ == "__main__":
    main()
