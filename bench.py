#!/usr/bin/env python3
"""Stage-training benchmark on one MI355X.

A step is one HPP-Round of the stage (Sec. 3.2): M micro-batches through forward and
backward in 1F1B order (K = 1), in-place gradient accumulation, one momentum-SGD update.
Inputs are synthetic, seeded, and resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfgN]

Without --workload the five benchmark configurations cfg1 .. cfg5 run one after the other and the
headline of the JSON line is cfg4 (the largest single-GPU workload); `per_config` carries all five.
Per configuration: W warm-up rounds, K timed rounds (wall clock between two synchronisations for
the headline rate; a HIP event pair per round for median and minimum), then a few more rounds with
every kernel launch timed, which give the kernel family with the largest share of the time, its
achieved rate against the HBM or MFMA peak, the launches per round, and a step-level fraction
(modelled bytes or flops of the whole round / round time / peak); last the CPU oracle on a bounded
sample of the same workload.  Prints ONE JSON line.
"""
import argparse
import glob
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def _cdiv(a, b):
    return -(-a // b)


def _dw_vw(h, w, stride):
    """Strip width (pixels per lane) of the depthwise register-window kernels; 0 = LDS kernels."""
    if stride == 2 and (h % 2 or w % 2):
        return 0
    if w % 4 == 0 and w // 4 <= 64:
        return 4
    if w % 2 == 0 and w // 2 <= 64:
        return 2
    return 1 if (stride == 1 and w <= 64) else 0


def kernel_model(cfg):
    """Algorithmic work of the kernel classes that can dominate a workload, from the layer list
    and the launch rules of the library (one entry per launch of one micro-batch):
    {profile kernel name: [(units, ...), ...]} with units = bytes (HBM-bound) or flops (MFMA)."""
    from asteroid_workloads import gen
    B = cfg.B
    out = {}
    shape = tuple(cfg.in_shape)
    first = True
    res_open = False
    # BatchNorm passes that the depthwise conv next to them takes over (fp32): the apply pass of a
    # BatchNorm(+ReLU) directly in front, the statistics pass of a BatchNorm directly behind
    lazy_bn, given_bn = set(), set()
    kinds = [L["kind"] for L in cfg.layers]
    for i, L in enumerate(cfg.layers):
        if L["kind"] == "conv2d" and cfg.dtype == "f32" and L["k"] == 3 and L["groups"] == L["cin"] == L["cout"] \
                and L.get("pad", 1) == 1 and not L.get("bias", False):
            if i >= 1 and kinds[i - 1] == "batchnorm2d":
                lazy_bn.add(i - 1)
            elif i >= 2 and kinds[i - 1] in ("relu", "relu6") and kinds[i - 2] == "batchnorm2d":
                lazy_bn.add(i - 2)
            if i + 1 < len(kinds) and kinds[i + 1] == "batchnorm2d":
                given_bn.add(i + 1)
    # statistics partials that a pointwise conv (no bias) leaves for the BatchNorm behind it: offered by the
    # 32- and 128-pixel-wavefront kernels while there are at most 256 pixel blocks
    stat_bn = set()
    shp = tuple(cfg.in_shape)
    outs = gen.layer_shapes(cfg.layers, cfg.in_shape)
    for i, L in enumerate(cfg.layers):
        if L["kind"] == "conv2d" and cfg.dtype == "f32" and L["k"] == 1 and L["groups"] == 1 and not L.get("bias", False) \
                and i + 1 < len(kinds) and kinds[i + 1] == "batchnorm2d" and (i + 1) not in given_bn:
            hw_, nq_ = shp[1] * shp[2], B * shp[1] * shp[2]
            ks = not (_cdiv(nq_, 128) * _cdiv(L["cout"], 32) < 256 and _cdiv(L["cin"], 8) >= 16)
            parts = _cdiv(nq_, 512) if (hw_ % 4 == 0 and nq_ >= 65536) else _cdiv(nq_, 128)
            if ks and parts <= 256:
                stat_bn.add(i + 1)
        shp = outs[i]
    for i, L in enumerate(cfg.layers):
        k = L["kind"]
        oshape = outs[i]
        if k == "res_begin":
            res_open = True
        if k == "conv2d" and cfg.dtype == "f32" and L["k"] == 1 and L["groups"] == 1:
            cin, cout = L["cin"], L["cout"]
            hw = shape[1] * shape[2]
            nq = B * hw

            def cls(m, kd):
                kg = _cdiv(kd, 8)
                if _cdiv(nq, 128) * _cdiv(m, 32) < 256 and kg >= 16:    # K split over 4 / 8 / 16 wavefronts
                    return "pkks" if kg <= 32 else ("pkks8" if kg <= 64 else "pkks16")
                if hw % 4 == 0 and nq >= 65536:
                    return "pk4"
                return "pk2" if kd > 32 else "pk1"
            fwd_names = {"pkks": "pw_conv_f32_pkks_kernel", "pkks8": "pw_conv_f32_pkks_kernel<8>",
                         "pkks16": "pw_conv_f32_pkks_kernel<16>", "pk4": "pw_conv_f32_pk4_kernel",
                         "pk2": "pw_conv_f32_pk_kernel<2>", "pk1": "pw_conv_f32_pk_kernel<1>"}
            wg_name = "pw_wgrad_f32_kernel<true>" if hw % 4 == 0 else "pw_wgrad_f32_kernel<false>"
            out.setdefault(fwd_names[cls(cout, cin)], []).append(4 * (cin + cout) * nq)      # forward
            if not first or cfg.needs_input_grad:
                extra = 4 * cin * nq if (res_open and cfg.layers[i - 1]["kind"] == "res_begin") else 0
                bc = cls(cin, cout)
                if bc in ("pkks8", "pkks16"):   # long K: input gradient and weight gradient as two launches
                    out.setdefault(fwd_names[bc], []).append(4 * (cin + cout) * nq + extra)
                    out.setdefault(wg_name, []).append(4 * (cin + cout) * nq)
                else:
                    # input gradient and weight-gradient partials in one launch: g and x in, dx out
                    out.setdefault("pw_bwd_dual_kernel<%s>" % bc, []).append(4 * (2 * cin + cout) * nq + extra)
            else:
                out.setdefault(wg_name, []).append(4 * (cin + cout) * nq)                   # g and x in
        if k == "conv2d" and cfg.dtype == "f32" and L["k"] == 3 and L["groups"] == 1 and L["stride"] == 1 \
                and L["pad"] == 1 and L["cin"] >= 8 and L["cout"] >= 8:
            # dense 3x3 on the matrix cores: flops of one product (forward; the input gradient is the same
            # kernel with the channel roles exchanged) and of the weight gradient
            c, h, w = shape
            flops = 2.0 * 9 * L["cin"] * L["cout"] * B * h * w
            out.setdefault("conv3x3_mfma_f32_kernel", []).append(flops)
            if not first or cfg.needs_input_grad:
                out.setdefault("conv3x3_mfma_f32_kernel", []).append(flops)
            wg = "conv3x3_wgrad_vec_mfma_f32_kernel" if w % 4 == 0 else "conv3x3_wgrad_mfma_f32_kernel"
            out.setdefault(wg, []).append(flops)
        if k == "conv2d" and cfg.dtype == "f32" and L["k"] == 5 and L["groups"] == L["cin"] == L["cout"]:
            c, h, w = shape
            oc, oh, ow = oshape
            out.setdefault("dwk_fwd_f32_kernel<s%d>" % L["stride"], []).append(4 * B * (c * h * w + oc * oh * ow))
            # upstream gradient and input in, input gradient out
            out.setdefault("dwk_bwd_f32_kernel<s%d>" % L["stride"], []).append(4 * B * (2 * c * h * w + oc * oh * ow))
        if k == "conv2d" and cfg.dtype == "f32" and L["k"] == 3 and L["groups"] == L["cin"] == L["cout"]:
            oc, oh, ow = oshape
            if _dw_vw(shape[1], shape[2], L["stride"]):
                name = "dw3x3_fwd_s%d_f32_kernel" % L["stride"]
            else:
                name = "dw3x3_fwd_f32_kernel"
            out.setdefault(name, []).append(4 * B * (shape[0] * shape[1] * shape[2] + oc * oh * ow))
        if k == "conv2d" and cfg.dtype == "f32" and L["k"] == 3 and L["groups"] == L["cin"] == L["cout"]:
            c, h, w = shape
            if _dw_vw(h, w, L["stride"]):
                oc, oh, ow = oshape
                name = "dw3x3_bwd_s%d_f32_kernel" % L["stride"]
                # g, x in; dx out; with a BatchNorm behind also the conv output (that BatchNorm's input)
                ny = 2 if (i + 1) in given_bn else 1
                out.setdefault(name, []).append(4 * B * (2 * c * h * w + ny * oc * oh * ow))
        if k == "batchnorm2d":
            c, h, w = shape
            vec = "<true>" if (h * w) % 4 == 0 else "<false>"
            n_el = B * c * h * w
            small = B * h * w <= 8192    # one block per channel, one launch per direction
            plain = i not in given_bn and i not in lazy_bn
            bwd_bytes = (12 if (not first or cfg.needs_input_grad) else 8) * n_el
            if small and plain and i not in stat_bn:
                out.setdefault("bn_fwd_onepass_kernel", []).append(8 * n_el)               # (+4 with a fused skip)
            else:
                if i not in given_bn and i not in stat_bn:
                    out.setdefault("bn_stats_partial_kernel" + vec, []).append(4 * n_el)
                if i not in lazy_bn:
                    out.setdefault("bn_apply_kernel" + vec, []).append(8 * n_el)          # (+4 with a fused skip)
            if small and plain:
                out.setdefault("bn_bwd_onepass_kernel", []).append(bwd_bytes)
            else:
                if i not in lazy_bn:     # else the depthwise conv behind leaves the sums
                    out.setdefault("bn_bwd_partial_kernel" + vec, []).append(8 * n_el)
                if i not in given_bn:    # else the depthwise conv in front forms the input gradient on load
                    # g and x in, dx out (no dx for a BatchNorm on the stage input when it is not wanted)
                    out.setdefault("bn_bwd_apply_kernel", []).append(bwd_bytes)
        if k == "conv2d" and cfg.dtype == "bf16":
            cin, cout, kk = L["cin"], L["cout"], L["k"] * L["k"]
            m = B * shape[1] * shape[2]

            halo = lambda kc, nn: L["k"] == 3 and kc % 64 == 0 and shape[2] <= 63   # the LDS-halo kernel's shapes

            def gcls(mm, nn, kc):
                if halo(kc, nn):
                    return "conv3x3_halo_kernel_n256" if nn > 128 else "conv3x3_halo_kernel_n128"
                return "gemm_bf16_kernel<128x128,im2col>" if _cdiv(mm, 128) * _cdiv(nn, 128) >= 256 \
                    else "gemm_bf16_kernel<64x64,im2col>"
            out.setdefault(gcls(m, cout, cin), []).append(2 * m * cout * kk * cin)
            if not first or cfg.needs_input_grad:
                out.setdefault(gcls(m, cin, cout), []).append(2 * m * cin * kk * cout)
            wg = "conv_wgrad_tr_kernel_n256" if cin > 128 else "conv_wgrad_tr_kernel_n128"
            out.setdefault(wg if m >= 48 else "gemm_bf16_kernel<128x128,wgrad_conv>", []).append(2 * m * cout * kk * cin)
        if cfg.dtype == "bf16" and k in ("linear", "mha"):
            rows = B * shape[0]

            def lcls(mm, nn, kc):
                if kc % 64 == 0 and nn % 8 == 0 and nn >= 64 and mm >= 64:      # the direct-to-LDS kernel's shapes
                    if _cdiv(mm, 256) * _cdiv(nn, 128) >= 160:
                        return "linear_dl_kernel_256x128"
                    return "linear_dl_kernel_128x128" if _cdiv(mm, 128) * _cdiv(nn, 128) >= 160 else "linear_dl_kernel_128x64"
                return "gemm_bf16_kernel<128x128,rows>" if _cdiv(mm, 128) * _cdiv(nn, 128) >= 256 \
                    else "gemm_bf16_kernel<64x64,rows>"
            mats = [(L["cin"], L["cout"])] if k == "linear" else [(L["d"], 3 * L["d"]), (L["d"], L["d"])]
            for cin, cout in mats:
                out.setdefault(lcls(rows, cout, cin), []).append(2 * rows * cin * cout)      # forward
                out.setdefault(lcls(rows, cin, cout), []).append(2 * rows * cin * cout)      # input gradient
                grouped = cin % 8 == 0 and cout % 8 == 0 and rows >= 48     # one launch for many layers' products
                out.setdefault("wgrad_grouped_kernel" if grouped else "gemm_bf16_kernel<128x128,wgrad_rows>",
                               []).append(2 * rows * cin * cout)
        if cfg.dtype == "bf16" and k == "mha":
            S, D = shape
            fl = 4 * S * D * B * S                                            # QK^T and PV
            out.setdefault("attention_fwd_kernel", []).append(fl)
            out.setdefault("attention_bwd_kernel", []).append(int(3.5 * fl))  # dK/dV role: S, dP, dV, dK; dQ role: S, dP, dQ
        if cfg.dtype == "bf16" and k == "layernorm":
            S, D = shape
            out.setdefault("layernorm_fwd_kernel", []).append(4 * B * S * D)      # bf16 in, bf16 out
            out.setdefault("layernorm_bwd_kernel", []).append(6 * B * S * D)      # g, x in; dx out
        if k == "res_add":
            res_open = False
        if k not in ("res_begin",):
            first = False
        shape = oshape
    return out


def kernel_bound(name):
    return "mfma" if name.startswith(("gemm_bf16", "attention", "conv3x3_", "conv_wgrad", "wgrad_grouped", "linear_dl")) else "hbm"


def family(name):
    """Kernel family of a profile name: template arguments and tile-size suffixes dropped."""
    return re.sub(r"_(n128|n256|256x128|128x128|128x64)$", "", name.split("<")[0])


def committed_traffic(workload, fam):
    """HBM bytes per launch of a kernel family from the committed rocprofv3 counter summaries
    (profiles/<workload>_*_hbm_counters.txt, lines `bench_family <family> traffic_bytes_per_launch <n>`:
    FETCH_SIZE and WRITE_SIZE of two --pmc runs, each scaled by what it reads for a plain copy)."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "%s_*_hbm_counters.txt" % workload))):
        with open(path) as f:
            for line in f:
                m = re.match(r"\s*bench_family\s+(\S+)\s+traffic_bytes_per_launch\s+(\d+)", line)
                if m and m.group(1) == fam:
                    return int(m.group(2))
    return None


# Learning rate of the updates inside bench.py's loops.  The configurations state 0.01 for ONE update; the
# bench runs tens of rounds back to back on the same unnormalised N(0,1) upstream gradients (|G| ~ 1e3), which
# at 0.01 drives the bf16 stages' weights to inf / NaN within a few rounds - and a round of the VGG stage on
# non-finite operands runs 6 % FASTER than on finite ones (3.65 against 3.89 ms: the matrix cores draw less
# power, the clock rises).  The same kernels, bytes and flops run for any value of the scalar, so the timed
# loop uses one that keeps every tensor finite over the whole run.  The parity tests use the stated 0.01.
BENCH_LR = 1e-9
REWARM_ROUNDS = 8   # untimed rounds in front of the per-kernel pass


def measure(workload, steps, warmup, cpu=True, profile_all=False, prof_rounds=3, K=1, forward_stream=False,
            two_streams=True):
    """One configuration: returns its record for the JSON line.  K = micro-batches in flight (stash
    slots); forward_stream: the forward passes run on a second stream beside the backward passes."""
    import torch
    import paper_2408_08015_amd as A
    from asteroid_workloads import get_config, gen

    cfg = get_config(workload)
    inp = gen.make_inputs(cfg)
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    stream = torch.cuda.current_stream()
    K = min(K, cfg.M)
    st = A.Stage(cfg.layers, cfg.B, cfg.M, K, cfg.in_shape, cfg.dtype, cfg.layout, cfg.needs_input_grad,
                 stream=stream.cuda_stream)
    st.set_params(inp["params"])
    fwd_stream = None
    if forward_stream:
        fwd_stream = A.stream_create()     # not torch.cuda.Stream(): its pool holds 32 streams per priority, and
        st.set_forward_stream(fwd_stream)  # the runtime deals all streams of a process onto four hardware queues
    B, M = cfg.B, cfg.M
    x = torch.from_numpy(inp["x"]).to(dev).to(tdt).contiguous()
    if cfg.loss_tail:
        labels = torch.from_numpy(inp["labels"]).to(dev)
        y = torch.zeros((B * M, gen.out_shape(cfg.layers, cfg.in_shape)[0]), device=dev)
        dy = None
    else:
        labels = None
        dy = torch.from_numpy(inp["dy"]).to(dev).to(tdt).contiguous()
        y = torch.zeros_like(dy)
    dx = torch.zeros_like(x) if cfg.needs_input_grad else None
    # one separately allocated buffer per micro-batch (16-byte aligned, as the ABI requires)
    mbs = lambda t: [t[m * B:(m + 1) * B].clone() if t is not None else None for m in range(M)]
    xs, ys, dys, dxs, labs = mbs(x), mbs(y), mbs(dy), mbs(dx), mbs(labels)
    loss = torch.zeros(M * 4, device=dev)
    ls = [loss[4 * m:4 * m + 1] if cfg.loss_tail else None for m in range(M)]

    def one_round():
        # K forward passes, then one backward / one forward (K = 1: F0 B0 F1 B1 ...), then the update
        for m in range(K):
            st.forward(m, xs[m], labs[m], ys[m], ls[m])
        for m in range(M):
            st.backward(m, dys[m], dxs[m])
            if m + K < M:
                st.forward(m + K, xs[m + K], labs[m + K], ys[m + K], ls[m + K])
        st.step(BENCH_LR, cfg.momentum)

    # the pool of HIP events for the per-kernel pass further down is created now (tens of thousands of
    # hipEventCreate calls): done later it would leave the GPU idle for a tenth of a second right before that pass
    st.profile_begin("", max_launches=prof_rounds * 20000)
    st.profile_end()
    for _ in range(warmup):
        one_round()
    # ---- the timed region: exactly `steps` rounds between two synchronisations; an event per round
    # boundary on the stage's stream (torch's current stream) for median / minimum
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record(stream)
    for i in range(steps):
        one_round()
        evs[i + 1].record(stream)
    t_enq = time.perf_counter()      # every launch enqueued; the GPU may still be working
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_round = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]
    ms_per_step = (t1 - t0) * 1e3 / steps

    # ---- every kernel launch timed with a HIP event pair attached to its dispatch (a pass of its own:
    # the events make the launches slower to enqueue)
    # After an idle moment the first 30 ms of work run at a lower clock (cfg4: 4.5 ms for the first round, 3.9 from
    # the eighth on), so the pass is preceded by untimed rounds, with no synchronisation in between.
    for _ in range(REWARM_ROUNDS):
        one_round()
    st.profile_begin("", max_launches=prof_rounds * 20000)
    for _ in range(prof_rounds):
        one_round()
    prof = st.profile_end()
    km = kernel_model(cfg)
    fams = {}
    for name, (n, ms) in prof.items():
        f = fams.setdefault(family(name), {"launches": 0, "ms": 0.0, "units": 0.0, "modelled": True, "bound": kernel_bound(name)})
        f["launches"] += n
        f["ms"] += ms
        units = [u for kn, u in km.items() if name.startswith(kn)]
        if units:
            f["units"] += sum(units[0]) * M * prof_rounds
        else:
            f["modelled"] = False
    tot_ms = sum(f["ms"] for f in fams.values())
    launches_per_step = sum(f["launches"] for f in fams.values()) / prof_rounds
    roofline = None
    ranked = sorted(fams.items(), key=lambda kv: -kv[1]["ms"])
    dom = next(((k, f) for k, f in ranked if f["modelled"] and f["units"] > 0), None)
    if dom:
        fam, f = dom
        bound = f["bound"]
        peak = HBM_PEAK_GBS if bound == "hbm" else MFMA_PEAK_TFLOPS[cfg.dtype]
        achieved = f["units"] / (f["ms"] * 1e-3) / (1e9 if bound == "hbm" else 1e12)
        roofline = {"bound": bound, "kernel": fam, "achieved": round(achieved, 1), "peak": peak,
                    "unit": "GB/s" if bound == "hbm" else "TFLOP/s", "frac": round(achieved / peak, 4),
                    "traffic": committed_traffic(workload, fam),
                    "algorithmic": int(f["units"] / f["launches"]), "launches": f["launches"],
                    "avg_us": round(f["ms"] * 1e3 / f["launches"], 2),
                    "share_of_kernel_time": round(f["ms"] / tot_ms, 3)}
    # step level: everything the model knows of one round against the round's time
    step_bound = "mfma" if cfg.dtype == "bf16" else "hbm"
    modelled = sum(sum(u) for kn, u in km.items() if kernel_bound(kn) == step_bound) * M
    t_med = statistics.median(per_round) * 1e-3
    step_peak = HBM_PEAK_GBS if step_bound == "hbm" else MFMA_PEAK_TFLOPS[cfg.dtype]
    step_ach = modelled / t_med / (1e9 if step_bound == "hbm" else 1e12)
    step_roofline = {"bound": step_bound, "modelled": int(modelled), "achieved": round(step_ach, 1), "peak": step_peak,
                     "unit": "GB/s" if step_bound == "hbm" else "TFLOP/s", "frac": round(step_ach / step_peak, 4)}
    if profile_all:
        print("%s: per-kernel HIP-event times over %d rounds (sum %.3f ms/round):" % (workload, prof_rounds, tot_ms / prof_rounds),
              file=sys.stderr)
        for k, v in sorted(prof.items(), key=lambda kv: -kv[1][1]):
            line = "  %-48s launches/step %6.1f  us/launch %9.2f  ms/step %8.4f  %5.1f%%" % (
                k, v[0] / prof_rounds, v[1] * 1e3 / v[0], v[1] / prof_rounds, 100 * v[1] / tot_ms)
            units = [u for n, u in km.items() if k.startswith(n)]
            if units:       # algorithmic work per launch / HIP-event time per launch
                per = sum(units[0]) / len(units[0])
                avg_s = v[1] * 1e-3 / v[0]
                if kernel_bound(k) == "hbm":
                    line += "  %7.1f MB/launch %7.0f GB/s  %4.0f%% of HBM peak" % (
                        per / 1e6, per / avg_s / 1e9, 100 * per / avg_s / 1e9 / HBM_PEAK_GBS)
                else:
                    line += "  %7.2f GF/launch %7.0f TF/s  %4.0f%% of MFMA peak" % (
                        per / 1e9, per / avg_s / 1e12, 100 * per / avg_s / 1e12 / MFMA_PEAK_TFLOPS[cfg.dtype])
            print(line, file=sys.stderr)
    mem = st.memory()
    st.close()
    if fwd_stream:
        A.stream_destroy(fwd_stream)
    # ---- the same rounds with K = 3 stashes and the forward passes on a second stream (the forward of a later
    # micro-batch runs beside the backward of an earlier one; bit-identical results): timed the same way,
    # reported beside the headline figure, never in its place
    two = None
    if two_streams and K == 1 and not forward_stream and cfg.M >= 2:
        K2 = min(3, cfg.M)
        st2 = A.Stage(cfg.layers, cfg.B, cfg.M, K2, cfg.in_shape, cfg.dtype, cfg.layout, cfg.needs_input_grad,
                      stream=stream.cuda_stream)
        st2.set_params(inp["params"])
        fs2 = A.stream_create()
        st2.set_forward_stream(fs2)

        def round2():
            for m in range(K2):
                st2.forward(m, xs[m], labs[m], ys[m], ls[m])
            for m in range(M):
                st2.backward(m, dys[m], dxs[m])
                if m + K2 < M:
                    st2.forward(m + K2, xs[m + K2], labs[m + K2], ys[m + K2], ls[m + K2])
            st2.step(BENCH_LR, cfg.momentum)

        for _ in range(warmup):
            round2()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(steps):
            round2()
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t2) * 1e3 / steps
        two = {"K": K2, "forward_stream": True, "ms_per_step": round(ms2, 4),
               "value": round(M * B / (ms2 * 1e-3), 1), "unit": "samples/s", "act_stashes": K2}
        st2.close()
        A.stream_destroy(fs2)
    del xs, ys, dys, dxs, x, y, dy, dx
    torch.cuda.empty_cache()
    rec = {
        "workload": "%s: %s, B=%d x M=%d, in %s %s" % (workload, cfg.name, B, M, "x".join(map(str, cfg.in_shape)), cfg.layout),
        "dtype": "f32" if cfg.dtype == "f32" else "bf16",
        "value": round(M * B / (ms_per_step * 1e-3), 1), "unit": "samples/s",
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(statistics.median(per_round), 4), "ms_per_step_min": round(min(per_round), 4),
        "host_enqueue_ms_per_step": round((t_enq - t0) * 1e3 / steps, 4),
        "launches_per_step": round(launches_per_step, 1),
        "K": K, "forward_stream": bool(forward_stream), "two_streams": two,
        "roofline": roofline, "step_roofline": step_roofline,
        "stage_bytes": {"mod": mem[0], "opt": mem[1], "act_per_mb": mem[2], "workspace": mem[3]},
        "cpu_baseline": cpu_baseline(cfg, inp) if cpu else None,
    }
    return rec, cfg


HEADLINE = "cfg4"   # the largest single-GPU configuration (3.55 TFLOP per round)


def run(args):
    workloads = [args.workload] if args.workload else ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"]
    head = args.workload or HEADLINE
    recs = {}
    for w in workloads:
        recs[w], cfg = measure(w, args.steps, args.warmup, cpu=not args.no_cpu_baseline, profile_all=args.profile_all,
                               K=args.K, forward_stream=args.forward_stream, two_streams=not args.no_two_streams)
        if w == head:
            head_cfg = cfg
    h = recs[head]
    out = {
        "metric": "stage train samples/sec (fwd+bwd+SGD, M micro-batches)",
        "value": h["value"], "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": h["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": h["dtype"], "data": "synthetic",
        "config": {"workload": h["workload"], "K": h["K"], "forward_stream": h["forward_stream"], "lr": BENCH_LR, "lr_of_the_configuration": head_cfg.lr, "momentum": head_cfg.momentum,
                   "ms_per_step_median": h["ms_per_step_median"], "ms_per_step_min": h["ms_per_step_min"],
                   "host_enqueue_ms_per_step": h["host_enqueue_ms_per_step"],
                   "launches_per_step": h["launches_per_step"], "stage_bytes": h["stage_bytes"]},
        "roofline": h["roofline"], "step_roofline": h["step_roofline"], "cpu_baseline": h["cpu_baseline"],
        "per_config": [recs[w] for w in workloads],
    }
    print(json.dumps(out))


def cpu_baseline(cfg, inp):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload."""
    from oracle import OracleStage, run_round
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    # sample: as many whole micro-batches as fit the time budget (at least one), then one update
    M, B = cfg.M, cfg.B
    st = OracleStage(cfg.layers, B, M, cfg.in_shape, cfg.layout, cfg.needs_input_grad,
                     storage="bf16" if cfg.dtype == "bf16" else "f64")
    st.set_params(inp["params"])
    target = inp["labels"] if cfg.loss_tail else inp["dy"]
    t0 = time.perf_counter()
    done = rounds = 0
    while True:    # whole micro-batches until about eight seconds have passed (at least one), at most four rounds
        part = 0
        for m in range(M):
            sl = slice(m * B, (m + 1) * B)
            st.forward(m, inp["x"][sl], target[sl] if cfg.loss_tail else None)
            st.backward(m, None if cfg.loss_tail else target[sl])
            part += 1
            if time.perf_counter() - t0 > 8.0:
                break
        st.stash.clear()
        st.step(cfg.lr, cfg.momentum)
        done += part
        rounds += 1
        if part < M or time.perf_counter() - t0 > 8.0 or rounds == 4:
            break
    dt = time.perf_counter() - t0
    return {"value": round(done * B / dt, 2), "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d micro-batches (B=%d, M=%d) forward+backward in %d round(s), one update per round; "
                      "numpy float64" % (done, B, M, rounds),
            "seconds": round(dt, 2)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None, help="one configuration only (default: cfg1 .. cfg5, headline cfg4)")
    ap.add_argument("--profile-all", action="store_true", help="time every kernel, table on stderr")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-two-streams", action="store_true", help="skip the extra K = 3 / forward-stream timing")
    ap.add_argument("--K", type=int, default=1, help="micro-batches in flight (stash slots): K forward passes, then 1F1B")
    ap.add_argument("--forward-stream", action="store_true",
                    help="forward passes on a second stream (needs --K 2 or more to overlap anything)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    run(args)


if __name__ == "__main__":
    main()
