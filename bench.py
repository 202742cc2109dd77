"""Benchmark: effective HBM GB/s of the fused layout chain on one MI355X.

A step is one execution of the composed map of the workload (one kernel launch
through the C ABI) on source/destination buffers that rotate through enough
independent sets that nothing survives in the last-level cache between steps.
Effective bytes = every needed source element read once + every destination
element written once.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
COLD_FOOTPRINT = 1 << 30


def _rotating_sets(torch, device, B, m, w, min_total):
    info = B.amap_describe(m)
    per_set = info.write_bytes + sum(int(__import__("numpy").prod(s)) * w.elem_size for s in w.src_shapes)
    n_sets = max(2, -(-min_total // per_set))
    host = w.sources()
    sets = []
    for _ in range(n_sets):
        srcs = [device.to_device(s) for s in host]
        dst = device.empty_dst(m, fill=0)
        arr = (C.c_void_p * len(srcs))(*[s.data_ptr() for s in srcs])
        sets.append((srcs, dst, arr))
    return sets


def _time_launches(torch, fn, sets, steps, warmup):
    for i in range(warmup):
        fn(sets[i % len(sets)])
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        fn(sets[i % len(sets)])
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    gpu_ms = e0.elapsed_time(e1) / steps
    return wall_ms, gpu_ms


def _time_legs(torch, legs, sets, steps, warmup, repeats=5, settle=150):
    """Median kernel-side ms per launch of each leg over `repeats` interleaved rounds.  A run of
    matrix-core launches first goes through the power controller's transient (the first ~10 ms of
    load run up to 20 % slower, whichever leg comes first), so `settle` untimed launches precede
    the rounds and the legs alternate instead of running one after the other."""
    for i in range(settle):
        legs[0](sets[i % len(sets)])
    per_leg = [[] for _ in legs]
    for _ in range(repeats):
        for k, fn in enumerate(legs):
            per_leg[k].append(_time_launches(torch, fn, sets, steps, warmup)[1])
    return [sorted(v)[len(v) // 2] for v in per_leg]


def _unfused_maps(B, w):
    """One map per operator: the program before data-movement elimination."""
    maps, shapes = [], [tuple(s) for s in w.src_shapes]
    for op in w.ops:
        m = B.amap_compose(shapes, w.elem_size, [op])
        maps.append(m)
        shapes = [B.dst_shape(m)]
    return maps


def _unfused_maps_views_free(B, w):
    """The chain as a framework runs it at best: reshape and leading-dimension slices are views (they
    cost nothing and are read through by the next copy), every other operator is one materialising copy."""
    maps, shapes, pending = [], [tuple(s) for s in w.src_shapes], []
    for op in w.ops:
        cur = B.dst_shape(B.amap_compose(shapes, w.elem_size, pending)) if pending else shapes[0]
        view = op[0] == "reshape" or (op[0] == "slice" and op[4] == 1 and all(e == 1 for e in cur[:op[1]]))
        if view and len(shapes) == 1:
            pending.append(op)
            continue
        m = B.amap_compose(shapes, w.elem_size, pending + [op])
        maps.append(m)
        shapes, pending = [B.dst_shape(m)], []
    return maps


def bench_workload(torch, device, B, synth, name, steps, warmup, with_unfused=True, with_hot=True, **kw):
    w = synth.workload(name, **kw)
    m = B.amap_compose(w.src_shapes, w.elem_size, w.ops)
    info = B.amap_describe(m)
    min_bytes = info.min_read_bytes + info.write_bytes
    stream = C.c_void_p(device.current_stream())
    sets = _rotating_sets(torch, device, B, m, w, COLD_FOOTPRINT)

    def fused(s):
        st = B.raw.amap_execute(s[2], C.c_void_p(s[1].data_ptr()), m.handle, stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    wall_ms, gpu_ms = _time_launches(torch, fused, sets, steps, warmup)
    hot_gpu = _time_launches(torch, fused, sets[:1], steps, warmup)[1] if with_hot else float("nan")
    res = {
        "workload": w.name, "min_bytes": int(min_bytes), "kernel": B.KERNEL_NAMES[info.kernel_id],
        "pieces": info.n_pieces, "cold_sets": len(sets),
        "fused_ms": wall_ms, "fused_kernel_ms": gpu_ms,
        "fused_gbs": min_bytes / wall_ms / 1e6, "fused_kernel_gbs": min_bytes / gpu_ms / 1e6,
        "hot_kernel_gbs": min_bytes / hot_gpu / 1e6,
    }
    if with_hot and len(sets) >= 4:
        # context, not the headline: the same launches issued round-robin on four streams, so that
        # the ramp-up of one launch overlaps the tail of another
        streams = [torch.cuda.Stream() for _ in range(4)]
        handles = [C.c_void_p(st.cuda_stream) for st in streams]

        def piped(i):
            s = sets[i % len(sets)]
            st = B.raw.amap_execute(s[2], C.c_void_p(s[1].data_ptr()), m.handle, handles[i % 4])
            if st != 0:
                raise RuntimeError(B.amap_status_str(st))

        torch.cuda.synchronize()
        for i in range(warmup):
            piped(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            piped(i)
        torch.cuda.synchronize()
        res["four_streams_gbs"] = min_bytes * steps / (time.perf_counter() - t0) / 1e9
    if with_unfused:
        maps = _unfused_maps(B, w)
        inter = [device.empty_dst(mm) for mm in maps]

        def unfused(s):
            cur = s[2]
            for k, mm in enumerate(maps):
                out = s[1] if k == len(maps) - 1 else inter[k]
                st = B.raw.amap_execute(cur, C.c_void_p(out.data_ptr()), mm.handle, stream)
                if st != 0:
                    raise RuntimeError(B.amap_status_str(st))
                cur = (C.c_void_p * 1)(out.data_ptr())

        u_wall, u_gpu = _time_launches(torch, unfused, sets, max(10, steps // 4), max(2, warmup // 4))
        res.update({"unfused_ms": u_wall, "unfused_gbs": min_bytes / u_wall / 1e6, "unfused_ops": len(maps),
                    "speedup_vs_unfused": u_wall / wall_ms})
        # the same with views free (what a framework's eager chain costs at best)
        vmaps = _unfused_maps_views_free(B, w)
        if vmaps:
            vbufs = [device.empty_dst(mm) for mm in vmaps]   # trailing views may leave the last copy larger than dst

            def views_free(s):
                cur = s[2]
                for mm, out in zip(vmaps, vbufs):
                    st = B.raw.amap_execute(cur, C.c_void_p(out.data_ptr()), mm.handle, stream)
                    if st != 0:
                        raise RuntimeError(B.amap_status_str(st))
                    cur = (C.c_void_p * 1)(out.data_ptr())

            v_wall, v_gpu = _time_launches(torch, views_free, sets, max(10, steps // 4), max(2, warmup // 4))
            res.update({"unfused_views_free_ms": v_wall, "unfused_views_free_copies": len(vmaps),
                        "speedup_vs_unfused_views_free": v_wall / wall_ms})
    del sets
    torch.cuda.empty_cache()
    return res


def bench_gemm(torch, device, B, synth, steps, warmup, fused_only=False):
    """Fused-prologue GEMM of cfg4 next to: materialise A with the same library, then the
    same GEMM kernel on the materialised A (identity map).  fused_only: nothing but the fused
    launches (for profiler runs)."""
    w = synth.workload("cfg4")
    m = B.amap_compose(w.src_shapes, 2, w.ops)
    M, K = B.dst_shape(m)
    N = w.gemm_n
    ident = B.amap_compose([(M, K)], 2, [])
    stream = C.c_void_p(device.current_stream())
    src_h, w_h = w.sources()[0], w.weight()
    per_set = src_h.nbytes + w_h.nbytes + M * N * 2 + M * K * 2
    sets = []
    for _ in range(max(2, -(-COLD_FOOTPRINT // per_set))):
        sets.append((device.to_device(src_h), device.to_device(w_h),
                     torch.empty((M, N), dtype=torch.int16, device="cuda"),
                     torch.empty((M, K), dtype=torch.int16, device="cuda")))

    def fused(s):
        st = B.raw.amap_gemm_fused(C.c_void_p(s[0].data_ptr()), m.handle, C.c_void_p(s[1].data_ptr()),
                                   C.c_int64(N), C.c_void_p(s[2].data_ptr()), stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    def unfused(s):
        arr = (C.c_void_p * 1)(s[0].data_ptr())
        st = B.raw.amap_execute(arr, C.c_void_p(s[3].data_ptr()), m.handle, stream)
        st = st or B.raw.amap_gemm_fused(C.c_void_p(s[3].data_ptr()), ident.handle, C.c_void_p(s[1].data_ptr()),
                                         C.c_int64(N), C.c_void_p(s[2].data_ptr()), stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    # the same product with the weight kept transposed ([N,K], read through a transpose map):
    # its k runs go to LDS as they are, no transposition in registers
    wt_map = B.amap_compose([(N, K)], 2, [("transpose", (1, 0))])

    def fused_wt(s):
        st = B.raw.amap_gemm_mapped(C.c_void_p(s[0].data_ptr()), m.handle, C.c_void_p(s[1].data_ptr()), wt_map.handle,
                                    None, C.c_void_p(s[2].data_ptr()), stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    def vendor(s):
        # context only: the vendor library's product on the materialised A of the unfused leg
        torch.matmul(s[3].view(torch.bfloat16), s[1].view(torch.bfloat16), out=s[2].view(torch.bfloat16))

    flops = 2.0 * M * N * K
    if fused_only:
        f_gpu = _time_launches(torch, fused, sets, steps, warmup)[1]
        return {"workload": "cfg4", "fused_ms": round(f_gpu, 5), "fused_tflops": round(flops / f_gpu / 1e9, 1),
                "algorithmic_bytes": src_h.nbytes + w_h.nbytes + M * N * 2}
    f_gpu, u_gpu, t_gpu, v_gpu = _time_legs(torch, [fused, unfused, fused_wt, vendor], sets, steps, warmup)
    del sets
    torch.cuda.empty_cache()
    return {"workload": "cfg4: C[8192,4096] = A[8192,1024] x W[1024,4096], A read through permute+reshape of [16,16,512,64]",
            "fused_transposed_weight_ms": round(t_gpu, 5), "fused_transposed_weight_tflops": round(flops / t_gpu / 1e9, 1),
            "fused_ms": round(f_gpu, 5), "fused_tflops": round(flops / f_gpu / 1e9, 1),
            "mfma_peak_tflops": 2500.0, "frac_of_mfma_peak": round(flops / f_gpu / 1e9 / 2500.0, 4),
            "unfused_ms": round(u_gpu, 5), "unfused_tflops": round(flops / u_gpu / 1e9, 1),
            "speedup_vs_unfused": round(u_gpu / f_gpu, 3), "dtype": "bf16 in, fp32 accumulate, bf16 out",
            "vendor_matmul_on_materialised_A_ms": round(v_gpu, 5),
            "protocol": "median of 5 interleaved rounds per leg, after 150 settling launches"}


def bench_gemm_store(torch, device, B, synth, steps, warmup):
    """QKV projection whose product is stored straight in the head-split layout of cfg2-fwd
    ([3,16,12,512,64]) next to: plain product, then the cfg2-fwd map as its own kernel."""
    w2 = synth.workload("cfg2_fwd")
    M, K, N = 16 * 512, 768, 2304
    a_map = B.amap_compose([(M, K)], 2, [])
    out_map = B.amap_compose([(M, N)], 2, [("reshape", (16, 512, 2304))] + list(w2.ops))
    stream = C.c_void_p(device.current_stream())
    per_set = (M * K + K * N + 2 * M * N) * 2
    sets = []
    for i in range(max(2, -(-COLD_FOOTPRINT // per_set))):
        g = torch.Generator(device="cuda").manual_seed(i)
        sets.append((torch.randint(-16000, 16000, (M, K), dtype=torch.int16, device="cuda", generator=g),
                     torch.randint(-16000, 16000, (K, N), dtype=torch.int16, device="cuda", generator=g),
                     torch.empty((M, N), dtype=torch.int16, device="cuda"),
                     torch.empty((M, N), dtype=torch.int16, device="cuda")))

    def fused(s):
        st = B.raw.amap_gemm_fused_store(C.c_void_p(s[0].data_ptr()), a_map.handle, C.c_void_p(s[1].data_ptr()),
                                         C.c_int64(N), out_map.handle, C.c_void_p(s[3].data_ptr()), stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    def unfused(s):
        st = B.raw.amap_gemm_fused(C.c_void_p(s[0].data_ptr()), a_map.handle, C.c_void_p(s[1].data_ptr()),
                                   C.c_int64(N), C.c_void_p(s[2].data_ptr()), stream)
        arr = (C.c_void_p * 1)(s[2].data_ptr())
        st = st or B.raw.amap_execute(arr, C.c_void_p(s[3].data_ptr()), out_map.handle, stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    f_gpu, u_gpu = _time_legs(torch, [fused, unfused], sets, steps, warmup)
    flops = 2.0 * M * N * K
    del sets
    torch.cuda.empty_cache()
    return {"workload": "QKV projection C[8192,2304] = A[8192,768] x W[768,2304] stored as [3,16,12,512,64]",
            "fused_ms": round(f_gpu, 5), "fused_tflops": round(flops / f_gpu / 1e9, 1),
            "unfused_ms": round(u_gpu, 5), "speedup_vs_unfused": round(u_gpu / f_gpu, 3)}


def bench_gemm_nchw(torch, device, B, synth, steps, warmup):
    """Pointwise convolution on a channel-major activation: the NCHW -> NHWC transposition of
    cfg1 (without its padding) folded into the A operand of the product with a [256,512] weight,
    next to: transposition as its own kernel, then the same GEMM on the NHWC copy."""
    n, c, h, wd, N = 32, 256, 56, 56, 512
    a_map = B.amap_compose([(n, c, h, wd)], 2, [("transpose", (0, 2, 3, 1)), ("reshape", (n * h * wd, c))])
    M, K = B.dst_shape(a_map)
    ident = B.amap_compose([(M, K)], 2, [])
    stream = C.c_void_p(device.current_stream())
    per_set = (2 * M * K + K * N + M * N) * 2
    sets = []
    for i in range(max(2, -(-COLD_FOOTPRINT // per_set))):
        g = torch.Generator(device="cuda").manual_seed(40 + i)
        sets.append((torch.randn((n, c, h, wd), device="cuda", generator=g).bfloat16().view(torch.int16),
                     (0.05 * torch.randn((K, N), device="cuda", generator=g)).bfloat16().view(torch.int16),
                     torch.empty((M, N), dtype=torch.int16, device="cuda"),
                     torch.empty((M, K), dtype=torch.int16, device="cuda")))

    def fused(s):
        st = B.raw.amap_gemm_fused(C.c_void_p(s[0].data_ptr()), a_map.handle, C.c_void_p(s[1].data_ptr()),
                                   C.c_int64(N), C.c_void_p(s[2].data_ptr()), stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    def unfused(s):
        arr = (C.c_void_p * 1)(s[0].data_ptr())
        st = B.raw.amap_execute(arr, C.c_void_p(s[3].data_ptr()), a_map.handle, stream)
        st = st or B.raw.amap_gemm_fused(C.c_void_p(s[3].data_ptr()), ident.handle, C.c_void_p(s[1].data_ptr()),
                                         C.c_int64(N), C.c_void_p(s[2].data_ptr()), stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    f_gpu, u_gpu = _time_legs(torch, [fused, unfused], sets, steps, warmup)
    flops = 2.0 * M * N * K
    min_bytes = (M * K + K * N + M * N) * 2
    del sets
    torch.cuda.empty_cache()
    return {"workload": "pointwise convolution C[100352,512] = NHWC view of x[32,256,56,56] (runs along m) x W[256,512]",
            "fused_ms": round(f_gpu, 5), "fused_tflops": round(flops / f_gpu / 1e9, 1),
            "fused_gbs": round(min_bytes / f_gpu / 1e6, 1),
            "unfused_ms": round(u_gpu, 5), "speedup_vs_unfused": round(u_gpu / f_gpu, 3)}


def bench_gemm_gather(torch, device, B, synth, steps, warmup):
    """Inception-style block end: the channel concat of four NCHW branches (cfg3's shapes at batch 128)
    and the NCHW -> NHWC transposition folded into the A operand of the following pointwise
    convolution, next to: cfg3's fused concat+transposition kernel, then the GEMM on its output."""
    w = synth.workload("cfg3", n=128)
    N = 256
    a_map = B.amap_compose(w.src_shapes, 2, list(w.ops) + [("reshape", (128 * 28 * 28, 320))])
    M, K = B.dst_shape(a_map)
    ident = B.amap_compose([(M, K)], 2, [])
    stream = C.c_void_p(device.current_stream())
    per_set = (2 * M * K + K * N + M * N) * 2
    sets = []
    for i in range(max(2, -(-COLD_FOOTPRINT // per_set))):
        g = torch.Generator(device="cuda").manual_seed(60 + i)
        srcs = [torch.randn(tuple(s), device="cuda", generator=g).bfloat16().view(torch.int16) for s in w.src_shapes]
        sets.append((srcs, (0.05 * torch.randn((K, N), device="cuda", generator=g)).bfloat16().view(torch.int16),
                     torch.empty((M, N), dtype=torch.int16, device="cuda"),
                     torch.empty((M, K), dtype=torch.int16, device="cuda"),
                     (C.c_void_p * len(srcs))(*[t.data_ptr() for t in srcs])))

    def fused(s):
        st = B.raw.amap_gemm_gather(s[4], a_map.handle, C.c_void_p(s[1].data_ptr()), None, C.c_int64(N), None,
                                    C.c_void_p(s[2].data_ptr()), stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    def unfused(s):
        st = B.raw.amap_execute(s[4], C.c_void_p(s[3].data_ptr()), a_map.handle, stream)
        st = st or B.raw.amap_gemm_fused(C.c_void_p(s[3].data_ptr()), ident.handle, C.c_void_p(s[1].data_ptr()),
                                         C.c_int64(N), C.c_void_p(s[2].data_ptr()), stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    f_gpu, u_gpu = _time_legs(torch, [fused, unfused], sets, steps, warmup)
    flops = 2.0 * M * N * K
    min_bytes = (M * K + K * N + M * N) * 2
    del sets
    torch.cuda.empty_cache()
    return {"workload": "pointwise convolution C[100352,256] on the channel concat of four NCHW branches "
                        "[128,{64,96,128,32},28,28] (A gathered from four sources, runs along m)",
            "fused_ms": round(f_gpu, 5), "fused_tflops": round(flops / f_gpu / 1e9, 1),
            "fused_gbs": round(min_bytes / f_gpu / 1e6, 1),
            "unfused_ms": round(u_gpu, 5), "speedup_vs_unfused": round(u_gpu / f_gpu, 3)}


def bench_multi(torch, device, B, synth, steps, warmup):
    """Q, K and V of cfg2-fwd as three separately allocated outputs: three amap_execute calls
    against one amap_execute_multi call (the same pieces, packed into one launch)."""
    w = synth.workload("cfg2_fwd")
    maps = [B.amap_compose(w.src_shapes, 2, synth.split_qkv_ops(t)) for t in range(3)]
    handles = (C.c_void_p * 3)(*[m.handle for m in maps])
    stream = C.c_void_p(device.current_stream())
    host = w.sources()
    per_set = 2 * host[0].nbytes
    sets = []
    for _ in range(max(2, -(-COLD_FOOTPRINT // per_set))):
        src = device.to_device(host[0])
        dsts = [device.empty_dst(m) for m in maps]
        sets.append((src, dsts, (C.c_void_p * 1)(src.data_ptr()), (C.c_void_p * 3)(*[d.data_ptr() for d in dsts])))

    def separate(s):
        for t in range(3):
            st = B.raw.amap_execute(s[2], C.c_void_p(s[1][t].data_ptr()), maps[t].handle, stream)
            if st != 0:
                raise RuntimeError(B.amap_status_str(st))

    def together(s):
        st = B.raw.amap_execute_multi(s[2], s[3], handles, 3, stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    s_wall, s_gpu = _time_launches(torch, separate, sets, steps, warmup)
    t_wall, t_gpu = _time_launches(torch, together, sets, steps, warmup)
    nbytes = 2 * host[0].nbytes
    del sets
    torch.cuda.empty_cache()
    return {"workload": "cfg2-fwd head split into three separately allocated outputs [16,12,512,64]",
            "min_bytes": nbytes, "three_calls_ms": round(s_gpu, 5), "three_calls_gbs": round(nbytes / s_gpu / 1e6, 1),
            "one_multi_call_ms": round(t_gpu, 5), "one_multi_call_gbs": round(nbytes / t_gpu / 1e6, 1),
            "speedup": round(s_gpu / t_gpu, 3)}


def bench_layout(torch, device, B, synth, steps, warmup):
    """Global layout assignment on the synthetic ResNet-like graph: relayout copies (count, bytes,
    time of running them as transpose maps) of the per-operator assignment against those left
    after propagation.  The local assignment's copies are rebuilt here from the same rules."""
    tensors, ops = synth.resnet_like_layout_graph(batch=32)
    g = B.LayoutGraph()
    for shape, fixed in tensors:
        g.tensor(shape, 2, fixed)
    for operands, outs, reqs, same in ops:
        g.op(operands, outs, reqs, same)
    rep = g.solve()
    stream = C.c_void_p(device.current_stream())

    def timed(maps):
        work = []
        for m in maps:
            info = B.amap_describe(m)
            src = torch.zeros(int(info.min_read_bytes // 2), dtype=torch.int16, device="cuda")
            work.append((m, (C.c_void_p * 1)(src.data_ptr()), device.empty_dst(m), src))

        def run(_):
            for m, arr, dst, _src in work:
                st = B.raw.amap_execute(arr, C.c_void_p(dst.data_ptr()), m.handle, stream)
                if st != 0:
                    raise RuntimeError(B.amap_status_str(st))
        return _time_launches(torch, run, [None], steps, warmup)[1] if work else 0.0

    glob = [m for _, _, _, m in g.copies()]
    # per-operator assignment: canonical order unless the operator asks for another one
    canon = lambda t: tuple(range(len(tensors[t][0])))
    written = {}
    for operands, outs, reqs, same in ops:
        for si, t in enumerate(operands):
            if outs[si]:
                written[t] = tuple(reqs[si]) if reqs and reqs[si] is not None else canon(t)
    local = []
    for operands, outs, reqs, same in ops:
        for si, t in enumerate(operands):
            if outs[si]:
                continue
            have = written.get(t, tensors[t][1] or canon(t))
            need = tuple(reqs[si]) if reqs and reqs[si] is not None else canon(t)
            if tuple(have) != need:
                shape = tensors[t][0]
                local.append(B.amap_transpose(B.amap_source(0, [shape[k] for k in have], 2), [have.index(d) for d in need]))
    return {"workload": "ResNet-like graph, 36 convolutions, bf16 activations, batch 32 (synthetic)",
            "copies_local": rep.n_copies_local, "copy_bytes_local": rep.copy_bytes_local,
            "copies_global": rep.n_copies_global, "copy_bytes_global": rep.copy_bytes_global,
            "sweeps": rep.n_sweeps, "local_copies_rebuilt": len(local),
            "local_ms": round(timed(local), 4), "global_ms": round(timed(glob), 4)}


def bench_graph(torch, device, B, synth, steps, warmup):
    """Graph-level data-movement elimination on the synthetic WaveNet-like graph: time of all
    layout operators run one at a time (each a materialising copy) against the composed maps
    that are left (non-identity loads of the compute operators + graph outputs).  The compute
    operators themselves are the same on both sides and are not run."""
    g = synth.wavenet_like_graph(layers=10, batch=8, channels=128, steps=4096, skip_steps=512)
    es = g.elem_size
    dme = B.GraphDME(g.nodes, g.outputs, es)
    rep = dme.eliminate()
    stream = C.c_void_p(device.current_stream())
    dt = torch.int16 if es == 2 else torch.int32
    shapes, buf = {}, {}
    single = []   # (map, source ids, dst id) of every layout operator on its own
    for i, n in enumerate(g.nodes):
        if n[0] == "input":
            shapes[i] = n[1]
        elif n[0] == "compute":
            shapes[i] = n[3]
        else:
            m = B.amap_compose([shapes[k] for k in n[2]], es, [n[1]])
            shapes[i] = B.dst_shape(m)
            single.append((m, n[2], i))
        buf[i] = torch.zeros(shapes[i], dtype=dt, device="cuda")
    composed = []  # (map, source ids, dst buffer)
    for cons, slot, m, ids in dme.loads():
        info = B.amap_describe(m)
        ident = len(ids) == 1 and info.n_pieces == 1 and info.kernel_id == B.AMAP_K_ROWS and \
            tuple(info.shape[k] for k in range(info.rank)) == tuple(shapes[ids[0]]) and info.fill_bytes == 0 and \
            info.min_read_bytes == info.write_bytes
        if cons >= 0 and ident:
            continue
        composed.append((m, ids, device.empty_dst(m)))

    def run(items, dst_of, st_handle=stream):
        for m, ids, d in items:
            arr = (C.c_void_p * max(1, len(ids)))(*[buf[k].data_ptr() for k in ids])
            st = B.raw.amap_execute(arr, C.c_void_p(dst_of(d).data_ptr()), m.handle, st_handle)
            if st != 0:
                raise RuntimeError(B.amap_status_str(st))

    u_wall, u_gpu = _time_launches(torch, lambda _: run(single, lambda d: buf[d]), [None], steps, warmup)
    o_wall, o_gpu = _time_launches(torch, lambda _: run(composed, lambda d: d), [None], steps, warmup)
    # the same composed maps replayed from a HIP graph (the calls allocate nothing and never synchronise)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        h = C.c_void_p(side.cuda_stream)
        run(composed, lambda d: d, h)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run(composed, lambda d: d, h)
    g_wall, g_gpu = _time_launches(torch, lambda _: graph.replay(), [None], steps, warmup)
    return {"workload": "WaveNet-like graph, 10 gated layers, bf16 [8,128,4096] activations (synthetic)",
            "layout_ops": rep.n_layout_ops, "pairs": rep.n_pairs, "pairs_left": rep.n_pairs_left,
            "rewrites": rep.n_rewrites, "loads": rep.n_loads, "mapped_loads": rep.n_mapped_loads,
            "moved_bytes_before": rep.moved_bytes_before,
            "moved_bytes_after_fused_consumers": rep.moved_bytes_after,
            "moved_bytes_after_materialised_loads": rep.moved_bytes_after + rep.mapped_load_bytes,
            "intermediate_bytes_eliminated": rep.intermediate_bytes,
            "kernels_before": len(single), "kernels_after": len(composed),
            "before_ms": round(u_gpu, 4), "after_ms": round(o_gpu, 4), "speedup": round(u_gpu / o_gpu, 3),
            "after_hip_graph_ms": round(g_gpu, 4)}


def bench_small_permute(torch, device, B, synth, steps, warmup):
    """Short dst rows at bandwidth sizes (>= 1 GiB moved per launch): the cross-lane form (one vector per
    lane, V x V blocks exchanged between lanes) against the register micro-transpose of the tile
    kernels, chosen with the planner's AMAP_XLANE switch (2: wherever it applies, 0: nowhere; unset:
    the planner's own choice)."""
    out = {}
    for name, kw in (("cfg0", {"n": 10240}), ("c8_nhwc", {"n": 8192})):
        row = {}
        for label, setting in (("cross_lane", "2"), ("micro_transpose", "0"), ("default", None)):
            if setting is None:
                os.environ.pop("AMAP_XLANE", None)
            else:
                os.environ["AMAP_XLANE"] = setting
            try:
                r = bench_workload(torch, device, B, synth, name, steps, warmup, with_unfused=False, with_hot=False, **kw)
            finally:
                os.environ.pop("AMAP_XLANE", None)
            row["min_bytes"] = r["min_bytes"]
            row[label] = {"kernel": r["kernel"], "kernel_ms": round(r["fused_kernel_ms"], 4),
                          "kernel_gbs": round(r["fused_kernel_gbs"], 1)}
        out[r["workload"]] = row
    return out


def cpu_baseline(synth, name, min_bytes, budget_s=12.0):
    from oracle import oracle
    w = synth.workload(name)
    srcs = w.sources()
    oracle.set_threads(1)
    oracle.run_chain(srcs, w.ops)  # warm-up pass (page faults)
    n, t0 = 0, time.perf_counter()
    while True:
        oracle.run_chain(srcs, w.ops)
        n += 1
        dt = time.perf_counter() - t0
        if dt > budget_s or n >= 20:
            break
    res = {"value": min_bytes * n / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
           "sample": f"{n} full passes of the {name} chain, operator by operator with materialised intermediates",
           "ms_per_pass": dt / n * 1e3}
    # the same oracle with its outermost loop spread over the host cores this process may use
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
    if cores > 1:
        oracle.set_threads(cores)
        oracle.run_chain(srcs, w.ops)
        n2, t0 = 0, time.perf_counter()
        while True:
            oracle.run_chain(srcs, w.ops)
            n2 += 1
            dt2 = time.perf_counter() - t0
            if dt2 > budget_s / 3 or n2 >= 20:
                break
        oracle.set_threads(1)
        res["all_cores"] = {"value": min_bytes * n2 / dt2 / 1e9, "unit": "GB/s", "cores": cores,
                            "ms_per_pass": dt2 / n2 * 1e3}
    return res


MAP_SOURCES = ["paper_2002_12798_amd/csrc/amap_kernels.hip", "paper_2002_12798_amd/csrc/amap_index.hpp",
               "paper_2002_12798_amd/csrc/amap_compose.cpp", "paper_2002_12798_amd/csrc/amap_plan.cpp",
               "paper_2002_12798_amd/csrc/amap_device.hpp"]
GEMM_SOURCES = ["paper_2002_12798_amd/csrc/amap_gemm.hip", "paper_2002_12798_amd/csrc/amap_compose.cpp"]
COPY_ELEMENTS = 53248000               # 2-byte elements moved by `--copy-only`: 106,496,000 B read and as many written


def _traffic_sources(workload):
    """The sources whose change invalidates a traffic record: those of the kernel that ran."""
    return GEMM_SOURCES if workload == "cfg4" else MAP_SOURCES


def _sources_hash(files):
    import hashlib
    h = hashlib.sha256()
    for f in files:
        h.update(open(os.path.join(ROOT, f), "rb").read())
    return h.hexdigest()


def measured_traffic(workload):
    """HBM bytes per launch from the committed rocprofv3 counter runs, or None if the
    kernel sources have changed since they were taken (or no counters exist for the workload)."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    files = _traffic_sources(workload)
    if rec.get("sources") != files or rec.get("sources_sha256") != _sources_hash(files):
        return None
    return round(rec["traffic_bytes_per_launch"])


def record_traffic(d, workload):
    """Turn rocprofv3 --pmc runs (csv, one counter set per run) into profiles/traffic_<workload>.json.
    Expected in `d`:  <tag>_<set>_counter_collection.csv  with tag = the workload and "copy"
    (`bench.py --copy-only`, the plain copy of known size that scales the counters) and set =
      FETCH_SIZE, WRITE_SIZE            the derived counters (KiB per dispatch)
      RD  (optional)                    TCC_EA0_RDREQ_sum TCC_EA0_RDREQ_32B_sum TCC_EA0_RDREQ_DRAM_sum TCC_BUBBLE_sum
      WR  (optional)                    TCC_EA0_WRREQ_sum TCC_EA0_WRREQ_64B_sum TCC_EA0_WRREQ_DRAM_sum
    RD / WR give a second reading from other counters: requests that went to DRAM, scaled by what the
    same counter reads per byte of the plain copy."""
    import csv
    import re
    import statistics
    # the map kernels (amap_pieces_kernel, amap_rows_kernel, amap_tile16_kernel) or the GEMM kernels
    kernel = "amap_gemm" if workload == "cfg4" else "amap_map"
    copy_bytes = 2 * COPY_ELEMENTS

    def means(tag, cset, kname):
        path = os.path.join(d, f"{tag}_{cset}_counter_collection.csv")
        if not os.path.exists(path):
            return None
        per, names = {}, set()
        for r in csv.DictReader(open(path)):
            n = r["Kernel_Name"]
            hit = ("amap_gemm" in n) if kname == "amap_gemm" else ("amap_" in n and "amap_gemm" not in n)
            if hit:
                names.add(re.search(r"amap_\w+", n).group(0))
                per.setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
        out = {k: (statistics.mean(v), len(v)) for k, v in per.items()}
        out["_kernels"] = sorted(names)
        return out

    files = _traffic_sources(workload)
    rec = {"workload": workload, "kernel": kernel, "sources": files, "sources_sha256": _sources_hash(files)}
    f, c = means(workload, "FETCH_SIZE", kernel), means("copy", "FETCH_SIZE", "amap_map")
    wf, wc = means(workload, "WRITE_SIZE", kernel), means("copy", "WRITE_SIZE", "amap_map")
    rec["kernel"] = f["_kernels"]
    rec["copy_kernel"] = c["_kernels"]
    rec["dispatches"] = f["FETCH_SIZE"][1]
    rec["fetch_kib_fused"], rec["fetch_kib_copy"] = f["FETCH_SIZE"][0], c["FETCH_SIZE"][0]
    rec["write_kib_fused"], rec["write_kib_copy"] = wf["WRITE_SIZE"][0], wc["WRITE_SIZE"][0]
    rec["fetch_factor"] = copy_bytes / (rec["fetch_kib_copy"] * 1024)
    rec["write_factor"] = copy_bytes / (rec["write_kib_copy"] * 1024)
    rec["read_bytes_per_launch"] = rec["fetch_kib_fused"] * 1024 * rec["fetch_factor"]
    rec["write_bytes_per_launch"] = rec["write_kib_fused"] * 1024 * rec["write_factor"]
    rec["traffic_bytes_per_launch"] = rec["read_bytes_per_launch"] + rec["write_bytes_per_launch"]
    rd, rdc = means(workload, "RD", kernel), means("copy", "RD", "amap_map")
    wr, wrc = means(workload, "WR", kernel), means("copy", "WR", "amap_map")
    if rd and rdc and wr and wrc:
        second = {"counters_fused": {k: v[0] for k, v in {**rd, **wr}.items() if k != "_kernels"},
                  "counters_copy": {k: v[0] for k, v in {**rdc, **wrc}.items() if k != "_kernels"}}
        second["bytes_per_dram_read_request_on_copy"] = copy_bytes / rdc["TCC_EA0_RDREQ_DRAM_sum"][0]
        second["bytes_per_dram_write_request_on_copy"] = copy_bytes / wrc["TCC_EA0_WRREQ_DRAM_sum"][0]
        second["read_bytes_per_launch"] = rd["TCC_EA0_RDREQ_DRAM_sum"][0] * second["bytes_per_dram_read_request_on_copy"]
        second["write_bytes_per_launch"] = wr["TCC_EA0_WRREQ_DRAM_sum"][0] * second["bytes_per_dram_write_request_on_copy"]
        second["traffic_bytes_per_launch"] = second["read_bytes_per_launch"] + second["write_bytes_per_launch"]
        rec["dram_request_counters"] = second
    out = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    json.dump(rec, open(out, "w"), indent=1)
    print(json.dumps(rec, indent=1))


def copy_ceiling(torch, device, B, n_bytes, steps, warmup):
    """Kernel-side GB/s of a plain copy that moves n_bytes in total (half read, half written) on cold
    rotating buffers: the identity map through this library and the vendor copy (Tensor.copy_), the
    better of the two.  What a kernel with no index arithmetic at all reaches at this size."""
    n = max(8, n_bytes // 4 // 8 * 8)
    m = B.amap_source(0, (n,), 2)
    n_sets = max(2, -(-COLD_FOOTPRINT // (4 * n)))
    sets = [(torch.zeros(n, dtype=torch.int16, device="cuda"), torch.empty(n, dtype=torch.int16, device="cuda"))
            for _ in range(n_sets)]
    stream = C.c_void_p(device.current_stream())

    def ours(s):
        st = B.raw.amap_execute((C.c_void_p * 1)(s[0].data_ptr()), C.c_void_p(s[1].data_ptr()), m.handle, stream)
        if st != 0:
            raise RuntimeError(B.amap_status_str(st))

    def vendor(s):
        s[1].copy_(s[0])

    t_ours = _time_launches(torch, ours, sets, steps, warmup)[1]
    t_vendor = _time_launches(torch, vendor, sets, steps, warmup)[1]
    del sets
    torch.cuda.empty_cache()
    return {"bytes": 4 * n, "identity_map_gbs": 4 * n / t_ours / 1e6, "vendor_copy_gbs": 4 * n / t_vendor / 1e6,
            "gbs": 4 * n / min(t_ours, t_vendor) / 1e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--scale", type=int, default=0,
                    help="batch extent of the workload instead of the named one (cfg1/cfg3: n, cfg2_*: b)")
    ap.add_argument("--no-extras", action="store_true", help="skip the other workloads and the CPU baseline")
    ap.add_argument("--copy-only", action="store_true",
                    help="launch only a plain copy (identity map) of 53,248,000 2-byte elements on cold buffers: "
                         "the known-size kernel that calibrates the rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--gemm-only", action="store_true", help="time only the fused-prologue GEMM (cfg4)")
    ap.add_argument("--next-only", action="store_true",
                    help="time only the repeat / tile / reversed-axis workloads and the graph-level elimination")
    ap.add_argument("--fused-only", action="store_true",
                    help="launch nothing but the fused kernel on cold buffers (for a clean rocprofv3 kernel summary); "
                         "with --gemm-only: nothing but the fused-prologue GEMM")
    ap.add_argument("--record-traffic", metavar="DIR",
                    help="no GPU work: turn the rocprofv3 --pmc csv files in DIR into profiles/traffic_<workload>.json")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if a.record_traffic:
        record_traffic(a.record_traffic, "cfg4" if a.gemm_only else a.workload)
        return

    import torch
    from paper_2002_12798_amd import binding as B
    from paper_2002_12798_amd import device, synth
    device.require_gpu()

    if a.copy_only:
        n = COPY_ELEMENTS
        m = B.amap_source(0, (n,), 2)
        sets = [(torch.zeros(n, dtype=torch.int16, device="cuda"), torch.empty(n, dtype=torch.int16, device="cuda"))
                for _ in range(11)]
        stream = C.c_void_p(device.current_stream())

        def copy(s):
            st = B.raw.amap_execute((C.c_void_p * 1)(s[0].data_ptr()), C.c_void_p(s[1].data_ptr()), m.handle, stream)
            if st != 0:
                raise RuntimeError(B.amap_status_str(st))

        wall, gpu = _time_launches(torch, copy, sets, a.steps, a.warmup)
        print(json.dumps({"workload": "plain copy of 106,496,000 B read + 106,496,000 B written per launch",
                          "read_bytes": 2 * n, "write_bytes": 2 * n, "kernel_ms": gpu, "gbs": 4 * n / gpu / 1e6}))
        return
    if a.gemm_only:
        print(json.dumps(bench_gemm(torch, device, B, synth, a.steps, a.warmup, fused_only=a.fused_only)))
        return
    if a.next_only:
        nxt = {}
        for name in synth.NEXT_WORKLOAD_NAMES:
            r = bench_workload(torch, device, B, synth, name, a.steps, a.warmup)
            nxt[r["workload"]] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()}
        print(json.dumps({"repeat_tile_reverse": nxt, "small_permute": bench_small_permute(torch, device, B, synth, 20, 3),
                          "graph_dme": bench_graph(torch, device, B, synth, 10, 2),
                          "execute_multi": bench_multi(torch, device, B, synth, a.steps, a.warmup),
                          "layout_assignment": bench_layout(torch, device, B, synth, 10, 2),
                          "fused_gemm_store": bench_gemm_store(torch, device, B, synth, a.steps, a.warmup),
                          "fused_gemm_nchw": bench_gemm_nchw(torch, device, B, synth, a.steps, a.warmup),
                          "fused_gemm_gather": bench_gemm_gather(torch, device, B, synth, a.steps, a.warmup)}))
        return
    if a.fused_only:
        a.no_extras = True
    scale_kw = {}
    if a.scale:
        scale_kw = {"b" if a.workload.startswith("cfg2") else "n": a.scale}
    main_res = bench_workload(torch, device, B, synth, a.workload, a.steps, a.warmup,
                              with_unfused=not a.fused_only, with_hot=not a.fused_only, **scale_kw)
    ceiling = None if a.fused_only else copy_ceiling(torch, device, B, main_res["min_bytes"], a.steps, a.warmup)
    extras = {}
    if not a.no_extras:
        for name, kw in [("cfg0", {}), ("cfg2_fwd", {}), ("cfg2_rev", {}), ("cfg3", {}),
                         ("cfg2_rev", {"b": 512}), ("cfg3", {"n": 1024})]:
            r = bench_workload(torch, device, B, synth, name, max(20, a.steps // 3), max(5, a.warmup // 3), **kw)
            extras[r["workload"]] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()}
    out = {
        "metric": "effective HBM GB/s of fused layout chain (% of MI355X peak) vs unfused chain",
        "value": round(main_res["fused_gbs"], 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(main_res["fused_ms"], 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16" if a.workload != "cfg0" else "u32",
        "data": "synthetic",
        "config": {"workload": f"{a.workload}: bf16 NCHW [32,256,56,56] -> NHWC + zero pad [32,58,58,256], one fused kernel"
                   if a.workload == "cfg1" else a.workload,
                   "cache": f"cold: {main_res['cold_sets']} rotating buffer sets (>= 1 GiB)",
                   "kernel": main_res["kernel"], "pieces": main_res["pieces"]},
        "pct_of_peak": round(100.0 * main_res["fused_gbs"] / HBM_PEAK_GBS, 2),
        "unfused_gbs": round(main_res.get("unfused_gbs", 0.0), 2),
        "speedup_vs_unfused": round(main_res.get("speedup_vs_unfused", 0.0), 3),
        "hot_cache_kernel_gbs": None if a.fused_only else round(main_res["hot_kernel_gbs"], 2),
        "four_streams_gbs": round(main_res["four_streams_gbs"], 2) if "four_streams_gbs" in main_res else None,
        "roofline": {"bound": "hbm", "achieved": round(main_res["fused_kernel_gbs"], 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(main_res["fused_kernel_gbs"] / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic(a.workload), "algorithmic_bytes": main_res["min_bytes"]},
    }
    if ceiling:
        # the same number of bytes moved by a plain copy: what the memory system gives a kernel of this size
        out["copy_ceiling_gbs"] = round(ceiling["gbs"], 2)
        out["copy_ceiling"] = {k: (round(v, 2) if isinstance(v, float) else v) for k, v in ceiling.items()}
        out["roofline"]["frac_of_copy_ceiling"] = round(main_res["fused_kernel_gbs"] / ceiling["gbs"], 4)
    if not a.no_extras:
        out["cpu_baseline"] = cpu_baseline(synth, a.workload, main_res["min_bytes"])
        out["other_workloads"] = extras
        out["fused_gemm"] = bench_gemm(torch, device, B, synth, max(20, a.steps // 3), max(5, a.warmup // 3))
        nxt = {}
        for name in synth.NEXT_WORKLOAD_NAMES:
            r = bench_workload(torch, device, B, synth, name, max(20, a.steps // 3), max(5, a.warmup // 3))
            nxt[r["workload"]] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()}
        out["repeat_tile_reverse"] = nxt
        out["fused_gemm_store"] = bench_gemm_store(torch, device, B, synth, max(20, a.steps // 3), max(5, a.warmup // 3))
        out["fused_gemm_nchw"] = bench_gemm_nchw(torch, device, B, synth, max(20, a.steps // 3), max(5, a.warmup // 3))
        out["fused_gemm_gather"] = bench_gemm_gather(torch, device, B, synth, max(20, a.steps // 3), max(5, a.warmup // 3))
        out["small_permute"] = bench_small_permute(torch, device, B, synth, 20, 3)
        out["execute_multi"] = bench_multi(torch, device, B, synth, max(20, a.steps // 3), max(5, a.warmup // 3))
        out["graph_dme"] = bench_graph(torch, device, B, synth, 10, 2)
        out["layout_assignment"] = bench_layout(torch, device, B, synth, 10, 2)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
