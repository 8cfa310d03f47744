#!/usr/bin/env python3
"""Decode-step benchmark of the HCAttention hot path on one MI355X.

A step is one decode step of the whole path over every layer of the workload: append + quantise
the new key (a1), scan the key cache (a2), top-k (a3), gather the selected values from pinned host
memory and attend (a4), and, every `evict_every` steps, accumulated-score eviction (a5).
Inputs are synthetic and seeded (synth_inputs.py) and resident (keys in HBM, values in pinned host
memory) before the timed region starts.

Prints one JSON line.
"""
import argparse
import faulthandler
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Model:
    """All layers of one workload: per-layer key cache / acc / pos / host values, shared scratch."""

    def __init__(self, w, layers, evict_every, total_steps, n_pipe=2, n_sel=3, evict_spare=False, fused=False,
                 host_chunks=0, host_threads=12, tune=None, n_pipe_sets=4, dual_scan="single"):
        import torch
        from paper_2507_19823_amd import binding as B
        self.torch, self.B, self.w = torch, B, w
        self.L = layers
        self.n0 = w.n
        self.evict_every = evict_every
        self.evict_spare = evict_spare
        self.cap = w.n + (evict_every if evict_every else total_steps) + 16
        self.vnew = total_steps + 16                  # value rows of appended tokens live in an HBM slice
        self.shape = B.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, self.cap, w.bits, w.group)
        self.rows = w.batch * w.n_kv_heads
        dev = "cuda"
        kb = B.hca_kcache_bytes(self.shape)
        self.kcache = [torch.empty(kb, dtype=torch.uint8, device=dev) for _ in range(layers)]
        self.acc = [torch.zeros(w.batch, w.n_kv_heads, self.cap, dtype=torch.float32, device=dev)
                    for _ in range(layers)]
        self.pos = [torch.arange(self.cap, dtype=torch.int32, device=dev).repeat(w.batch, w.n_kv_heads, 1).contiguous()
                    for _ in range(layers)]
        # one spare (cache, acc, pos) set: eviction writes the compacted layer into it and the buffers swap
        self.spare = (torch.empty(kb, dtype=torch.uint8, device=dev),
                      torch.zeros(w.batch, w.n_kv_heads, self.cap, dtype=torch.float32, device=dev),
                      torch.zeros(w.batch, w.n_kv_heads, self.cap, dtype=torch.int32, device=dev))
        self.v_host = [None] * layers
        self.v_hbm = [torch.zeros(w.batch, w.n_kv_heads, self.vnew, 128, dtype=torch.float16, device=dev)
                      for _ in range(layers)]
        # score buffers of the pipeline slots; with the fused scan + top-k a selection workspace per slot instead
        self.fused = fused
        self.host_chunks, self.host_threads, self.tune = host_chunks, host_threads, dict(tune or {})
        self.gap_report = False
        self.sels = [torch.empty(w.batch, w.n_kv_heads, self.cap, dtype=torch.float32, device=dev)
                     for _ in range(1 if fused else max(3, n_sel))]
        self.ws_sel = [torch.empty(B.hca_workspace_bytes(self.shape, w.k, 1), dtype=torch.uint8, device=dev)
                       for _ in range(max(3, n_sel) if fused else 0)]
        self.sel = self.sels[0]
        self.sel_ev = [dict(score_done=torch.cuda.Event(), sel_free=torch.cuda.Event()) for _ in range(3)]
        self.ws_main = torch.empty(B.hca_workspace_bytes(self.shape, w.k, self.n0), dtype=torch.uint8, device=dev)
        self.ws_topk = torch.empty(B.hca_workspace_bytes(self.shape, w.k, 1), dtype=torch.uint8, device=dev)
        wsa = B.hca_workspace_bytes(self.shape, w.k, 1)
        self.pipe = []
        self.n_pipe_sets = n_pipe_sets
        self.dual_scan = dual_scan
        self.layer_idx_on = False
        self.layer_idx = None
        # The layer whose results are checked against the oracle: one whose set of selection buffers is not taken
        # again later in the step (so its top-k indices are still there when the step ends), and among those the
        # one whose first eviction comes latest (the check covers the timed steps up to that eviction).
        self.verify_layer, self.verify_until = 0, total_steps - 1
        cands = range(max(0, layers - n_pipe_sets), layers)
        if evict_every:
            first = {l: (evict_every - 1 - l) % evict_every for l in cands}
            self.verify_layer = max(cands, key=lambda l: first[l])
            self.verify_until = first[self.verify_layer]
        else:
            self.verify_layer = max(cands)
        for _ in range(n_pipe_sets):
            self.pipe.append(dict(
                idx=torch.zeros(w.batch, w.n_kv_heads, w.k, dtype=torch.int32, device=dev),
                count=torch.zeros(w.batch, w.n_kv_heads, dtype=torch.int32, device=dev),
                ws=torch.empty(wsa, dtype=torch.uint8, device=dev),
                sel_done=torch.cuda.Event(), gather_done=torch.cuda.Event(),
                topk_done=torch.cuda.Event(), pipe_free=torch.cuda.Event()))
        self.layer_done = [torch.cuda.Event() for _ in range(layers)]
        self.y = torch.zeros(layers, w.batch, w.n_q_heads, 128, dtype=torch.float32, device=dev)
        self.n = [[0] * w.batch for _ in range(layers)]
        self.sm_scale = 1.0 / (128.0 ** 0.5)
        self.step_count = 0

    def build(self, phys_value_layers):
        """Generate each layer's context on the GPU, quantise it into the key cache (bulk a1) and park
        the values in pinned host memory.  Returns seconds spent in the bulk quantise calls."""
        import synth_inputs as S
        torch, B, w = self.torch, self.B, self.w
        tq = 0.0
        for l in range(self.L):
            d = S.make_layer(w, l, device="cuda", want_values=(l < phys_value_layers))
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            B.hca_quantize_keys(self.shape, self.kcache[l], d["keys"], w.n, self.n[l], None, None, None)
            e1.record()
            torch.cuda.synchronize()
            tq += e0.elapsed_time(e1) * 1e-3          # stream time of the call, not the host's wait for it
            self.n[l] = [w.n] * w.batch
            vh = None
            if l < phys_value_layers:
                try:
                    vh = torch.empty(w.batch, w.n_kv_heads, w.n, 128, dtype=torch.float16, pin_memory=True)
                except RuntimeError as e:          # the box refuses more pinned memory: share from here on
                    log(f"pinned allocation for layer {l} refused ({str(e).splitlines()[0]}); "
                        f"mapping logical layers onto {l} physical value layers")
                    phys_value_layers = l
            if vh is not None:
                vh.copy_(d["values"])
                self.v_host[l] = vh
                if self.host_chunks:                  # the host threads will read this store at random rows
                    t0 = time.perf_counter()
                    torch.cuda.synchronize()
                    B.hca_host_prefault(vh, 16)
                    self.prefault_s = getattr(self, "prefault_s", 0.0) + time.perf_counter() - t0
            elif phys_value_layers > 0:
                self.v_host[l] = self.v_host[l % phys_value_layers]   # logical layer shares a physical store
            if l == 0:
                self.layer0 = {"q": d["q"].cpu()}
            if l == self.verify_layer:                # the layer the oracle replays (cpu_baseline leg, verification)
                self.layerv = {k: (v.cpu() if v is not None and hasattr(v, "cpu") else v) for k, v in d.items()}
            del d
        self.phys = phys_value_layers
        return tq

    def make_steps(self, total_steps):
        """Pre-generate the appended token and the query of every (step, layer); values go to the host store."""
        import synth_inputs as S
        torch, w = self.torch, self.w
        self.k_new, self.q = [], []
        for t in range(total_steps):
            ks, qs = [], []
            for l in range(self.L):
                k_new, v_new, q = S.make_step(w, l, t)
                self.v_hbm[l][:, :, t] = v_new[:, :, 0].cuda()
                ks.append(k_new)
                qs.append(q)
            self.k_new.append(torch.stack(ks).cuda())
            self.q.append(torch.stack(qs).cuda())
        torch.cuda.synchronize()

    def scan_select(self, l, t, st, pipe, ev=None):
        """a1 + a2 + a3 of layer l, decode step t, on stream st."""
        if self.fused:
            B, w, n = self.B, self.w, self.n[l]
            B.hca_quantize_keys(self.shape, self.kcache[l], self.k_new[t][l], 1, n, self.acc[l], self.pos[l],
                                [self.n0 + t] * w.batch, st)
            self.n[l] = n = [x + 1 for x in n]
            if ev is not None:
                ev[0].record(st)
            B.hca_score_topk(self.shape, self.kcache[l], self.q[t][l], n, w.k, pipe["idx"], pipe["count"],
                             self.ws_main, st)
            if ev is not None:
                ev[1].record(st)
            return
        self.scan(l, t, st, self.sel, ev)
        self.B.hca_topk(self.shape, self.sel, self.n[l], self.w.k, pipe["idx"], pipe["count"], self.ws_main, st)

    def scan(self, l, t, st, sel, ev=None):
        """a1 + a2 of layer l, decode step t, on stream st: append the new key, scan the cache."""
        B, w = self.B, self.w
        n = self.n[l]
        B.hca_quantize_keys(self.shape, self.kcache[l], self.k_new[t][l], 1, n, self.acc[l], self.pos[l],
                            [self.n0 + t] * w.batch, st)
        n = [x + 1 for x in n]
        self.n[l] = n
        if ev is not None:
            ev[0].record(st)
        B.hca_score_qkeys(self.shape, self.kcache[l], self.q[t][l], n, sel, None, None, st)
        if ev is not None:
            ev[1].record(st)

    def gather(self, l, gst, pipe):
        """host-link half of a4: selected value rows -> staging, on the gather stream."""
        vh = self.v_host[l]
        self.B.hca_gather_values(self.shape, pipe["idx"], pipe["count"], self.w.k, self.pos[l], vh, vh.shape[2],
                                 vh.shape[2], self.v_hbm[l], self.vnew, pipe["ws"], gst)

    def attend_evict(self, l, t, st, pipe):
        """compute half of a4 (+ accumulated scores) and, when due, a5."""
        B, w = self.B, self.w
        B.hca_attend_gathered(self.shape, self.kcache[l], self.q[t][l], pipe["idx"], pipe["count"], w.k,
                              self.sm_scale, self.y[l], self.acc[l], pipe["ws"], st)
        if self.evict_due(l, t):
            sk, sa_, sp = self.spare
            B.hca_evict(self.shape, self.kcache[l], self.acc[l], self.pos[l], self.n[l], self.n0,
                        self.evict_every, None, self.ws_main, sk, sa_, sp, st)
            self.spare = (self.kcache[l], self.acc[l], self.pos[l])
            self.kcache[l], self.acc[l], self.pos[l] = sk, sa_, sp
            self.n[l] = [min(x, self.n0) for x in self.n[l]]

    def native_pipeline(self, sa, sb, sg, sc, timing_slots, timing_stride=1):
        """Hands the four streams and the pipeline buffers to the library's step driver."""
        import ctypes as C
        B, w = self.B, self.w
        d = B.hca_pipeline_desc()
        d.stream_scan, d.stream_topk = sa.cuda_stream, sb.cuda_stream
        d.stream_gather, d.stream_attend = sg.cuda_stream, sc.cuda_stream
        if self.fused:
            d.fused_select = 1
            for i, wbuf in enumerate(self.ws_sel):
                d.ws_select[i] = wbuf.data_ptr()
            d.n_sel = len(self.ws_sel)
        else:
            for i, sbuf in enumerate(self.sels):
                d.sel[i] = sbuf.data_ptr()
            d.n_sel = len(self.sels)
        d.timing_layer_stride = timing_stride
        d.n_pipe = self.n_pipe_sets
        d.dual_scan = {"single": 0, "dual": 1, "pair": 2}[self.dual_scan] if self.fused else 0
        for i in range(self.n_pipe_sets):
            d.idx[i] = self.pipe[i]["idx"].data_ptr()
            d.count[i] = self.pipe[i]["count"].data_ptr()
            d.ws_attend[i] = self.pipe[i]["ws"].data_ptr()
        if self.layer_idx_on:
            # one selection result per layer: the selections run in step with the scans, a set of staging buffers is
            # claimed only by the gather stage
            self.layer_idx = self.torch.zeros(self.L, w.batch, w.n_kv_heads, w.k, dtype=self.torch.int32, device="cuda")
            self.layer_count = self.torch.zeros(self.L, w.batch, w.n_kv_heads, dtype=self.torch.int32, device="cuda")
            d.layer_idx, d.layer_count = self.layer_idx.data_ptr(), self.layer_count.data_ptr()
            d.layer_idx_stride = w.batch * w.n_kv_heads * w.k
        d.ws_topk, d.ws_evict = self.ws_topk.data_ptr(), self.ws_main.data_ptr()
        if timing_slots > 0:
            pairs = B.hca_scan_stamp_pairs(self.shape, self.cap)
            self.stamps = self.torch.zeros(timing_slots, self.L, pairs, 2, dtype=self.torch.int64, device="cuda")
            d.scan_stamps, d.scan_stamp_pairs = self.stamps.data_ptr(), pairs
            if self.gap_report:
                self.gstamps = self.torch.zeros(timing_slots, self.L, 1024, 2, dtype=self.torch.int64, device="cuda")
                d.gather_stamps = self.gstamps.data_ptr()
        if self.evict_spare:
            d.spare_kcache, d.spare_acc, d.spare_pos = (x.data_ptr() for x in self.spare)
        d.host_chunks, d.host_threads = self.host_chunks, self.host_threads
        for name, val in self.tune.items():           # this pipeline's own launch-shape knobs
            setattr(d, name, val)
        self.pl = B.hca_pipeline_create(self.shape, self.L, d, timing_slots)
        self.pl_layers = (B.hca_layer * self.L)()
        for l in range(self.L):
            ly = self.pl_layers[l]
            ly.kcache, ly.acc, ly.pos = self.kcache[l].data_ptr(), self.acc[l].data_ptr(), self.pos[l].data_ptr()
            ly.v_host, ly.v_hbm = self.v_host[l].data_ptr(), self.v_hbm[l].data_ptr()
            ly.y = self.y[l].data_ptr()
        self.pl_n = (C.c_int64 * (self.L * w.batch))(*[x for l in range(self.L) for x in self.n[l]])

    def decode_step_native(self, t, timing_slot=-1):
        """One decode step through hca_pipeline_step (same kernels as decode_step_staged)."""
        w = self.w
        for l in range(self.L):
            self.pl_layers[l].k_new = self.k_new[t][l].data_ptr()
            self.pl_layers[l].q = self.q[t][l].data_ptr()
        import ctypes as C
        evict = (C.c_int64 * self.L)(*[self.n0 if self.evict_due(l, t) else 0 for l in range(self.L)])
        vh = self.v_host[0]
        self.B.hca_pipeline_step(self.pl, self.pl_layers, self.pl_n, self.n0 + t, w.k, vh.shape[2], vh.shape[2],
                                 self.vnew, self.sm_scale, evict, self.evict_every, timing_slot)

    def evict_due(self, l, t):
        """Every layer is evicted once per `evict_every` steps; the layers are staggered over the period
        so that each step carries its share instead of one step carrying all of them."""
        return bool(self.evict_every) and (t + 1 + l) % self.evict_every == 0

    def decode_step_staged(self, t, sa, sb, sg, sc, events=None):
        """One decode step over all layers as a four-stage pipeline across layers, one stream per stage:
        sa: append + key scan, sb: top-k, sg: host-link gather, sc: attend (+ eviction when due).
        Layer l's stages follow each other through events; different layers overlap, so the step is
        paced by its slowest stage (the gather) instead of by the sum of the stages."""
        B, w = self.B, self.w
        for l in range(self.L):
            s3, pipe = self.sel_ev[l % 3], self.pipe[l % 4]
            sel = self.sels[l % 3]
            sa.wait_event(s3["sel_free"])            # top-k of the previous user of this score buffer
            sa.wait_event(self.layer_done[l])        # this layer's attend / evict of the previous step
            self.scan(l, t, sa, sel, None if events is None else events[l])
            s3["score_done"].record(sa)
            sb.wait_event(s3["score_done"])
            sb.wait_event(pipe["pipe_free"])         # attend of the previous user of idx / staging
            B.hca_topk(self.shape, sel, self.n[l], w.k, pipe["idx"], pipe["count"], self.ws_topk, sb)
            s3["sel_free"].record(sb)
            pipe["topk_done"].record(sb)
            sg.wait_event(pipe["topk_done"])
            self.gather(l, sg, pipe)
            pipe["gather_done"].record(sg)
            sc.wait_event(pipe["gather_done"])
            self.attend_evict(l, t, sc, pipe)
            pipe["pipe_free"].record(sc)
            self.layer_done[l].record(sc)

    def decode_step(self, t, main, side, overlap=True, events=None):
        """One decode step over all layers.  With overlap, the gather of layer l runs on the side stream
        under the key scan and top-k of layer l+1; the main stream never waits for the host link
        except right before the attend that needs it."""
        prev = None
        for l in range(self.L):
            pipe = self.pipe[l & 1]
            ev = None
            if events is not None:
                ev = events[l]
            self.scan_select(l, t, main, pipe, ev)
            if overlap:
                pipe["sel_done"].record(main)
                side.wait_event(pipe["sel_done"])
                self.gather(l, side, pipe)
                pipe["gather_done"].record(side)
                if prev is not None:
                    pp = self.pipe[prev & 1]
                    main.wait_event(pp["gather_done"])
                    self.attend_evict(prev, t, main, pp)
                prev = l
            else:
                self.gather(l, main, pipe)
                self.attend_evict(l, t, main, pipe)
        if prev is not None:
            pp = self.pipe[prev & 1]
            main.wait_event(pp["gather_done"])
            self.attend_evict(prev, t, main, pp)


def per_layer_latency(cfg, main, side, link_peak, iters=8, fused=False, streams=None):
    """One layer of workload `cfg` (synth_inputs.CONFIGS), decode steps issued back to back on one stream with no
    overlap between layers: time from query ready to y ready (quantise-append, scan, top-k, gather,
    attend).  For config 5 the cache is first evicted to its 50% cap, as the config says."""
    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    w = S.CONFIGS[cfg]
    warm = 3
    m = Model(w, 1, 0, 2 * iters + warm, fused=fused)
    m.build(1)
    m.make_steps(2 * iters + warm)
    t = 0
    for _ in range(2):
        m.decode_step(t, main, side, overlap=False)
        t += 1
    resident = w.n + 2
    if cfg == 5:
        B.hca_evict(m.shape, m.kcache[0], m.acc[0], m.pos[0], m.n[0], w.evict_keep, 2, None, m.ws_main,
                    None, None, None, main)
        m.n[0] = [w.evict_keep] * w.batch
        resident = w.evict_keep
    m.decode_step(t, main, side, overlap=False)
    t += 1
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    sc = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))] for _ in range(iters)]
    for i in range(iters):
        ev[i][0].record(main)
        m.decode_step(t + i, main, side, overlap=False, events=sc[i])
        ev[i][1].record(main)
    torch.cuda.synchronize()
    lat = sorted(a.elapsed_time(b) for a, b in ev)[iters // 2]
    scan = sorted(x[0][0].elapsed_time(x[0][1]) for x in sc)[iters // 2]
    code_bytes = 128 * w.bits // 8 + (128 // w.group) * 4
    scan_bytes = w.batch * w.n_kv_heads * (resident + iters // 2) * (code_bytes + 4)
    score_topk_ms = scan if fused else None          # fused: the bracket holds the whole hca_score_topk call
    # the gather alone, as the path issues it
    pipe = m.pipe[0]
    g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    g0.record(main)
    for _ in range(iters):
        m.gather(0, main, pipe)
    g1.record(main)
    torch.cuda.synchronize()
    gms = g0.elapsed_time(g1) / iters
    gbytes = w.batch * w.n_kv_heads * w.k * 256
    if fused and streams is not None:
        # the selecting scan alone: the same layer through the step driver (one layer: nothing overlaps), timed
        # by the driver's HIP events around the launch
        m.native_pipeline(*streams, iters)
        for i in range(iters):
            m.decode_step_native(t + iters + i, i)
            torch.cuda.synchronize()
        per = sorted(B.hca_pipeline_scan_ms(m.pl, i, 1)[0] for i in range(iters))
        bracket = per[iters // 2]                    # HIP events around the launch: the kernel plus its dispatch
        # the kernel's own duration, as rocprofv3 reports it and as the main roofline figure is taken: from the
        # per-wave wall-clock stamps of the launch, first wave start to last wave end
        st_ = m.stamps[:, 0]
        starts = torch.where(st_[..., 0] > 0, st_[..., 0], torch.full_like(st_[..., 0], 1 << 62)).amin(-1)
        own = sorted(((st_[..., 1].amax(-1) - starts).double() / B.hca_wall_clock_khz()).tolist())
        scan = own[iters // 2]
        scan_bytes = w.batch * w.n_kv_heads * (resident + iters + iters // 2) * code_bytes
        B.hca_pipeline_destroy(m.pl)
    out = {"workload": w.name, "resident_tokens": resident, "ms_per_layer": lat, "score_topk_ms": score_topk_ms,
           "scan_event_bracket_ms": bracket if fused and streams is not None else None,
           "key_scan_ms": scan, "key_scan_GBs": scan_bytes / scan / 1e6, "key_scan_frac_of_hbm_peak": scan_bytes / scan / 1e6 / HBM_PEAK_GBS,
           "gather_ms": gms, "gather_GBs": gbytes / gms / 1e6, "gather_frac_of_link_peak": gbytes / gms / 1e6 / link_peak}
    del m
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch._C._host_emptyCache()
    return out


def per_layer_latency_hybrid(cfg, stream, host_threads, iters=8):
    """One layer of workload `cfg`, decode steps one after another, with the hybrid value side: the step driver
    with one layer and all four stages on one stream (nothing can overlap: the next step's append waits for this
    step's output), 5/8 of every row's chunks of selected tokens summed by the host threads while the rest is
    gathered over the link.  Time from the first kernel of a step to its y, mean over `iters` steps enqueued back
    to back.  For config 5 the cache is first evicted to its 50% cap, as in per_layer_latency."""
    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    w = S.CONFIGS[cfg]
    warm = 3
    nsplit = -(-w.k // 256)
    hc = max(1, round(nsplit * 5 / 8))
    m = Model(w, 1, 0, iters + warm + 2, n_sel=3, fused=True, host_chunks=hc, host_threads=host_threads)
    m.build(1)
    m.make_steps(iters + warm + 2)
    resident = w.n + warm
    if cfg == 5:
        B.hca_evict(m.shape, m.kcache[0], m.acc[0], m.pos[0], m.n[0], w.evict_keep, 2, None, m.ws_main,
                    None, None, None, stream)
        m.n[0] = [w.evict_keep] * w.batch
        resident = w.evict_keep + warm
        torch.cuda.synchronize()
    m.layer_idx_on = True
    m.native_pipeline(stream, stream, stream, stream, 0)
    for t in range(warm):
        m.decode_step_native(t)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(iters):
        m.decode_step_native(warm + i)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    status = B.hca_pipeline_host_status(m.pl)
    B.hca_pipeline_destroy(m.pl)
    del m
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch._C._host_emptyCache()
    return {"ms_per_layer": ms, "resident_tokens": resident, "host_chunks_of": [hc, nsplit],
            "host_threads": host_threads, "host_timeouts_bad_rows": list(status),
            "how": "hca_pipeline_step with one layer and one stream for all four stages, scan and top-k fused; "
                   "steps enqueued back to back, each waits for the one before"}


def per_layer_latency_grouped(cfg, groups, streams, iters=8, fused=True):
    """One layer of workload `cfg` (synth_inputs.CONFIGS) with its rows (sequences x KV heads) cut into `groups` parts that
    go through the four stages as a pipeline: the gather of one part overlaps the scan of the next.  Unlike
    the overlap across layers this is legal in a real model, where the next layer's query does not exist yet:
    all parts belong to the same layer and use the same query.  The parts are handed to the step driver as its
    "layers".  The enqueue of the whole layer is hidden behind a spinning gate kernel on the scan stream, as a
    serving loop would hide it behind the preceding non-attention work; the time runs from the gate's end to
    the last part's y."""
    import dataclasses
    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    w = S.CONFIGS[cfg]
    gb = min(groups, w.batch)
    gh = groups // gb
    assert gb * gh == groups and w.batch % gb == 0 and w.n_kv_heads % gh == 0
    wg = dataclasses.replace(w, name=f"{w.name}/{groups}parts", batch=w.batch // gb,
                             n_q_heads=w.n_q_heads // gh, n_kv_heads=w.n_kv_heads // gh)
    warm = 3
    m = Model(wg, groups, 0, iters + warm, n_sel=groups, fused=fused)
    m.build(groups)
    m.make_steps(iters + warm)
    sa, sb, sg, sc = streams
    m.native_pipeline(sa, sb, sg, sc, 0)
    t = 0
    for _ in range(2):
        m.decode_step_native(t)
        t += 1
    torch.cuda.synchronize()
    if cfg == 5:
        for l in range(groups):
            n_l = [m.pl_n[l * wg.batch + b] for b in range(wg.batch)]
            B.hca_evict(m.shape, m.kcache[l], m.acc[l], m.pos[l], n_l, w.evict_keep, 2, None, m.ws_main,
                        None, None, None, sa)
            for b in range(wg.batch):
                m.pl_n[l * wg.batch + b] = w.evict_keep
        torch.cuda.synchronize()
    m.decode_step_native(t)
    t += 1
    torch.cuda.synchronize()
    # gate length: long enough for the host to enqueue every part
    with torch.cuda.stream(sa):
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record(sa)
        torch.cuda._sleep(1_000_000)
        c1.record(sa)
    torch.cuda.synchronize()
    cycles_per_ms = 1_000_000 / c0.elapsed_time(c1)
    gate = int(cycles_per_ms * (0.5 + 0.35 * groups))
    lat = []
    for i in range(iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(sa):
            torch.cuda._sleep(gate)
        e0.record(sa)
        h0 = time.perf_counter()
        m.decode_step_native(t + i)
        host_ms = (time.perf_counter() - h0) * 1e3
        e1.record(sc)
        torch.cuda.synchronize()
        lat.append((e0.elapsed_time(e1), host_ms))
    lat.sort()
    ms, host_ms = lat[iters // 2]
    B.hca_pipeline_destroy(m.pl)
    del m
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch._C._host_emptyCache()
    return {"parts": groups, "ms_per_layer": ms, "host_enqueue_ms": host_ms, "gate_ms": gate / cycles_per_ms}


def other_config_step(cfg, layers, phys, steps, streams, args, tune):
    """ms per decode step of another workload through the same step driver and settings as the headline run
    (a few steps; `layers` logical layers on `phys` physical value stores)."""
    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    w = S.CONFIGS[cfg]
    warm = 2
    nsplit = -(-w.k // 256)
    hc = min(nsplit, round(args.host_chunks * nsplit / 16)) if args.host_chunks else 0
    m = Model(w, layers, args.evict_every, steps + warm, n_sel=layers if layers >= 3 else 3, fused=not args.no_fused_select,
              host_chunks=hc, host_threads=args.host_threads, tune=tune, n_pipe_sets=args.pipe_sets,
              dual_scan=args.scan_mode)
    m.build(phys)
    m.make_steps(steps + warm)
    m.layer_idx_on = not args.slot_idx
    m.native_pipeline(*streams, 0)
    for t in range(warm):
        m.decode_step_native(t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(warm, warm + steps):
        m.decode_step_native(t)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    status = B.hca_pipeline_host_status(m.pl) if hc else (0, 0)
    B.hca_pipeline_destroy(m.pl)
    out = {"workload": w.name, "layers": layers, "physical_value_layers": m.phys, "batch": w.batch,
           "resident_tokens_per_layer": w.n + warm + steps, "top_k": w.k, "steps": steps, "ms_per_step": ms,
           "ms_per_layer": ms / layers, "context_tokens_scored_per_s": w.batch * w.n * layers / ms * 1e3,
           "host_chunks_of": [hc, nsplit], "host_timeouts_bad_rows": list(status)}
    del m
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch._C._host_emptyCache()
    return out


def vq_probe(w, iters, g=32, c=256):
    """Codebook form of the key path on one layer of the workload: bulk assignment (tokens/s), table build
    + lookup scan (time, bytes of the index matrix streamed + scores written against the HBM peak - the bound now
    that the table reads are free of bank conflicts - and table bytes read from LDS against the LDS peak).
    c > 256 (the paper's own c = 8192): 16-bit indices, the table is read through L2; the codebook is then c sampled
    sub-vectors per group without Lloyd rounds (the host trainer would take minutes at that size, and the kernels'
    time does not depend on where the centroids lie)."""
    import numpy as np
    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    G = w.n_q_heads // w.n_kv_heads
    cap = w.n + 16
    shape = B.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, cap)
    d = S.make_layer(w, 0, device="cuda", want_values=False)
    rng = np.random.default_rng(1000 * w.config + 7)
    # codebooks from the library's host trainer on the first 8192 tokens of each KV head of sequence 0
    t0 = time.perf_counter()
    cen = []
    wide = c > 256 or g * c * G > 32768
    for h in range(w.n_kv_heads):
        kval = d["keys"][0, h, :(8192 if not wide else 32768)].cpu().numpy()
        init = np.stack([rng.choice(kval.shape[0], c, replace=False) for _ in range(g)]).astype(np.int32)
        if wide:
            sub = kval.astype(np.float32).reshape(kval.shape[0], g, 128 // g)
            cen.append(np.stack([sub[init[i], i] for i in range(g)]))
        else:
            cen.append(B.hca_vq_train(kval, g, c, init, 4)[0])
    t_train = time.perf_counter() - t0
    cen = torch.from_numpy(np.stack(cen)).cuda()
    cb = B.make_codebook(g, c, cen)
    P = [torch.empty(B.hca_vq_pcache_bytes(shape, cb), dtype=torch.uint8, device="cuda") for _ in range(2)]
    lut = torch.empty(B.hca_vq_lut_bytes(shape, cb) // 4, dtype=torch.float32, device="cuda")
    sel = torch.empty(w.batch, w.n_kv_heads, cap, dtype=torch.float32, device="cuda")
    n0 = [0] * w.batch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    B.hca_vq_assign(shape, cb, P[1], d["keys"], w.n, n0)
    e0.record()
    B.hca_vq_assign(shape, cb, P[0], d["keys"], w.n, n0)
    e1.record()
    torch.cuda.synchronize()
    assign_ms = e0.elapsed_time(e1)
    n = [w.n] * w.batch
    q = d["q"]
    for i in range(3):
        B.hca_vq_score(shape, cb, P[i & 1], q, n, lut, sel)
    torch.cuda.synchronize()
    e0.record()
    for i in range(iters):
        B.hca_vq_score(shape, cb, P[i & 1], q, n, lut, sel)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    rows = w.batch * w.n_kv_heads
    hbm_bytes = rows * w.n * (g * (2 if wide else 1) + 4)
    lds_bytes = rows * w.n * g * G * 4
    # LDS: 256 compute units x 256 B per clock (16-byte reads, measured: 4 clocks per conflict-free wave read)
    # x 2.4 GHz.  Assignment: per centroid and channel one subtract and one fused multiply-add = 3 flop.
    lds_peak = 256 * 256 * 2.4
    assign_flop = rows * w.n * g * c * (128 // g) * 3
    out = {"workload": w.name, "groups": g, "codewords": c, "train_s_host": t_train,
           "assign_ms": assign_ms, "assign_token_heads_per_s": rows * w.n / assign_ms * 1e3,
           "assign_roofline": {"bound": "alu", "achieved": assign_flop / assign_ms / 1e9, "peak": 157.3,
                               "unit": "TFLOP/s", "frac": assign_flop / assign_ms / 1e9 / 157.3},
           "score_ms": ms, "index_bytes_per_token_head": g * (2 if wide else 1),
           "table": "through LDS, a slice of groups at a time" if wide else "LDS",
           "context_tokens_scored_per_s": w.batch * w.n / ms * 1e3,
           "score_roofline": {"bound": "hbm", "achieved": hbm_bytes / ms / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": hbm_bytes / ms / 1e6 / HBM_PEAK_GBS,
                              "lds_GBs": lds_bytes / ms / 1e6, "lds_frac": lds_bytes / ms / 1e6 / lds_peak}}
    del P, lut, sel, d
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return out


def selection_probe(w, iters=10):
    """Times the two selection calls on the scores of one real scan of the workload's first layer:
    hca_topk (k fixed) and hca_topp (Eq. 4, tau = 0.9 and 0.99, cut at the same k)."""
    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    cap = w.n + 16
    shape = B.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, cap, w.bits, w.group)
    d = S.make_layer(w, 0, device="cuda", want_values=False)
    kc = torch.empty(B.hca_kcache_bytes(shape), dtype=torch.uint8, device="cuda")
    B.hca_quantize_keys(shape, kc, d["keys"], w.n, [0] * w.batch)
    n = [w.n] * w.batch
    sel = torch.empty(w.batch, w.n_kv_heads, cap, dtype=torch.float32, device="cuda")
    B.hca_score_qkeys(shape, kc, d["q"], n, sel)
    idx = torch.zeros(w.batch, w.n_kv_heads, w.k, dtype=torch.int32, device="cuda")
    count = torch.zeros(w.batch, w.n_kv_heads, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.hca_workspace_bytes(shape, w.k, 1), dtype=torch.uint8, device="cuda")
    sm = 1.0 / (128.0 ** 0.5)
    out = {"workload": w.name, "k": w.k}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(f):
        for _ in range(2):
            f()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(iters):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    lse = torch.zeros(w.batch, w.n_q_heads, dtype=torch.float32, device="cuda")
    out["scan_ms"] = timed(lambda: B.hca_score_qkeys(shape, kc, d["q"], n, sel))
    out["scan_with_lse_ms"] = timed(lambda: B.hca_score_qkeys_lse(shape, kc, d["q"], n, sm, sel, lse, ws))
    out["topk_ms"] = timed(lambda: B.hca_topk(shape, sel, n, w.k, idx, count, ws))
    for tau in (0.9, 0.99):
        ms = timed(lambda: B.hca_topp(shape, sel, n, sm, tau, w.k, idx, count, None, ws))
        out[f"topp_tau{tau}"] = {"ms": ms, "selected_per_kv_head": count.cpu().reshape(-1).tolist()}
    del kc, sel, d
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return out


def paper_form_probe(w, streams, layers=8, steps=6, g=32, c=256, tau=0.9):
    """Decode steps in the paper's own form on `layers` layers of the workload: codebook key cache (Sec. 3.1),
    table-lookup scores (Eq. 3), cumulative-weight selection (Eq. 4, cut at the workload's k), gather of the
    selected value rows from pinned host memory, softmax-weighted sum.  First on one stream, calls in order:
    the time per layer is what a layer costs when nothing overlaps.  Then the same steps through the library's
    step driver (four stages on `streams`, layers overlapping).  With the synthetic planted queries the
    selection keeps only a few tokens per head (the count is reported), so the gather is short here."""
    import numpy as np
    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    G = w.n_q_heads // w.n_kv_heads
    cap = w.n + 2 * steps + 16
    shape = B.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, cap)
    rng = np.random.default_rng(1000 * w.config + 11)
    P, cens, cbs, vh, pos, acc, qs, kn = [], [], [], [], [], [], [], []
    for l in range(layers):
        d = S.make_layer(w, l, device="cuda", want_values=True)
        cen = []
        for h in range(w.n_kv_heads):
            kval = d["keys"][0, h, :(4096 if c <= 256 else 32768)].cpu().numpy()
            init = np.stack([rng.choice(kval.shape[0], c, replace=False) for _ in range(g)]).astype(np.int32)
            if c <= 256:
                cen.append(B.hca_vq_train(kval, g, c, init, 2)[0])
            else:      # sampled sub-vectors as centroids: the host trainer would take minutes at this size
                sub = kval.astype(np.float32).reshape(kval.shape[0], g, 128 // g)
                cen.append(np.stack([sub[init[i], i] for i in range(g)]))
        cens.append(torch.from_numpy(np.stack(cen)).cuda())
        cbs.append(B.make_codebook(g, c, cens[-1]))
        P.append(torch.empty(B.hca_vq_pcache_bytes(shape, cbs[-1]), dtype=torch.uint8, device="cuda"))
        pos.append(torch.zeros(w.batch, w.n_kv_heads, cap, dtype=torch.int32, device="cuda"))
        acc.append(torch.zeros(w.batch, w.n_kv_heads, cap, dtype=torch.float32, device="cuda"))
        B.hca_vq_assign(shape, cbs[-1], P[-1], d["keys"], w.n, [0] * w.batch, acc[-1], pos[-1], [0] * w.batch)
        v = torch.empty(w.batch, w.n_kv_heads, w.n, 128, dtype=torch.float16, pin_memory=True)
        v.copy_(d["values"])
        vh.append(v)
        st = [S.make_step(w, l, t) for t in range(2 * steps)]
        kn.append([x[0].cuda() for x in st])
        qs.append([x[2].cuda() for x in st])
        del d
    lut = torch.empty(B.hca_vq_lut_bytes(shape, cbs[0]) // 4, dtype=torch.float32, device="cuda")
    sel = torch.empty(w.batch, w.n_kv_heads, cap, dtype=torch.float32, device="cuda")
    idx = torch.zeros(w.batch, w.n_kv_heads, w.k, dtype=torch.int32, device="cuda")
    count = torch.zeros(w.batch, w.n_kv_heads, dtype=torch.int32, device="cuda")
    y = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    vnew = torch.zeros(w.batch, w.n_kv_heads, 2 * steps, 128, dtype=torch.float16, device="cuda")
    ws = torch.empty(B.hca_vq_workspace_bytes(shape, cbs[0], w.k, 1), dtype=torch.uint8, device="cuda")
    sm = 1.0 / (128.0 ** 0.5)
    kept = []

    def step(t):
        n = [w.n + t] * w.batch
        for l in range(layers):
            B.hca_vq_assign(shape, cbs[l], P[l], kn[l][t], 1, n, acc[l], pos[l], n)
            n1 = [x + 1 for x in n]
            B.hca_vq_score(shape, cbs[l], P[l], qs[l][t], n1, lut, sel)
            B.hca_topp(shape, sel, n1, sm, tau, w.k, idx, count, None, ws)
            B.hca_gather_values(shape, idx, count, w.k, pos[l], vh[l], w.n, w.n, vnew, 2 * steps, ws)
            B.hca_vq_attend_gathered(shape, cbs[l], P[l], lut, idx, count, w.k, sm, y, acc[l], ws)

    step(0)
    torch.cuda.synchronize()
    kept = count.cpu().reshape(-1).tolist()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for t in range(1, steps):
        step(t)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / (steps - 1)
    out = {"workload": w.name, "layers": layers, "groups": g, "codewords": c, "tau": tau, "k_cut": w.k,
           "ms_per_layer": ms / layers, "context_tokens_scored_per_s": w.batch * w.n * layers / ms * 1e3,
           "selected_per_kv_head_last_layer": kept}
    # the same form through the step driver: steps `steps` .. 2 * steps - 1 on the caches as they stand
    import ctypes as C
    d = B.hca_pipeline_desc()
    d.stream_scan, d.stream_topk, d.stream_gather, d.stream_attend = (x.cuda_stream for x in streams)
    sels = [torch.empty(w.batch, w.n_kv_heads, cap, dtype=torch.float32, device="cuda") for _ in range(layers)]
    luts = [torch.empty(B.hca_vq_lut_bytes(shape, cbs[0]) // 4, dtype=torch.float32, device="cuda") for _ in range(layers)]
    ys = torch.zeros(layers, w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    keep = []
    for i, t_ in enumerate(sels):
        d.sel[i] = t_.data_ptr()
    d.n_sel = layers
    for i in range(4):
        a = torch.zeros(w.batch, w.n_kv_heads, w.k, dtype=torch.int32, device="cuda")
        b = torch.zeros(w.batch, w.n_kv_heads, dtype=torch.int32, device="cuda")
        cws = torch.empty(B.hca_vq_workspace_bytes(shape, cbs[0], w.k, 1), dtype=torch.uint8, device="cuda")
        keep += [a, b, cws]
        d.idx[i], d.count[i], d.ws_attend[i] = a.data_ptr(), b.data_ptr(), cws.data_ptr()
    wt = torch.zeros(B.hca_vq_workspace_bytes(shape, cbs[0], w.k, 1), dtype=torch.uint8, device="cuda")
    d.ws_topk = wt.data_ptr()
    d.vq_groups, d.vq_codewords, d.topp_tau = g, c, tau
    pl = B.hca_pipeline_create(shape, layers, d, 0)
    ly = (B.hca_layer * layers)()
    for l in range(layers):
        ly[l].kcache, ly[l].acc, ly[l].pos = P[l].data_ptr(), acc[l].data_ptr(), pos[l].data_ptr()
        ly[l].v_host, ly[l].v_hbm, ly[l].y = vh[l].data_ptr(), vnew.data_ptr(), ys[l].data_ptr()
        ly[l].vq_centroids, ly[l].vq_lut = cens[l].data_ptr(), luts[l].data_ptr()
    nres = (C.c_int64 * (layers * w.batch))(*([w.n + steps] * (layers * w.batch)))

    def driver_step(t):
        for l in range(layers):
            ly[l].k_new, ly[l].q = kn[l][t].data_ptr(), qs[l][t].data_ptr()
        B.hca_pipeline_step(pl, ly, nres, w.n + t, w.k, w.n, w.n, 2 * steps, sm, None, 0, -1)

    torch.cuda.synchronize()
    driver_step(steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps + 1, 2 * steps):
        driver_step(t)
    torch.cuda.synchronize()
    ms_p = (time.perf_counter() - t0) * 1e3 / (steps - 1)
    out["pipelined_ms_per_layer"] = ms_p / layers
    out["pipelined_context_tokens_scored_per_s"] = w.batch * w.n * layers / ms_p * 1e3
    B.hca_pipeline_destroy(pl)
    del P, vh, lut, sel, sels, luts, keep, wt
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch._C._host_emptyCache()
    return out


def cpu_split_probe(w, threads=16, iters=6):
    """The paper's CPU-GPU split of the value side on one layer of the workload, beside the graded gather
    path: after scan + top-k, (a) hca_attend_weights writes fp16 weights and value-row numbers into pinned
    host memory and hca_host_weighted_sum forms y on the host cores; (b) hca_gather_values +
    hca_attend_gathered.  Reports link bytes per layer and the time of each form (stream time for the GPU
    parts, wall clock for the host sum)."""
    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    cap = w.n + 16
    shape = B.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, cap, w.bits, w.group)
    d = S.make_layer(w, 0, device="cuda", want_values=True)
    kc = torch.empty(B.hca_kcache_bytes(shape), dtype=torch.uint8, device="cuda")
    B.hca_quantize_keys(shape, kc, d["keys"], w.n, [0] * w.batch)
    n = [w.n] * w.batch
    sel = torch.empty(w.batch, w.n_kv_heads, cap, dtype=torch.float32, device="cuda")
    idx = torch.zeros(w.batch, w.n_kv_heads, w.k, dtype=torch.int32, device="cuda")
    count = torch.zeros(w.batch, w.n_kv_heads, dtype=torch.int32, device="cuda")
    pos = torch.arange(cap, dtype=torch.int32, device="cuda").repeat(w.batch, w.n_kv_heads, 1).contiguous()
    ws = torch.empty(B.hca_workspace_bytes(shape, w.k, 1), dtype=torch.uint8, device="cuda")
    y = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    vh = torch.empty(w.batch, w.n_kv_heads, w.n, 128, dtype=torch.float16, pin_memory=True)
    vh.copy_(d["values"])
    w16 = torch.zeros(w.batch, w.n_q_heads, w.k, dtype=torch.float16).pin_memory()
    vrow = torch.zeros(w.batch, w.n_kv_heads, w.k, dtype=torch.int32).pin_memory()
    cnt_h = torch.zeros(w.batch, w.n_kv_heads, dtype=torch.int32).pin_memory()
    yh = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32)
    sm = 1.0 / (128.0 ** 0.5)
    B.hca_score_qkeys(shape, kc, d["q"], n, sel)
    B.hca_topk(shape, sel, n, w.k, idx, count, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    gpu_ms, host_ms = [], []
    for _ in range(iters):
        e0.record()
        B.hca_attend_weights(shape, kc, d["q"], idx, count, w.k, pos, sm, None, w16, vrow, None, ws)
        cnt_h.copy_(count, non_blocking=True)
        e1.record()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.hca_host_weighted_sum(shape, vrow, cnt_h, w.k, w16, vh, w.n, yh, threads)
        host_ms.append((time.perf_counter() - t0) * 1e3)
        gpu_ms.append(e0.elapsed_time(e1))
    gath = []
    for _ in range(iters):
        e0.record()
        B.hca_gather_values(shape, idx, count, w.k, pos, vh, w.n, w.n, None, 0, ws)
        B.hca_attend_gathered(shape, kc, d["q"], idx, count, w.k, sm, y, None, ws)
        e1.record()
        torch.cuda.synchronize()
        gath.append(e0.elapsed_time(e1))
    torch.cuda.synchronize()
    diff = float((y.cpu() - yh).abs().max() / y.abs().max().cpu())
    rows = w.batch * w.n_kv_heads
    G = w.n_q_heads // w.n_kv_heads
    out = {"workload": w.name, "k": w.k, "host_threads": threads,
           "split_link_bytes_per_layer": rows * w.k * (4 + 2 * G), "gather_link_bytes_per_layer": rows * w.k * 256,
           "split_gpu_weights_ms": sorted(gpu_ms)[iters // 2], "split_host_sum_ms": sorted(host_ms)[iters // 2],
           "gather_plus_attend_ms": sorted(gath)[iters // 2], "max_rel_diff_between_the_two": diff}
    del kc, sel, vh, d
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch._C._host_emptyCache()
    return out


def prefill_blocks(w, sizes=(1024, 4096, 16384, 65536, 262144)):
    """Key compression as a block-wise prefill hands it over (App. B: the keys of a block are quantised when the
    block's attention is done): the context arrives in blocks of T tokens per sequence and every block is appended
    with one call - hca_quantize_keys (uniform codes, 4-bit / group 32 and 2-bit / group 64) or hca_vq_assign
    (codebook indices, g = 32, c = 256 and the paper's c = 8192).  The paper gives no block size; the sweep covers
    1 Ki to 256 Ki tokens.  Per block size: time per call (median of HIP-event brackets around each call), tokens
    per second, and the fraction of the bound - HBM bytes (256 B of fp16 key read + the codes written per token and
    KV head) for the uniform form, fp32 vector flops (one subtract + one fused multiply-add per centroid and channel)
    for the assignment.  Uniform and c = 256 run over 1 Mi / 256 Ki tokens per sequence, c = 8192 over 32 Ki (at
    least two blocks where the size allows)."""
    import numpy as np
    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    rows = w.batch * w.n_kv_heads
    d = S.make_layer(w, 0, device="cuda", want_values=False)
    keys = d["keys"]
    out = {"workload": w.name, "block_sizes": list(sizes)}

    def run(call, total, T):
        blocks = [keys[:, :, a:a + T].contiguous() for a in range(0, total, T)]
        n = [0] * w.batch
        call(blocks[0], T, n)                        # warm-up (the cache is refilled from slot 0 below)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in blocks]
        for (e0, e1), blk in zip(ev, blocks):
            e0.record()
            call(blk, T, n)
            e1.record()
            n = [x + T for x in n]
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev)
        return ms[len(ms) // 2], len(blocks)

    for bits, group in ((4, 32), (2, 64)):
        shape = B.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.n, bits, group)
        kc = torch.empty(B.hca_kcache_bytes(shape), dtype=torch.uint8, device="cuda")
        code_bytes = 128 * bits // 8 + (128 // group) * 4
        res = []
        for T in sizes:
            total = max(min(w.n, 1 << 20), T)
            ms, nb = run(lambda blk, T_, n: B.hca_quantize_keys(shape, kc, blk, T_, n), total, T)
            gbs = rows * T * (256 + code_bytes) / ms / 1e6
            res.append({"block_tokens": T, "blocks": nb, "ms_per_block": ms, "tokens_per_s": w.batch * T / ms * 1e3,
                        "GBs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS})
        out[f"uniform_{bits}bit_group{group}"] = res
        del kc
    shape = B.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.n)
    rng = np.random.default_rng(1000 * w.config + 8)
    for c, total_cap in ((256, 1 << 18), (8192, 1 << 15)):
        g = 32
        sub = keys[0, :, :32768].float().reshape(w.n_kv_heads, 32768, g, 128 // g)
        pick = torch.from_numpy(np.stack([rng.choice(32768, c, replace=False) for _ in range(g)])).cuda()
        cen = torch.stack([torch.stack([sub[h, pick[i], i] for i in range(g)]) for h in range(w.n_kv_heads)]).contiguous()
        cb = B.make_codebook(g, c, cen)
        P = torch.empty(B.hca_vq_pcache_bytes(shape, cb), dtype=torch.uint8, device="cuda")
        res = []
        for T in sizes:
            total = max(total_cap, T)
            ms, nb = run(lambda blk, T_, n: B.hca_vq_assign(shape, cb, P, blk, T_, n), total, T)
            tf = rows * T * g * c * (128 // g) * 3 / ms / 1e9          # the exhaustive exact search's flops
            r = {"block_tokens": T, "blocks": nb, "ms_per_block": ms, "tokens_per_s": w.batch * T / ms * 1e3}
            if T >= 1024 and c >= 512 and T * c >= (1 << 21):
                # the library's bulk form from this size on: two passes of v_mfma_f32_32x32x16_f16 over every
                # (token, group, centroid), 16 products each, then the exact search on the shortlist only
                mt = rows * T * g * c * 2 * 16 * 2 / ms / 1e9
                r.update({"form": "matrix-core shortlist + exact chain on the shortlist", "matrix_TFLOPs": mt,
                          "frac_of_f16_matrix_peak": mt / 2500.0, "exhaustive_search_equivalent_TFLOPs": tf})
            else:
                r.update({"form": "exact chain over every centroid (vector ALU)", "TFLOPs": tf,
                          "frac_of_fp32_vector_peak": tf / 157.3})
            res.append(r)
        out[f"codebook_g{g}_c{c}"] = res
        del P, cen
    del d, keys
    torch.cuda.empty_cache()
    return out


def correlated_selection(w, iters=12):
    """hca_score_topk on one layer of `w` whose keys resemble their neighbours (synth_inputs.make_correlated_layer,
    runs of up to 64 and of up to 4096 slots), beside the same call on the independent keys of the main workload:
    time per call, spread of the candidate counts, rows that needed the second scan.  The results are the same
    sets as hca_score_qkeys + hca_topk give (checked here on the GPU; against the oracle in the tests)."""
    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    from paper_2507_19823_amd.session import LayerState
    R = w.batch * w.n_kv_heads
    out = {"workload": w.name, "k": w.k}
    for name, run_max in (("independent", 0), ("runs_up_to_64", 64), ("runs_up_to_4096", 4096)):
        d = (S.make_layer(w, 0, device="cuda", want_values=False) if run_max == 0 else
             S.make_correlated_layer(w, 0, device="cuda", run_max=run_max))
        st = LayerState(w.batch, w.n_q_heads, w.n_kv_heads, w.n + 32, w.bits, w.group, k_max=w.k, want_z=False)
        for a in range(0, w.n, 1 << 18):
            st.quantize(d["keys"][:, :, a:a + (1 << 18)].contiguous())
        q = d["q"]
        del d
        idx = torch.zeros(R, w.k, dtype=torch.int32, device="cuda")
        count = torch.zeros(R, dtype=torch.int32, device="cuda")
        st.score(q)
        st.topk(w.k)
        for _ in range(3):
            B.hca_score_topk(st.shape, st.kcache, q, st.n, w.k, idx, count, st.ws)
        torch.cuda.synchronize()
        same = bool(torch.equal(idx.view(-1), st.idx.reshape(-1)))
        ms = []
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(iters):
            e0.record()
            B.hca_score_topk(st.shape, st.kcache, q, st.n, w.k, idx, count, st.ws)
            e1.record()
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        cand = torch.zeros(R, dtype=torch.int32, device="cuda")
        resc = torch.zeros(R, dtype=torch.int32, device="cuda")
        B.hca_score_topk_report(st.shape, st.n, st.ws, cand, resc)
        torch.cuda.synchronize()
        out[name] = {"score_topk_ms": sorted(ms)[iters // 2], "candidates_min": int(cand.min()),
                     "candidates_max": int(cand.max()), "rows_rescanned": int(resc.sum()),
                     "same_sets_as_scan_plus_topk": same}
        del st, idx, count
        torch.cuda.empty_cache()
    return out


def scan_only(w, iters):
    """Key-scan kernel alone on one layer (two cache copies alternate), preceded by a plain 1 GiB
    device copy whose FETCH_SIZE / WRITE_SIZE readings calibrate the counters (profiles/)."""
    import torch
    from paper_2507_19823_amd import binding as B
    m = Model(w, 2, 0, 1)
    m.build(0)
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)                                    # calibration dispatch: reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    q = m.layer0["q"].cuda()
    for i in range(3):
        B.hca_score_qkeys(m.shape, m.kcache[i & 1], q, m.n[0], m.sel, None, None)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        B.hca_score_qkeys(m.shape, m.kcache[i & 1], q, m.n[0], m.sel, None, None)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    code_bytes = 128 * w.bits // 8 + (128 // w.group) * 4
    by = w.batch * w.n_kv_heads * w.n * (code_bytes + 4)
    print(json.dumps({"mode": "scan", "workload": w.name, "ms": ms, "bytes_per_launch": by,
                      "GBs": by / ms / 1e6, "frac": by / ms / 1e6 / HBM_PEAK_GBS}), flush=True)


def select_only(w, iters):
    """hca_score_topk alone on one layer (two cache copies alternate): the selecting scan and the small kernels
    around it, preceded by the same 1 GiB calibration copy as --mode scan."""
    import torch
    from paper_2507_19823_amd import binding as B
    m = Model(w, 2, 0, 1, fused=True)
    m.build(0)
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)                                    # calibration dispatch: reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    q = m.layer0["q"].cuda()
    pipe = m.pipe[0]

    def call(i):
        B.hca_score_topk(m.shape, m.kcache[i & 1], q, m.n[0], w.k, pipe["idx"], pipe["count"], m.ws_main)

    for i in range(3):
        call(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        call(i)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    code_bytes = 128 * w.bits // 8 + (128 // w.group) * 4
    print(json.dumps({"mode": "select", "workload": w.name, "score_topk_ms": ms,
                      "scan_algorithmic_bytes_per_launch": w.batch * w.n_kv_heads * w.n * code_bytes}), flush=True)


def gather_only(w, iters):
    """Value gather alone at the workload's shape: k selected rows of 256 B per (sequence, KV head) read from a
    pinned host store at random rows (drawn here; the store's contents do not matter), against the host link's
    rate for one large pinned copy measured in the same process."""
    import torch
    from paper_2507_19823_amd import binding as B
    cap = w.n + 16
    shape = B.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, cap, w.bits, w.group)
    R, k = w.batch * w.n_kv_heads, w.k
    big = torch.empty(1 << 28, dtype=torch.uint8, pin_memory=True)
    dbig = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    dbig.copy_(big, non_blocking=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(8):
        dbig.copy_(big, non_blocking=True)
    torch.cuda.synchronize()
    link_peak = 8 * (1 << 28) / (time.perf_counter() - t0) / 1e9
    del big, dbig
    g = torch.Generator().manual_seed(1000 * w.config + 3)
    idx = torch.stack([torch.randperm(w.n, generator=g)[:k].sort().values for _ in range(R)]).to(torch.int32)
    idx = idx.reshape(w.batch, w.n_kv_heads, k).cuda()
    count = torch.full((w.batch, w.n_kv_heads), k, dtype=torch.int32, device="cuda")
    pos = torch.arange(cap, dtype=torch.int32).repeat(w.batch, w.n_kv_heads, 1).contiguous().cuda()
    vh = torch.empty(w.batch, w.n_kv_heads, w.n, 128, dtype=torch.float16, pin_memory=True)
    vh.view(torch.int16).random_(0, 30000)
    ws = torch.empty(B.hca_workspace_bytes(shape, k, 1), dtype=torch.uint8, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ts = []
    for _ in range(iters + 1):
        e0.record()
        B.hca_gather_values(shape, idx, count, k, pos, vh, w.n, w.n, None, 0, ws)
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    ms = sum(ts[1:]) / iters
    by = R * k * 256
    print(json.dumps({"mode": "gather", "workload": w.name, "ms": ms, "bytes_per_launch": by, "GBs": by / ms / 1e6,
                      "host_link_peak_GBs": link_peak, "frac_of_link_peak": by / ms / 1e6 / link_peak}), flush=True)


def run_cpu_baseline(model, w, budget_s=12.0, max_steps=32, min_steps=0):
    """Times the oracle, as it stands, on layer 0 of the same workload: consecutive decode steps
    (append one token, score every resident token, top-k, attend with accumulated-score update)
    until about `budget_s` seconds of CPU work are done."""
    import numpy as np
    import oracle
    import synth_inputs as S
    d = model.layerv
    lv = model.verify_layer
    R = w.batch * w.n_kv_heads
    oc = oracle.Cache(R, w.n + max_steps, 128, w.bits, w.group)
    t0 = time.perf_counter()
    oracle.quantize(oc, d["keys"].numpy().reshape(R, w.n, 128))
    t_build = time.perf_counter() - t0
    V = np.zeros((R, w.n + max_steps, 128), np.float16)
    V[:, :w.n] = d["values"].numpy().reshape(R, w.n, 128)
    pos = np.tile(np.arange(w.n + max_steps, dtype=np.int32), (R, 1))
    acc = np.zeros((R, w.n + max_steps), np.float32)
    parts = np.zeros(4)
    steps, scored = 0, 0
    results = []                                      # (top-k index sets, outputs) of every replayed step
    while steps < max_steps and (parts.sum() < budget_s or steps < min_steps):
        k_new, v_new, q = S.make_step(w, lv, steps)
        V[:, w.n + steps] = v_new.numpy().reshape(R, 128)
        q16 = q.numpy().reshape(-1, 128)
        t0 = time.perf_counter()
        oracle.quantize(oc, k_new.numpy().reshape(R, 1, 128))
        t1 = time.perf_counter()
        sel, _ = oracle.score(oc, q16, want_z=False)
        t2 = time.perf_counter()
        idx, count = oracle.topk(sel, oc.n, w.k)
        t3 = time.perf_counter()
        y, _ = oracle.attend(oc, q16, idx, count, pos, V, model.sm_scale, acc=acc)
        t4 = time.perf_counter()
        results.append((idx, y))
        parts += (t1 - t0, t2 - t1, t3 - t2, t4 - t3)
        steps += 1
        scored += w.batch * int(oc.n[0])
    total = float(parts.sum())
    cores = len(os.sched_getaffinity(0))
    return results, {
        "value": scored / total, "unit": "context tokens scored/s",
        # the oracle's only parallel loop runs over the (sequence, KV head) rows: OpenMP threads beyond them idle
        "cores": min(oracle.num_threads(), R), "cores_available": cores, "omp_threads": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"{steps} consecutive decode steps of ONE layer (layer {lv}) of {w.name}, every resident token of "
                  f"all {w.n_kv_heads} KV heads scored per step, no eviction (append {parts[0]:.3f}s, score "
                  f"{parts[1]:.3f}s, top-k {parts[2]:.3f}s, attend {parts[3]:.3f}s); the oracle's own bulk "
                  f"quantise of the context ({t_build:.1f}s) is not in the timed part",
        "seconds": total,
    }


def main():
    faulthandler.enable()
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4, help="workload id in synth_inputs.CONFIGS (2, 3, 4 or 5)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers")
    ap.add_argument("--host-gib", type=float, default=60.0,
                    help="pinned host memory budget for values (the GPU boxes refuse more than 65 GiB in total)")
    ap.add_argument("--evict-every", type=int, default=16)
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE",
                    help="launch-shape knob passed to hca_tune (gather_wgs, gather_unroll, score_bpw, score_depth)")
    ap.add_argument("--evict-spare", action="store_true",
                    help="native pipeline: evict out of place into a spare buffer set, in slices behind the attends "
                         "(default: in place, which moves only the slots from the first dropped one on)")
    ap.add_argument("--host-chunks", type=int, default=14,
                    help="hybrid value side of the native step driver: of every row's selected tokens the first N "
                         "chunks of 256 are summed by host threads from the value store, the rest gathered (0: all gathered)")
    ap.add_argument("--host-threads", type=int, default=14, help="worker threads of the hybrid value side")
    ap.add_argument("--scan-mode", default="pair", choices=["single", "dual", "pair"],
                    help="native step driver with the fused selection: single = one scan launch per layer on one stream; "
                         "dual = even layers scan + select on one stream, odd layers on a second one, so that two scans "
                         "overlap; pair = one scan launch per two layers")
    ap.add_argument("--pipe-sets", type=int, default=8, choices=[4, 5, 6, 7, 8],
                    help="native step driver: sets of selection / staging buffers, i.e. layers in flight between top-k and attend")
    ap.add_argument("--resident", type=int, default=0,
                    help="--mode scan / select: tokens per sequence instead of the workload's context length")
    ap.add_argument("--slot-idx", action="store_true",
                    help="native pipeline: the selection results share the n_pipe sets of staging buffers (the first "
                         "form) instead of one result buffer per layer")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gap-report", action="store_true",
                    help="log the largest idle times between consecutive scan launches with their step.layer")
    ap.add_argument("--timeline-out", default="", metavar="PATH",
                    help="with --gap-report: write the merged timeline of scan launches and gathers around one step "
                         "boundary (wall-clock stamps, us) to this file")
    ap.add_argument("--no-fused-select", action="store_true",
                    help="scan and top-k as two calls with a score buffer between them (hca_score_qkeys, hca_topk) "
                         "instead of hca_score_topk; always so with --pipeline staged / gather / none")
    ap.add_argument("--sel-buffers", type=int, default=32,
                    help="score buffers of the native step driver (one per layer: the scan never waits for one)")
    ap.add_argument("--bracket-stride", type=int, default=4,
                    help="HIP-event bracket around the scan of every n-th layer (the in-kernel stamps time all of them)")
    ap.add_argument("--pipeline", default="native", choices=["native", "staged", "gather", "none"],
                    help="native: the library's four-stage step driver; staged: the same pipeline enqueued from Python; "
                         "gather: only the gather overlaps; none: serial")
    ap.add_argument("--vq-codewords", type=int, default=256, help="--mode vq: centroids per group (up to 8192)")
    ap.add_argument("--no-latency", action="store_true", help="skip the per-layer latency probes at 128K / 1M / 4M")
    ap.add_argument("--latency-parts", type=int, nargs="*", default=[],
                    help="row splits tried by the pipelined per-layer latency probe")
    ap.add_argument("--stages", type=int, default=4, choices=[3, 4],
                    help="native pipeline: 4 = scan | top-k | gather | attend; 3 = top-k shares the scan stream")
    ap.add_argument("--mode", default="step", choices=["step", "scan", "select", "vq", "gather", "prefill"],
                    help="scan: only the key-scan kernel on one layer plus a 1 GiB copy for counter calibration; "
                         "select: the same for hca_score_topk (selecting scan, sampling, selection); "
                         "vq: the codebook form of the key path (assignment, table, lookup scan) on one layer; "
                         "gather: only the value gather at the workload's shape, against the host link's copy rate")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus N with N > 1 is not supported "
              "(one process, one MI355X, no collectives).", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth_inputs as S
    from paper_2507_19823_amd import binding as B
    B.lib()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    tune = {}
    for kv in args.tune:
        name, val = kv.split("=")
        if args.pipeline == "native" and args.mode == "step" and name != "host_spin_us":
            tune[name] = int(val)                     # the step driver takes its knobs from its own descriptor
        else:
            B.hca_tune(name, int(val))

    if args.pipeline == "native" and args.host_chunks and "gather_wgs" not in tune:
        tune["gather_wgs"] = 4                        # the gather moves an eighth of the rows: half the workgroups do
    w = S.CONFIGS[args.config]
    # a 32 Ki-token layer (20 MiB of codes) would sit in the last-level cache if it were scanned over and over:
    # the small workload is run as 16 layers, i.e. 16 cache copies in rotation
    L = args.layers or (16 if args.config == 2 else w.layers)
    if args.resident and args.mode in ("scan", "select"):
        import dataclasses
        w = dataclasses.replace(w, n=args.resident)
    if args.mode == "scan":
        return scan_only(w, args.steps)
    if args.mode == "select":
        return select_only(w, args.steps)
    if args.mode == "gather":
        return gather_only(w, args.steps)
    if args.mode == "prefill":
        print(json.dumps(dict(mode="prefill", **prefill_blocks(w))), flush=True)
        return
    if args.mode == "vq":
        print(json.dumps(dict(mode="vq", **vq_probe(w, args.steps, c=args.vq_codewords))), flush=True)
        return
    # host link: peak (one large pinned copy) and the gather as the path issues it
    # The boxes expose 4 hardware queues per process and HIP deals streams onto them round-robin, so
    # exactly four streams are used (the default one included): one per pipeline stage, none shared.
    main_s = [torch.cuda.current_stream()]
    gath_s = [torch.cuda.Stream()]
    extra = [torch.cuda.Stream(), torch.cuda.Stream()]
    _ = [x.cuda_stream for x in main_s + gath_s + extra]
    big = torch.empty(1 << 28, dtype=torch.uint8, pin_memory=True)
    dbig = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    dbig.copy_(big, non_blocking=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(16):
        dbig.copy_(big, non_blocking=True)
    torch.cuda.synchronize()
    link_peak = 16 * (1 << 28) / (time.perf_counter() - t0) / 1e9
    del dbig

    latency = {}
    if not args.no_latency:
        for name, c in (("128K", 3), ("1M", 4), ("4M", 5)):
            latency[name] = per_layer_latency(c, main_s[0], gath_s[0], link_peak)
            latency[name]["ms_per_layer_serial"] = latency[name]["ms_per_layer"]
            log(f"latency probe {name}: {latency[name]['ms_per_layer']:.3f} ms per layer, stages one after another")
            # the same with scan and top-k as one call (hca_score_topk); key_scan_ms is then the whole call
            f = per_layer_latency(c, main_s[0], gath_s[0], link_peak, fused=True,
                                  streams=(main_s[0], extra[0], gath_s[0], extra[1]))
            latency[name]["fused_select"] = {"ms_per_layer": f["ms_per_layer"], "score_topk_ms": f["score_topk_ms"],
                                             "select_scan_ms": f["key_scan_ms"], "select_scan_GBs": f["key_scan_GBs"],
                                             "select_scan_frac_of_hbm_peak": f["key_scan_frac_of_hbm_peak"],
                                             "select_scan_timed_by": "per-wave wall-clock stamps of the launch (first wave "
                                                                     "start to last wave end, the kernel's own duration)",
                                             "select_scan_event_bracket_ms": f.get("scan_event_bracket_ms")}
            log(f"latency probe {name}: {f['ms_per_layer']:.3f} ms per layer with scan and top-k fused "
                f"({f['score_topk_ms']:.3f} ms for the two; the selecting scan alone {f['key_scan_ms']:.3f} ms)")
            if args.pipeline == "native" and args.host_threads > 0:
                h = per_layer_latency_hybrid(c, main_s[0], args.host_threads)
                latency[name]["hybrid_value_side"] = h
                log(f"latency probe {name}: {h['ms_per_layer']:.3f} ms per layer with scan and top-k fused and "
                    f"{h['host_chunks_of'][0]} of {h['host_chunks_of'][1]} chunks of the value side on the host")
            for parts in args.latency_parts:
                g = per_layer_latency_grouped(c, parts, (main_s[0], extra[0], gath_s[0], extra[1]))
                log(f"latency probe {name}: {g['ms_per_layer']:.3f} ms per layer as {parts} pipelined parts "
                    f"(host enqueue {g['host_enqueue_ms']:.2f} ms behind a {g['gate_ms']:.2f} ms gate)")
                latency[name].setdefault("pipelined_parts", []).append(g)
                if g["host_enqueue_ms"] < g["gate_ms"] and g["ms_per_layer"] < latency[name]["ms_per_layer"]:
                    latency[name]["ms_per_layer"] = g["ms_per_layer"]
                    latency[name]["parts"] = parts

    codebook = selection = paper_form = cpu_split = None
    if not args.no_latency:
        codebook = vq_probe(S.CONFIGS[4], 10)
        log(f"codebook key path at 1M: table + lookup scan {codebook['score_ms']:.3f} ms per layer")
        paper_form = paper_form_probe(S.CONFIGS[4], (main_s[0], extra[0], gath_s[0], extra[1]))
        log(f"paper-form decode step at 1M: {paper_form['ms_per_layer']:.3f} ms per layer on one stream, "
            f"{paper_form['pipelined_ms_per_layer']:.3f} ms through the step driver")
        # the same with the paper's own codebook size (g = 32, c = 8192: 16-bit indices, table through LDS in slices)
        paper_form["c8192"] = paper_form_probe(S.CONFIGS[4], (main_s[0], extra[0], gath_s[0], extra[1]), layers=4, c=8192)
        log(f"paper-form decode step at 1M, c = 8192: {paper_form['c8192']['ms_per_layer']:.3f} ms per layer on one "
            f"stream, {paper_form['c8192']['pipelined_ms_per_layer']:.3f} ms through the step driver")
        cpu_split = cpu_split_probe(S.CONFIGS[4])
        log(f"value side at 1M, k 4096: gather + attend {cpu_split['gather_plus_attend_ms']:.3f} ms; paper's split "
            f"{cpu_split['split_gpu_weights_ms']:.3f} ms on the GPU + {cpu_split['split_host_sum_ms']:.3f} ms on the host")
        selection = selection_probe(S.CONFIGS[4])
        log(f"selection at 1M: top-k {selection['topk_ms']:.3f} ms, Eq. 4 at tau 0.9 {selection['topp_tau0.9']['ms']:.3f} ms")

    others = None
    correlated = None
    prefill = None
    if not args.no_latency and args.config == 4:
        prefill = prefill_blocks(w)
        log("block-wise key compression, fraction of the bound by block size "
            + "; ".join(f"{k_}: " + " ".join(f"{r.get('frac_of_hbm_peak', r.get('frac_of_fp32_vector_peak', r.get('frac_of_f16_matrix_peak'))):.2f}" for r in v_)
                        for k_, v_ in prefill.items() if isinstance(v_, list) and v_ and isinstance(v_[0], dict)))
    if not args.no_latency and args.config == 4:
        correlated = correlated_selection(w)
        log("fused selection at 1M, ms per call (candidates min..max, second scans): " + "; ".join(
            f"{k_} {v_['score_topk_ms']:.3f} ({v_['candidates_min']}..{v_['candidates_max']}, {v_['rows_rescanned']})"
            for k_, v_ in correlated.items() if isinstance(v_, dict)))
    if not args.no_latency and args.pipeline == "native" and args.config == 4:
        # the same step driver on the other stacks (a few steps each; the headline stays config 4)
        st4 = (main_s[0], extra[0], gath_s[0], extra[1])
        others = {"cfg3": other_config_step(3, 1, 1, 16, st4, args, tune)}
        log(f"config 3 through the step driver: {others['cfg3']['ms_per_step']:.3f} ms per step")
        others["cfg5"] = other_config_step(5, 8, 2, 6, st4, args, tune)
        others["cfg5"]["note"] = ("8 of the 32 layers on 2 physical value stores (the full stack needs 256 GiB of pinned "
                                  "memory), 4 Mi resident tokens per layer; ms_per_layer x 32 extrapolates the stack")
        log(f"config 5 through the step driver, 8 layers: {others['cfg5']['ms_per_step']:.3f} ms per step "
            f"({others['cfg5']['ms_per_layer']:.3f} ms per layer)")
    total_steps = args.steps + args.warmup
    fused = args.pipeline == "native" and not args.no_fused_select
    model = Model(w, L, args.evict_every, total_steps, n_sel=min(L, args.sel_buffers), evict_spare=args.evict_spare,
                  fused=fused, host_chunks=args.host_chunks if args.pipeline == "native" else 0,
                  host_threads=args.host_threads, tune=tune, n_pipe_sets=args.pipe_sets, dual_scan=args.scan_mode)
    layer_v_gib = w.batch * w.n_kv_heads * w.n * 256 / 2 ** 30
    phys = max(1, min(L, int(args.host_gib / layer_v_gib)))
    t0 = time.perf_counter()
    tq = model.build(phys)
    model.make_steps(total_steps)
    phys = model.phys
    log(f"setup {time.perf_counter() - t0:.1f}s: {L} layers, {phys} physical value layers "
        f"({phys * layer_v_gib:.1f} GiB pinned), bulk quantise {tq:.3f}s")
    bulk_tokens = L * w.batch * w.n_kv_heads * w.n
    code_bytes = 128 * w.bits // 8 + (128 // w.group) * 4

    main, side = main_s[0], gath_s[0]

    model.gap_report = args.gap_report
    model.layer_idx_on = args.pipeline == "native" and not args.slot_idx
    if args.pipeline == "native":
        model.native_pipeline(main, main if args.stages == 3 else extra[0], side, extra[1], args.steps,
                              args.bracket_stride)

    def run_step(t, ev=None):
        if args.pipeline == "native":
            model.decode_step_native(t, -1 if ev is None else t - args.warmup)
        elif args.pipeline == "staged":
            model.decode_step_staged(t, main, extra[0], side, extra[1], ev)
        else:
            model.decode_step(t, main, side, args.pipeline == "gather", ev)

    cal_src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)                            # calibration dispatch for counter runs: reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    del cal_src, cal_dst
    for t in range(args.warmup):
        run_step(t)
    if args.pipeline == "native" and fused:
        torch.cuda.synchronize()                      # the warm-up steps' selections are not counted
        for wsl in model.ws_sel:
            B.hca_score_topk_monitor(model.shape, wsl, None, True)
    torch.cuda.synchronize()
    log("warmup done")
    events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(L)]
              for _ in range(args.steps)]
    # what the check against the oracle needs: the verification layer's top-k indices and output of the timed steps
    # up to its first eviction, copied aside behind each of those steps. Each copy rides the stream that writes its
    # source (indices: the top-k stream; output: the attend stream), so it is ordered before the next step's
    # writes and no stream waits for another.
    captured = {}
    vslot = model.verify_layer % model.n_pipe_sets if args.pipeline == "native" else 0
    topk_s = main if args.stages == 3 else extra[0]

    def capture(t):
        with torch.cuda.stream(topk_s):
            ci = (model.layer_idx[model.verify_layer] if model.layer_idx is not None else model.pipe[vslot]["idx"]).clone()
        with torch.cuda.stream(extra[1]):
            cy = model.y[model.verify_layer].clone()
        captured[t] = (ci, cy)

    step_end = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    host_done = []
    step_end[0].record(extra[1])                      # the attend stream: a step's last kernels run there
    t0 = time.perf_counter()
    host_steps = []
    for t in range(args.warmup, total_steps):
        h0 = time.perf_counter()
        run_step(t, events[t - args.warmup])
        if args.pipeline == "native" and not args.no_cpu_baseline and t <= model.verify_until and len(captured) < 6:
            capture(t)
        step_end[t - args.warmup + 1].record(extra[1] if args.pipeline in ("native", "staged") else main)
        host_steps.append((time.perf_counter() - h0) * 1e3)
        host_done.append((time.perf_counter() - t0) * 1e3)
    host_dt = time.perf_counter() - t0
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    log(f"timed region done: {dt:.3f}s for {args.steps} steps (host enqueue {host_dt:.3f}s; per step ms: "
        + " ".join(f"{x:.2f}" for x in host_steps) + ")")
    if args.pipeline == "native":
        gpu_done = [step_end[0].elapsed_time(step_end[i + 1]) for i in range(args.steps)]
        log("host lead per step (GPU end of step - host end of its enqueue, ms): "
            + " ".join(f"{g - h:.2f}" for g, h in zip(gpu_done, host_done)))
    ms_per_step = dt * 1e3 / args.steps
    host_side = None
    if args.pipeline == "native" and model.host_chunks:
        to, bad = B.hca_pipeline_host_status(model.pl)
        ju, tu = B.hca_pipeline_host_times(model.pl)
        host_side = {"wait_timeouts": to, "bad_rows": bad, "host_us_per_layer": ju, "host_us_per_chunk": tu}
        log(f"hybrid value side: host threads {ju:.1f} us per layer, {tu:.1f} us per chunk; timeouts {to}, bad rows {bad}")
    tokens_per_step = w.batch * w.n * L
    value = tokens_per_step / (dt / args.steps)
    bracket_ms = None
    if args.pipeline == "native":
        # event bracket around each scan launch (includes the wait for the other stages' kernels to make
        # room) and the kernel's own duration from the per-wave wall-clock stamps (first start to last end)
        per = [x for slot in range(args.steps) for x in B.hca_pipeline_scan_ms(model.pl, slot, L) if x >= 0]
        bracket_ms = sum(per) / len(per)
        st_ = model.stamps
        starts = torch.where(st_[..., 0] > 0, st_[..., 0], torch.full_like(st_[..., 0], 1 << 62)).amin(-1)
        ends = st_[..., 1].amax(-1)
        layers_per_launch = 1
        if fused and args.scan_mode == "pair" and L % 2 == 0:
            # one launch scans two layers: its duration runs from the first wave of either to the last wave of either
            layers_per_launch = 2
            starts = starts.reshape(args.steps, L // 2, 2).amin(-1)
            ends = ends.reshape(args.steps, L // 2, 2).amax(-1)
        khz = B.hca_wall_clock_khz()
        scan_ms = float((ends - starts).double().mean()) / khz
        flat_s, flat_e = starts.reshape(-1).double(), ends.reshape(-1).double()
        gaps = (flat_s[1:] - flat_e[:-1]) / khz * 1e3
        log("key scan launches: mean %.1f us; idle between consecutive ones: mean %.1f us, median %.1f us" % (
            scan_ms * 1e3, float(gaps.mean()), float(gaps.median())))
        if args.gap_report:
            edges = [0, 10, 20, 30, 50, 80, 120, 200, 400, 100000]
            hist = []
            for a, b in zip(edges[:-1], edges[1:]):
                m = (gaps >= a) & (gaps < b)
                hist.append(f"[{a},{b}): {int(m.sum())} gaps, {float(gaps[m].sum()) / args.steps:.0f} us/step")
            log("scan gap histogram: " + "; ".join(hist))
            # mean pause before each launch of a step (launch 0: the pause across the step boundary), over the steps
            nl_ = starts.shape[1]
            by_launch = torch.cat([gaps.new_zeros(1), gaps]).reshape(args.steps, nl_)[1:].mean(0)
            log("mean pause before launch i of a step, us: " + " ".join(f"{float(x):.0f}" for x in by_launch))
            gs = model.gstamps
            g_start = torch.where(gs[..., 0] > 0, gs[..., 0], torch.full_like(gs[..., 0], 1 << 62)).amin(-1).reshape(-1).double()
            g_end = gs[..., 1].amax(-1).reshape(-1).double()
            ggaps = (g_start[1:] - g_end[:-1]) / khz * 1e3
            gdur = (g_end - g_start) / khz * 1e3
            log("gathers: mean %.1f us; idle between consecutive ones: mean %.1f us, median %.1f us" % (
                float(gdur.mean()), float(ggaps.mean()), float(ggaps.median())))
            # merged timeline of scan launches and gathers around one step boundary (wall-clock stamps, us)
            try:
                if not args.timeline_out:
                    raise RuntimeError("no --timeline-out path given")
                sb_, ge_ = starts.reshape(-1).double() / khz * 1e3, ends.reshape(-1).double() / khz * 1e3
                per = sb_.numel() // args.steps
                mid = (args.steps // 2) * per
                base = float(sb_[mid])
                ev_ = [(float(sb_[i]) - base, float(ge_[i]) - base, f"scan  launch {i % per} step {i // per}")
                       for i in range(mid - per // 2, mid + per // 2)]
                gi0 = (args.steps // 2) * L
                ev_ += [(float(g_start[i]) / khz * 1e3 - base, float(g_end[i]) / khz * 1e3 - base, f"gather layer {i % L} step {i // L}")
                        for i in range(gi0 - L // 2, gi0 + L // 2)]
                with open(args.timeline_out, "w") as f:
                    for a_, b_, n_ in sorted(ev_):
                        f.write(f"{a_:10.1f} {b_:10.1f} {n_}\n")
            except Exception as e:                    # a diagnostic only
                log(f"no timeline written: {e}")
            gtop = torch.topk(ggaps, 24)
            log("largest gather gaps (us @ step.layer): " + " ".join(
                "%.0f@%d.%d" % (float(v), (int(i) + 1) // L, (int(i) + 1) % L) for v, i in zip(gtop.values, gtop.indices)))
            top = torch.topk(gaps, 24)
            # a gap sits before launch (i + 1) of the flat list; a launch scans layers_per_launch layers
            log("largest gaps (us @ step.first layer of the launch behind the gap): " + " ".join(
                "%.0f@%d.%d" % (float(v), (int(i) + 1) // nl_, ((int(i) + 1) % nl_) * layers_per_launch)
                for v, i in zip(top.values, top.indices)))
    else:
        layers_per_launch = 1
        events = [e for step_events in events for e in step_events]
        scan_ms = sum(a.elapsed_time(b) for a, b in events) / len(events)
    scan_bytes = layers_per_launch * w.batch * w.n_kv_heads * (w.n + 1) * (code_bytes + (0 if fused else 4))
    achieved = scan_bytes / (scan_ms * 1e-3) / 1e9

    traffic = None
    pair = fused and layers_per_launch == 2
    pmc = os.path.join(ROOT, "profiles", ("select_scan_pair_cfg4_1m_pmc.md" if pair else "select_scan_cfg4_1m_pmc.md")
                       if fused else "score_kernel_cfg4_1m_pmc.md")
    kernel = ("score_select_pair_kernel (the selecting scan; two layers per launch)" if pair else
              "score_select_step_kernel (the selecting scan; one launch per layer)" if fused else "score_kernel")
    if args.config == 4 and os.path.exists(pmc):     # measured with rocprofv3 --pmc, see that file
        for line in open(pmc):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])
    out = {
        "metric": "context tokens scored/s + per-layer decode latency at 128K/1M/4M (HBM GB/s %)",
        "value": value, "unit": "context tokens scored/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "context": w.n, "layers": L, "q_heads": w.n_q_heads,
                   "kv_heads": w.n_kv_heads, "key_bits": w.bits, "group": w.group, "top_k": w.k,
                   "evict_every": args.evict_every,
                   "eviction_case": ("in place; M = the context length, the newest evict_every slots protected: the dropped "
                                     "slots are the newest never-selected ones just below the protected window (ties go "
                                     "against the higher slot) and the keep-set's threshold is 0, so one counting pass "
                                     "over the accumulated scores and a short tail move are paid (~0.06 ms per layer); "
                                     "an eviction whose first dropped slot is early costs about 0.7 ms per layer, one "
                                     "whose threshold is not 0 four more passes") if args.evict_every else None,
                   "values": "context rows in pinned host fp16, appended rows in an HBM slice",
                   "physical_value_layers": phys, "pipeline": args.pipeline,
                   "value_side": (f"hybrid: {model.host_chunks} of {-(-w.k // 256)} chunks of 256 selected tokens per row "
                                  f"summed by {model.host_threads} host threads from the value store, the rest gathered"
                                  if model.host_chunks else "all selected rows gathered over the host link"),
                   "selection": "hca_score_topk (scan + top-k fused)" if fused else "hca_score_qkeys + hca_topk"},
        "pipelined_ms_per_layer": ms_per_step / L,
        "per_layer_decode_latency": latency,
        "steps_other_configs": others,
        "codebook_key_path": codebook,
        "selection": selection,
        "fused_selection_on_correlated_keys": correlated,
        "prefill_block_compression": prefill,
        "paper_form_step": paper_form,
        "value_side_cpu_split": cpu_split,
        "bulk_quantize_tokens_per_s": bulk_tokens / tq,
        "bulk_quantize_GBs": bulk_tokens * (256 + code_bytes) / tq / 1e9,
        "host_link_peak_GBs": link_peak,
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": (f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of the same kernel alone, recorded in "
                                        f"profiles/{os.path.basename(pmc)} (not a counter of this run)") if traffic else None,
                     "layers_per_launch": layers_per_launch,
                     "avg_launch_ms": scan_ms, "bytes_per_launch": scan_bytes,
                     "avg_event_bracket_ms": bracket_ms,
                     # the same kernel at the same shape with no other kernel beside it (latency probe above)
                     "frac_alone": (latency.get("1M", {}).get("fused_select", {}).get("select_scan_frac_of_hbm_peak") if fused
                                    else latency.get("1M", {}).get("key_scan_frac_of_hbm_peak")) if args.config == 4 else None},
    }
    if args.pipeline == "native":
        # per row and set of selection buffers, over every fused selection of the timed steps: the fewest and the most
        # pairs a first scan let through, and how many selections needed the second scan
        if fused:
            mon = torch.zeros(len(model.ws_sel), model.rows, 4, dtype=torch.int32, device="cuda")
            for i, wsl in enumerate(model.ws_sel):
                B.hca_score_topk_monitor(model.shape, wsl, mon[i], False)
            torch.cuda.synchronize()
            mon = mon.cpu()
            out["selection_monitor"] = {"scope": "every row of every layer, every timed step",
                                        "selections": int(mon[..., 0].sum()),
                                        "expected_selections": args.steps * L * model.rows,
                                        "candidates_min": int(mon[..., 1].min()), "candidates_max": int(mon[..., 2].max()),
                                        "rows_rescanned": int(mon[..., 3].sum())}
        out["hybrid_value_side"] = host_side
        B.hca_pipeline_destroy(model.pl)              # ends the driver's host threads before the oracle is timed
    out["verified"] = None
    if not args.no_cpu_baseline:
        want = max(captured) + 1 if captured else 0
        results, out["cpu_baseline"] = run_cpu_baseline(model, w, min_steps=want)
        if captured:
            import numpy as np
            worst, checked, sets_ok = 0.0, [], True
            for t, (gi, gy) in sorted(captured.items()):
                oi, oy = results[t]
                gi = gi.cpu().numpy().reshape(oi.shape)
                if not np.array_equal(gi, oi):
                    log(f"VERIFICATION FAILED: step {t}, layer {model.verify_layer}: top-k index sets differ from the oracle's")
                    out["verified"], sets_ok = False, False
                    break
                gy = gy.cpu().numpy().reshape(oy.shape)
                err = float(np.max(np.abs(gy - oy).max(-1) / np.maximum(np.abs(oy).max(-1), 1e-30)))
                worst = max(worst, err)
                checked.append(t)
            else:
                out["verified"] = bool(worst <= 2e-3)
            out["verification"] = {"layer": model.verify_layer, "steps": checked, "of_timed_steps": f"{args.warmup}..{total_steps - 1}",
                                   "top_k_sets": "bit-exact" if sets_ok else "differ",
                                   "max_rel_err_y": worst, "tolerance": 2e-3,
                                   "against": "the oracle's replay of the same layer from step 0 (cpu_baseline leg)"}
    print(json.dumps(out), flush=True)
    if out["verified"] is False:
        log("result printed; the timed region's outputs do NOT match the oracle")
        sys.exit(1)
    log("result printed")


if __name__ == "__main__":
    main()
