"""Runs a stack of SpC layers (a list of layer dicts as produced by
``synth.unet_layers``) through the C-ABI binding: all kernel maps are built up front by
``spc_build_kmaps_network`` (network-wide voxel indexing, Section 5.5), then every layer
is one ``spc_conv_forward`` call.  Skip connections are realised without a copy: the two
producers write into the two column halves of one buffer (row pitch arguments).

``SpcNetwork.capture_step`` records the whole step of one cloud size (pack + sort, feature
permutation, map build on several streams, all feature layers) into one HIP graph: a step
enqueues some 150 small kernels and as many event operations, which costs the host about as
much time as the GPU needs to run them; replaying the graph removes the host from the loop."""
from __future__ import annotations

import torch

from . import binding as B


class SpcNetwork:
    def __init__(self, layers, weights, dataflow=None, hybrid_t=None):
        """weights: list of device tensors [K^3, cin, cout]; dataflow: None (OS everywhere), a
        single B.DATAFLOW_* value, or one value per layer.  hybrid_t: None, or one entry per layer,
        each None (use `dataflow`) or the threshold of the hybrid dual dataflow for that layer."""
        self.layers = layers
        self.weights = weights
        n = len(layers)
        if dataflow is None:
            dataflow = B.DATAFLOW_OS
        self.dataflow = [dataflow] * n if isinstance(dataflow, int) else list(dataflow)
        self.hybrid_t = [None] * n if hybrid_t is None else list(hybrid_t)
        self.maps = None
        self.size_hints = None  # per layer: n_out seen by the last learn_sizes()
        self._packed = None  # per layer: weights in the MFMA operand layout, or None
        # concat plan: tensor name -> (buffer name, column offset); a buffer holds [src | skip]
        self._placement = {}
        for l in layers:
            if l["skip"] is not None:
                buf = "cat_" + l["name"]
                src_w = next(x["cout"] for x in layers if x["save"] == l["src"])
                self._placement[l["src"]] = (buf, 0, l["cin"])
                self._placement[l["skip"]] = (buf, src_w, l["cin"])

    def build_maps(self, v0_keys, desc, streams=None, flags=0, use_hints=False):
        """use_hints: hand the level sizes of the last learn_sizes() to the new maps, so that the feature
        kernels are chosen for those sizes without anybody waiting for the true counts."""
        req = []
        for l, df, t in zip(self.layers, self.dataflow, self.hybrid_t):
            # a hybrid layer asks for exactly the split it will use: dense offsets in the matrix, sparse ones in lists
            layout = (B.LAYOUT_BOTH | B.LAYOUT_HYBRID_T(t)) if t is not None else (B.LAYOUT_OS if df == B.DATAFLOW_OS else B.LAYOUT_WS)
            req.append((l["K"], l["in_stride"], l["layer_stride"], l["transposed"], layout))
        self.maps = B.spc_build_kmaps_network(v0_keys, desc, req, streams, flags)
        if use_hints and self.size_hints is not None:
            for m, h in zip(self.maps, self.size_hints):
                m.set_size_hint(h)
        return self.maps

    def learn_sizes(self):
        """Remembers every layer's output count of the current maps (waits for the build)."""
        self.size_hints = [m.n_out for m in self.maps]
        return self.size_hints

    def destroy_maps(self):
        if self.maps:
            for m in self.maps:
                m.destroy()
        self.maps = None

    def prepare_weights(self):
        """Re-orders every layer's weights once into the layout the MFMA kernels read (layers whose
        shape those kernels do not take directly keep their plain weights)."""
        self._packed = []
        for w, df, t in zip(self.weights, self.dataflow, self.hybrid_t):
            cin, cout = w.shape[1], w.shape[2]
            ok = w.dtype in (torch.float16, torch.bfloat16) and cout % 32 == 0
            if df == B.DATAFLOW_WS or t is not None:
                ok = ok and cout in (32, 64, 128, 256)
            self._packed.append(B.spc_conv_prepare_weights(w) if ok else None)

    def forward(self, feats, keep=False, static_rows=None):
        """feats: [n0, cin] device tensor in sorted-voxel order.  Returns the last layer's output
        (and, with keep=True, the dict of all saved tensors).
        static_rows: None -> every tensor has exactly its level's voxel count, which the host waits
        for once per level.  An int (an upper bound of every level's count, e.g. n0) -> every tensor
        gets that many rows, of which the first n_out are written; nothing waits, so the call can be
        captured into a graph."""
        assert self.maps is not None, "call build_maps first"
        if self._packed is None:
            self.prepare_weights()
        T = {"input": feats}
        bufs = {}
        y = None
        for j, l in enumerate(self.layers):
            m = self.maps[j]
            n_out = m.n_out if static_rows is None else int(static_rows)
            x = T[l["src"]]
            if l["skip"] is not None:
                buf, _, _ = self._placement[l["src"]]
                x = bufs[buf]  # both halves were written in place by their producers
            out = None
            if l["save"] in self._placement:
                buf, col, width = self._placement[l["save"]]
                if buf not in bufs:
                    bufs[buf] = torch.empty((n_out, width), dtype=feats.dtype, device=feats.device)
                out = bufs[buf][:, col:col + l["cout"]]
            flags = B.CONV_RELU if l["relu"] else 0
            w = self.weights[j]
            if self._packed[j] is not None:
                w, flags = self._packed[j], flags | B.CONV_PACKED_WEIGHTS
            y = B.spc_conv_forward(m, x, w, self.dataflow[j], flags, out=out, n_out=n_out, hybrid_t=self.hybrid_t[j])
            T[l["save"]] = y
        return (y, T) if keep else y

    def tune(self, v0_keys, desc, feats, reps=5):
        """One-time tuning of the hybrid dual dataflow (Section 5.4): on the sample cloud given, every
        layer's feature computation is timed for every threshold t = 0 (pure weight-stationary) ..
        L1max + 1 (pure output-stationary) by the library (spc_conv_tune_threshold), with the extra
        kernel-map build time of the layouts a threshold needs added, and the fastest threshold is
        kept.  Returns one row per layer:
        (name, best t, {t: microseconds}).  Afterwards build_maps / forward use the chosen settings."""
        n = len(self.layers)
        ev = lambda: torch.cuda.Event(enable_timing=True)

        def timed(fn):
            fn()
            a, b = ev(), ev()
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps * 1e3

        # activations of every layer with the current settings, and maps that hold both layouts
        self.build_maps(v0_keys, desc)
        _, T = self.forward(feats, keep=True)
        self.destroy_maps()
        req = [(l["K"], l["in_stride"], l["layer_stride"], l["transposed"], B.LAYOUT_BOTH) for l in self.layers]
        maps = B.spc_build_kmaps_network(v0_keys, desc, req)
        if self._packed is None:
            self.prepare_weights()
        rows = []
        build_cost = {}
        for j, l in enumerate(self.layers):
            geo = (l["K"], l["in_stride"], l["layer_stride"], l["transposed"])
            if geo not in build_cost:  # what the weight-stationary lists add to this geometry's map build
                in_keys = v0_keys
                t_os = timed(lambda: B.spc_build_kmaps_network(in_keys, desc, [geo + (B.LAYOUT_OS,)])[0].destroy())
                t_both = timed(lambda: B.spc_build_kmaps_network(in_keys, desc, [geo + (B.LAYOUT_BOTH,)])[0].destroy())
                build_cost[geo] = max(t_both - t_os, 0.0)
            x = T[l["src"]]
            if l["skip"] is not None:
                x = torch.cat([T[l["src"]], T[l["skip"]]], dim=1)
            w = self.weights[j]
            cout = w.shape[2]
            wp = B.spc_conv_prepare_weights(w) if (w.dtype != torch.float32 and cout % 32 == 0) else None
            out = torch.empty((maps[j].n_out, cout), dtype=x.dtype, device=x.device)
            l1_max = 3 if l["K"] == 2 else 3 * (l["K"] - 1) // 2
            best, us, _ = B.spc_conv_tune_threshold(maps[j], x, w, wp, flags=B.CONV_RELU if l["relu"] else 0, reps=reps,
                                                    ws_build_us=build_cost[geo], out=out)
            times = dict(enumerate(us))
            rows.append((l["name"], best, times))
            if best == l1_max + 1:
                self.dataflow[j], self.hybrid_t[j] = B.DATAFLOW_OS, None
            elif best == 0:
                self.dataflow[j], self.hybrid_t[j] = B.DATAFLOW_WS, None
            else:
                self.hybrid_t[j] = best
        for m in maps:
            m.destroy()
        self._packed = None  # the packable set depends on the dataflow of each layer
        return rows

    def capture_step(self, coords, feats_raw, desc, streams=None, flags=0):
        """Records one full step for clouds of coords.shape[0] voxels into a HIP graph and returns a
        CapturedStep.  Runs the step once eagerly first: that fills the library's block cache on the
        streams used (so the capture allocates nothing) and learns the level sizes the kernels are
        chosen for.  `coords` [n0,4] int32 and `feats_raw` [n0,cin] are the graph's input buffers:
        overwrite them in place, then replay."""
        return CapturedStep(self, coords, feats_raw, desc, streams, flags)


class CapturedStep:
    def __init__(self, net, coords, feats_raw, desc, streams, flags):
        n0 = coords.shape[0]
        dev = coords.device
        self.net, self.coords, self.feats_raw = net, coords, feats_raw
        self.ws = torch.empty(B.spc_pack_workspace_bytes(n0, desc), dtype=torch.uint8, device=dev)
        self.keys = torch.empty(n0, dtype=torch.int32 if desc.key_bits == 32 else torch.int64, device=dev)
        self.perm = torch.empty(n0, dtype=torch.int32, device=dev)
        self.feats = torch.empty_like(feats_raw)
        self.stream = torch.cuda.Stream(device=dev)
        side = list(streams) if streams else []

        def step(static):
            B.spc_pack_coords(coords, desc, True, 0, None, self.ws, self.keys, self.perm)
            B.spc_permute_rows(feats_raw, self.perm, self.feats)
            net.build_maps(self.keys, desc, [torch.cuda.current_stream()] + side, flags, use_hints=static)
            if not static:
                net.learn_sizes()
            return net.forward(self.feats, static_rows=n0 if static else None)

        self.stream.wait_stream(torch.cuda.current_stream(dev))
        with torch.cuda.stream(self.stream):
            step(False)
            net.destroy_maps()
            step(True)  # same allocation pattern as the capture
            net.destroy_maps()
        torch.cuda.synchronize(dev)
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph, stream=self.stream, capture_error_mode="relaxed"):
            self.output = step(True)
        self.maps = net.maps  # alive as long as the graph
        net.maps = None

    def replay(self):
        self.graph.replay()

    def n_out(self) -> int:
        """Valid rows of `output` after the latest replay (drains the device)."""
        return self.maps[-1].n_out

    def destroy(self):
        self.graph = None
        for m in self.maps or []:
            m.destroy()
        self.maps = None
