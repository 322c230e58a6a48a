"""Runs a stack of SpC layers (a list of layer dicts as produced by
``synth.unet_layers``) through the C-ABI binding: all kernel maps are built up front by
``spc_build_kmaps_network`` (network-wide voxel indexing, Section 5.5), then every layer
is one ``spc_conv_forward`` call.  Skip connections are realised without a copy: the two
producers write into the two column halves of one buffer (row pitch arguments)."""
from __future__ import annotations

import torch

from . import binding as B


class SpcNetwork:
    def __init__(self, layers, weights, dataflow=None):
        """weights: list of device tensors [K^3, cin, cout]; dataflow: None (OS everywhere), a
        single B.DATAFLOW_* value, or one value per layer."""
        self.layers = layers
        self.weights = weights
        n = len(layers)
        if dataflow is None:
            dataflow = B.DATAFLOW_OS
        self.dataflow = [dataflow] * n if isinstance(dataflow, int) else list(dataflow)
        self.maps = None
        self._packed = None  # per layer: weights in the MFMA operand layout, or None
        # concat plan: tensor name -> (buffer name, column offset); a buffer holds [src | skip]
        self._placement = {}
        for l in layers:
            if l["skip"] is not None:
                buf = "cat_" + l["name"]
                src_w = next(x["cout"] for x in layers if x["save"] == l["src"])
                self._placement[l["src"]] = (buf, 0, l["cin"])
                self._placement[l["skip"]] = (buf, src_w, l["cin"])

    def build_maps(self, v0_keys, desc, streams=None, flags=0):
        req = []
        for l, df in zip(self.layers, self.dataflow):
            layout = B.LAYOUT_OS if df == B.DATAFLOW_OS else B.LAYOUT_WS
            req.append((l["K"], l["in_stride"], l["layer_stride"], l["transposed"], layout))
        self.maps = B.spc_build_kmaps_network(v0_keys, desc, req, streams, flags)
        return self.maps

    def destroy_maps(self):
        if self.maps:
            for m in self.maps:
                m.destroy()
        self.maps = None

    def prepare_weights(self):
        """Re-orders every layer's weights once into the layout the MFMA kernels read (layers whose
        shape those kernels do not take directly keep their plain weights)."""
        self._packed = []
        for w, df in zip(self.weights, self.dataflow):
            cin, cout = w.shape[1], w.shape[2]
            ok = w.dtype in (torch.float16, torch.bfloat16) and cin % 16 == 0 and cout % 32 == 0
            if df == B.DATAFLOW_WS:
                ok = ok and cout in (32, 64, 128, 256)
            self._packed.append(B.spc_conv_prepare_weights(w) if ok else None)

    def forward(self, feats, keep=False):
        """feats: [n0, cin] device tensor in sorted-voxel order.  Returns the last layer's output
        (and, with keep=True, the dict of all saved tensors)."""
        assert self.maps is not None, "call build_maps first"
        if self._packed is None:
            self.prepare_weights()
        T = {"input": feats}
        bufs = {}
        y = None
        for j, l in enumerate(self.layers):
            m = self.maps[j]
            n_out = m.n_out
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
            if self._packed[j] is not None and x.stride(0) % 8 == 0 and x.data_ptr() % 16 == 0:
                w, flags = self._packed[j], flags | B.CONV_PACKED_WEIGHTS
            y = B.spc_conv_forward(m, x, w, self.dataflow[j], flags, out=out, n_out=n_out)
            T[l["save"]] = y
        return (y, T) if keep else y
