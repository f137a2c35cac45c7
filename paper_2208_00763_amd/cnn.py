"""Layer chaining for the complete-model experiment (Section "Complete model evaluation"):
conv layers through the packed DNN path, each followed by the un-accelerated epilogue
(ReLU, requantise, optional 2x2 max-pool) that writes the next layer's bit-dense input.

Orchestration only: every step runs in libhikonv kernels on the caller's stream.
"""
import torch

from . import binding as hk


class PackedCnn:
    """Pre-packs the weights of a list of conv layers once; forward() runs the chain."""

    def __init__(self, weights, specs, act_bits=4, w_bits=4, w_signed=True, wide=True, m=0, tight=0, fused=True,
                 keep_accs=True, objective=hk.OBJ_PAPER_OPS):
        """fused: "layer" = one kernel per layer (hikonv_conv2d_fused: the convolution's store stage
        writes the next layer's packed activation words; layers it does not cover fall back to the
        next form); True = a convolution kernel and an epilogue kernel that writes the next
        layer's packed words (hikonv_epilogue_pack); False = the epilogue writes bit-dense rows
        that the next layer packs.  keep_accs (fused == "layer" only): also store every layer's
        int32 accumulators (the last layer's are always stored).  objective: what the planner
        optimises for every layer (Algorithm 1's operations per multiply, or the modelled cost)."""
        self.layers = []
        width, acc = (32, 64) if wide else (24, 32)
        for w_dev, spec in zip(weights, specs):
            co, c, kh, kw = w_dev.shape
            plan = hk.hikonv_plan_ex(bits_a=act_bits, bits_w=w_bits, a_signed=0, w_signed=int(w_signed), L_A=width,
                                     L_B=width, L_acc=acc, mode=hk.MODE_DNN, M=m, taps=kw, tight=tight,
                                     objective=objective, max_N=hk.LAYER_MAX_N)
            packed = torch.empty(hk.hikonv_packed_weights_bytes(plan, co, c, kh, kw), dtype=torch.uint8,
                                 device=w_dev.device)
            hk.hikonv_pack_weights(plan, w_dev, co, c, kh, kw, packed)
            self.layers.append(dict(plan=plan, packed=packed, co=co, c=c, kh=kh, kw=kw, pad=spec["pad"],
                                    pool=spec["pool"]))
        self.act_bits = act_bits
        self.fused = fused
        self.keep_accs = keep_accs
        self.layer_kernel = [fused == "layer"] * len(self.layers)   # cleared where the fused kernel does not apply
        self.buffers = None

    def _allocate(self, n, h, w):
        bufs = []
        for layer in self.layers:
            ho = h + 2 * layer["pad"] - layer["kh"] + 1
            wo = w + 2 * layer["pad"] - layer["kw"] + 1
            ws = torch.empty(hk.hikonv_conv2d_workspace_bytes(layer["plan"], n, layer["c"], h, w, layer["co"],
                                                              layer["kh"], layer["kw"], 1, layer["pad"], True),
                             dtype=torch.uint8, device="cuda")
            acc = torch.empty(n * layer["co"] * ho * wo, dtype=torch.int32, device="cuda")
            h2, w2 = (ho // 2, wo // 2) if layer["pool"] else (ho, wo)
            row_bytes = hk.hikonv_bitdense_row_bytes(w2, self.act_bits)
            nxt = torch.empty(n * layer["co"] * h2 * row_bytes, dtype=torch.uint8, device="cuda")
            bufs.append(dict(ws=ws, acc=acc, nxt=nxt, h=h, w=w, ho=ho, wo=wo))
            h, w = h2, w2
        self.buffers = (n, bufs)

    def forward(self, x_bitdense, n, h, w, shifts, qmax=15):
        """x_bitdense: [n][c0][h] bit-dense rows.  Returns (int32 accumulators of the last layer,
        list of per-layer int32 accumulator tensors)."""
        if self.buffers is None or self.buffers[0] != n or self.buffers[1][0]["h"] != h or self.buffers[1][0]["w"] != w:
            self._allocate(n, h, w)
        cur, fmt = x_bitdense, hk.FMT_BITDENSE
        accs = []
        bufs = self.buffers[1]
        for i, (layer, buf) in enumerate(zip(self.layers, bufs)):
            last = i + 1 == len(self.layers)
            if self.layer_kernel[i]:
                nxt = None if last else self.layers[i + 1]
                try:
                    hk.hikonv_conv2d_fused(
                        layer["plan"], cur, fmt, n, layer["c"], buf["h"], buf["w"], layer["packed"], layer["co"],
                        layer["kh"], layer["kw"], layer["pad"], buf["ws"], buf["acc"] if (self.keep_accs or last) else None,
                        0 if last else shifts[i], qmax, layer["pool"], None if last else nxt["plan"],
                        0 if last else nxt["co"], 0 if last else nxt["kh"], 0 if last else nxt["kw"],
                        0 if last else nxt["pad"], None if last else bufs[i + 1]["ws"])
                    accs.append(buf["acc"])
                    cur, fmt = None, hk.FMT_PACKED
                    continue
                except hk.HikonvError as err:
                    if err.code != hk.EUNSUPPORTED:
                        raise
                    self.layer_kernel[i] = False        # refused on the host, nothing was launched
            hk.hikonv_conv2d_prepacked(layer["plan"], cur, fmt, n, layer["c"], buf["h"], buf["w"],
                                       layer["packed"], layer["co"], layer["kh"], layer["kw"], 1, layer["pad"],
                                       buf["ws"], buf["acc"])
            accs.append(buf["acc"])
            if i + 1 == len(self.layers):
                break
            if self.fused:
                nxt = self.layers[i + 1]
                hk.hikonv_epilogue_pack(buf["acc"], n, layer["co"], buf["ho"], buf["wo"], shifts[i], qmax,
                                        layer["pool"], nxt["plan"], nxt["co"], nxt["kh"], nxt["kw"], 1, nxt["pad"],
                                        bufs[i + 1]["ws"])
                cur, fmt = None, hk.FMT_PACKED
            else:
                hk.hikonv_epilogue(buf["acc"], n, layer["co"], buf["ho"], buf["wo"], shifts[i], qmax, layer["pool"],
                                   self.act_bits, hk.FMT_BITDENSE, buf["nxt"])
                cur = buf["nxt"]
        return accs[-1], accs


class UnpackedCnn:
    """The same chain on the baseline kernels: every layer is the direct convolution with one
    v_mad_i32_i24 per low-bit product (hikonv_conv2d_unpacked), followed by the same epilogue
    writing one value per byte.  The counterpart of the paper's unpacked complete model."""

    def __init__(self, weights, specs, act_bits=4, w_bits=4, w_signed=True):
        self.layers = [dict(w=w_dev, co=w_dev.shape[0], c=w_dev.shape[1], kh=w_dev.shape[2], kw=w_dev.shape[3],
                            pad=spec["pad"], pool=spec["pool"]) for w_dev, spec in zip(weights, specs)]
        self.act_bits, self.w_bits = act_bits, w_bits
        self.sign = hk.signedness(False, w_signed)
        self.buffers = None

    def _allocate(self, n, h, w):
        bufs = []
        for layer in self.layers:
            ho = h + 2 * layer["pad"] - layer["kh"] + 1
            wo = w + 2 * layer["pad"] - layer["kw"] + 1
            acc = torch.empty(n * layer["co"] * ho * wo, dtype=torch.int32, device="cuda")
            h2, w2 = (ho // 2, wo // 2) if layer["pool"] else (ho, wo)
            nxt = torch.empty(n * layer["co"] * h2 * w2, dtype=torch.uint8, device="cuda")
            bufs.append(dict(acc=acc, nxt=nxt, h=h, w=w, ho=ho, wo=wo))
            h, w = h2, w2
        self.buffers = (n, bufs)

    def forward(self, x_bytes, n, h, w, shifts, qmax=15):
        """x_bytes: [n][c0][h][w], one value per byte.  Returns (last accumulators, all accumulators)."""
        if self.buffers is None or self.buffers[0] != n or self.buffers[1][0]["h"] != h or self.buffers[1][0]["w"] != w:
            self._allocate(n, h, w)
        cur, accs, bufs = x_bytes, [], self.buffers[1]
        for i, (layer, buf) in enumerate(zip(self.layers, bufs)):
            hk.hikonv_conv2d_unpacked(self.act_bits, self.w_bits, self.sign, cur, n, layer["c"], buf["h"], buf["w"],
                                      layer["w"], layer["co"], layer["kh"], layer["kw"], 1, layer["pad"], buf["acc"])
            accs.append(buf["acc"])
            if i + 1 == len(self.layers):
                break
            hk.hikonv_epilogue(buf["acc"], n, layer["co"], buf["ho"], buf["wo"], shifts[i], qmax, layer["pool"],
                               self.act_bits, hk.FMT_INT8, buf["nxt"])
            cur = buf["nxt"]
        return accs[-1], accs
