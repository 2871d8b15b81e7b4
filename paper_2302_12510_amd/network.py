"""Chained DyBit inference over a layer list (the ResNet-18 / ResNet-50 workloads).

Per convolution / linear layer, on one stream and without host synchronisation:
    absmax scale of the fp32 input -> quantize to DyBit codes -> dybit_conv2d against the
    pre-quantized weights with the folded batch-norm shift as bias (and ReLU) -> fp32 output.
This is the paper's dataflow with the write-back quantization done as a separate pass
(Sec. III-B: activations and weights are stored as DyBit codes, partial sums stay FP).  Where a
layer's output goes to the next encoder unchanged (or through a max-pool of non-negative values,
which keeps the maximum), its max|y| is taken in the convolution's epilogue
(dybit_conv2d_ex + dybit_scale_from_absmax) instead of by a pass over the fp32 tensor; the
identity shortcut of a residual block is added in the same epilogue, before the ReLU.
Pooling runs on the fp32 tensors with torch ops; it is glue, not part of the library.
A layer with op "dwconv" (depthwise convolution, the building block of the depthwise-separable
network of Sec. IV; filter [kh][kw][C]) runs through dybit_dwconv2d_wb in both chains: it reads the
codes its producer wrote and writes codes for its consumer like a dense convolution.

With `forward(x, static=True)` after a `calibrate(x)` the chain follows the paper's dataflow to
the letter: the scales of all activation tensors are fixed (those of the calibration input), every
convolution whose consumers agree on a format encodes its results in its own epilogue
(dybit_conv2d_wb) and the next layer reads those codes; the fp32 tensor is only written where a
shortcut, a pooling or the network output needs it, and no pass over an fp32 tensor remains except
behind the pooling layers.  The scales need not come from an offline calibration: with
`forward(x, static=True, track=True)` every epilogue also takes max|result| of the pass, and
`advance_scales()` turns those maxima into the scales of the next pass (previous-iteration scales).

`code_shortcuts=True` removes the remaining fp32 tensors of the static chain: the identity shortcut of a
residual block is read as the DyBit codes its tensor was stored as (dybit_conv2d_wb_rc adds
scale * value(code), the number a decoder in front of the adder would deliver), and a max-pool whose readers
all take codes of one format pools the codes themselves (dybit_maxpool2d_codes; the encoder is monotone, so
this equals encoding the pooled fp32 tensor bit for bit).  fp32 then remains only in front of the average
pool and at the output.

`per_channel=True` gives every output channel of every layer its own weight scale (row-wise max-abs,
dybit_quantize_rows; the convolutions then run through dybit_conv2d_pc; depthwise filters: one scale per
channel, dybit_quantize_cols); activations keep one scale per tensor.

Formats: weights are signed; an activation tensor is unsigned when it is the output of a
ReLU or of a pooling of such outputs, signed otherwise (the network input).  Layer-wise
bitwidths come from a table {layer name: (bits_W, bits_A)}, as the search of Sec. III-C
would produce.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _pad_channels(cin: int, bits_a: int, bits_w: int) -> int:
    """Smallest channel count >= cin whose packed pixel ends on a byte boundary for both formats."""
    c = cin
    while (c * bits_a) % 8 or (c * bits_w) % 8:
        c += 1
    return c


def _pad_few_channels(cin: int, kh: int, kw: int, bits_a: int, bits_w: int):
    """Layout of a convolution with few input channels (an image network's first layer) that lets the
    library fetch whole runs of neighbouring taps: channels padded to a divisor of 16 and the filter
    rows padded with zero taps until kw * channels is a multiple of 16; when a filter row is then
    exactly 32 codes, the filter also gets an even number of rows, which puts the layer on the tiled
    kernels.  Zero weights change no result; the caller uses this layout only for inputs where the
    larger filter leaves the output size unchanged.
    Returns (channels, kh, kw) or None when the layer does not qualify."""
    if cin >= 16:
        return None
    for c in (1, 2, 4, 8):
        if c >= cin and (c * bits_a) % 8 == 0 and (c * bits_w) % 8 == 0:
            k2 = kw
            while (k2 * c) % 16:
                k2 += 1
            return (c, kh + (kh % 2 if k2 * c == 32 else 0), k2)
    return None


class DybitNetwork:
    def __init__(self, layers, weights, bitwidths, device="cuda", epilogue_absmax=True, per_channel=False,
                 code_shortcuts=False):
        self.layers = layers
        self.code_shortcuts = code_shortcuts and not per_channel   # static chain: shortcuts and max-pools on codes
        self.per_channel = per_channel           # True: one weight scale per output channel (dybit_quantize_rows, dybit_conv2d_pc)
        self.epilogue_absmax = epilogue_absmax   # False: every scale from a pass over the fp32 tensor
        self.bitwidths = bitwidths
        self.device = device
        self.params = {}
        for l in layers:
            if l["op"] == "dwconv":                  # depthwise: filter [kh][kw][C]
                w, b = weights[l["name"]]
                bw, ba = bitwidths[l["name"]]
                wd = torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32)).to(device).reshape(-1)
                if per_channel:                      # one scale per channel: the columns of the [kh*kw][C] filter
                    sw, wq = B.dybit_quantize_cols(wd.reshape(-1, w.shape[2]), bw, True)
                else:
                    sw = B.dybit_absmax_scale(wd, bw, True)
                    wq = B.dybit_quantize(wd, sw, bw, True)
                self.params[l["name"]] = {"w_fmt": (bw, True), "w_scale": sw, "w_codes": wq,
                                          "bias": torch.from_numpy(b).to(device), "a_bits": ba, "k": w.shape[0], "kw": w.shape[1],
                                          "cin": w.shape[2], "cpad": w.shape[2], "cout": w.shape[2]}
                continue
            if l["op"] not in ("conv", "fc"):
                continue
            w, b = weights[l["name"]]
            bw, ba = bitwidths[l["name"]]
            cout, kh, kw, cin = w.shape
            w_fmt = (bw, True)

            def layout(cpad, khp, kwp):
                wp = np.zeros((cout, khp, kwp, cpad), dtype=np.float32)
                wp[:, :kh, :kw, :cin] = w
                wd = torch.from_numpy(wp).to(device).reshape(-1)
                if per_channel:
                    sw, wq = B.dybit_quantize_rows(wd.reshape(cout, -1), *w_fmt)
                else:
                    sw = B.dybit_absmax_scale(wd, *w_fmt)      # zero padding changes neither the scale nor a code
                    wq = B.dybit_quantize(wd, sw, *w_fmt)
                return {"w_fmt": w_fmt, "w_scale": sw, "w_codes": wq,
                        "bias": torch.from_numpy(b).to(device), "cin": cin, "cpad": cpad, "cout": cout,
                        "k": khp, "kw": kwp, "a_bits": ba}

            self.params[l["name"]] = layout(_pad_channels(cin, ba, bw), kh, kw)
            few = _pad_few_channels(cin, kh, kw, ba, bw) if l["op"] == "conv" else None
            if few is not None and few != (self.params[l["name"]]["cpad"], kh, kw):
                self.params[l["name"]]["few"] = layout(*few)   # used when the larger filter keeps the output size

        self._plan_write_back()
        self.static_scale = None                 # layer name -> device scale of its input, set by calibrate()

    def _plan_write_back(self):
        """Per conv layer: the format its consumers want its output in (if they agree and the packed
        rows are whole words), whether anyone needs the fp32 tensor, and (code_shortcuts) whether its
        shortcut is read as codes; per max-pool: whether it pools codes."""
        nonneg = {"input": False}
        produced_by = {}
        coded = ("conv", "fc", "dwconv")             # layers that read codes
        for l in self.layers:
            if l["op"] in coded:
                nonneg[l["name"]] = bool(l.get("relu"))
                produced_by[l["name"]] = l
            else:
                nonneg[l["name"]] = nonneg[l["src"]]
        self.a_fmt = {l["name"]: (self.params[l["name"]]["a_bits"], not nonneg[l["src"]])
                      for l in self.layers if l["op"] in coded}
        last = self.layers[-1]["name"]
        readers = lambda t: [u for u in self.layers if u["src"] == t]
        adders = lambda t: [u for u in self.layers if u.get("add") == t]
        pools = {l["name"]: l for l in self.layers if l["op"] == "maxpool"}

        def common_format(convs, channels):
            """The one format the coded readers of a tensor of `channels` channels agree on, or None."""
            fmts = {self.a_fmt[u["name"]] for u in convs}
            if len(fmts) != 1 or not all(self.params[u["name"]]["cpad"] == channels for u in convs):
                return None
            f = next(iter(fmts))
            return f if (channels * f[0]) % 32 == 0 else None

        # a max-pool may pool codes when all its readers take codes of one 2-, 4- or 8-bit format
        pool_fmt = {}
        for name, l in pools.items():
            src = produced_by.get(l["src"])
            rd = readers(name)
            f = common_format(rd, self.params[src["name"]]["cout"]) if src and rd and all(u["op"] in coded for u in rd) else None
            pool_fmt[name] = f if (self.code_shortcuts and f and f[0] in (2, 4, 8) and src["op"] == "conv") else None
        while True:
            fmt_of = {}
            for name, l in produced_by.items():
                rd = readers(name)
                convs = [u for u in rd if u["op"] in coded]
                through = [pool_fmt[u["name"]] for u in rd if u["op"] == "maxpool" and pool_fmt[u["name"]]]
                f = common_format(convs, self.params[name]["cout"]) if convs else (through[0] if through else None)
                if f and any(t != f for t in through):
                    f = None
                if f and not (l["op"] == "conv" or (l["op"] == "dwconv" and f[0] in (4, 8))):   # the depthwise epilogue packs 4- and 8-bit codes
                    f = None
                fmt_of[name] = f
            # a layer can read its shortcut as codes when it writes codes itself (the decoder sits in that epilogue)
            takes_codes = lambda u: self.code_shortcuts and fmt_of.get(u["name"]) is not None
            # a tensor that is only ever added as a shortcut (the projection of a downsampling block) has no reader
            # to dictate a format: 8-bit codes under a scale of its own
            own = set()
            for name, l in produced_by.items():
                if (self.code_shortcuts and l["op"] == "conv" and not readers(name) and adders(name) and name != last
                        and all(takes_codes(u) for u in adders(name)) and (self.params[name]["cout"] * 8) % 32 == 0):
                    own.add(name)
            for name in own:
                fmt_of[name] = (8, not produced_by[name].get("relu"))
            dropped = [n for n, f in pool_fmt.items()
                       if f and (fmt_of[pools[n]["src"]] != f or not all(takes_codes(u) for u in adders(n)))]
            if not dropped:
                break
            for n in dropped:
                pool_fmt[n] = None
        self.pool_fmt = pool_fmt
        self.plan = {}
        for name, l in produced_by.items():
            f = fmt_of[name]
            rd = readers(name)
            convs = [u for u in rd if u["op"] in coded] or [u for p in rd if p["op"] == "maxpool" for u in readers(p["name"])]
            others = [u for u in rd if u["op"] not in coded and not (u["op"] == "maxpool" and pool_fmt[u["name"]])]
            add_ok = f is not None and f[0] != 2 and all(takes_codes(u) for u in adders(name))
            need_fp32 = name == last or f is None or bool(others) or (bool(adders(name)) and not add_ok)
            shortcut = l.get("add")
            src_fmt = (fmt_of.get(shortcut) if shortcut in produced_by else pool_fmt.get(shortcut)) if shortcut else None
            self.plan[name] = {"fmt": f, "scale_of": ("out:" + name if name in own else convs[0]["name"]) if f else None,
                               "fp32": need_fp32,
                               "shortcut_codes": bool(shortcut) and takes_codes(l) and src_fmt is not None and src_fmt[0] != 2}

    def _layer_params(self, l, height: int, width: int):
        """Parameters of a conv layer for an input of the given size: the few-channel layout (filter
        padded with zero taps) if the layer has one and it yields the same output size."""
        p = self.params[l["name"]]
        few = p.get("few")
        if few is not None:
            same = all((n + 2 * l["pad"] - few[k]) // l["stride"] == (n + 2 * l["pad"] - p[k]) // l["stride"]
                       for n, k in ((height, "k"), (width, "kw")))
            if same:
                return few
        return p

    def calibrate(self, x: torch.Tensor) -> None:
        """Fixes the scale of every activation tensor to the one a dynamic forward pass over x uses."""
        scales = {}

        def keep(name, rec):
            scales[name] = rec["a_scale"].clone()
            plan = self.plan[name]
            if plan["scale_of"] == "out:" + name:           # encoded under a scale of its own: that of this pass's values
                scales[plan["scale_of"]] = B.dybit_absmax_scale(rec["y"].reshape(-1), *plan["fmt"])

        self.forward(x, record=keep)
        self.static_scale = scales

    def forward(self, x: torch.Tensor, record=None, static: bool = False, track: bool = False) -> torch.Tensor:
        """x: NHWC float32 on the device.  `record(name, dict)` receives, per conv/fc layer, the
        tensors needed to check that layer in isolation (input, scale, codes, raw output).
        static=True: the scales of the activation tensors are given (calibrate(), or the previous pass:
        see advance_scales()) and the write-back is fused (see the module text).
        track=True (static chain): every layer also folds max|result| of this pass into a word of its
        own, from which advance_scales() derives the scales of the next pass."""
        if static:
            return self._forward_static(x, record, track)
        acts = {"input": x}
        nonneg = {"input": False}
        known_max = {}                       # tensor name -> device scalar holding max|tensor|
        encoded = {}                         # (tensor name, format, padded channels) -> (scale, codes)
        n_fused = sum(1 for l in self.layers if l["op"] in ("conv", "fc", "dwconv"))
        max_words = torch.zeros(max(n_fused, 1), dtype=torch.float32, device=x.device)
        next_word = 0
        out = x
        for l in self.layers:
            name, op = l["name"], l["op"]
            src = acts[l["src"]]
            if op == "maxpool":
                y = torch.nn.functional.max_pool2d(src.permute(0, 3, 1, 2), l["k"], l["stride"], l["pad"])
                out = y.permute(0, 2, 3, 1).contiguous()
                nonneg[name] = nonneg[l["src"]]
                if nonneg[name] and l["src"] in known_max and l["k"] >= l["stride"]:
                    known_max[name] = known_max[l["src"]]     # every element is in some window
            elif op == "avgpool":
                out = src.mean(dim=(1, 2), keepdim=True)
                nonneg[name] = nonneg[l["src"]]
            elif op == "dwconv":
                Bn, H, W, C = src.shape
                p = self.params[name]
                a_fmt = (p["a_bits"], not nonneg[l["src"]])
                flat = src.reshape(-1)
                key = (l["src"], a_fmt, C)
                if key in encoded:
                    sa, qa = encoded[key]
                elif l["src"] in known_max:
                    sa, qa = encoded[key] = B.dybit_quantize_absmax(flat, known_max[l["src"]], *a_fmt)
                else:
                    sa = B.dybit_absmax_scale(flat, *a_fmt)
                    qa = B.dybit_quantize(flat, sa, *a_fmt)
                    encoded[key] = (sa, qa)
                relu = bool(l.get("relu"))
                word = None
                if self.epilogue_absmax:
                    word = max_words[next_word:next_word + 1]
                    next_word += 1
                    known_max[name] = word
                out, _ = B.dybit_dwconv2d_wb(Bn, H, W, C, p["k"], p["kw"], l["stride"], l["pad"], qa, a_fmt, sa,
                                             p["w_codes"], p["w_fmt"], p["w_scale"], p["bias"], relu, word,
                                             per_channel=self.per_channel)
                if record is not None:
                    record(name, {"x": src, "a_fmt": a_fmt, "a_scale": sa, "a_codes": qa, "y": out, "shortcut": None,
                                  "relu": relu, "stride": l["stride"], "pad": l["pad"], **p})
                nonneg[name] = relu
            else:
                Bn, H, W, C = src.shape
                p = self._layer_params(l, H, W) if op == "conv" else self.params[name]
                a_fmt = (p["a_bits"], not nonneg[l["src"]])
                key = (l["src"], a_fmt, p["cpad"])                  # two consumers of one tensor in one format share its codes
                pad_kernel = p["cpad"] != C and p["cpad"] % 4 == 0 and key not in encoded
                if pad_kernel:
                    # channels padded with zero codes by the encoder itself (zero padding keeps the maximum)
                    if l["src"] in known_max:
                        sa = B.dybit_scale_from_absmax(known_max[l["src"]], *a_fmt)
                    else:
                        sa = B.dybit_absmax_scale(src.reshape(-1), *a_fmt)
                    qa = B.dybit_quantize_pad(src.reshape(-1, C), p["cpad"], sa, *a_fmt)
                    encoded[key] = (sa, qa)
                    if record is not None:
                        src = torch.nn.functional.pad(src, (0, p["cpad"] - C))
                elif p["cpad"] != C:
                    src = torch.nn.functional.pad(src, (0, p["cpad"] - C))
                flat = src.reshape(-1)
                if key in encoded:
                    sa, qa = encoded[key]
                elif l["src"] in known_max:                     # zero padding of channels keeps the maximum
                    sa, qa = encoded[key] = B.dybit_quantize_absmax(flat, known_max[l["src"]], *a_fmt)
                else:
                    sa = B.dybit_absmax_scale(flat, *a_fmt)
                    qa = B.dybit_quantize(flat, sa, *a_fmt)
                    encoded[key] = (sa, qa)
                relu = bool(l.get("relu"))
                k = p["k"]
                stride, pad = (l["stride"], l["pad"]) if op == "conv" else (1, 0)
                conv_args = (Bn, H, W, p["cpad"], p["cout"], k, p["kw"], stride, pad,
                             qa, a_fmt, sa, p["w_codes"], p["w_fmt"], p["w_scale"])
                shortcut = acts[l["add"]] if l.get("add") else None
                word = None
                if self.epilogue_absmax:
                    word = max_words[next_word:next_word + 1]
                    next_word += 1
                    known_max[name] = word
                if self.per_channel:
                    y, _ = B.dybit_conv2d_pc(*conv_args, p["bias"], shortcut, relu, word)
                else:
                    y = B.dybit_conv2d_ex(*conv_args, p["bias"], shortcut, relu, word)
                if record is not None:
                    record(name, {"x": src, "a_fmt": a_fmt, "a_scale": sa, "a_codes": qa, "y": y, "shortcut": shortcut,
                                  "relu": relu, "stride": stride, "pad": pad, "k": k, **p})
                out = y
                nonneg[name] = bool(l.get("relu"))
            acts[name] = out
        return out.reshape(out.shape[0], -1)

    def capture(self, x: torch.Tensor, static: bool = False):
        """Records one forward pass over the (fixed) input buffer x into a HIP graph.  Returns
        (graph, logits): `graph.replay()` reruns every launch of the pass without host work per launch
        and rewrites `logits` in place; new inputs are copied into x before a replay.  The pass contains
        kernels only (the library clears its words with small kernels, never with memset nodes)."""
        side = torch.cuda.Stream()                       # default priority
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                    # warm-up outside the capture: allocator, lazy initialisation
            for _ in range(2):
                self.forward(x, static=static)
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            logits = self.forward(x, static=static)
        return graph, logits

    def advance_scales(self) -> None:
        """Previous-iteration scales (Sec. III-B writes results back as codes, and with tensor-level scales
        the encoder needs max|result| before the results exist): after a forward(static=True, track=True)
        the scale of every activation tensor that a tracked layer produced becomes the max-abs scale of
        the values that pass produced.  The next pass encodes under those scales (a tensor that grew beyond
        its previous maximum saturates at the all-ones code).  Device work only: one small kernel per tensor."""
        if getattr(self, "_tracked", None) is None:
            raise RuntimeError("run forward(static=True, track=True) first")
        origin = {}                                     # tensor name -> producing layer whose maximum it carries
        nonneg = {"input": False}
        for l in self.layers:
            name, op = l["name"], l["op"]
            if op in ("conv", "fc", "dwconv"):
                origin[name] = name
                nonneg[name] = bool(l.get("relu"))
            else:
                nonneg[name] = nonneg[l["src"]]
                if op == "maxpool" and nonneg[name] and l["k"] >= l["stride"] and l["src"] in origin:
                    origin[name] = origin[l["src"]]     # every element is in some window: the maximum survives
        for l in self.layers:
            if l["op"] in ("conv", "fc", "dwconv") and l["src"] in origin:
                B.dybit_scale_from_absmax(self._tracked[origin[l["src"]]], *self.a_fmt[l["name"]], out=self.static_scale[l["name"]])
            own = self.plan.get(l["name"], {}).get("scale_of")
            if own == "out:" + l["name"]:
                B.dybit_scale_from_absmax(self._tracked[l["name"]], *self.plan[l["name"]]["fmt"], out=self.static_scale[own])

    def _forward_static(self, x: torch.Tensor, record=None, track: bool = False) -> torch.Tensor:
        if self.static_scale is None:
            raise RuntimeError("calibrate() first: the static chain needs a scale per activation tensor")
        words = None
        if track:
            names = [l["name"] for l in self.layers if l["op"] in ("conv", "fc", "dwconv")]
            buf = torch.zeros(len(names), dtype=torch.float32, device=x.device)
            words = {n: buf[i:i + 1] for i, n in enumerate(names)}
        self._tracked = words
        acts = {"input": x}                  # fp32 tensors (None where only codes were written)
        codes = {}                           # tensor name -> (format, scale, packed codes)
        shapes = {"input": tuple(x.shape)}
        out = x
        for l in self.layers:
            name, op = l["name"], l["op"]
            src = acts[l["src"]]
            if op == "dwconv":
                a_fmt = self.a_fmt[name]
                sa = self.static_scale[name]
                Bn, H, W, C = shapes[l["src"]]
                p = self.params[name]
                if l["src"] in codes and codes[l["src"]][0] == a_fmt:
                    qa = codes[l["src"]][2]                         # written by the producer's epilogue
                else:
                    qa = B.dybit_quantize(src.reshape(-1), sa, *a_fmt)
                relu = bool(l.get("relu"))
                plan = self.plan[name]
                y_scale = None if plan["fmt"] is None else self.static_scale[plan["scale_of"]]
                y, y_codes = B.dybit_dwconv2d_wb(Bn, H, W, C, p["k"], p["kw"], l["stride"], l["pad"], qa, a_fmt, sa,
                                                 p["w_codes"], p["w_fmt"], p["w_scale"], p["bias"], relu,
                                                 None if words is None else words[name],
                                                 plan["fmt"], y_scale, per_channel=self.per_channel,
                                                 fp32=plan["fp32"] or plan["fmt"] is None)
                if y_codes is not None:
                    codes[name] = (plan["fmt"], y_scale, y_codes)
                if record is not None:
                    record(name, {"a_fmt": a_fmt, "a_scale": sa, "a_codes": qa, "in_shape": (Bn, H, W, C), "y": y,
                                  "y_codes": y_codes, "y_fmt": plan["fmt"], "y_scale": y_scale, "shortcut": None,
                                  "relu": relu, "stride": l["stride"], "pad": l["pad"], **p})
                out = y
                shapes[name] = (Bn, (H + 2 * l["pad"] - p["k"]) // l["stride"] + 1,
                                (W + 2 * l["pad"] - p["kw"]) // l["stride"] + 1, C)
                acts[name] = out
                continue
            if op == "maxpool" and self.pool_fmt[name]:
                f, s_in, q_in = codes[l["src"]]                 # the codes the producer wrote, pooled as codes
                Bn, H, W, C = shapes[l["src"]]
                q = B.dybit_maxpool2d_codes(Bn, H, W, C, l["k"], l["stride"], l["pad"], q_in, f)
                codes[name] = (f, s_in, q)
                shapes[name] = (Bn, q.shape[1], q.shape[2], C)
                acts[name] = None
                if record is not None:
                    record(name, {"op": "maxpool", "fmt": f, "x_codes": q_in, "y_codes": q, "in_shape": (Bn, H, W, C),
                                  "k": l["k"], "stride": l["stride"], "pad": l["pad"]})
                continue
            if op == "maxpool":
                y = torch.nn.functional.max_pool2d(src.permute(0, 3, 1, 2), l["k"], l["stride"], l["pad"])
                out = y.permute(0, 2, 3, 1).contiguous()
            elif op == "avgpool":
                out = src.mean(dim=(1, 2), keepdim=True)
            else:
                a_fmt = self.a_fmt[name]
                sa = self.static_scale[name]
                Bn, H, W, C = shapes[l["src"]]
                p = self._layer_params(l, H, W) if op == "conv" else self.params[name]
                if l["src"] in codes and codes[l["src"]][0] == a_fmt:
                    qa = codes[l["src"]][2]                         # written by the producer's epilogue
                elif p["cpad"] != C and p["cpad"] % 4 == 0:
                    qa = B.dybit_quantize_pad(src.reshape(-1, C), p["cpad"], sa, *a_fmt)
                else:
                    if p["cpad"] != C:
                        src = torch.nn.functional.pad(src, (0, p["cpad"] - C))
                    qa = B.dybit_quantize(src.reshape(-1), sa, *a_fmt)
                relu = bool(l.get("relu"))
                k = p["k"]
                stride, pad = (l["stride"], l["pad"]) if op == "conv" else (1, 0)
                conv_args = (Bn, H, W, p["cpad"], p["cout"], k, p["kw"], stride, pad,
                             qa, a_fmt, sa, p["w_codes"], p["w_fmt"], p["w_scale"])
                shortcut = acts[l["add"]] if l.get("add") else None
                plan = self.plan[name]
                y_codes = None
                word = None if words is None else words[name]
                if plan["shortcut_codes"]:
                    r_fmt, r_scale, r_codes = codes[l["add"]]
                    y_scale = self.static_scale[plan["scale_of"]]
                    y, y_codes = B.dybit_conv2d_wb_rc(*conv_args, plan["fmt"], y_scale, r_codes, r_fmt, r_scale, p["bias"], relu,
                                                      word, fp32=plan["fp32"])
                    codes[name] = (plan["fmt"], y_scale, y_codes)
                    if record is not None:                      # what the epilogue added: the decoded codes
                        shortcut = B.dybit_dequantize(r_codes.reshape(-1), r_codes.numel() * 8 // r_fmt[0], r_scale, *r_fmt)
                        shortcut = shortcut.reshape(y_codes.shape[0], y_codes.shape[1], y_codes.shape[2], p["cout"])
                elif plan["fmt"] is not None:
                    y_scale = self.static_scale[plan["scale_of"]]
                    if self.per_channel:
                        y, y_codes = B.dybit_conv2d_pc(*conv_args, p["bias"], shortcut, relu, word, plan["fmt"], y_scale,
                                                       fp32=plan["fp32"])
                    else:
                        y, y_codes = B.dybit_conv2d_wb(*conv_args, plan["fmt"], y_scale, p["bias"], shortcut, relu, word,
                                                       fp32=plan["fp32"])
                    codes[name] = (plan["fmt"], y_scale, y_codes)
                elif self.per_channel:
                    y, _ = B.dybit_conv2d_pc(*conv_args, p["bias"], shortcut, relu, word)
                else:
                    y = B.dybit_conv2d_ex(*conv_args, p["bias"], shortcut, relu, word)
                if record is not None:
                    record(name, {"a_fmt": a_fmt, "a_scale": sa, "a_codes": qa, "in_shape": (Bn, H, W, p["cpad"]),
                                  "y": y, "y_codes": y_codes, "y_fmt": plan["fmt"],
                                  "y_scale": None if y_codes is None else y_scale, "shortcut": shortcut,
                                  "relu": relu, "stride": stride, "pad": pad, "k": k, **p})
                out = y
                Ho = (H + 2 * pad - k) // stride + 1
                Wo = (W + 2 * pad - p["kw"]) // stride + 1
                shapes[name] = (Bn, Ho, Wo, p["cout"])
            if op in ("maxpool", "avgpool"):
                shapes[name] = tuple(out.shape)
            acts[name] = out
        return out.reshape(out.shape[0], -1)

    def layer_work(self, batch: int, hw: int):
        """Per conv/fc layer, for an input of batch x hw x hw: the GEMM shape (K on the real channel
        count), the number of input activations, the operand widths and whether a shortcut is added --
        what a per-layer roofline needs."""
        sizes = {"input": hw}
        out = []
        for l in self.layers:
            s = sizes[l["src"]]
            if l["op"] == "maxpool":
                sizes[l["name"]] = (s + 2 * l["pad"] - l["k"]) // l["stride"] + 1
            elif l["op"] == "avgpool":
                sizes[l["name"]] = 1
            else:
                bw, ba = self.bitwidths[l["name"]]
                if l["op"] == "fc":
                    sizes[l["name"]] = 1
                    m, n, k, n_in = batch, l["cout"], l["cin"], batch * l["cin"]
                else:
                    o = (s + 2 * l["pad"] - l["k"]) // l["stride"] + 1
                    sizes[l["name"]] = o
                    m, n, k = batch * o * o, l["cout"], l["k"] * l["k"] * l["cin"]
                    n_in = batch * s * s * l["cin"]
                out.append({"name": l["name"], "M": m, "N": n, "K": k, "inputs": n_in, "bits_w": bw, "bits_a": ba,
                            "shortcut": bool(l.get("add"))})
        return out

    def gemm_shapes(self, batch: int, hw: int):
        """(name, M, N, K) of every conv/fc layer for an input of batch x hw x hw (K counted on
        the real channel count, not the padded one)."""
        sizes = {"input": hw}
        shapes = []
        for l in self.layers:
            s = sizes[l["src"]]
            if l["op"] == "maxpool":
                sizes[l["name"]] = (s + 2 * l["pad"] - l["k"]) // l["stride"] + 1
            elif l["op"] == "avgpool":
                sizes[l["name"]] = 1
            elif l["op"] == "fc":
                sizes[l["name"]] = 1
                shapes.append((l["name"], batch, l["cout"], l["cin"]))
            else:
                o = (s + 2 * l["pad"] - l["k"]) // l["stride"] + 1
                sizes[l["name"]] = o
                shapes.append((l["name"], batch * o * o, l["cout"], l["k"] * l["k"] * l["cin"]))
        return shapes
