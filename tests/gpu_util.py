"""Helpers for the GPU parity tests: device buffers through torch, calls through the C ABI."""
import numpy as np
import torch

import paper_2208_00763_amd as hk
from oracle import direct


def dev(a: np.ndarray) -> torch.Tensor:
    """numpy (int8/uint8/int32) -> contiguous CUDA tensor of the same bytes."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.int8:
        return torch.from_numpy(a.view(np.uint8)).cuda()
    return torch.from_numpy(a).cuda()


GUARD_BYTES = 256         # untouched-guard region on each side of a buffer the library writes
GUARD_I32 = -77777


class Guarded:
    """An output buffer of `count` elements with untouched-guard regions before and after it.

    `view` is what the library gets (it starts 256 bytes + `offset` elements into the
    allocation, so its alignment is 256 bytes plus `offset` elements); `result()` checks
    that neither guard region was written and returns the payload as numpy."""

    def __init__(self, count, dtype=torch.int32, fill=GUARD_I32, offset=0):
        guard = GUARD_BYTES // torch.empty(0, dtype=dtype).element_size()
        self.count, self.fill, self.front = int(count), fill, guard + offset
        self.buf = torch.full((self.front + self.count + guard,), fill, dtype=dtype, device="cuda")
        self.view = self.buf[self.front:self.front + self.count]

    def check(self):
        assert bool((self.buf[:self.front] == self.fill).all()), "wrote before the start of the output"
        assert bool((self.buf[self.front + self.count:] == self.fill).all()), "wrote past the end of the output"

    def result(self):
        torch.cuda.synchronize()
        self.check()
        return self.view.cpu().numpy()


# kernel form that conv1d_plan puts into its plans (a fixture of the 1-D tests switches it, so that
# every case runs on the lane-exchange kernel and on the library's own choice)
CONV1D_DEFAULTS = {"kernel": 0}


def conv1d_plan(bits, a_signed, w_signed, taps, tight=0, bits_w=None):
    return hk.hikonv_plan_ex(bits_a=bits, bits_w=bits_w or bits, a_signed=int(a_signed), w_signed=int(w_signed),
                             L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, taps=taps, tight=tight,
                             kernel=CONV1D_DEFAULTS["kernel"])


def compact(x_np: np.ndarray, bits: int, bipolar=False) -> torch.Tensor:
    """[rows][len] bytes -> bit-dense rows on the device, through hikonv_compact."""
    rows, length = x_np.shape
    row_bytes = hk.hikonv_bitdense_row_bytes(length, bits)
    out = Guarded(rows * row_bytes, torch.uint8, 0xA5)       # sized exactly: nothing behind the last row
    hk.hikonv_compact(dev(x_np), rows, length, bits, bipolar, out.view)
    torch.cuda.synchronize()
    out.check()
    return out.view


def run_conv1d(x_np, g_np, bits, a_signed, w_signed, mode, fmt, packed=True, plan=None, y_offset=0):
    """y_offset: int32 elements by which the output pointer is moved off its 256-byte alignment
    (a multiple of 4: the entry points ask for 16-byte alignment)."""
    rows, length = x_np.shape
    taps = g_np.shape[0]
    out_len = length + taps - 1 if mode == hk.OUT_FULL else max(length - taps + 1, 0)
    out = Guarded(rows * out_len, offset=y_offset)
    y = out.view
    x_d = compact(x_np, bits) if fmt == hk.FMT_BITDENSE else dev(x_np)
    g_d = dev(g_np)
    if packed:
        plan = plan or conv1d_plan(bits, a_signed, w_signed, taps)
        hk.hikonv_conv1d(plan, x_d, fmt, rows, length, g_d, taps, mode, y)
    else:
        hk.hikonv_conv1d_unpacked(bits, bits, hk.signedness(a_signed, w_signed), x_d, fmt, rows, length, g_d, taps,
                                  mode, y)
    return out.result().reshape(rows, out_len)


def oracle_conv1d(x_np, g_np, mode):
    return direct.conv1d(x_np, g_np, direct.FULL if mode == hk.OUT_FULL else direct.VALID)


# layer kernel form and flags that dnn_plan puts into its plans (test fixtures switch them to
# reach both kernels and the 64-bit-address stores on small shapes)
LAYER_DEFAULTS = {"kernel": 0, "flags": 0}


def dnn_plan(bits_a, bits_w, a_signed, w_signed, taps, m, wide=True, bipolar=False, tight=0, max_n=None,
             objective=hk.OBJ_PAPER_OPS):
    """A layer plan the layer kernels can run (N <= LAYER_MAX_N unless max_n says otherwise)."""
    width = 32 if wide else 24
    return hk.hikonv_plan_ex(bits_a=bits_a, bits_w=bits_w, a_signed=int(a_signed), w_signed=int(w_signed),
                             bipolar=int(bipolar), L_A=width, L_B=width, L_acc=64 if wide else 32,
                             mode=hk.MODE_DNN, M=m, taps=taps, tight=tight, objective=objective,
                             max_N=hk.LAYER_MAX_N if max_n is None else max_n,
                             kernel=LAYER_DEFAULTS["kernel"], flags=LAYER_DEFAULTS["flags"])


def run_conv2d(plan, x_np, w_np, stride, pad, fmt=hk.FMT_INT8, prepacked=False):
    n, c, h, w = x_np.shape
    co, _, kh, kw = w_np.shape
    ho, wo = (h + 2 * pad - kh) // stride + 1, (w + 2 * pad - kw) // stride + 1
    out = Guarded(n * co * ho * wo)
    y = out.view
    if fmt == hk.FMT_BITDENSE:
        x_d = compact(x_np.reshape(n * c * h, w), plan.bits_a, bool(plan.bipolar))
    else:
        x_d = dev(x_np)
    w_d = dev(w_np)
    ws_bytes = hk.hikonv_conv2d_workspace_bytes(plan, n, c, h, w, co, kh, kw, stride, pad, prepacked)
    assert ws_bytes > 0
    wsg = Guarded(ws_bytes, torch.uint8, 0x5A)
    ws = wsg.view
    if prepacked:
        pwg = Guarded(hk.hikonv_packed_weights_bytes_ex(plan, co, c, 1, kh, kw, stride), torch.uint8, 0x5A)
        pw = pwg.view
        hk.hikonv_pack_weights_ex(plan, w_d, co, c, 1, kh, kw, stride, pw)
        hk.hikonv_conv2d_prepacked(plan, x_d, fmt, n, c, h, w, pw, co, kh, kw, stride, pad, ws, y)
        torch.cuda.synchronize()
        pwg.check()
    else:
        hk.hikonv_conv2d(plan, x_d, fmt, n, c, h, w, w_d, co, kh, kw, stride, pad, ws, y)
    res = out.result()
    wsg.check()
    return res.reshape(n, co, ho, wo)


def run_conv3d(plan, x_np, w_np, stride, pad, fmt=hk.FMT_INT8, prepacked=False):
    n, c, d, h, w = x_np.shape
    co, _, kd, kh, kw = w_np.shape
    do, ho, wo = ((d + 2 * pad - kd) // stride + 1, (h + 2 * pad - kh) // stride + 1,
                  (w + 2 * pad - kw) // stride + 1)
    count = n * co * do * ho * wo
    out = Guarded(count)
    y = out.view
    x_d = compact(x_np.reshape(n * c * d * h, w), plan.bits_a, bool(plan.bipolar)) if fmt == hk.FMT_BITDENSE else dev(x_np)
    w_d = dev(w_np)
    ws_bytes = hk.hikonv_conv3d_workspace_bytes(plan, n, c, d, h, w, co, kd, kh, kw, stride, pad, prepacked)
    assert ws_bytes > 0
    wsg = Guarded(ws_bytes, torch.uint8, 0x5A)
    ws = wsg.view
    if prepacked:
        pwg = Guarded(hk.hikonv_packed_weights_bytes_ex(plan, co, c, kd, kh, kw, stride), torch.uint8, 0x5A)
        pw = pwg.view
        hk.hikonv_pack_weights_ex(plan, w_d, co, c, kd, kh, kw, stride, pw)
        hk.hikonv_conv3d(plan, x_d, fmt, n, c, d, h, w, pw, True, co, kd, kh, kw, stride, pad, ws, y)
        torch.cuda.synchronize()
        pwg.check()
    else:
        hk.hikonv_conv3d(plan, x_d, fmt, n, c, d, h, w, w_d, False, co, kd, kh, kw, stride, pad, ws, y)
    res = out.result()
    wsg.check()
    return res.reshape(n, co, do, ho, wo)


def oracle_cnn(x, weights, specs, shifts=None):
    """Layer-by-layer oracle forward; the per-layer requantisation shift is chosen here so that
    the 99th percentile of the positive accumulators maps to at most 15 (or taken from `shifts`)."""
    given = shifts
    accs, shifts = [], []
    cur = x
    for i, (w, spec) in enumerate(zip(weights, specs)):
        acc = direct.conv2d(cur, w, 1, spec["pad"])
        accs.append(acc)
        if i + 1 == len(weights):
            break
        pos = acc[acc > 0]
        p99 = int(np.percentile(pos, 99)) if pos.size else 0
        shift = 0
        while (p99 >> shift) > 15:
            shift += 1
        if given is not None:
            shift = given[i]
        shifts.append(shift)
        q = direct.relu_requant(acc, shift, 15)
        if spec["pool"]:
            q = direct.maxpool2x2(q)
        cur = q.view(np.uint8)
    return accs, shifts
