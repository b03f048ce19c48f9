"""A container for models whose binary layers are stored with 1-bit weights.

The paper's model converter (Sec. 2.2.3) reads a trained model and packs the weights of its
QConvolution and QFullyConnected layers 32 to 1 (ResNet-18: 44.7 MB -> 1.5 MB).  This module
is that step for this library: `convert` packs every binary layer's weights with the HIP pack
kernel and computes its alpha; `save` / `load` move the result to and from one file;
`to_device` turns a loaded layer into the operands the layer calls take (a convolution's
private row layout is rebuilt on the GPU from the stored bits).

File layout (little endian): 8 bytes magic "BMXW0001", uint64 length of a UTF-8 JSON header,
the header, then the arrays, each starting at a multiple of 64 bytes from the start of the
file.  The header is {"layers": [{"name", "kind": "fc" | "conv", "shape": fp32 weight shape,
"bits": [offset, rows, words], "alpha": [offset, rows]}, ...]}: "bits" are uint64 words, row r
= output feature / filter r, element k of the row (for a convolution k runs over (c, kh, kw),
the OIHW order flattened) in bit k % 64 of word k / 64, 1 = weight >= 0; "alpha" is fp32.
Nothing here computes: packing, alpha and unpacking are library calls.
"""
import json
import struct

import numpy as np

MAGIC = b"BMXW0001"
ALIGN = 64


def convert(weights, device="cuda"):
    """weights: {name: fp32 numpy array, 2-D [out, in] or 4-D [O, C, KH, KW]} -> list of layer
    records holding host copies of the packed bits and alpha (computed on `device`)."""
    import torch
    from . import binding as B
    layers = []
    for name, w in weights.items():
        w = np.ascontiguousarray(w, dtype=np.float32)
        if w.ndim not in (2, 4):
            raise ValueError("%s: binary layers have 2-D or 4-D weights" % name)
        t = torch.from_numpy(w).to(device)
        flat = t.reshape(w.shape[0], -1)
        bits = B.binarize_pack(flat, 1).cpu().numpy().view(np.uint64)
        alpha = B.alpha_mean_abs(flat).cpu().numpy()
        layers.append({"name": name, "kind": "fc" if w.ndim == 2 else "conv", "shape": list(w.shape),
                       "bits": bits, "alpha": alpha})
    return layers


def save(path, layers):
    """Write layer records (as from `convert`) to `path`; returns the number of bytes written."""
    table, blobs = [], []
    pos = 0  # relative to the start of the array section

    def place(a):
        nonlocal pos
        pos = (pos + ALIGN - 1) // ALIGN * ALIGN
        off = pos
        blobs.append((off, a.tobytes()))
        pos += a.nbytes
        return off

    for L in layers:
        bits = np.ascontiguousarray(L["bits"], dtype="<u8")
        alpha = np.ascontiguousarray(L["alpha"], dtype="<f4")
        rows = int(L["shape"][0])
        k = int(np.prod(L["shape"][1:]))
        if bits.shape != (rows, (k + 63) // 64) or alpha.shape != (rows,):
            raise ValueError("%s: packed arrays do not fit shape %s" % (L["name"], L["shape"]))
        table.append({"name": L["name"], "kind": L["kind"], "shape": [int(v) for v in L["shape"]],
                      "bits": [place(bits), rows, int(bits.shape[1])], "alpha": [place(alpha), rows]})
    header = json.dumps({"layers": table}).encode()
    start = (len(MAGIC) + 8 + len(header) + ALIGN - 1) // ALIGN * ALIGN
    with open(path, "wb") as f:
        f.write(MAGIC)
        f.write(struct.pack("<Q", len(header)))
        f.write(header)
        f.write(b"\0" * (start - f.tell()))
        for off, data in blobs:
            f.write(b"\0" * (start + off - f.tell()))
            f.write(data)
        return f.tell()


def load(path):
    """Read a file written by `save`: list of layer records with numpy arrays (copies)."""
    with open(path, "rb") as f:
        data = f.read()
    if data[:8] != MAGIC:
        raise ValueError("%s: not a packed-weights file" % path)
    (hlen,) = struct.unpack_from("<Q", data, 8)
    if 16 + hlen > len(data):
        raise ValueError("%s: truncated header" % path)
    table = json.loads(data[16:16 + hlen].decode())["layers"]
    start = (16 + hlen + ALIGN - 1) // ALIGN * ALIGN
    out = []
    for T in table:
        boff, rows, words = T["bits"]
        aoff, arows = T["alpha"]
        if start + boff + rows * words * 8 > len(data) or start + aoff + arows * 4 > len(data):
            raise ValueError("%s: layer %s lies outside the file" % (path, T["name"]))
        bits = np.frombuffer(data, dtype="<u8", count=rows * words, offset=start + boff).reshape(rows, words)
        alpha = np.frombuffer(data, dtype="<f4", count=arows, offset=start + aoff)
        out.append({"name": T["name"], "kind": T["kind"], "shape": T["shape"], "bits": bits.copy(),
                    "alpha": alpha.copy()})
    return out


def to_device(layer, device="cuda"):
    """A loaded layer as the operands of the layer calls: (Wp, alpha) device tensors; Wp is the
    packed matrix of `binary_fc*` for an fc layer and the row layout of `binary_conv2d*` for a
    convolution (rebuilt on the GPU: bits -> +-1 floats -> bmx_pack_conv_weights)."""
    import torch
    from . import binding as B
    bits = torch.from_numpy(layer["bits"].view(np.int64)).to(device)
    alpha = torch.from_numpy(layer["alpha"]).to(device)
    if layer["kind"] == "fc":
        return bits, alpha
    O, C, KH, KW = layer["shape"]
    w = B.unpack_pm1(bits, C * KH * KW).reshape(O, C, KH, KW)
    return B.pack_conv_weights(w), alpha
