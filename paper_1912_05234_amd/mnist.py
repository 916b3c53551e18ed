"""Reader for the IDX files MNIST is distributed in (Section 4.2 trains on 60000 and classifies
10000 of its 28x28 images) and the pixel scaling used here.

The data set itself is not part of this repository.  An IDX file is a big-endian header -- two
zero bytes, a type code (0x08 = unsigned byte), the number of dimensions, then one 32-bit extent
per dimension -- followed by the items in row-major order; files may be gzip-compressed.
"""
import gzip
import struct

import numpy as np


def read_idx(path):
    """The unsigned-byte array stored in an IDX file (optionally .gz)."""
    opener = gzip.open if str(path).endswith(".gz") else open
    with opener(path, "rb") as f:
        data = f.read()
    if len(data) < 4:
        raise ValueError("%s: too short for an IDX header" % path)
    zero, dtype_code, ndim = struct.unpack(">HBB", data[:4])
    if zero != 0 or dtype_code != 0x08:
        raise ValueError("%s: not an unsigned-byte IDX file (header %r)" % (path, data[:4]))
    if ndim < 1 or len(data) < 4 + 4 * ndim:
        raise ValueError("%s: truncated IDX header" % path)
    shape = struct.unpack(">" + "I" * ndim, data[4:4 + 4 * ndim])
    count = int(np.prod(shape, dtype=np.int64))
    body = data[4 + 4 * ndim:]
    if len(body) != count:
        raise ValueError("%s: header promises %d items, file holds %d" % (path, count, len(body)))
    return np.frombuffer(body, dtype=np.uint8).reshape(shape)


def write_idx(path, array):
    """Writes an unsigned-byte array as IDX (used to make fixtures; gzip if the name ends in .gz)."""
    array = np.ascontiguousarray(array, dtype=np.uint8)
    header = struct.pack(">HBB", 0, 0x08, array.ndim) + struct.pack(">" + "I" * array.ndim, *array.shape)
    opener = gzip.open if str(path).endswith(".gz") else open
    with opener(path, "wb") as f:
        f.write(header + array.tobytes())


def load_images(path):
    """float32 [n,28,28] in [0,1]: bytes divided by 255."""
    a = read_idx(path)
    if a.ndim != 3 or a.shape[1:] != (28, 28):
        raise ValueError("%s: expected [n,28,28] images, found %r" % (path, a.shape))
    return a.astype(np.float32) / np.float32(255.0)


def load_labels(path):
    """int32 [n] in 0..9."""
    a = read_idx(path)
    if a.ndim != 1 or (a.size and a.max() > 9):
        raise ValueError("%s: expected a vector of labels 0..9" % path)
    return a.astype(np.int32)
