"""Library of stored chunk caches and its disk format (oracle side, TEST INFRASTRUCTURE).

Sec. 3.1 items 2-3 and the serving workflow of Sec. 3.1: the KV cache of an uploaded
file is computed once, kept for serving, copied to disk, and deleted when its time is
up.  Sec. 3.2: at the start of a request every referenced cache is looked up; it is in
GPU memory, in CPU memory, on disk, or missing (expired / never stored).  The paper
names these places and the expiry, nothing more, so the model below is the plain
statement of that: a mapping id -> (K, V of every layer, place, expiry time).  A
cache holds bytes; a store returns exactly the bytes it was given or reports the
cache missing.

The file layout is this build's own (the paper gives none).  All fields little endian:
    0   8 bytes  "MPICKV01"
    8   u64      id
   16   i32      len (tokens)        20  i32  n_layers
   24   i32      n_kv_heads          28  i32  head_dim
   32   i32      dtype (0 fp32, 1 bf16)   36  i32  0
   40   u64      block_bytes = len * n_kv_heads * head_dim * element size
   48   u64      payload_off (a multiple of 4096)
   56   u64      checksum of bytes [0, 56)
   64   u64 x 2 x n_layers   checksum of the K block and of the V block of every layer
   payload_off:  K block of layer 0, V block of layer 0, K block of layer 1, ...
checksum of n 8-byte words w_0 .. w_{n-1}:  (n + sum_i w_i * P^(i+1)) mod 2^64 with
P = 0x9E3779B97F4A7C15.  P is odd, so every power is invertible mod 2^64 and a change
of any single word changes the sum.
"""
import os
import struct

import numpy as np

MISSING, HBM, HOST, DISK = 0, 1, 2, 3
MAGIC = b"MPICKV01"
P = 0x9E3779B97F4A7C15
MASK = (1 << 64) - 1
ELEM = {0: 4, 1: 2}


def checksum(data):
    """data: bytes-like whose length is a multiple of 8."""
    w = np.frombuffer(data, dtype="<u8")
    if w.size == 0:
        return 0
    with np.errstate(over="ignore"):
        powers = np.multiply.accumulate(np.full(w.size, P, dtype=np.uint64))
        total = np.add.reduce(w.astype(np.uint64) * powers, dtype=np.uint64)
    return (int(total) + w.size) & MASK


def file_name(chunk_id):
    return "%016x.mpickv" % chunk_id


def write_chunk_file(path, chunk_id, k, v, dtype_code):
    """k, v: arrays [n_layers][len][Hkv][D] of the storage type (bf16 as uint16)."""
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    n_layers, length, n_kv, d = k.shape
    block = length * n_kv * d * ELEM[dtype_code]
    assert k.nbytes == v.nbytes == n_layers * block and block % 8 == 0
    table_end = 64 + 16 * n_layers
    payload_off = (table_end + 4095) // 4096 * 4096
    head = MAGIC + struct.pack("<QiiiiiiQQ", chunk_id, length, n_layers, n_kv, d, dtype_code, 0, block, payload_off)
    head += struct.pack("<Q", checksum(head))
    sums = b""
    for layer in range(n_layers):
        sums += struct.pack("<QQ", checksum(k[layer].tobytes()), checksum(v[layer].tobytes()))
    with open(path, "wb") as f:
        f.write(head + sums)
        f.write(b"\0" * (payload_off - table_end))
        for layer in range(n_layers):
            f.write(k[layer].tobytes())
            f.write(v[layer].tobytes())


def read_chunk_file(path):
    """Returns (id, dtype_code, K bytes per layer, V bytes per layer, (len, Hkv, D)); raises
    ValueError when the file is not what the layout above says (bad magic, sizes, sums)."""
    with open(path, "rb") as f:
        raw = f.read()
    if len(raw) < 64 or raw[:8] != MAGIC:
        raise ValueError("not a chunk cache file")
    chunk_id, length, n_layers, n_kv, d, dtype_code, zero, block, payload_off = struct.unpack("<QiiiiiiQQ", raw[8:56])
    if struct.unpack("<Q", raw[56:64])[0] != checksum(raw[:56]):
        raise ValueError("header checksum")
    if dtype_code not in ELEM or min(length, n_layers, n_kv, d) <= 0 or block != length * n_kv * d * ELEM[dtype_code]:
        raise ValueError("header fields")
    if payload_off % 4096 or payload_off < 64 + 16 * n_layers or len(raw) != payload_off + 2 * n_layers * block:
        raise ValueError("file size")
    ks, vs = [], []
    for layer in range(n_layers):
        want_k, want_v = struct.unpack("<QQ", raw[64 + 16 * layer: 80 + 16 * layer])
        at = payload_off + 2 * layer * block
        kb, vb = raw[at: at + block], raw[at + block: at + 2 * block]
        if checksum(kb) != want_k or checksum(vb) != want_v:
            raise ValueError("block checksum, layer %d" % layer)
        ks.append(kb)
        vs.append(vb)
    return chunk_id, dtype_code, ks, vs, (length, n_kv, d)


class ChunkStore:
    """id -> stored cache.  put() replaces; a cache whose expiry time has come is deleted by
    expire(now) and is MISSING afterwards (expires_at < 0: kept for ever)."""

    def __init__(self):
        self.entries = {}

    def put(self, chunk_id, k, v, place, expires_at=-1):
        assert place in (HBM, HOST, DISK)
        self.entries[chunk_id] = dict(k=np.array(k, copy=True), v=np.array(v, copy=True), place=place,
                                      expires_at=expires_at)

    def move(self, chunk_id, place):
        assert place in (HBM, HOST, DISK)
        self.entries[chunk_id]["place"] = place

    def drop(self, chunk_id):
        self.entries.pop(chunk_id, None)

    def expire(self, now):
        gone = sorted(i for i, e in self.entries.items() if 0 <= e["expires_at"] <= now)
        for i in gone:
            del self.entries[i]
        return gone

    def lookup(self, ids):
        place = [self.entries[i]["place"] if i in self.entries else MISSING for i in ids]
        length = [self.entries[i]["k"].shape[1] if i in self.entries else 0 for i in ids]
        return place, length

    def layer(self, chunk_id, layer):
        e = self.entries[chunk_id]
        return e["k"][layer], e["v"][layer]
