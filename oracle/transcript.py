"""SHA-256 Fiat-Shamir transcript.

The paper's protocols are interactive: the verifier sends a uniform field
element after every round polynomial (App. B, both protocols).  Here each such
message is replaced by a hash of everything sent so far.  The byte format is
this build's own; the HIP library implements the same format independently.

The transcript is ONE byte stream, and everything derived from it is a plain SHA-256
of an extension of it:

  stream_0          = "zkdl-mi355x/v3" zero-padded to 56 bytes || u64le(seed)      (64 bytes)
  absorb(label, m)  : stream <- stream || u8(len label) || label || u64le(len m) || m
                      (len label <= 32)
  challenges(n)     : for i < n: d0 = SHA256(stream || 0xF0 || u32le(i)),
                                 d1 = SHA256(stream || 0xF1 || u32le(i)),
                                 c_i = int_le(d0 || d1) mod r
                      then stream <- stream || 0xF2 || zero bytes up to the next multiple of 64
                      (n = 0: nothing happens)
  challenge()       = challenges(1)[0]
  digest()          = SHA256(stream)

A prover keeps the SHA-256 chaining value after the last whole block and the bytes of the
unfinished block.  After a draw the stream is block-aligned, so the usual step of a sumcheck
round - absorb a 106-byte frame, draw one challenge - is one compression for the frame's first
64 bytes, followed by three independent compressions from that chaining value: the two hashes
of the draw (their last block holds the frame's remaining 42 bytes, the five bytes of the draw
and the padding) and the block that extends the stream.  The n challenges of one draw are one
hash latency on a parallel machine, not n.

Field elements are absorbed as 32-byte canonical little-endian strings.
Test infrastructure; not used by the product.
"""
import hashlib
import struct

from .field import R_MOD, to_le

DOMAIN = b"zkdl-mi355x/v3"
MAX_LABEL = 32


class Transcript:
    def __init__(self, seed=0):
        self._h = hashlib.sha256()
        self._len = 0
        self._append(DOMAIN + b"\x00" * (56 - len(DOMAIN)) + struct.pack("<Q", seed))
        self.challenges = []          # every challenge drawn, in order

    def _append(self, data):
        self._h.update(data)
        self._len += len(data)

    def absorb(self, label, data):
        label = bytes(label)
        data = bytes(data)
        assert len(label) <= MAX_LABEL
        self._append(bytes([len(label)]) + label + struct.pack("<Q", len(data)) + data)

    def absorb_fr(self, label, elements):
        self.absorb(label, b"".join(to_le(e) for e in elements))

    def absorb_u32(self, label, words):
        self.absorb(label, b"".join(struct.pack("<I", w) for w in words))

    def _fork(self, tail):
        f = self._h.copy()
        f.update(tail)
        return f.digest()

    def challenges_vec(self, n):
        out = []
        for i in range(n):
            idx = struct.pack("<I", i)
            out.append(int.from_bytes(self._fork(b"\xf0" + idx) + self._fork(b"\xf1" + idx), "little") % R_MOD)
        if n > 0:
            self._append(b"\xf2")
            self._append(b"\x00" * (-self._len % 64))
        self.challenges.extend(out)
        return out

    def challenge(self):
        return self.challenges_vec(1)[0]

    def digest(self):
        return self._h.digest()
