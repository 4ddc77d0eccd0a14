"""SHA-256 Fiat-Shamir transcript.

The paper's protocols are interactive: the verifier sends a uniform field
element after every round polynomial (App. B, both protocols).  Here each such
message is replaced by a hash of everything sent so far.  The byte format is
this build's own; the HIP library implements the same format independently.

The transcript is ONE byte stream, always a whole number of 64-byte blocks, and
everything derived from it is a plain SHA-256 of a prefix-extension of it:

  stream_0          = "zkdl-mi355x/v2" zero-padded to 56 bytes || u64le(seed)      (one block)
  absorb(label, m)  : stream <- stream || pad64(u8(len label) || label || u64le(len m) || m)
                      (pad64: zero bytes up to the next multiple of 64; len label <= 32)
  challenges(n)     : for i < n: d0 = SHA256(stream || 0xF0 || u32le(i)),
                                 d1 = SHA256(stream || 0xF1 || u32le(i)),
                                 c_i = int_le(d0 || d1) mod r
                      then stream <- stream || 0xF2 || 63 zero bytes   (n = 0: nothing happens)
  challenge()       = challenges(1)[0]
  digest()          = SHA256(stream)

Because the stream is block-aligned, a prover needs the SHA-256 chaining value
after the last block only: an absorb costs one compression per 64 bytes of
message, and each hash of a draw is one more compression from that chaining
value (its block holds the five bytes and the padding), all of them independent.
The n challenges of one draw are therefore one hash latency on a parallel
machine, not n.

Field elements are absorbed as 32-byte canonical little-endian strings.
Test infrastructure; not used by the product.
"""
import hashlib
import struct

from .field import R_MOD, to_le

DOMAIN = b"zkdl-mi355x/v2"
MAX_LABEL = 32


class Transcript:
    def __init__(self, seed=0):
        self._h = hashlib.sha256()
        self._h.update(DOMAIN + b"\x00" * (56 - len(DOMAIN)) + struct.pack("<Q", seed))
        self.challenges = []          # every challenge drawn, in order

    def absorb(self, label, data):
        label = bytes(label)
        data = bytes(data)
        assert len(label) <= MAX_LABEL
        frame = bytes([len(label)]) + label + struct.pack("<Q", len(data)) + data
        self._h.update(frame + b"\x00" * (-len(frame) % 64))

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
            self._h.update(b"\xf2" + b"\x00" * 63)
        self.challenges.extend(out)
        return out

    def challenge(self):
        return self.challenges_vec(1)[0]

    def digest(self):
        return self._h.digest()
