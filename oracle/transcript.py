"""SHA-256 Fiat-Shamir transcript.

The paper's protocols are interactive: the verifier sends a uniform field
element after every round polynomial (App. B, both protocols).  Here each such
message is replaced by a hash of everything sent so far.  The byte format is
this build's own; the HIP library implements the same format independently.

  state_0           = SHA256("zkdl-mi355x/v1" || u64le(seed))
  absorb(label, m)  : state <- SHA256(state || u8(len label) || label || u64le(len m) || m)
  challenge()       : d0 = SHA256(state || 0x00); d1 = SHA256(state || 0x01)
                      c  = int_le(d0 || d1) mod r
                      state <- SHA256(state || 0x02)

Field elements are absorbed as 32-byte canonical little-endian strings.
Test infrastructure; not used by the product.
"""
import hashlib
import struct

from .field import R_MOD, to_le

DOMAIN = b"zkdl-mi355x/v1"


class Transcript:
    def __init__(self, seed=0):
        self.state = hashlib.sha256(DOMAIN + struct.pack("<Q", seed)).digest()
        self.challenges = []          # every challenge drawn, in order

    def absorb(self, label, data):
        label = bytes(label)
        data = bytes(data)
        assert len(label) < 256
        self.state = hashlib.sha256(
            self.state + bytes([len(label)]) + label + struct.pack("<Q", len(data)) + data
        ).digest()

    def absorb_fr(self, label, elements):
        self.absorb(label, b"".join(to_le(e) for e in elements))

    def absorb_u32(self, label, words):
        self.absorb(label, b"".join(struct.pack("<I", w) for w in words))

    def challenge(self):
        d0 = hashlib.sha256(self.state + b"\x00").digest()
        d1 = hashlib.sha256(self.state + b"\x01").digest()
        c = int.from_bytes(d0 + d1, "little") % R_MOD
        self.state = hashlib.sha256(self.state + b"\x02").digest()
        self.challenges.append(c)
        return c

    def challenges_vec(self, n):
        return [self.challenge() for _ in range(n)]

    def digest(self):
        return self.state
