"""SHA-256 Fiat-Shamir transcript.

The paper's protocols are interactive: the verifier sends a uniform field
element after every round polynomial (App. B, both protocols).  Here each such
message is replaced by a hash of everything sent so far.  The byte format is
this build's own; the HIP library implements the same format independently.

  state_0           = SHA256("zkdl-mi355x/v1" || u64le(seed))
  absorb(label, m)  : state <- SHA256(state || u8(len label) || label || u64le(len m) || m)
  challenges(n)     : for i < n: d0 = SHA256(state || 0x00 || u32le(i)),
                                 d1 = SHA256(state || 0x01 || u32le(i)),
                                 c_i = int_le(d0 || d1) mod r
                      then state <- SHA256(state || 0x02)   (n = 0: nothing happens)
  challenge()       = challenges(1)[0]

The n challenges of one draw depend on the state only, so a point u in F^m is
one hash latency on a parallel machine, not m.

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

    def challenges_vec(self, n):
        out = []
        for i in range(n):
            idx = struct.pack("<I", i)
            d0 = hashlib.sha256(self.state + b"\x00" + idx).digest()
            d1 = hashlib.sha256(self.state + b"\x01" + idx).digest()
            out.append(int.from_bytes(d0 + d1, "little") % R_MOD)
        if n > 0:
            self.state = hashlib.sha256(self.state + b"\x02").digest()
        self.challenges.extend(out)
        return out

    def challenge(self):
        return self.challenges_vec(1)[0]

    def digest(self):
        return self.state
