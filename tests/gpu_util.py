"""Helpers for the GPU parity tests: move a workload to the device, run the library through the
Python binding of the C ABI, and fetch the results."""
import struct

import numpy as np
import torch

from paper_2206_05279_amd import binding as pb


class DeviceWorkload:
    def __init__(self, wl):
        self.wl = wl
        self.geom = pb.make_geom(*wl.geom)
        dev = torch.device("cuda:0")
        self.img = torch.from_numpy(wl.img).to(dev)
        self.mu = torch.from_numpy(wl.mu).to(dev)
        self.log_scale = torch.from_numpy(wl.log_scale).to(dev)
        self.chan_coef = torch.from_numpy(wl.chan_coef).to(dev)
        ws_bytes, self.max_coded = pb.pilc_workspace_size(self.geom)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.coded = torch.zeros(self.max_coded + 16, dtype=torch.uint8, device=dev)
        self.out = torch.zeros_like(self.img)

    def encode(self, check=True, capacity=None):
        coded = self.coded if capacity is None else self.coded[:capacity]
        rc, nbytes = pb.pilc_encode(self.geom, self.img, self.mu, self.log_scale, self.chan_coef,
                                    self.workspace, coded, check=check)
        self.nbytes = nbytes
        return rc, nbytes

    def coded_numpy(self):
        return self.coded[: self.nbytes].cpu().numpy()

    def decode(self, coded=None, nbytes=None, check=True):
        coded = self.coded if coded is None else coded
        nbytes = self.nbytes if nbytes is None else nbytes
        self.out.fill_(0xA5)
        rc = pb.pilc_decode(self.geom, coded, nbytes, self.mu, self.log_scale, self.chan_coef,
                            self.workspace, self.out, check=check)
        return rc

    def decoded_numpy(self):
        return self.out.cpu().numpy()


def parse_container(coded: np.ndarray):
    b = coded.tobytes()
    assert b[:4] == b"PILC"
    lanes = struct.unpack_from("<I", b, 40)[0]
    payload = struct.unpack_from("<Q", b, 48)[0]
    offs = np.frombuffer(b, dtype="<u4", count=lanes + 1, offset=64)
    start = 64 + 4 * (lanes + 1)
    return lanes, payload, offs, coded[start:]


def first_difference(a: np.ndarray, b: np.ndarray) -> str:
    if a.size != b.size:
        return "sizes differ: %d vs %d" % (a.size, b.size)
    d = np.flatnonzero(a != b)
    return "identical" if d.size == 0 else "first difference at byte %d of %d (%d differ)" % (
        d[0], a.size, d.size)
