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


class DevicePieces:
    """A piece workload on the device with tables built by the library."""

    def __init__(self, prec_bits, mass, sym, dist, build=True):
        dev = torch.device("cuda:0")
        self.m, self.mass_np, self.sym_np, self.dist_np = prec_bits, mass, sym, dist
        self.d, self.x = mass.shape
        self.shape = pb.make_ansai_shape(sym.shape[0], sym.shape[1], prec_bits, self.d, self.x)
        self.mass = torch.from_numpy(np.ascontiguousarray(mass, dtype=np.uint32)).to(dev)
        self.sym = torch.from_numpy(sym).to(dev)
        self.dist = torch.from_numpy(dist).to(dev)
        self.tables = torch.zeros(pb.pilc_ansai_table_bytes(prec_bits, self.d, self.x), dtype=torch.uint8,
                                  device=dev)
        ws_bytes, self.max_coded = pb.pilc_ansai_workspace_size(self.shape)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.coded = torch.zeros(self.max_coded + 16, dtype=torch.uint8, device=dev)
        self.out = torch.zeros_like(self.sym)
        self.nbytes = 0
        if build:
            pb.pilc_ansai_build_tables(prec_bits, self.d, self.x, self.mass, self.tables)

    def encode(self, check=True, capacity=None, sym=None, dist=None):
        coded = self.coded if capacity is None else self.coded[:capacity]
        rc, self.nbytes = pb.pilc_ansai_encode(self.shape, self.sym if sym is None else sym,
                                               self.dist if dist is None else dist, self.tables,
                                               self.workspace, coded, check=check)
        return rc, self.nbytes

    def coded_numpy(self):
        return self.coded[: self.nbytes].cpu().numpy()

    def decode(self, coded=None, nbytes=None, check=True, dist=None):
        coded = self.coded if coded is None else coded
        nbytes = self.nbytes if nbytes is None else nbytes
        self.out.fill_(0xA5)
        return pb.pilc_ansai_decode(self.shape, coded, nbytes, self.dist if dist is None else dist,
                                    self.tables, self.workspace, self.out, check=check)

    def decoded_numpy(self):
        return self.out.cpu().numpy()

    def table_views(self):
        """delta, phi, theta, nbits, next as numpy arrays read back from the device blob: a
        256-byte header, {delta, phi} pairs in rows of 256 per distribution (one more pair closes
        them), then the symbol table
        and the (next << 4 | 15 - nbits) table (16-bit entries up to M = 12, 32-bit above), each
        part 256-byte aligned."""
        blob = self.tables.cpu().numpy()
        up = lambda v: (v + 255) & ~255
        entries = self.d << self.m
        enc = np.frombuffer(blob, dtype="<u4", count=2 * self.d * 256, offset=256).reshape(self.d, 256, 2)
        enc = enc[:, : self.x]
        th_off = up(256 + 8 * (self.d * 256 + 1))
        theta = np.frombuffer(blob, dtype=np.uint8, count=entries, offset=th_off).reshape(self.d, -1)
        nb_off = up(th_off + entries)
        nb = np.frombuffer(blob, dtype="<u4" if self.m > 12 else "<u2", count=entries, offset=nb_off)
        nb = nb.astype(np.uint32).reshape(self.d, -1)
        return enc[:, :, 0].astype(np.int32), enc[:, :, 1], theta, (15 - (nb & 15)).astype(np.uint8), nb >> 4


class DeviceMix:
    """A mixture workload (synth_mix.MixWorkload) on the device."""

    def __init__(self, wl):
        self.wl = wl
        self.k = wl.num_comp
        self.geom = pb.make_geom(*wl.geom)
        dev = torch.device("cuda:0")
        self.img = torch.from_numpy(wl.img).to(dev)
        self.mu = torch.from_numpy(wl.mu).to(dev)
        self.log_scale = torch.from_numpy(wl.log_scale).to(dev)
        self.weight = torch.from_numpy(wl.weight).to(dev)
        self.chan_coef = torch.from_numpy(wl.chan_coef).to(dev)
        ws_bytes, self.max_coded = pb.pilc_workspace_size(self.geom)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.coded = torch.zeros(self.max_coded + 16, dtype=torch.uint8, device=dev)
        self.out = torch.zeros_like(self.img)
        self.nbytes = 0

    def encode(self, check=True, capacity=None, weight=None, k=None):
        coded = self.coded if capacity is None else self.coded[:capacity]
        rc, self.nbytes = pb.pilc_mix_encode(self.geom, self.k if k is None else k, self.img, self.mu,
                                             self.log_scale, self.weight if weight is None else weight,
                                             self.chan_coef, self.workspace, coded, check=check)
        return rc, self.nbytes

    def coded_numpy(self):
        return self.coded[: self.nbytes].cpu().numpy()

    def decode(self, coded=None, nbytes=None, check=True, weight=None, k=None):
        coded = self.coded if coded is None else coded
        nbytes = self.nbytes if nbytes is None else nbytes
        self.out.fill_(0xA5)
        return pb.pilc_mix_decode(self.geom, self.k if k is None else k, coded, nbytes, self.mu,
                                  self.log_scale, self.weight if weight is None else weight,
                                  self.chan_coef, self.workspace, self.out, check=check)

    def decoded_numpy(self):
        return self.out.cpu().numpy()
