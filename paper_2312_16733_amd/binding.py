"""ctypes binding of include/subnetact.h (same names, argument marshalling only)."""
import ctypes as C
import os

import numpy as np

MAX_STAGES, MAX_DEPTH, NAME_LEN, N_KCLASS = 8, 16, 48, 12
FAMILY = {"tiny": 0, "resnet": 1, "mbv3": 2, "transformer": 3}
DTYPE = {"fp32": 0, "bf16": 1}
ACT = {"none": 0, "relu": 1, "hswish": 2, "gelu": 3}

_HERE = os.path.dirname(os.path.abspath(__file__))


class SnaError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"sna_status {status}: {text}")
        self.status = status


class ArchDesc(C.Structure):
    _fields_ = [("family", C.c_int32), ("dtype", C.c_int32), ("n_classes", C.c_int32),
                ("in_ch", C.c_int32), ("stem_ch", C.c_int32), ("n_stages", C.c_int32),
                ("stage_ch", C.c_int32 * MAX_STAGES), ("stage_stride", C.c_int32 * MAX_STAGES),
                ("stage_max_depth", C.c_int32 * MAX_STAGES),
                ("block_max_mid", (C.c_int32 * MAX_DEPTH) * MAX_STAGES),
                ("block_max_aux", (C.c_int32 * MAX_DEPTH) * MAX_STAGES),
                ("stage_se", C.c_int32 * MAX_STAGES), ("stage_act", C.c_int32 * MAX_STAGES),
                ("tail_ch", C.c_int32), ("fc_ch", C.c_int32),
                ("hidden", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn", C.c_int32), ("seq_len", C.c_int32), ("max_layers", C.c_int32),
                ("max_res", C.c_int32)]


class SubnetCfgC(C.Structure):
    _fields_ = [("subnet_id", C.c_int32), ("n_stages", C.c_int32),
                ("depth", C.c_int32 * MAX_STAGES), ("stage_out_ch", C.c_int32 * (MAX_STAGES + 1)),
                ("block_mid_ch", (C.c_int32 * MAX_DEPTH) * MAX_STAGES),
                ("block_aux_ch", (C.c_int32 * MAX_DEPTH) * MAX_STAGES),
                ("block_kernel", (C.c_int32 * MAX_DEPTH) * MAX_STAGES),
                ("in_h", C.c_int32), ("in_w", C.c_int32)]


class TensorInfo(C.Structure):
    _fields_ = [("name", C.c_char * NAME_LEN), ("kind", C.c_int32), ("dtype", C.c_int32),
                ("dims", C.c_int32 * 4), ("c_pad", C.c_int32), ("offset", C.c_int64),
                ("bytes", C.c_int64)]


class NormInfo(C.Structure):
    _fields_ = [("name", C.c_char * NAME_LEN), ("channels", C.c_int32), ("offset", C.c_int32)]


def library_path() -> str:
    return os.path.join(_HERE, "libsubnetact.so")


_lib = None


def lib():
    """Load libsubnetact.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise SnaError(-8, f"{path} is not built: run `python -m paper_2312_16733_amd.build` "
                           "(or __graft_entry__.build()) first")
    L = C.CDLL(path)
    ap = C.POINTER(ArchDesc)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.sna_last_error.restype = C.c_char_p
    L.sna_tensor_count.argtypes = [ap]; L.sna_tensor_count.restype = i32
    L.sna_norm_count.argtypes = [ap]; L.sna_norm_count.restype = i32
    L.sna_tensor_info_get.argtypes = [ap, i32, C.POINTER(TensorInfo)]; L.sna_tensor_info_get.restype = i32
    L.sna_norm_info_get.argtypes = [ap, i32, C.POINTER(NormInfo)]; L.sna_norm_info_get.restype = i32
    L.sna_weights_bytes.argtypes = [ap]; L.sna_weights_bytes.restype = i64
    L.sna_stats_row_len.argtypes = [ap]; L.sna_stats_row_len.restype = i64
    L.sna_workspace_bytes.argtypes = [ap, i32, i32]; L.sna_workspace_bytes.restype = i64
    L.sna_supernet_load.argtypes = [ap, vp, sz, vp, sz, i32, i32, vp, sz, vp, C.POINTER(vp)]
    L.sna_supernet_load.restype = i32
    L.sna_subnet_forward.argtypes = [vp, C.POINTER(SubnetCfgC), i32, C.POINTER(i32), i32, vp, vp, vp, vp]
    L.sna_subnet_forward.restype = i32
    L.sna_subnet_tune.argtypes = L.sna_subnet_forward.argtypes; L.sna_subnet_tune.restype = i32
    L.sna_subnet_forward_static.argtypes = L.sna_subnet_forward.argtypes; L.sna_subnet_forward_static.restype = i32
    L.sna_static_scratch_bytes.argtypes = []; L.sna_static_scratch_bytes.restype = i64
    L.sna_subnet_calibrate.argtypes = [vp, vp, i32, vp, vp, vp, vp]; L.sna_subnet_calibrate.restype = i32
    L.sna_tuned_count.argtypes = [vp]; L.sna_tuned_count.restype = i32
    L.sna_tuning_export.argtypes = [vp, C.c_char_p, i64]; L.sna_tuning_export.restype = i64
    L.sna_tuning_import.argtypes = [vp, C.c_char_p, i64]; L.sna_tuning_import.restype = i32
    L.sna_supernet_free.argtypes = [vp]; L.sna_supernet_free.restype = None
    L.sna_last_forward_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i32)]; L.sna_last_forward_info.restype = i32
    L.sna_profile_enable.argtypes = [vp, i32]; L.sna_profile_enable.restype = i32
    L.sna_set_k_split.argtypes = [vp, i32]; L.sna_set_k_split.restype = i32
    L.sna_set_tile_variant.argtypes = [vp, i32]; L.sna_set_tile_variant.restype = i32
    L.sna_tile_variant_count.argtypes = []; L.sna_tile_variant_count.restype = i32
    L.sna_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64), C.POINTER(C.c_double),
                                   C.POINTER(C.c_double)]
    L.sna_profile_read.restype = i32
    L.sna_profile_class_name.argtypes = [i32]; L.sna_profile_class_name.restype = C.c_char_p
    L.sna_profile_read_launches.argtypes = [vp, C.c_char_p, i64]; L.sna_profile_read_launches.restype = i64
    _lib = L
    return L


def _check(st):
    if st < 0:
        raise SnaError(st, lib().sna_last_error().decode())
    return st


# ---------------------------------------------------------------- descriptions
def arch_desc_from_spec(spec, max_res=None) -> ArchDesc:
    """Fill the C architecture description from any object with the family's attributes."""
    a = ArchDesc()
    a.family, a.dtype, a.n_classes = FAMILY[spec.family], DTYPE[spec.dtype], spec.n_classes
    if spec.family == "transformer":
        a.n_stages = 1
        a.hidden, a.n_heads, a.head_dim, a.ffn = spec.hidden, spec.n_heads, spec.head_dim, spec.ffn
        a.seq_len, a.max_layers = spec.seq_len, spec.max_layers
        a.max_res = spec.seq_len
        return a
    a.in_ch, a.stem_ch, a.n_stages = spec.in_ch, spec.stem_ch, spec.n_stages
    a.max_res = max_res or max(spec.res_choices)
    for s in range(spec.n_stages):
        a.stage_ch[s] = spec.stage_ch[s]
        a.stage_max_depth[s] = spec.max_depth[s]
        a.stage_stride[s] = 2 if spec.family == "tiny" else spec.stage_stride[s]
        for j in range(spec.max_depth[s]):
            if spec.family == "resnet":
                a.block_max_mid[s][j] = spec.max_mid(s)
            elif spec.family == "mbv3":
                a.block_max_mid[s][j] = spec.max_mid(s, j)
                a.block_max_aux[s][j] = spec.max_sq(s, j)
        if spec.family == "mbv3":
            a.stage_se[s] = int(spec.stage_se[s])
            a.stage_act[s] = ACT[spec.stage_act[s]]
    if spec.family == "mbv3":
        a.tail_ch, a.fc_ch = spec.tail_ch, spec.fc_ch
    return a


def cfg_to_c(cfg) -> SubnetCfgC:
    c = SubnetCfgC()
    c.subnet_id, c.n_stages, c.in_h, c.in_w = cfg.subnet_id, cfg.n_stages, cfg.in_h, cfg.in_w
    for s, d in enumerate(cfg.depth):
        c.depth[s] = d
    for s, v in enumerate(cfg.stage_out_ch):
        c.stage_out_ch[s] = v
    for name in ("block_mid_ch", "block_aux_ch", "block_kernel"):
        src, dst = getattr(cfg, name), getattr(c, name)
        for s, row in enumerate(src):
            for j, v in enumerate(row):
                dst[s][j] = v
    return c


def tensor_infos(arch: ArchDesc):
    L = lib()
    n = _check(L.sna_tensor_count(C.byref(arch)))
    out = []
    for i in range(n):
        ti = TensorInfo()
        _check(L.sna_tensor_info_get(C.byref(arch), i, C.byref(ti)))
        out.append(ti)
    return out


def norm_infos(arch: ArchDesc):
    L = lib()
    n = _check(L.sna_norm_count(C.byref(arch)))
    out = []
    for i in range(n):
        ni = NormInfo()
        _check(L.sna_norm_info_get(C.byref(arch), i, C.byref(ni)))
        out.append(ni)
    return out


def _bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array holding bf16-representable values -> their 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    if np.any(u & np.uint32(0xFFFF)):
        raise ValueError("value is not representable in bfloat16")
    return (u >> np.uint32(16)).astype(np.uint16)


def pack_weights(arch: ArchDesc, tensors: dict) -> np.ndarray:
    """name -> fp32 ndarray (max-size shapes)  =>  the library's weight blob (uint8, host)."""
    blob = np.zeros(_check(lib().sna_weights_bytes(C.byref(arch))), dtype=np.uint8)
    for ti in tensor_infos(arch):
        name = ti.name.decode()
        a = np.asarray(tensors[name], dtype=np.float32)
        nd = {0: 4, 1: 3, 2: 2, 3: 1}[ti.kind]
        want = tuple(ti.dims[:nd])
        if a.shape != want:
            raise ValueError(f"{name}: shape {a.shape} != {want}")
        if ti.kind == 0 and ti.c_pad > ti.dims[3]:          # stored input channels are zero-padded
            a = np.concatenate([a, np.zeros(a.shape[:3] + (ti.c_pad - ti.dims[3],), np.float32)], axis=3)
        raw = _bf16_bits(a).tobytes() if ti.dtype == DTYPE["bf16"] else a.tobytes()
        assert len(raw) == ti.bytes, name
        blob[ti.offset:ti.offset + ti.bytes] = np.frombuffer(raw, dtype=np.uint8)
    return blob


def pack_stats(arch: ArchDesc, stats: dict, n_subnets: int) -> np.ndarray:
    """name -> [n_subnets][4][C_max]  =>  fp32 [n_subnets][4][row_len]."""
    row = _check(lib().sna_stats_row_len(C.byref(arch)))
    out = np.zeros((n_subnets, 4, max(row, 1)), dtype=np.float32)
    for ni in norm_infos(arch):
        a = stats[ni.name.decode()]
        assert a.shape == (n_subnets, 4, ni.channels), ni.name
        out[:, :, ni.offset:ni.offset + ni.channels] = a
    return out


# ---------------------------------------------------------------- the two calls
def supernet_load(arch, weights_dev_ptr, weights_bytes, stats_dev_ptr, stats_bytes, n_subnets,
                  max_batch, workspace_dev_ptr, workspace_bytes, stream=0):
    h = C.c_void_p()
    _check(lib().sna_supernet_load(C.byref(arch), weights_dev_ptr, weights_bytes, stats_dev_ptr,
                                   stats_bytes, n_subnets, max_batch, workspace_dev_ptr,
                                   workspace_bytes, stream, C.byref(h)))
    return h


def subnet_forward(handle, cfgs_c, req_cfg, inputs_dev_ptr, logits_dev_ptr, hidden_dev_ptr=None, stream=0,
                   tune=False, static=False):
    n_cfgs = len(cfgs_c)
    arr = cfgs_c if isinstance(cfgs_c, C.Array) else (SubnetCfgC * n_cfgs)(*cfgs_c)
    rc = np.ascontiguousarray(req_cfg, dtype=np.int32)
    fn = lib().sna_subnet_tune if tune else (lib().sna_subnet_forward_static if static else lib().sna_subnet_forward)
    _check(fn(handle, arr, n_cfgs, rc.ctypes.data_as(C.POINTER(C.c_int32)),
              len(rc), inputs_dev_ptr, logits_dev_ptr, hidden_dev_ptr, stream))


class Supernet:
    """A resident SuperNet: torch owns the device buffers, the library borrows them."""

    def __init__(self, spec, tensors: dict, stats: dict, n_subnets: int, max_batch: int,
                 device="cuda:0", max_res=None):
        import torch
        self.torch = torch
        self.spec = spec
        self.device = torch.device(device)
        self.arch = arch_desc_from_spec(spec, max_res)
        self.n_subnets, self.max_batch = n_subnets, max_batch
        self.act_dtype = torch.bfloat16 if spec.dtype == "bf16" else torch.float32
        self.weights = torch.from_numpy(pack_weights(self.arch, tensors)).to(self.device)
        self.stats = torch.from_numpy(pack_stats(self.arch, stats, n_subnets)).to(self.device)
        ws = _check(lib().sna_workspace_bytes(C.byref(self.arch), n_subnets, max_batch))
        self.workspace = torch.empty(ws, dtype=torch.uint8, device=self.device)
        self.weight_bytes = self.weights.numel()
        self.stats_bytes = self.stats.numel() * 4
        stream = torch.cuda.current_stream(self.device).cuda_stream
        self.handle = supernet_load(self.arch, self.weights.data_ptr(), self.weights.numel(),
                                    self.stats.data_ptr(), self.stats.numel() * 4, n_subnets, max_batch,
                                    self.workspace.data_ptr(), ws, stream)
        self._cfg_cache = {}

    def close(self):
        if self.handle is not None:
            lib().sna_supernet_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prepare_cfgs(self, cfgs):
        return (SubnetCfgC * len(cfgs))(*[cfg_to_c(c) for c in cfgs])

    def _request_elems(self, cfg_c) -> int:
        """Input elements one request of this cfg occupies."""
        if self.spec.family == "transformer":
            return int(cfg_c.in_h) * self.spec.hidden
        return int(cfg_c.in_h) * int(cfg_c.in_w) * self.spec.in_ch

    def _check_buffers(self, cfgs_c, req_cfg, inputs, logits, hidden):
        """The library trusts the caller's buffer sizes; refuse tensors shorter than the routed requests need."""
        n = len(req_cfg)
        if n > self.max_batch:
            return                                      # the library's to report, as are bad indices and cfgs
        need = 0
        for r in req_cfg:
            if not 0 <= int(r) < len(cfgs_c):
                return
            c = cfgs_c[int(r)]
            if not (0 < c.in_h <= self.arch.max_res and 0 < c.in_w <= max(self.arch.max_res, 1)):
                return
            need += self._request_elems(c)
        if inputs.numel() < need:
            raise ValueError(f"inputs hold {inputs.numel()} elements, the {n} routed requests need {need}")
        if logits is not None and logits.numel() < n * self.spec.n_classes:
            raise ValueError(f"logits hold {logits.numel()} elements, need {n * self.spec.n_classes}")
        if hidden is not None and hidden.numel() < n * self.spec.seq_len * self.spec.hidden:
            raise ValueError(f"hidden holds {hidden.numel()} elements, need {n * self.spec.seq_len * self.spec.hidden}")

    def tune(self, cfgs, req_cfg, inputs, hidden=None, stream=None):
        """One forward that also measures the tile variants of every layer shape it meets."""
        return self.forward(cfgs, req_cfg, inputs, hidden=hidden, stream=stream, tune=True)

    def calibrate(self, cfg, inputs, logits=None, stream=None):
        """SubnetNorm calibration of one cfg on `inputs` (device tensor, requests concatenated): fills
        row cfg.subnet_id of the resident statistics table; returns that forward's logits."""
        torch = self.torch
        cfgs_c = self.prepare_cfgs([cfg])
        assert inputs.dtype == self.act_dtype and inputs.is_contiguous() and inputs.device == self.device
        per = self._request_elems(cfgs_c[0])
        if per <= 0 or inputs.numel() % per:
            raise ValueError(f"inputs hold {inputs.numel()} elements, not a whole number of requests of {per}")
        n = inputs.numel() // per
        if logits is None:
            logits = torch.empty((n, self.spec.n_classes), dtype=torch.float32, device=self.device)
        elif logits.numel() < n * self.spec.n_classes:
            raise ValueError(f"logits hold {logits.numel()} elements, need {n * self.spec.n_classes}")
        if stream is None:
            stream = torch.cuda.current_stream(self.device).cuda_stream
        _check(lib().sna_subnet_calibrate(self.handle, cfgs_c, n, inputs.data_ptr(), self.stats.data_ptr(),
                                          logits.data_ptr(), stream))
        return logits

    def stats_table(self) -> dict:
        """The resident statistics table read back: name -> fp32 [n_subnets][4][C_max]."""
        host = self.stats.cpu().numpy().reshape(self.n_subnets, 4, -1)
        return {ni.name.decode(): host[:, :, ni.offset:ni.offset + ni.channels].copy() for ni in norm_infos(self.arch)}

    def tuned_count(self):
        return int(lib().sna_tuned_count(self.handle))

    def tuning_export(self) -> str:
        n = int(lib().sna_tuning_export(self.handle, None, 0))
        buf = C.create_string_buffer(n + 1)
        lib().sna_tuning_export(self.handle, buf, n + 1)
        return buf.value.decode()

    def tuning_import(self, text: str):
        b = text.encode()
        _check(lib().sna_tuning_import(self.handle, b, len(b)))

    def forward(self, cfgs, req_cfg, inputs, logits=None, hidden=None, stream=None, tune=False, static=False):
        """inputs: device tensor of the architecture's dtype, requests concatenated (flat is fine).
        static=True calls sna_subnet_forward_static (pass `logits` too if the caller must not allocate)."""
        torch = self.torch
        cfgs_c = cfgs if isinstance(cfgs, C.Array) else self.prepare_cfgs(cfgs)
        n = len(req_cfg)
        assert inputs.dtype == self.act_dtype and inputs.is_contiguous() and inputs.device == self.device
        self._check_buffers(cfgs_c, req_cfg, inputs, logits, hidden)
        if logits is None:
            logits = torch.empty((n, self.spec.n_classes), dtype=torch.float32, device=self.device)
        if stream is None:
            stream = torch.cuda.current_stream(self.device).cuda_stream
        subnet_forward(self.handle, cfgs_c, req_cfg, inputs.data_ptr(), logits.data_ptr(),
                       hidden.data_ptr() if hidden is not None else None, stream, tune=tune, static=static)
        return logits

    def last_forward_info(self):
        m, l = C.c_int64(), C.c_int32()
        _check(lib().sna_last_forward_info(self.handle, C.byref(m), C.byref(l)))
        return m.value, l.value

    def set_tile_variant(self, variant):
        _check(lib().sna_set_tile_variant(self.handle, int(variant)))

    def set_k_split(self, mode):
        _check(lib().sna_set_k_split(self.handle, int(mode)))

    def profile_enable(self, on: bool):
        _check(lib().sna_profile_enable(self.handle, int(on)))

    def profile_read_launches(self) -> str:
        n = lib().sna_profile_read_launches(self.handle, None, 0)
        if n < 0:
            raise SnaError(-1, lib().sna_last_error().decode())
        buf = C.create_string_buffer(n + 1)
        lib().sna_profile_read_launches(self.handle, buf, n + 1)
        return buf.value.decode()

    def profile_read(self):
        ms = (C.c_double * N_KCLASS)(); la = (C.c_int64 * N_KCLASS)()
        fl = (C.c_double * N_KCLASS)(); by = (C.c_double * N_KCLASS)()
        _check(lib().sna_profile_read(self.handle, ms, la, fl, by))
        out = {}
        for k in range(N_KCLASS):
            name = lib().sna_profile_class_name(k).decode()
            if name and la[k]:
                out[name] = {"ms": ms[k], "launches": la[k], "flops": fl[k], "bytes": by[k]}
        return out
