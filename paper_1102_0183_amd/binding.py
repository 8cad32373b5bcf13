"""Thin ctypes binding of the cnn355 C ABI (include/cnn355.h).

Argument marshalling only: every step of the network runs in the HIP kernels of
libcnn355.so.  PyTorch is used for device memory (the workspace, images, labels, outputs)
and for the stream handle; nothing here computes.  There is no CPU fallback: if the
library cannot be loaded this module raises.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

OK, E_SYNTAX, E_SHAPE, E_ARG, E_WORKSPACE, E_HIP, E_STATE = 0, -1, -2, -3, -4, -5, -6
LAYER_INPUT, LAYER_CONV, LAYER_POOL, LAYER_FC = 0, 1, 2, 3
MODE_STAGES, MODE_PERSISTENT, MODE_RESIDENT = 0, 1, 2
OUTPUT_SOFTMAX_XENT, OUTPUT_TANH_SQERR = 0, 1

_lib = None


class CnnError(RuntimeError):
    def __init__(self, code, what, msg=""):
        super().__init__("cnn355: %s failed with code %d%s" % (what, code, (": " + msg) if msg else ""))
        self.code = code


def lib():
    """Load libcnn355.so (built beforehand by build.py; compiled here only if it is missing)."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            path = _build.build(force=True)
        L = C.CDLL(path)
        vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int32
        sig = {
            "cnn_arch_info": (C.c_int, [C.c_char_p, vp, vp, i32]),
            "cnn_arch_info_xy": (C.c_int, [C.c_char_p, vp, vp, i32]),
            "cnn_workspace_bytes": (C.c_int, [C.c_char_p, vp]),
            "cnn_plan_text": (C.c_int, [C.c_char_p, vp, sz]),
            "cnn_get_plan_text": (C.c_int, [vp, vp, sz]),
            "cnn_create": (C.c_int, [C.c_char_p, vp, sz, vp, vp]),
            "cnn_destroy": (None, [vp]),
            "cnn_deform_images": (C.c_int, [vp, vp, sz, vp, sz, C.c_int, C.c_int, C.c_int, vp, C.c_uint64, C.c_uint64, vp, vp]),
            "cnn_set_connection_table": (C.c_int, [vp, C.c_int, vp]),
            "cnn_set_fixed_frontend": (C.c_int, [vp, C.c_int, C.c_int, C.c_int, vp, vp]),
            "cnn_num_weights": (sz, [vp]),
            "cnn_image_size": (sz, [vp]),
            "cnn_num_layers": (C.c_int, [vp]),
            "cnn_num_classes": (C.c_int, [vp]),
            "cnn_layer_info": (C.c_int, [vp, C.c_int, vp]),
            "cnn_layer_info_xy": (C.c_int, [vp, C.c_int, vp]),
            "cnn_get_weights": (C.c_int, [vp, vp, sz]),
            "cnn_set_weights": (C.c_int, [vp, vp, sz]),
            "cnn_forward": (C.c_int, [vp, vp, vp]),
            "cnn_train_step": (C.c_int, [vp, vp, i32, C.c_float]),
            "cnn_train_many": (C.c_int, [vp, vp, vp, sz, C.c_float]),
            "cnn_forward_many": (C.c_int, [vp, vp, sz, vp]),
            "cnn_set_mode": (C.c_int, [vp, C.c_int]),
            "cnn_get_mode": (C.c_int, [vp]),
            "cnn_mode_supported": (C.c_int, [vp, C.c_int]),
            "cnn_set_team": (C.c_int, [vp, C.c_int, C.c_int]),
            "cnn_forward_batch_scratch_bytes": (C.c_int, [vp, sz, vp]),
            "cnn_forward_batch": (C.c_int, [vp, vp, sz, vp, vp, sz, sz]),
            "cnn_forward_batch_static": (C.c_int, [vp, vp, sz, vp, sz]),
            "cnn_set_output_units": (C.c_int, [vp, C.c_int]),
            "cnn_get_output_units": (C.c_int, [vp]),
            "cnn_set_matrix_cores": (C.c_int, [vp, C.c_int]),
            "cnn_set_launch_graph": (C.c_int, [vp, C.c_int]),
            "cnn_set_grid": (C.c_int, [vp, C.c_int]),
            "cnn_set_spin_limit": (C.c_int, [vp, C.c_uint]),
            "cnn_set_barrier": (C.c_int, [vp, C.c_int]),
            "cnn_synchronize": (C.c_int, [vp]),
            "cnn_get_activation": (C.c_int, [vp, C.c_int, vp]),
            "cnn_get_delta": (C.c_int, [vp, C.c_int, vp]),
            "cnn_get_argmax": (C.c_int, [vp, C.c_int, vp]),
            "cnn_get_loss": (C.c_int, [vp, vp]),
            "cnn_debug_gradients": (C.c_int, [vp, vp, i32, vp]),
            "cnn_get_stage_times": (C.c_int, [vp, vp, C.c_int, vp]),
            "cnn_measure_crossing": (C.c_int, [vp, C.c_int, C.c_int, C.c_int, vp]),
            "cnn_measure_launch": (C.c_int, [vp, C.c_int, vp]),
            "cnn_debug_forward_batch_layer": (C.c_int, [vp, vp, C.c_size_t, C.c_int, vp, vp, vp, C.c_size_t]),
            "cnn_resident_spec_source": (C.c_int, [vp, vp, C.c_size_t]),
            "cnn_load_resident_code": (C.c_int, [vp, C.c_char_p]),
            "cnn_resident_code_active": (C.c_int, [vp]),
            "cnn_last_error": (C.c_char_p, [vp]),
        }
        for name, (res, args) in sig.items():
            f = getattr(L, name)
            f.restype = res
            f.argtypes = args
        _lib = L
    return _lib


FORWARD_BATCH_STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = ["cnn_arch_info", "cnn_arch_info_xy", "cnn_workspace_bytes", "cnn_plan_text", "cnn_get_plan_text", "cnn_create", "cnn_destroy",
           "cnn_set_connection_table", "cnn_set_fixed_frontend", "cnn_num_weights", "cnn_image_size",
           "cnn_num_layers", "cnn_num_classes", "cnn_layer_info", "cnn_layer_info_xy", "cnn_get_weights", "cnn_set_weights",
           "cnn_forward", "cnn_train_step", "cnn_train_many", "cnn_forward_many",
           "cnn_forward_batch_scratch_bytes", "cnn_forward_batch", "cnn_forward_batch_static", "cnn_set_mode",
           "cnn_get_mode", "cnn_mode_supported", "cnn_set_team", "cnn_set_output_units", "cnn_get_output_units",
           "cnn_set_matrix_cores", "cnn_set_launch_graph", "cnn_set_grid", "cnn_set_spin_limit", "cnn_set_barrier", "cnn_synchronize", "cnn_get_activation",
           "cnn_get_delta", "cnn_get_argmax", "cnn_get_loss", "cnn_debug_gradients", "cnn_get_stage_times", "cnn_measure_crossing", "cnn_measure_launch",
           "cnn_resident_spec_source", "cnn_load_resident_code", "cnn_resident_code_active", "cnn_debug_forward_batch_layer",
           "cnn_deform_images", "cnn_last_error"]


def _err(handle=None):
    m = lib().cnn_last_error(handle)
    return m.decode() if m else ""


class DeformParams(C.Structure):
    """cnn_deform_params of the header, field for field."""
    _fields_ = [("max_translation", C.c_float), ("max_rotation", C.c_float), ("max_scaling", C.c_float),
                ("max_shear", C.c_float), ("sigma", C.c_float), ("alpha", C.c_float), ("fill", C.c_float)]


def deform_images(d_src, d_dst, n, params, seed, first_index, d_src_index=None, d_displacement=None, stream=None):
    """cnn_deform_images: d_src [n_src][C][H][W] and d_dst [>= n][C][H][W] float32 device tensors; params a
    DeformParams (or None: NULL); d_src_index an int32 device tensor of n entries or None; d_displacement a
    float32 device tensor [n][2][H][W] or None.  Asynchronous on `stream` (a torch stream; None: the current)."""
    import torch
    for t in (d_src, d_dst):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.dim() == 4
    n_src, Cc, H, W = d_src.shape
    assert tuple(d_dst.shape[1:]) == (Cc, H, W) and d_dst.shape[0] >= n
    if d_src_index is not None:
        assert d_src_index.is_cuda and d_src_index.dtype == torch.int32 and d_src_index.is_contiguous()
        assert d_src_index.numel() >= n
    if d_displacement is not None:
        assert d_displacement.is_cuda and d_displacement.dtype == torch.float32 and d_displacement.is_contiguous()
        assert d_displacement.numel() >= n * 2 * H * W
    st = (stream or torch.cuda.current_stream(d_src.device)).cuda_stream
    rc = lib().cnn_deform_images(st, d_src.data_ptr(), int(n_src), d_dst.data_ptr(), int(n), int(Cc), int(H), int(W),
                                 C.addressof(params) if params is not None else None, int(seed), int(first_index),
                                 d_src_index.data_ptr() if d_src_index is not None else None,
                                 d_displacement.data_ptr() if d_displacement is not None else None)
    if rc:
        raise CnnError(rc, "cnn_deform_images", _err())


def arch_info(arch):
    """Host-only: list of dicts {kind, maps, h, w, K, S, Kx, Sx} (K, S: the y values), layer 0 = input."""
    n = C.c_int32()
    rc = lib().cnn_arch_info_xy(arch.encode(), C.addressof(n), None, 0)
    if rc:
        raise CnnError(rc, "cnn_arch_info_xy(%r)" % arch, _err())
    info = np.zeros((n.value, 8), dtype=np.int32)
    rc = lib().cnn_arch_info_xy(arch.encode(), C.addressof(n), info.ctypes.data, n.value)
    if rc:
        raise CnnError(rc, "cnn_arch_info_xy(%r)" % arch, _err())
    return [dict(kind=int(r[0]), maps=int(r[1]), h=int(r[2]), w=int(r[3]), K=int(r[4]), S=int(r[5]),
                 Kx=int(r[6]), Sx=int(r[7])) for r in info]


def workspace_bytes(arch):
    n = C.c_size_t()
    rc = lib().cnn_workspace_bytes(arch.encode(), C.addressof(n))
    if rc:
        raise CnnError(rc, "cnn_workspace_bytes(%r)" % arch, _err())
    return int(n.value)


def plan_text(arch):
    """Host-only: the stage list of one training step, one line per stage."""
    buf = C.create_string_buffer(1 << 14)
    rc = lib().cnn_plan_text(arch.encode(), buf, len(buf))
    if rc:
        raise CnnError(rc, "cnn_plan_text(%r)" % arch, _err())
    return buf.value.decode()


def resident_plan(arch, fan_in=0, n_ranks=0, xcd_stride=0):
    """Development aid, host-only: the resident-mode plan of an architecture, parsed: {"numbers": {name: value},
    "conv": [{field: value}], "fc": [...], "regions": [(name, first_float, floats)]}, or {"unsupported": reason}.
    fan_in > 0: output map j of every conv layer above the first reads input maps j .. j + fan_in - 1 (mod M_i);
    fan_in = -d: M_i / d of them in every layer."""
    f = lib().cnn355_resident_plan_text
    f.restype = C.c_int
    f.argtypes = [C.c_char_p, C.c_int, C.c_int, C.c_int, C.c_char_p, C.c_size_t]
    buf = C.create_string_buffer(1 << 16)
    rc = f(arch.encode(), fan_in, n_ranks, xcd_stride, buf, len(buf))
    if rc:
        raise CnnError(rc, "cnn355_resident_plan_text(%r)" % arch, _err())
    plan = {"numbers": {}, "conv": [], "fc": [], "regions": []}
    for line in buf.value.decode().splitlines():
        w = line.split()
        if w[0] == "unsupported":
            return {"unsupported": " ".join(w[1:])}
        if w[0] in ("conv", "fc"):
            plan[w[0]].append({w[k]: int(w[k + 1]) for k in range(2, len(w), 2)})
        elif w[0] == "region":
            plan["regions"].append((w[1], int(w[2]), int(w[3])))
        else:
            plan["numbers"][w[0]] = int(w[1])
    return plan


def resident_spec_source_for(arch, fan_in=0, n_ranks=0, xcd_stride=0):
    """Development aid, host-only: what Cnn.resident_spec_source() returns for a handle of this architecture with the
    tables of resident_plan() and the default output units, on a device of 256 compute units."""
    f = lib().cnn355_resident_spec_source_for
    f.restype = C.c_int
    f.argtypes = [C.c_char_p, C.c_int, C.c_int, C.c_int, C.c_char_p, C.c_size_t]
    buf = C.create_string_buffer(1 << 16)
    rc = f(arch.encode(), fan_in, n_ranks, xcd_stride, buf, len(buf))
    if rc < 0:
        raise CnnError(rc, "cnn355_resident_spec_source_for(%r)" % arch, _err())
    return buf.value.decode()


class Cnn:
    """One network on the current HIP device.  The workspace is a torch uint8 tensor owned here."""

    def __init__(self, arch, device="cuda:0", stream=None):
        import torch
        self._torch = torch
        self.arch = arch
        self.device = torch.device(device)
        nbytes = workspace_bytes(arch)
        with torch.cuda.device(self.device):
            self.workspace = torch.zeros(nbytes + 256, dtype=torch.uint8, device=self.device)
            base = self.workspace.data_ptr()
            self._ws_ptr = (base + 255) // 256 * 256
            s = torch.cuda.current_stream(self.device) if stream is None else stream
            self._stream = s
            torch.cuda.synchronize(self.device)
            h = C.c_void_p()
            rc = lib().cnn_create(arch.encode(), self._ws_ptr, nbytes, s.cuda_stream, C.addressof(h))
        if rc:
            raise CnnError(rc, "cnn_create(%r)" % arch, _err())
        self._h = h

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().cnn_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ck(self, rc, what):
        if rc:
            raise CnnError(rc, what, _err(self._h))

    # ---- structure
    def set_connection_table(self, conv_index, table):
        t = np.ascontiguousarray(table, dtype=np.uint8)
        self._ck(lib().cnn_set_connection_table(self._h, int(conv_index), t.ctypes.data),
                 "cnn_set_connection_table")

    def set_fixed_frontend(self, filters, src_channel, n_src_channels):
        f = np.ascontiguousarray(filters, dtype=np.float32)
        s = np.ascontiguousarray(src_channel, dtype=np.int32)
        self._ck(lib().cnn_set_fixed_frontend(self._h, int(f.shape[0]), int(f.shape[-1]),
                                              int(n_src_channels), f.ctypes.data, s.ctypes.data),
                 "cnn_set_fixed_frontend")

    @property
    def num_weights(self):
        return int(lib().cnn_num_weights(self._h))

    @property
    def image_size(self):
        return int(lib().cnn_image_size(self._h))

    @property
    def num_layers(self):
        return int(lib().cnn_num_layers(self._h))

    @property
    def num_classes(self):
        return int(lib().cnn_num_classes(self._h))

    def layer_info(self, layer):
        info = np.zeros(8, dtype=np.int32)
        self._ck(lib().cnn_layer_info_xy(self._h, int(layer), info.ctypes.data), "cnn_layer_info_xy")
        return dict(kind=int(info[0]), maps=int(info[1]), h=int(info[2]), w=int(info[3]),
                    K=int(info[4]), S=int(info[5]), Kx=int(info[6]), Sx=int(info[7]))

    def set_mode(self, mode):
        self._ck(lib().cnn_set_mode(self._h, int(mode)), "cnn_set_mode")

    def plan_text(self):
        """The stage list of one training step of this network as it is now, one line per stage."""
        buf = C.create_string_buffer(1 << 14)
        self._ck(lib().cnn_get_plan_text(self._h, buf, len(buf)), "cnn_get_plan_text")
        return buf.value.decode()

    @property
    def mode(self):
        return int(lib().cnn_get_mode(self._h))

    def mode_supported(self, mode):
        return bool(lib().cnn_mode_supported(self._h, int(mode)))

    def set_team(self, n_ranks=0, xcd_stride=0):
        self._ck(lib().cnn_set_team(self._h, int(n_ranks), int(xcd_stride)), "cnn_set_team")

    def set_launch_graph(self, images_per_graph):
        """Stage mode: replay graphs of the launches of this many images (0: launch every stage by itself)."""
        self._ck(lib().cnn_set_launch_graph(self._h, int(images_per_graph)), "cnn_set_launch_graph")

    def set_output_units(self, kind):
        """OUTPUT_SOFTMAX_XENT (default) or OUTPUT_TANH_SQERR."""
        self._ck(lib().cnn_set_output_units(self._h, int(kind)), "cnn_set_output_units")

    @property
    def output_units(self):
        return lib().cnn_get_output_units(self._h)

    def set_matrix_cores(self, on):
        self._ck(lib().cnn_set_matrix_cores(self._h, 1 if on else 0), "cnn_set_matrix_cores")

    def set_grid(self, n_workgroups):
        self._ck(lib().cnn_set_grid(self._h, int(n_workgroups)), "cnn_set_grid")

    def set_barrier(self, kind):
        self._ck(lib().cnn_set_barrier(self._h, int(kind)), "cnn_set_barrier")

    def set_spin_limit(self, polls):
        self._ck(lib().cnn_set_spin_limit(self._h, int(polls)), "cnn_set_spin_limit")

    # ---- weights
    def set_weights(self, w):
        w = np.ascontiguousarray(w, dtype=np.float32)
        self._ck(lib().cnn_set_weights(self._h, w.ctypes.data, w.size), "cnn_set_weights")

    def get_weights(self):
        w = np.empty(self.num_weights, dtype=np.float32)
        self._ck(lib().cnn_get_weights(self._h, w.ctypes.data, w.size), "cnn_get_weights")
        return w

    # ---- the hot path (device tensors in, device tensors out; asynchronous)
    def _dev_f32(self, t, n):
        torch = self._torch
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == n, \
            "expected a contiguous float32 device tensor of %d elements" % n
        return t.data_ptr()

    def forward(self, d_image, d_probs=None):
        p = None if d_probs is None else self._dev_f32(d_probs, self.num_classes)
        self._ck(lib().cnn_forward(self._h, self._dev_f32(d_image, self.image_size), p), "cnn_forward")

    def train_step(self, d_image, label, lr):
        self._ck(lib().cnn_train_step(self._h, self._dev_f32(d_image, self.image_size), int(label),
                                      float(lr)), "cnn_train_step")

    def train_many(self, d_images, d_labels, lr, n=None):
        torch = self._torch
        n = d_labels.numel() if n is None else int(n)
        assert d_labels.is_cuda and d_labels.dtype == torch.int32 and d_labels.is_contiguous()
        assert d_labels.numel() >= n and d_images.numel() >= n * self.image_size
        assert d_images.is_cuda and d_images.dtype == torch.float32 and d_images.is_contiguous()
        self._ck(lib().cnn_train_many(self._h, d_images.data_ptr(), d_labels.data_ptr(), n, float(lr)),
                 "cnn_train_many")

    def forward_many(self, d_images, n, d_probs=None):
        torch = self._torch
        assert d_images.is_cuda and d_images.dtype == torch.float32 and d_images.is_contiguous()
        assert d_images.numel() >= n * self.image_size
        p = None if d_probs is None else self._dev_f32(d_probs, n * self.num_classes)
        self._ck(lib().cnn_forward_many(self._h, d_images.data_ptr(), int(n), p), "cnn_forward_many")

    def forward_batch_scratch_bytes(self, batch):
        n = C.c_size_t(0)
        self._ck(lib().cnn_forward_batch_scratch_bytes(self._h, int(batch), C.byref(n)),
                 "cnn_forward_batch_scratch_bytes")
        return n.value

    def forward_batch(self, d_images, n, d_probs, d_scratch, batch):
        """Forward pass of n images, `batch` at a time, every layer one matrix product over the
        batch.  d_scratch: a uint8 device tensor of at least forward_batch_scratch_bytes(batch)."""
        torch = self._torch
        assert d_images.is_cuda and d_images.dtype == torch.float32 and d_images.is_contiguous()
        assert d_images.numel() >= n * self.image_size
        assert d_scratch.is_cuda and d_scratch.dtype == torch.uint8 and d_scratch.is_contiguous()
        p = self._dev_f32(d_probs, n * self.num_classes)
        self._ck(lib().cnn_forward_batch(self._h, d_images.data_ptr(), int(n), p, d_scratch.data_ptr(),
                                         d_scratch.numel(), int(batch)), "cnn_forward_batch")

    def debug_forward_batch_layer(self, d_images, n, trainable_layer, d_scratch):
        """Outputs of one trainable layer of the batched forward pass for n images run as one batch: (n, floats)."""
        torch = self._torch
        assert d_images.is_cuda and d_images.dtype == torch.float32 and d_images.is_contiguous()
        assert d_images.numel() >= n * self.image_size
        biggest = max(i["maps"] * i["h"] * i["w"] for i in (self.layer_info(l) for l in range(self.num_layers)))
        out = np.empty((n, biggest), dtype=np.float32)
        per = C.c_size_t(0)
        self._ck(lib().cnn_debug_forward_batch_layer(self._h, d_images.data_ptr(), int(n), int(trainable_layer),
                                                     out.ctypes.data, C.byref(per), d_scratch.data_ptr(), d_scratch.numel()),
                 "cnn_debug_forward_batch_layer")
        return out.reshape(-1)[:n * per.value].reshape(n, per.value).copy()

    def measure_crossing(self, n_ranks, words_per_rank, rounds=200):
        """Microseconds one exchange of words_per_rank tagged words per rank among n_ranks workgroups takes."""
        us = C.c_float(0)
        self._ck(lib().cnn_measure_crossing(self._h, int(n_ranks), int(words_per_rank), int(rounds), C.byref(us)),
                 "cnn_measure_crossing")
        return us.value

    def measure_launch(self, rounds=500):
        """Microseconds per launch of an empty kernel, back to back on the handle's stream."""
        us = C.c_float(0)
        self._ck(lib().cnn_measure_launch(self._h, int(rounds), C.byref(us)), "cnn_measure_launch")
        return us.value

    def resident_spec_source(self):
        """The header text that describes this handle's network to the resident kernel's source (see specialize.py)."""
        n = lib().cnn_resident_spec_source(self._h, None, 0)
        if n < 0:
            raise CnnError(n, "cnn_resident_spec_source", _err(None))
        buf = C.create_string_buffer(n + 1)
        lib().cnn_resident_spec_source(self._h, buf, n + 1)
        return buf.value.decode()

    def load_resident_code(self, path):
        """Run resident-mode calls in the kernel of the code object at `path`, compiled for this handle's plan."""
        self._ck(lib().cnn_load_resident_code(self._h, os.fsencode(path)), "cnn_load_resident_code")

    @property
    def resident_code_active(self):
        return bool(lib().cnn_resident_code_active(self._h))

    def forward_batch_static(self, d_images, n, d_probs, batch):
        """forward_batch with the scratch memory taken from the library's own device array (at most
        FORWARD_BATCH_STATIC_SCRATCH_BYTES): nothing is allocated anywhere."""
        torch = self._torch
        assert d_images.is_cuda and d_images.dtype == torch.float32 and d_images.is_contiguous()
        assert d_images.numel() >= n * self.image_size
        p = self._dev_f32(d_probs, n * self.num_classes)
        self._ck(lib().cnn_forward_batch_static(self._h, d_images.data_ptr(), int(n), p, int(batch)),
                 "cnn_forward_batch_static")

    def synchronize(self):
        self._ck(lib().cnn_synchronize(self._h), "cnn_synchronize")

    # ---- parity taps (synchronous, host results)
    def activation(self, layer):
        i = self.layer_info(layer)
        a = np.empty((i["maps"], i["h"], i["w"]), dtype=np.float32)
        self._ck(lib().cnn_get_activation(self._h, int(layer), a.ctypes.data), "cnn_get_activation")
        return a

    def delta(self, layer):
        i = self.layer_info(layer)
        a = np.empty((i["maps"], i["h"], i["w"]), dtype=np.float32)
        self._ck(lib().cnn_get_delta(self._h, int(layer), a.ctypes.data), "cnn_get_delta")
        return a

    def argmax(self, layer):
        i = self.layer_info(layer)
        a = np.empty((i["maps"], i["h"], i["w"]), dtype=np.uint8)
        self._ck(lib().cnn_get_argmax(self._h, int(layer), a.ctypes.data), "cnn_get_argmax")
        return a

    def loss(self):
        v = C.c_float()
        self._ck(lib().cnn_get_loss(self._h, C.addressof(v)), "cnn_get_loss")
        return float(v.value)

    def stage_times(self):
        """Persistent mode: [(work_us, barrier_us)] per stage for the last image of the last call."""
        buf = np.zeros(2 * 128, dtype=np.float32)
        n = C.c_int()
        self._ck(lib().cnn_get_stage_times(self._h, buf.ctypes.data, 128, C.addressof(n)),
                 "cnn_get_stage_times")
        return [(float(buf[2 * k]), float(buf[2 * k + 1])) for k in range(n.value)]

    def resident_static_id(self):
        """Development aid: which compiled-in network the resident plan equals (0: none)."""
        f = lib().cnn355_resident_static_id
        f.restype = C.c_int
        f.argtypes = [C.c_void_p]
        return int(f(self._h))

    def resident_ranks(self):
        """Development aid: workgroups in the resident plan's team (0: the network cannot run in resident mode)."""
        f = lib().cnn355_resident_ranks
        f.restype = C.c_int
        f.argtypes = [C.c_void_p]
        return int(f(self._h))

    def resident_streams(self):
        """Development aid: whether the resident plan streams the inputs of the layers above the first."""
        f = lib().cnn355_resident_streams
        f.restype = C.c_int
        f.argtypes = [C.c_void_p]
        return bool(f(self._h))

    def resident_pull_shares(self, conv_index):
        """Development aid: ranks that share the delta pull into one input map of a conv layer of the resident plan."""
        f = lib().cnn355_resident_pull_shares
        f.restype = C.c_int
        f.argtypes = [C.c_void_p, C.c_int]
        return int(f(self._h, conv_index))

    def raw_stamps(self, n=128):
        """Development aid: device timestamps (100 MHz ticks) left by the last call."""
        buf = np.zeros(n, dtype=np.uint64)
        f = lib().cnn355_read_status_stamps
        f.restype = C.c_int
        f.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
        self._ck(f(self._h, buf.ctypes.data, n), "cnn355_read_status_stamps")
        return buf

    def debug_gradients(self, d_image, label):
        g = np.empty(self.num_weights, dtype=np.float32)
        self._ck(lib().cnn_debug_gradients(self._h, self._dev_f32(d_image, self.image_size), int(label),
                                           g.ctypes.data), "cnn_debug_gradients")
        return g
