"""ctypes binding of libtc.so: argument marshalling only.

Every function of include/tc.h is reachable under its own name through
`load_library().tc_*`; the classes below only pack arguments (shapes, byte
strings, device pointers taken from torch tensors) and raise TcError on a
negative status."""
import ctypes
import os

TC_OK = 0
TC_ERR_ARG, TC_ERR_SHAPE, TC_ERR_RANGE, TC_ERR_NOMEM, TC_ERR_HIP, TC_ERR_VERIFY, TC_ERR_STATE = -1, -2, -3, -4, -5, -6, -7
TC_I8, TC_I16, TC_FR, TC_F16 = 1, 2, 3, 4
TC_SRS_SUFFIX, TC_SRS_FIXED_BASE, TC_SRS_MONOMIAL, TC_SRS_OPEN_TABLE = 1, 2, 4, 8
TC_INTERP_NEWTON, TC_INTERP_GREGORY, TC_INTERP_BARYCENTRIC = 0, 1, 2
TC_LEAF_ENTRIES, TC_LEAF_TENSORS = 0, 1
TC_PROF_BUCKET_ACC, TC_PROF_NODE_COMMIT, TC_PROF_NODE_COMMIT_UPPER, TC_PROF_VERIFY_CHAIN = 0, 1, 2, 3
TC_MAX_ORDER, TC_MAX_STEPS = 4, 16
TC_ALU_MAD, TC_ALU_MAD_CARRY, TC_ALU_FP_MUL, TC_ALU_FP_SQR, TC_ALU_FP_MUL_F64, TC_ALU_FP_SQR_F64 = 0, 1, 2, 3, 4, 5
TC_ALU_FP28_MUL, TC_ALU_FP28_SQR = 6, 7
TC_OPT_ACC_SUBRUN, TC_OPT_ACC_FANIN, TC_OPT_FR_WINDOW, TC_OPT_CHECK_LEVEL = 0, 1, 2, 3
TC_STATIC_MAX_TERMS, TC_STATIC_SCRATCH_BYTES = 1 << 18, 32 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))
_ERR_NAMES = {-1: "TC_ERR_ARG", -2: "TC_ERR_SHAPE", -3: "TC_ERR_RANGE", -4: "TC_ERR_NOMEM", -5: "TC_ERR_HIP",
              -6: "TC_ERR_VERIFY", -7: "TC_ERR_STATE"}


class TcError(RuntimeError):
    def __init__(self, code, message=""):
        super().__init__("%s (%d): %s" % (_ERR_NAMES.get(code, "TC_ERR"), code, message))
        self.code = code


class tc_tree_desc(ctypes.Structure):
    _fields_ = [
        ("m", ctypes.c_int),
        ("grid", ctypes.c_uint32 * TC_MAX_ORDER),
        ("node_shape", ctypes.c_uint32 * TC_MAX_ORDER),
        ("node_srs", ctypes.c_void_p),
        ("leaf_kind", ctypes.c_int),
        ("d_payload", ctypes.c_void_p),
        ("dtype", ctypes.c_int),
        ("leaf_srs", ctypes.POINTER(ctypes.c_void_p)),
        ("d_leaf_scalars", ctypes.POINTER(ctypes.c_void_p)),
        ("leaf_dtype", ctypes.POINTER(ctypes.c_int)),
    ]


class tc_path(ctypes.Structure):
    _fields_ = [
        ("n_steps", ctypes.c_int),
        ("m", ctypes.c_int * TC_MAX_STEPS),
        ("shape", (ctypes.c_uint32 * TC_MAX_ORDER) * TC_MAX_STEPS),
        ("kappa", (ctypes.c_uint32 * TC_MAX_ORDER) * TC_MAX_STEPS),
    ]


def library_path():
    return os.path.join(_HERE, "libtc.so")


_LIBS = {}


def load_library(path=None):
    """Loads libtc.so (or the library at `path`) and declares the prototypes of include/tc.h."""
    path = os.path.abspath(path or library_path())
    if path in _LIBS:
        return _LIBS[path]
    if not os.path.exists(path):
        raise FileNotFoundError(
            "%s is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`; "
            "there is no fallback implementation" % path)
    L = ctypes.CDLL(path)
    vp, u8p, u32p = ctypes.c_void_p, ctypes.c_char_p, ctypes.POINTER(ctypes.c_uint32)
    sig = {
        "tc_ctx_create": (ctypes.c_int, [ctypes.POINTER(vp), ctypes.c_int, vp]),
        "tc_ctx_destroy": (None, [vp]),
        "tc_last_error": (ctypes.c_char_p, [vp]),
        "tc_ctx_sync": (ctypes.c_int, [vp]),
        "tc_ctx_profile": (ctypes.c_int, [vp, ctypes.c_int]),
        "tc_ctx_profile_read": (ctypes.c_int, [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                               ctypes.POINTER(ctypes.c_uint64)]),
        "tc_ctx_profile_units": (ctypes.c_int, [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_uint64)]),
        "tc_ctx_alu_rate": (ctypes.c_int, [vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]),
        "tc_ctx_field_op": (ctypes.c_int, [vp, ctypes.c_int, vp, vp, ctypes.c_size_t, vp]),
        "tc_ctx_set_option": (ctypes.c_int, [vp, ctypes.c_int, ctypes.c_int64]),
        "tc_ctx_get_option": (ctypes.c_int, [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]),
        "tc_setup_from_trapdoor": (ctypes.c_int, [vp, u8p, ctypes.c_int, u32p, ctypes.c_uint32, ctypes.POINTER(vp)]),
        "tc_srs_destroy": (None, [vp]),
        "tc_srs_size": (ctypes.c_uint64, [vp, ctypes.c_int]),
        "tc_srs_get_point": (ctypes.c_int, [vp, vp, ctypes.c_int, ctypes.c_uint64, vp]),
        "tc_srs_export": (ctypes.c_int, [vp, vp, vp, ctypes.POINTER(ctypes.c_size_t)]),
        "tc_srs_import": (ctypes.c_int, [vp, vp, ctypes.c_size_t, ctypes.POINTER(vp)]),
        "tc_terkle_export": (ctypes.c_int, [vp, vp, vp, ctypes.POINTER(ctypes.c_size_t)]),
        "tc_terkle_import": (ctypes.c_int, [vp, ctypes.POINTER(tc_tree_desc), vp, ctypes.c_size_t, ctypes.POINTER(vp)]),
        "tc_encode_tensor": (ctypes.c_int, [vp, vp, ctypes.c_int, ctypes.c_size_t, ctypes.c_float, vp]),
        "tc_quant_scale": (ctypes.c_int, [vp, vp, ctypes.c_size_t, vp]),
        "tc_encode_tensor_scaled": (ctypes.c_int, [vp, vp, ctypes.c_int, ctypes.c_size_t, vp, vp]),
        "tc_encode_batch_scaled": (ctypes.c_int, [vp, ctypes.c_int, vp, vp, vp, vp]),
        "tc_commit": (ctypes.c_int, [vp, vp, vp, ctypes.c_int, vp]),
        "tc_commit_batch": (ctypes.c_int, [vp, ctypes.c_int, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                           ctypes.POINTER(ctypes.c_int), vp]),
        "tc_commit_static": (ctypes.c_int, [vp, vp, vp, ctypes.c_int, vp]),
        "tc_alloc_calls": (ctypes.c_uint64, []),
        "tc_open": (ctypes.c_int, [vp, vp, vp, ctypes.c_int, u32p, vp, vp]),
        "tc_vk_from_trapdoor": (ctypes.c_int, [u8p, ctypes.c_int, ctypes.POINTER(vp)]),
        "tc_vk_destroy": (None, [vp]),
        "tc_verify": (ctypes.c_int, [vp, vp, ctypes.c_int, u32p, u8p, u32p, u8p, u8p]),
        "tc_terkle_build": (ctypes.c_int, [vp, ctypes.POINTER(tc_tree_desc), ctypes.POINTER(vp)]),
        "tc_tree_destroy": (None, [vp]),
        "tc_terkle_root": (ctypes.c_int, [vp, vp]),
        "tc_terkle_levels": (ctypes.c_int, [vp]),
        "tc_terkle_level_info": (ctypes.c_int, [vp, ctypes.c_int, u32p, ctypes.POINTER(ctypes.c_uint64)]),
        "tc_terkle_node": (ctypes.c_int, [vp, vp, ctypes.c_int, ctypes.c_uint64, vp]),
        "tc_path_from_grid": (ctypes.c_int, [ctypes.c_int, u32p, u32p, ctypes.c_int, u32p, ctypes.c_int, u32p, u32p,
                                             ctypes.POINTER(tc_path)]),
        "tc_terkle_open": (ctypes.c_int, [vp, vp, u32p, u32p, vp, ctypes.POINTER(ctypes.c_size_t)]),
        "tc_terkle_open_batch": (ctypes.c_int, [vp, vp, ctypes.c_int, u32p, u32p, vp, ctypes.c_size_t,
                                                ctypes.POINTER(ctypes.c_size_t)]),
        "tc_verify_path": (ctypes.c_int, [vp, vp, ctypes.POINTER(tc_path), u8p, u8p, vp, ctypes.c_size_t]),
        "tc_verify_paths_batch": (ctypes.c_int, [vp, vp, ctypes.c_int, ctypes.POINTER(tc_path), u8p, u8p, vp,
                                                 ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t),
                                                 ctypes.POINTER(ctypes.c_int)]),
        "tc_terkle_update": (ctypes.c_int, [vp, vp, u32p, u32p, ctypes.c_int64]),
        "tc_interpolate": (ctypes.c_int, [vp, ctypes.c_int, u32p, vp, ctypes.c_int, vp]),
        "tc_interpolate_form": (ctypes.c_int, [vp, ctypes.c_int, u32p, vp, ctypes.c_int, ctypes.c_int, vp]),
        "tc_divide_by_linear": (ctypes.c_int, [vp, ctypes.c_int, u32p, vp, ctypes.c_int, ctypes.c_uint32, vp, vp]),
        "tc_hill_alpha": (ctypes.c_int, [ctypes.POINTER(ctypes.c_double), ctypes.c_size_t, ctypes.c_size_t,
                                         ctypes.POINTER(ctypes.c_double)]),
        "tc_layer_benefits": (ctypes.c_int, [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double), ctypes.c_size_t,
                                             ctypes.POINTER(ctypes.c_double)]),
        "tc_select_layers": (ctypes.c_int, [ctypes.c_size_t, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                            ctypes.c_size_t, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                            ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]),
        "tc_vkp_from_trapdoor": (ctypes.c_int, [u8p, ctypes.c_int, ctypes.POINTER(vp)]),
        "tc_vkp_destroy": (None, [vp]),
        "tc_vkp_get": (ctypes.c_int, [vp, ctypes.c_int, vp]),
        "tc_pairing": (ctypes.c_int, [u8p, u8p, vp]),
        "tc_verify_pairing": (ctypes.c_int, [vp, ctypes.c_int, u32p, u8p, u32p, u8p, u8p]),
        "tc_verify_path_pairing": (ctypes.c_int, [vp, ctypes.POINTER(tc_path), u8p, u8p, vp, ctypes.c_size_t]),
        "tc_verify_paths_pairing_batch": (ctypes.c_int, [vp, ctypes.c_int, ctypes.POINTER(tc_path), u8p, u8p, vp,
                                                         ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t),
                                                         ctypes.POINTER(ctypes.c_int)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)              # AttributeError here = the library does not export a declared symbol
        fn.restype = res
        fn.argtypes = args
    L._tc_signatures = sig
    _LIBS[path] = L
    return L


def _f64(values):
    values = [float(v) for v in values]
    return (ctypes.c_double * max(len(values), 1))(*values)


def hill_alpha(eigenvalues, chi, lib=None):
    lib = lib or load_library()
    out = ctypes.c_double()
    rc = lib.tc_hill_alpha(_f64(eigenvalues), len(eigenvalues), chi, ctypes.byref(out))
    if rc != TC_OK:
        raise TcError(rc, "tc_hill_alpha")
    return out.value


def layer_benefits(alpha, params, lib=None):
    lib = lib or load_library()
    out = (ctypes.c_double * len(alpha))()
    rc = lib.tc_layer_benefits(_f64(alpha), _f64(params), len(alpha), out)
    if rc != TC_OK:
        raise TcError(rc, "tc_layer_benefits")
    return list(out)


def select_layers(nu, phi, beta, lib=None):
    """-> (value, [(start, end) or None per verifier])"""
    lib = lib or load_library()
    value = ctypes.c_double()
    s = (ctypes.c_int64 * max(len(beta), 1))()
    e = (ctypes.c_int64 * max(len(beta), 1))()
    rc = lib.tc_select_layers(len(nu), _f64(nu), _f64(phi), len(beta), _f64(beta), ctypes.byref(value), s, e)
    if rc != TC_OK:
        raise TcError(rc, "tc_select_layers")
    return value.value, [None if s[k] < 0 else (s[k], e[k]) for k in range(len(beta))]


class PairingVerifier:
    """Public verification with the pairing: host only, needs neither a GPU nor a Context."""

    def __init__(self, tau_bytes, m=TC_MAX_ORDER, lib=None):
        self.lib = lib or load_library()
        self.handle = ctypes.c_void_p()
        rc = self.lib.tc_vkp_from_trapdoor(bytes(tau_bytes), m, ctypes.byref(self.handle))
        if rc != TC_OK:
            raise TcError(rc, "tc_vkp_from_trapdoor")
        self.m = m

    def key(self, axis):
        out = ctypes.create_string_buffer(192)
        rc = self.lib.tc_vkp_get(self.handle, axis, out)
        if rc != TC_OK:
            raise TcError(rc, "tc_vkp_get")
        return out.raw

    def pairing(self, p_g1, q_g2):
        out = ctypes.create_string_buffer(576)
        rc = self.lib.tc_pairing(bytes(p_g1), bytes(q_g2), out)
        if rc != TC_OK:
            raise TcError(rc, "tc_pairing")
        return out.raw

    def verify(self, shape, commitment, kappa, y, pi):
        rc = self.lib.tc_verify_pairing(self.handle, len(shape), _u32(shape), bytes(commitment), _u32(kappa), bytes(y),
                                        b"".join(pi))
        if rc == TC_ERR_VERIFY:
            return False
        if rc != TC_OK:
            raise TcError(rc, "tc_verify_pairing")
        return True

    def verify_path(self, path, root, leaf_value, proof):
        rc = self.lib.tc_verify_path_pairing(self.handle, ctypes.byref(path), bytes(root), bytes(leaf_value),
                                             bytes(proof), len(proof))
        if rc == TC_ERR_VERIFY:
            return False
        if rc != TC_OK:
            raise TcError(rc, "tc_verify_path_pairing")
        return True

    def verify_paths(self, paths, roots, leaf_values, proofs):
        n = len(paths)
        stride = max([len(p) for p in proofs] + [1])
        buf = b"".join(p + bytes(stride - len(p)) for p in proofs)
        lens = (ctypes.c_size_t * max(n, 1))(*[len(p) for p in proofs])
        arr = (tc_path * max(n, 1))(*paths)
        res = (ctypes.c_int * max(n, 1))()
        rc = self.lib.tc_verify_paths_pairing_batch(self.handle, n, arr, b"".join(roots), b"".join(leaf_values), buf,
                                                    stride, lens, res)
        if rc != TC_OK:
            raise TcError(rc, "tc_verify_paths_pairing_batch")
        return [res[i] == TC_OK for i in range(n)]

    def close(self):
        if self.handle:
            self.lib.tc_vkp_destroy(self.handle)
            self.handle = None


def _u32(values):
    values = [int(v) for v in values]
    return (ctypes.c_uint32 * max(len(values), 1))(*values)


def _ptr(x):
    """Device pointer of a torch tensor, address of a numpy array (host-emulation tests) or an int."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return ctypes.c_void_p(x.data_ptr())
    if hasattr(x, "ctypes"):
        return ctypes.c_void_p(x.ctypes.data)
    return ctypes.c_void_p(int(x))


class Srs:
    def __init__(self, ctx, handle, shape, flags):
        self.ctx, self.handle, self.shape, self.flags = ctx, handle, tuple(shape), flags

    def size(self, first_axis=0):
        return int(self.ctx.lib.tc_srs_size(self.handle, first_axis))

    def point(self, index, first_axis=0):
        out = ctypes.create_string_buffer(96)
        self.ctx._check(self.ctx.lib.tc_srs_get_point(self.ctx.handle, self.handle, first_axis, index, out))
        return out.raw

    def export(self):
        """The SRS as the bytes of its flat file."""
        n = ctypes.c_size_t(0)
        self.ctx._check(self.ctx.lib.tc_srs_export(self.ctx.handle, self.handle, None, ctypes.byref(n)))
        buf = ctypes.create_string_buffer(n.value)
        self.ctx._check(self.ctx.lib.tc_srs_export(self.ctx.handle, self.handle, buf, ctypes.byref(n)))
        return buf.raw[: n.value]

    def close(self):
        if self.handle:
            self.ctx.lib.tc_srs_destroy(self.handle)
            self.handle = None


class Tree:
    def __init__(self, ctx, handle, desc_keepalive, grid, node_shape, leaf_kind, leaf_shapes=None):
        self.ctx, self.handle, self._keep = ctx, handle, desc_keepalive
        self.grid, self.node_shape, self.leaf_kind, self.leaf_shapes = tuple(grid), tuple(node_shape), leaf_kind, leaf_shapes

    @property
    def root(self):
        out = ctypes.create_string_buffer(96)
        self.ctx._check(self.ctx.lib.tc_terkle_root(self.handle, out))
        return out.raw

    @property
    def levels(self):
        return int(self.ctx.lib.tc_terkle_levels(self.handle))

    def level_info(self, level):
        grid = (ctypes.c_uint32 * TC_MAX_ORDER)()
        n = ctypes.c_uint64()
        self.ctx._check(self.ctx.lib.tc_terkle_level_info(self.handle, level, grid, ctypes.byref(n)))
        return tuple(grid[: len(self.grid)]), int(n.value)

    def node(self, level, index):
        out = ctypes.create_string_buffer(96)
        self.ctx._check(self.ctx.lib.tc_terkle_node(self.ctx.handle, self.handle, level, index, out))
        return out.raw

    def path(self, leaf_index, inner_index=None):
        return self.ctx.path_from_grid(self.grid, self.node_shape, self.leaf_kind, leaf_index,
                                       None if inner_index is None else self._leaf_shape(leaf_index), inner_index)

    def _leaf_shape(self, leaf_index):
        flat = 0
        for i, g in zip(leaf_index, self.grid):
            flat = flat * g + int(i)
        return self.leaf_shapes[flat]

    def open(self, leaf_index, inner_index=None):
        (proof,) = self.open_batch([leaf_index], None if inner_index is None else [inner_index])
        return proof

    def open_batch(self, leaf_indices, inner_indices=None, stride=8192):
        count = len(leaf_indices)
        flat_leaf = [int(v) for li in leaf_indices for v in li]
        flat_inner = [int(v) for ii in (inner_indices or []) for v in ii]
        buf = ctypes.create_string_buffer(stride * max(count, 1))
        lens = (ctypes.c_size_t * max(count, 1))()
        self.ctx._check(self.ctx.lib.tc_terkle_open_batch(
            self.ctx.handle, self.handle, count, _u32(flat_leaf), _u32(flat_inner) if inner_indices else None,
            buf, stride, lens))
        return [buf.raw[i * stride : i * stride + lens[i]] for i in range(count)]

    def export(self):
        """Every node commitment of the tree as the bytes of its flat file."""
        n = ctypes.c_size_t(0)
        self.ctx._check(self.ctx.lib.tc_terkle_export(self.ctx.handle, self.handle, None, ctypes.byref(n)))
        buf = ctypes.create_string_buffer(n.value)
        self.ctx._check(self.ctx.lib.tc_terkle_export(self.ctx.handle, self.handle, buf, ctypes.byref(n)))
        return buf.raw[: n.value]

    def update(self, leaf_index, delta, inner_index=None):
        """One entry changed by `delta` (the caller updates its own buffer): recompute the path and the root."""
        self.ctx._check(self.ctx.lib.tc_terkle_update(self.ctx.handle, self.handle, _u32(leaf_index),
                                                      _u32(inner_index) if inner_index is not None else None, int(delta)))

    def close(self):
        if self.handle:
            self.ctx.lib.tc_tree_destroy(self.handle)
            self.handle = None


class Context:
    """One GPU context.  `stream` is a raw hipStream_t (int) or None for the default stream."""

    def __init__(self, device=0, stream=None, lib=None):
        self.lib = lib or load_library()
        h = ctypes.c_void_p()
        rc = self.lib.tc_ctx_create(ctypes.byref(h), int(device), ctypes.c_void_p(stream) if stream else None)
        if rc != TC_OK:
            raise TcError(rc, "tc_ctx_create failed (is a GPU visible?)")
        self.handle = h
        self._vk = {}

    def _check(self, rc):
        if rc != TC_OK:
            raise TcError(rc, self.lib.tc_last_error(self.handle).decode())

    def sync(self):
        self._check(self.lib.tc_ctx_sync(self.handle))

    def profile(self, enable=True):
        self._check(self.lib.tc_ctx_profile(self.handle, 1 if enable else 0))

    def profile_read(self, kind):
        ms, n = ctypes.c_double(), ctypes.c_uint64()
        self._check(self.lib.tc_ctx_profile_read(self.handle, kind, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, int(n.value)

    def profile_units(self, kind):
        units = ctypes.c_uint64()
        self._check(self.lib.tc_ctx_profile_units(self.handle, kind, ctypes.byref(units)))
        return int(units.value)

    def set_option(self, option, value):
        self._check(self.lib.tc_ctx_set_option(self.handle, option, int(value)))

    def get_option(self, option):
        v = ctypes.c_int64()
        rc = self.lib.tc_ctx_get_option(self.handle, option, ctypes.byref(v))
        if rc != TC_OK:
            raise TcError(rc, "bad option")
        return int(v.value)

    def field_op(self, op, a, b, n, out):
        self._check(self.lib.tc_ctx_field_op(self.handle, op, _ptr(a), _ptr(b), n, _ptr(out)))

    def alu_rate(self, kind, waves_per_simd):
        """multiply-adds/s (kinds 0, 1) or Fp products/s (kinds 2, 3) with that many waves on every SIMD"""
        out = ctypes.c_double()
        self._check(self.lib.tc_ctx_alu_rate(self.handle, kind, waves_per_simd, ctypes.byref(out)))
        return out.value

    def close(self):
        for vk in self._vk.values():
            self.lib.tc_vk_destroy(vk)
        self._vk = {}
        if self.handle:
            self.lib.tc_ctx_destroy(self.handle)
            self.handle = None

    # -- Setup ---------------------------------------------------------------------------
    def setup_from_trapdoor(self, tau_bytes, shape, flags=0):
        h = ctypes.c_void_p()
        m = len(shape)
        self._check(self.lib.tc_setup_from_trapdoor(self.handle, bytes(tau_bytes), m, _u32(shape), flags, ctypes.byref(h)))
        return Srs(self, h, shape, flags)

    def srs_import(self, data):
        """An SRS from the bytes that Srs.export wrote (shape and flags come from the file)."""
        h = ctypes.c_void_p()
        data = bytes(data)
        self._check(self.lib.tc_srs_import(self.handle, data, len(data), ctypes.byref(h)))
        m = int.from_bytes(data[24:28], "little")
        shape = tuple(int.from_bytes(data[28 + 4 * j : 32 + 4 * j], "little") for j in range(m))
        return Srs(self, h, shape, int.from_bytes(data[20:24], "little"))

    # -- encode / commit / open ------------------------------------------------------------
    def encode_tensor(self, src, src_dtype, n, inv_scale, dst):
        self._check(self.lib.tc_encode_tensor(self.handle, _ptr(src), src_dtype, n, float(inv_scale), _ptr(dst)))

    def quant_scale(self, src, n, inv_scale_out):
        """inv_scale_out: device buffer of one float32 that receives 32767 / max|x| over the n fp16 values of src."""
        self._check(self.lib.tc_quant_scale(self.handle, _ptr(src), n, _ptr(inv_scale_out)))

    def encode_tensor_scaled(self, src, src_dtype, n, inv_scale_dev, dst):
        self._check(self.lib.tc_encode_tensor_scaled(self.handle, _ptr(src), src_dtype, n, _ptr(inv_scale_dev), _ptr(dst)))

    def encode_batch_scaled(self, srcs, ns, inv_scales_dev, dsts):
        """Scale and quantisation of several fp16 tensors in shared launches; inv_scales_dev: len(srcs) float32 on the device."""
        k = len(srcs)
        a_src = (ctypes.c_void_p * k)(*[_ptr(x).value for x in srcs])
        a_dst = (ctypes.c_void_p * k)(*[_ptr(x).value for x in dsts])
        a_n = (ctypes.c_size_t * k)(*[int(v) for v in ns])
        self._check(self.lib.tc_encode_batch_scaled(self.handle, k, a_src, a_n, _ptr(inv_scales_dev), a_dst))

    def commit(self, srs, scalars, dtype):
        out = ctypes.create_string_buffer(96)
        self._check(self.lib.tc_commit(self.handle, srs.handle, _ptr(scalars), dtype, out))
        return out.raw

    def commit_batch(self, srs_list, scalars_list, dtypes):
        n = len(srs_list)
        out = ctypes.create_string_buffer(96 * max(n, 1))
        a = (ctypes.c_void_p * max(n, 1))(*[s.handle for s in srs_list])
        b = (ctypes.c_void_p * max(n, 1))(*[_ptr(s) for s in scalars_list])
        c = (ctypes.c_int * max(n, 1))(*dtypes)
        self._check(self.lib.tc_commit_batch(self.handle, n, a, b, c, out))
        return [out.raw[96 * i : 96 * (i + 1)] for i in range(n)]

    def commit_static(self, srs, scalars, dtype, out):
        """The commitment without any allocation; `out` is a device buffer of 96 bytes, written asynchronously."""
        self._check(self.lib.tc_commit_static(self.handle, srs.handle, _ptr(scalars), dtype, _ptr(out)))

    def alloc_calls(self):
        return int(self.lib.tc_alloc_calls())

    def open(self, srs, scalars, dtype, kappa):
        y = ctypes.create_string_buffer(32)
        pi = ctypes.create_string_buffer(96 * len(srs.shape))
        self._check(self.lib.tc_open(self.handle, srs.handle, _ptr(scalars), dtype, _u32(kappa), y, pi))
        return y.raw, [pi.raw[96 * i : 96 * (i + 1)] for i in range(len(srs.shape))]

    # -- coefficient route -----------------------------------------------------------------------
    def interpolate(self, shape, scalars, dtype, coeffs_out):
        self._check(self.lib.tc_interpolate(self.handle, len(shape), _u32(shape), _ptr(scalars), dtype, _ptr(coeffs_out)))

    def interpolate_form(self, shape, scalars, dtype, form, coeffs_out):
        self._check(self.lib.tc_interpolate_form(self.handle, len(shape), _u32(shape), _ptr(scalars), dtype, form, _ptr(coeffs_out)))

    def divide_by_linear(self, shape, coeffs, axis, kappa_axis, quotient_out, remainder_out):
        self._check(self.lib.tc_divide_by_linear(self.handle, len(shape), _u32(shape), _ptr(coeffs), axis, kappa_axis,
                                                 _ptr(quotient_out), _ptr(remainder_out)))

    # -- verify ------------------------------------------------------------------------------
    def vk_from_trapdoor(self, tau_bytes, m=TC_MAX_ORDER):
        key = (bytes(tau_bytes), m)
        if key not in self._vk:
            h = ctypes.c_void_p()
            rc = self.lib.tc_vk_from_trapdoor(bytes(tau_bytes), m, ctypes.byref(h))
            if rc != TC_OK:
                raise TcError(rc, "tc_vk_from_trapdoor")
            self._vk[key] = h
        return self._vk[key]

    def verify(self, vk, shape, commitment, kappa, y, pi):
        rc = self.lib.tc_verify(self.handle, vk, len(shape), _u32(shape), bytes(commitment), _u32(kappa), bytes(y),
                                b"".join(pi))
        if rc == TC_ERR_VERIFY:
            return False
        self._check(rc)
        return True

    # -- Terkle ------------------------------------------------------------------------------
    def _tree(self, d, keep, grid, node_shape, leaf_kind, leaf_shapes, file_bytes):
        """tc_terkle_build, or tc_terkle_import when the bytes of an exported tree are given."""
        h = ctypes.c_void_p()
        if file_bytes is None:
            self._check(self.lib.tc_terkle_build(self.handle, ctypes.byref(d), ctypes.byref(h)))
        else:
            file_bytes = bytes(file_bytes)
            self._check(self.lib.tc_terkle_import(self.handle, ctypes.byref(d), file_bytes, len(file_bytes), ctypes.byref(h)))
        return Tree(self, h, keep, grid, node_shape, leaf_kind, leaf_shapes)

    def terkle_build_entries(self, node_srs, payload, dtype, grid, node_shape, from_file=None):
        d = tc_tree_desc()
        d.m = len(grid)
        for j, (g, s) in enumerate(zip(grid, node_shape)):
            d.grid[j], d.node_shape[j] = int(g), int(s)
        d.node_srs = node_srs.handle
        d.leaf_kind = TC_LEAF_ENTRIES
        d.d_payload = _ptr(payload)
        d.dtype = dtype
        return self._tree(d, (d, payload, node_srs), grid, node_shape, TC_LEAF_ENTRIES, None, from_file)

    def terkle_build_tensors(self, node_srs, leaf_srs, leaf_scalars, leaf_dtypes, grid, node_shape, from_file=None):
        n = len(leaf_srs)
        d = tc_tree_desc()
        d.m = len(grid)
        for j, (g, s) in enumerate(zip(grid, node_shape)):
            d.grid[j], d.node_shape[j] = int(g), int(s)
        d.node_srs = node_srs.handle
        d.leaf_kind = TC_LEAF_TENSORS
        a = (ctypes.c_void_p * n)(*[s.handle for s in leaf_srs])
        b = (ctypes.c_void_p * n)(*[_ptr(s) for s in leaf_scalars])
        c = (ctypes.c_int * n)(*leaf_dtypes)
        d.leaf_srs, d.d_leaf_scalars, d.leaf_dtype = a, b, c
        return self._tree(d, (d, a, b, c, leaf_scalars, leaf_srs, node_srs), grid, node_shape, TC_LEAF_TENSORS,
                          [s.shape for s in leaf_srs], from_file)

    def path_from_grid(self, grid, node_shape, leaf_kind, leaf_index, inner_shape=None, inner_index=None):
        p = tc_path()
        rc = self.lib.tc_path_from_grid(len(grid), _u32(grid), _u32(node_shape), leaf_kind, _u32(leaf_index),
                                        len(inner_shape) if inner_shape else 0,
                                        _u32(inner_shape) if inner_shape else None,
                                        _u32(inner_index) if inner_index is not None else None, ctypes.byref(p))
        if rc != TC_OK:
            raise TcError(rc, "tc_path_from_grid")
        return p

    def verify_path(self, vk, path, root, leaf_value, proof):
        rc = self.lib.tc_verify_path(self.handle, vk, ctypes.byref(path), bytes(root), bytes(leaf_value), bytes(proof),
                                     len(proof))
        if rc == TC_ERR_VERIFY:
            return False
        self._check(rc)
        return True

    def verify_paths_batch(self, vk, paths, roots, leaf_values, proofs):
        n = len(paths)
        stride = max([len(p) for p in proofs] + [1])
        buf = b"".join(p + bytes(stride - len(p)) for p in proofs)
        lens = (ctypes.c_size_t * max(n, 1))(*[len(p) for p in proofs])
        arr = (tc_path * max(n, 1))(*paths)
        res = (ctypes.c_int * max(n, 1))()
        self._check(self.lib.tc_verify_paths_batch(self.handle, vk, n, arr, b"".join(roots), b"".join(leaf_values), buf,
                                                   stride, lens, res))
        return [res[i] == TC_OK for i in range(n)]
