"""ctypes binding of the C ABI declared in include/cfdecode.h.

Argument marshalling only: every step of the decode block runs inside the HIP
library.  There is no fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("CFDECODE_LIB") or os.path.join(_PKG, "libcfdecode.so")   # override: A/B builds
_lib = None

EXPORTED_SYMBOLS = ("cf_create", "cf_destroy", "cf_decode_block", "cf_decode_block_static", "cf_decode_block_packed", "cf_decode_layer", "cf_decode_layer_rows",
                    "cf_decode_stack",
                    "cf_pack_weights",
                    "cf_packed_sizes", "cf_status", "cf_debug_export",
                    "cf_set_tuning", "cf_get_plan", "cf_algorithmic_bytes", "cf_strerror", "cf_last_hip_error",
                    "cf_team_create", "cf_team_destroy", "cf_team_reduce", "cf_team_gather", "cf_team_status",
                    "cf_team_set_spin_limit",
                    "cf_mla_create", "cf_mla_destroy", "cf_mla_decode", "cf_mla_status", "cf_mla_set_spin_limit",
                    "cf_mla_algorithmic_bytes", "cf_mla_set_splits", "cf_mla_debug_export",
                    "cf_splithead_create", "cf_splithead_destroy", "cf_splithead_pack", "cf_splithead_decode",
                    "cf_splithead_status", "cf_splithead_set_spin_limit",
                    "cf_ffn_create", "cf_ffn_destroy", "cf_ffn_decode", "cf_ffn_status", "cf_ffn_set_spin_limit",
                    "cf_ffn_algorithmic_bytes")

CF_FLAG_DEBUG_EXPORT = 1


class CfConfig(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("max_batch", ctypes.c_int32), ("max_seq", ctypes.c_int32),
                ("rope_base", ctypes.c_float), ("flags", ctypes.c_int32)]


class MlaConfig(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32), ("nope_dim", ctypes.c_int32),
                ("rope_dim", ctypes.c_int32), ("kv_lora_rank", ctypes.c_int32), ("v_head_dim", ctypes.c_int32),
                ("max_batch", ctypes.c_int32), ("max_seq", ctypes.c_int32), ("rope_base", ctypes.c_float)]


class FfnConfig(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("max_batch", ctypes.c_int32),
                ("activation", ctypes.c_int32)]


FFN_SILU = 0
FFN_GELU = 1


class CfError(RuntimeError):
    def __init__(self, code, msg, hip=0):
        super().__init__("cfdecode error %d (%s)%s" % (code, msg, " hip=%d" % hip if hip else ""))
        self.code = code


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libcfdecode.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError("%s not built: run `python -c 'import __graft_entry__ as g; g.build()'`" % _LIB_PATH)
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        lib.cf_create.argtypes = [ctypes.POINTER(CfConfig), ctypes.POINTER(vp)]
        lib.cf_destroy.argtypes = [vp]
        lib.cf_decode_block.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, vp, vp]
        lib.cf_decode_block_packed.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, vp, vp]
        lib.cf_decode_block_static.argtypes = [ctypes.POINTER(CfConfig), i32, vp, vp, vp, vp, vp, i32, vp, vp]
        lib.cf_decode_block_static.restype = ctypes.c_int
        lib.cf_decode_layer.argtypes = [vp, i32, vp, vp, ctypes.c_float, i32, i32, vp, vp, vp, vp, i32, vp, vp]
        lib.cf_decode_layer_rows.argtypes = [vp, i32, vp, vp, ctypes.c_float, i32, i32, vp, vp, vp, vp, vp, i32, vp, vp]
        lib.cf_pack_weights.argtypes = [vp, vp, vp, vp, vp, vp]
        lib.cf_packed_sizes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
        lib.cf_status.argtypes = [vp, vp]
        lib.cf_debug_export.argtypes = [vp, i32, vp, ctypes.c_size_t, vp]
        lib.cf_set_tuning.argtypes = [vp, i32, i32, i32, i32]
        lib.cf_get_plan.argtypes = [vp, ctypes.POINTER(i32), i32]
        lib.cf_algorithmic_bytes.argtypes = [ctypes.POINTER(CfConfig), i32, i32]
        lib.cf_algorithmic_bytes.restype = ctypes.c_int64
        lib.cf_strerror.argtypes = [ctypes.c_int]
        lib.cf_strerror.restype = ctypes.c_char_p
        lib.cf_last_hip_error.argtypes = [vp]
        lib.cf_team_create.argtypes = [i32, ctypes.c_size_t, ctypes.POINTER(vp)]
        lib.cf_team_destroy.argtypes = [vp]
        lib.cf_team_reduce.argtypes = [vp, i32, i32, i32, vp, vp, ctypes.c_size_t, i32, vp]
        lib.cf_team_gather.argtypes = [vp, i32, i32, vp, vp, ctypes.c_size_t, i32, vp]
        lib.cf_team_status.argtypes = [vp, vp]
        lib.cf_team_set_spin_limit.argtypes = [vp, i32]
        lib.cf_mla_create.argtypes = [ctypes.POINTER(MlaConfig), ctypes.POINTER(vp)]
        lib.cf_mla_destroy.argtypes = [vp]
        lib.cf_mla_decode.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
        lib.cf_mla_status.argtypes = [vp, vp]
        lib.cf_mla_set_spin_limit.argtypes = [vp, i32]
        lib.cf_mla_set_splits.argtypes = [vp, i32]
        lib.cf_mla_debug_export.argtypes = [vp, i32, vp, ctypes.c_size_t, vp]
        lib.cf_mla_algorithmic_bytes.argtypes = [ctypes.POINTER(MlaConfig), i32, i32]
        lib.cf_mla_algorithmic_bytes.restype = ctypes.c_int64
        lib.cf_splithead_create.argtypes = [ctypes.POINTER(CfConfig), i32, ctypes.POINTER(vp)]
        lib.cf_splithead_destroy.argtypes = [vp]
        lib.cf_splithead_pack.argtypes = [vp, vp, vp, vp]
        lib.cf_splithead_decode.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, vp]
        lib.cf_splithead_status.argtypes = [vp, vp]
        lib.cf_splithead_set_spin_limit.argtypes = [vp, i32]
        for name in ("cf_splithead_create", "cf_splithead_destroy", "cf_splithead_pack", "cf_splithead_decode",
                     "cf_splithead_status", "cf_splithead_set_spin_limit"):
            getattr(lib, name).restype = ctypes.c_int
        for name in ("cf_team_create", "cf_team_destroy", "cf_team_reduce", "cf_team_gather", "cf_team_status",
                     "cf_team_set_spin_limit",
                    "cf_mla_create", "cf_mla_destroy", "cf_mla_decode", "cf_mla_status", "cf_mla_set_spin_limit",
                    "cf_mla_set_splits", "cf_mla_debug_export"):
            getattr(lib, name).restype = ctypes.c_int
        lib.cf_ffn_create.argtypes = [ctypes.POINTER(FfnConfig), ctypes.POINTER(vp)]
        lib.cf_ffn_destroy.argtypes = [vp]
        lib.cf_ffn_decode.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
        lib.cf_ffn_status.argtypes = [vp, vp]
        lib.cf_ffn_set_spin_limit.argtypes = [vp, i32]
        lib.cf_ffn_algorithmic_bytes.argtypes = [ctypes.POINTER(FfnConfig), i32]
        lib.cf_ffn_algorithmic_bytes.restype = ctypes.c_int64
        for name in ("cf_ffn_create", "cf_ffn_destroy", "cf_ffn_decode", "cf_ffn_status", "cf_ffn_set_spin_limit"):
            getattr(lib, name).restype = ctypes.c_int
        lib.cf_decode_stack.argtypes = [vp, i32, i32, vp, ctypes.POINTER(vp), ctypes.c_float, i32, i32, ctypes.POINTER(vp),
                                        ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), i32, vp, vp]
        for name in ("cf_create", "cf_destroy", "cf_decode_block", "cf_decode_block_packed", "cf_decode_layer", "cf_decode_layer_rows",
                     "cf_decode_stack",
                    "cf_pack_weights",
                     "cf_packed_sizes", "cf_status", "cf_debug_export",
                     "cf_set_tuning", "cf_get_plan", "cf_last_hip_error"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def algorithmic_bytes(cfg: CfConfig, batch: int, pos: int) -> int:
    return int(load_library().cf_algorithmic_bytes(ctypes.byref(cfg), batch, pos))


def decode_block_static(cfg: CfConfig, batch, x, w_qkv, w_o, k_cache, v_cache, pos, out, stream=0):
    """cf_decode_block_static: the decode step without a handle, on the library's fixed scratch array."""
    lib = load_library()
    rc = lib.cf_decode_block_static(ctypes.byref(cfg), batch, x, w_qkv, w_o, k_cache, v_cache, pos, out, stream)
    if rc != 0:
        raise CfError(rc, lib.cf_strerror(rc).decode())


PLAN_FIELDS = ("workgroups", "team_size", "k_splits", "rows_per_split", "kv_splits", "tokens_per_split",
               "out_col_blocks", "out_cols_per_block", "out_row_splits", "lds_bytes")


class DecodeBlock:
    """One handle of the library.  Tensors are passed as raw device addresses
    (e.g. torch_tensor.data_ptr()); `stream` is a hipStream_t value."""

    def __init__(self, d_model, n_q_heads, n_kv_heads, head_dim, max_batch, max_seq, rope_base, debug=False):
        self._lib = load_library()
        self.cfg = CfConfig(d_model, n_q_heads, n_kv_heads, head_dim, max_batch, max_seq, rope_base,
                            CF_FLAG_DEBUG_EXPORT if debug else 0)
        self._h = ctypes.c_void_p()
        self._check(self._lib.cf_create(ctypes.byref(self.cfg), ctypes.byref(self._h)))

    def _check(self, rc):
        if rc != 0:
            hip = self._lib.cf_last_hip_error(self._h) if self._h else 0
            raise CfError(rc, self._lib.cf_strerror(rc).decode(), hip)

    def decode_block(self, batch, x, w_qkv, w_o, k_cache, v_cache, pos, out, stream=0):
        rc = self._lib.cf_decode_block(self._h, batch, x, w_qkv, w_o, k_cache, v_cache, pos, out, stream)
        if rc != 0:
            self._check(rc)

    def packed_sizes(self):
        a, b = ctypes.c_size_t(), ctypes.c_size_t()
        self._check(self._lib.cf_packed_sizes(self._h, ctypes.byref(a), ctypes.byref(b)))
        return int(a.value), int(b.value)

    def pack_weights(self, w_qkv, w_o, w_qkv_packed, w_o_packed, stream=0):
        self._check(self._lib.cf_pack_weights(self._h, w_qkv, w_o, w_qkv_packed, w_o_packed, stream))

    def decode_block_packed(self, batch, x, w_qkv_packed, w_o_packed, k_cache, v_cache, pos, out, stream=0):
        rc = self._lib.cf_decode_block_packed(self._h, batch, x, w_qkv_packed, w_o_packed, k_cache, v_cache, pos,
                                              out, stream)
        if rc != 0:
            self._check(rc)

    def decode_layer(self, batch, x, norm_weight, eps, residual, packed, w_qkv, w_o, k_cache, v_cache, pos, out, stream=0):
        rc = self._lib.cf_decode_layer(self._h, batch, x, norm_weight, eps, int(residual), int(packed), w_qkv, w_o,
                                       k_cache, v_cache, pos, out, stream)
        if rc != 0:
            self._check(rc)

    def decode_layer_rows(self, batch, x, norm_weight, eps, residual, packed, w_qkv, w_o, k_cache, v_cache, row_pos,
                          max_pos, out, stream=0):
        rc = self._lib.cf_decode_layer_rows(self._h, batch, x, norm_weight, eps, int(residual), int(packed), w_qkv, w_o,
                                            k_cache, v_cache, row_pos, max_pos, out, stream)
        if rc != 0:
            self._check(rc)

    def decode_layer_rows_rc(self, batch, x, norm_weight, eps, residual, packed, w_qkv, w_o, k_cache, v_cache, row_pos,
                             max_pos, out, stream=0) -> int:
        return int(self._lib.cf_decode_layer_rows(self._h, batch, x, norm_weight, eps, int(residual), int(packed), w_qkv,
                                                  w_o, k_cache, v_cache, row_pos, max_pos, out, stream))

    def decode_layer_rc(self, batch, x, norm_weight, eps, residual, packed, w_qkv, w_o, k_cache, v_cache, pos, out,
                        stream=0) -> int:
        return int(self._lib.cf_decode_layer(self._h, batch, x, norm_weight, eps, int(residual), int(packed), w_qkv, w_o,
                                             k_cache, v_cache, pos, out, stream))

    def decode_block_rc(self, batch, x, w_qkv, w_o, k_cache, v_cache, pos, out, stream=0) -> int:
        """Same call, returning the library's code instead of raising (for error-path tests)."""
        return int(self._lib.cf_decode_block(self._h, batch, x, w_qkv, w_o, k_cache, v_cache, pos, out, stream))

    def status(self, stream=0):
        self._check(self._lib.cf_status(self._h, stream))

    def decode_stack_rc(self, batch, x, norm_weights, eps, residual, packed, w_qkv, w_o, k_cache, v_cache, pos, out,
                        stream=0) -> int:
        """w_qkv, w_o, k_cache, v_cache: sequences of device addresses, one per layer; norm_weights: such a sequence
        or None."""
        n = len(w_qkv)
        assert len(w_o) == n and len(k_cache) == n and len(v_cache) == n and (norm_weights is None or len(norm_weights) == n)
        arr = lambda seq: (ctypes.c_void_p * n)(*[ctypes.c_void_p(int(a)) for a in seq])
        nw = arr(norm_weights) if norm_weights is not None else None
        return int(self._lib.cf_decode_stack(self._h, n, batch, x, nw, float(eps), int(residual), int(packed), arr(w_qkv),
                                             arr(w_o), arr(k_cache), arr(v_cache), pos, out, stream))

    def decode_stack(self, *args, **kw):
        rc = self.decode_stack_rc(*args, **kw)
        if rc != 0:
            self._check(rc)

    def set_tuning(self, workgroups=0, k_splits=0, kv_splits=0, spin_limit_us=0):
        self._check(self._lib.cf_set_tuning(self._h, workgroups, k_splits, kv_splits, spin_limit_us))

    def plan(self) -> dict:
        arr = (ctypes.c_int32 * len(PLAN_FIELDS))()
        self._check(self._lib.cf_get_plan(self._h, arr, len(PLAN_FIELDS)))
        return dict(zip(PLAN_FIELDS, list(arr)))

    def debug_export(self, what, host_array, stream=0):
        """host_array: contiguous float32 numpy array of shape [batch, n_q_heads, head_dim]."""
        self._check(self._lib.cf_debug_export(self._h, what, host_array.ctypes.data, host_array.nbytes, stream))

    def close(self):
        if self._h:
            self._lib.cf_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


TEAM_SUM, TEAM_MAX = 0, 1
TEAM_ROUNDS, TEAM_TWO_KERNELS, TEAM_DIRECT, TEAM_TWO_HOPS = 0, 1, 2, 3     # how the ranks exchange their data (argument `mode`)


class TeamCollectives:
    """Handle of the team-collective entry points (cf_team_*).  Tensors are raw device addresses of fp32 data."""

    def __init__(self, max_ranks, max_elems):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        self._check(self._lib.cf_team_create(max_ranks, max_elems, ctypes.byref(self._h)))

    def _check(self, rc):
        if rc != 0:
            raise CfError(rc, self._lib.cf_strerror(rc).decode())

    def reduce(self, teams, team_size, op, src, dst, elems, mode=TEAM_ROUNDS, stream=0):
        self._check(self._lib.cf_team_reduce(self._h, teams, team_size, op, src, dst, elems, int(mode), stream))

    def reduce_rc(self, teams, team_size, op, src, dst, elems, mode=TEAM_ROUNDS, stream=0) -> int:
        return int(self._lib.cf_team_reduce(self._h, teams, team_size, op, src, dst, elems, int(mode), stream))

    def gather(self, teams, team_size, src, dst, elems, mode=TEAM_ROUNDS, stream=0):
        self._check(self._lib.cf_team_gather(self._h, teams, team_size, src, dst, elems, int(mode), stream))

    def gather_rc(self, teams, team_size, src, dst, elems, mode=TEAM_ROUNDS, stream=0) -> int:
        return int(self._lib.cf_team_gather(self._h, teams, team_size, src, dst, elems, int(mode), stream))

    def status(self, stream=0):
        self._check(self._lib.cf_team_status(self._h, stream))

    def set_spin_limit(self, us):
        self._check(self._lib.cf_team_set_spin_limit(self._h, us))

    def close(self):
        if self._h:
            self._lib.cf_team_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class MlaBlock:
    """Handle of the fused MLA decode block (cf_mla_*).  Tensors are raw device addresses of fp16 data."""

    def __init__(self, d_model, n_heads, nope_dim, rope_dim, kv_lora_rank, v_head_dim, max_batch, max_seq, rope_base):
        self._lib = load_library()
        self.cfg = MlaConfig(d_model, n_heads, nope_dim, rope_dim, kv_lora_rank, v_head_dim, max_batch, max_seq, rope_base)
        self._h = ctypes.c_void_p()
        self._check(self._lib.cf_mla_create(ctypes.byref(self.cfg), ctypes.byref(self._h)))

    def _check(self, rc):
        if rc != 0:
            raise CfError(rc, self._lib.cf_strerror(rc).decode())

    def decode(self, batch, x, w_q, w_kv, w_up, w_down, w_o, kv_cache, pos, out, stream=0):
        rc = self._lib.cf_mla_decode(self._h, batch, x, w_q, w_kv, w_up, w_down, w_o, kv_cache, pos, out, stream)
        if rc != 0:
            self._check(rc)

    def decode_rc(self, batch, x, w_q, w_kv, w_up, w_down, w_o, kv_cache, pos, out, stream=0) -> int:
        return int(self._lib.cf_mla_decode(self._h, batch, x, w_q, w_kv, w_up, w_down, w_o, kv_cache, pos, out, stream))

    def status(self, stream=0):
        self._check(self._lib.cf_mla_status(self._h, stream))

    def algorithmic_bytes(self, batch, pos) -> int:
        return int(self._lib.cf_mla_algorithmic_bytes(ctypes.byref(self.cfg), batch, pos))

    def set_spin_limit(self, us):
        self._check(self._lib.cf_mla_set_spin_limit(self._h, us))

    def set_splits(self, max_splits):
        self._check(self._lib.cf_mla_set_splits(self._h, max_splits))

    def debug_export(self, what, host_array, stream=0):
        """what 0: q_lat, 1: q_rope, 2: z of the last call, into a C-contiguous float32 numpy array of that shape."""
        assert host_array.dtype.name == "float32" and host_array.flags["C_CONTIGUOUS"]
        self._check(self._lib.cf_mla_debug_export(self._h, what, host_array.ctypes.data, host_array.nbytes, stream))

    def close(self):
        if self._h:
            self._lib.cf_mla_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class FfnBlock:
    """Handle of the fused feed-forward block (cf_ffn_*).  Tensors are raw device addresses of fp16 data."""

    def __init__(self, d_model, d_ff, max_batch, activation=FFN_SILU):
        self._lib = load_library()
        self.cfg = FfnConfig(d_model, d_ff, max_batch, activation)
        self._h = ctypes.c_void_p()
        self._check(self._lib.cf_ffn_create(ctypes.byref(self.cfg), ctypes.byref(self._h)))

    def _check(self, rc):
        if rc != 0:
            raise CfError(rc, self._lib.cf_strerror(rc).decode())

    def decode(self, batch, z, w1, w2, w3, out, stream=0):
        rc = self._lib.cf_ffn_decode(self._h, batch, z, w1, w2, w3, out, stream)
        if rc != 0:
            self._check(rc)

    def decode_rc(self, batch, z, w1, w2, w3, out, stream=0) -> int:
        return int(self._lib.cf_ffn_decode(self._h, batch, z, w1, w2, w3, out, stream))

    def status(self, stream=0):
        self._check(self._lib.cf_ffn_status(self._h, stream))

    def algorithmic_bytes(self, batch) -> int:
        return int(self._lib.cf_ffn_algorithmic_bytes(ctypes.byref(self.cfg), batch))

    def set_spin_limit(self, us):
        self._check(self._lib.cf_ffn_set_spin_limit(self._h, us))

    def close(self):
        if self._h:
            self._lib.cf_ffn_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class SplitHeadBlock:
    """Handle of the SplitHead variant of the decode block (cf_splithead_*): batch 1, one KV head per query head.
    Tensors are raw device addresses of fp16 data."""

    def __init__(self, d_model, n_heads, head_dim, max_seq, rope_base, team_size):
        self._lib = load_library()
        self.cfg = CfConfig(d_model, n_heads, n_heads, head_dim, 1, max_seq, rope_base, 0)
        self.team_size = int(team_size)
        self._h = ctypes.c_void_p()
        self._check(self._lib.cf_splithead_create(ctypes.byref(self.cfg), self.team_size, ctypes.byref(self._h)))

    def _check(self, rc):
        if rc != 0:
            raise CfError(rc, self._lib.cf_strerror(rc).decode())

    def pack(self, w_qkv, w_qkv_members, stream=0):
        self._check(self._lib.cf_splithead_pack(self._h, w_qkv, w_qkv_members, stream))

    def decode(self, x, w_qkv_members, w_o, k_cache, v_cache, pos, out, stream=0):
        rc = self._lib.cf_splithead_decode(self._h, x, w_qkv_members, w_o, k_cache, v_cache, pos, out, stream)
        if rc != 0:
            self._check(rc)

    def decode_rc(self, x, w_qkv_members, w_o, k_cache, v_cache, pos, out, stream=0) -> int:
        return int(self._lib.cf_splithead_decode(self._h, x, w_qkv_members, w_o, k_cache, v_cache, pos, out, stream))

    def status(self, stream=0):
        self._check(self._lib.cf_splithead_status(self._h, stream))

    def set_spin_limit(self, us):
        self._check(self._lib.cf_splithead_set_spin_limit(self._h, us))

    def close(self):
        if self._h:
            self._lib.cf_splithead_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
