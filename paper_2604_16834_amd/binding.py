"""Thin ctypes binding of the C boundary declared in ``include/ckks.h``.

Argument marshalling only: every function below has the name of the C entry point it calls and
hands it raw device pointers of PyTorch tensors (PyTorch is used for device memory and streams,
nothing else).  Polynomial data are ``torch.int64`` tensors holding the uint64 residues bit for
bit (``from_host`` / ``to_host`` convert from and to numpy ``uint64``).  There is no fallback: if
the compiled library is missing the import of this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libckks_mi355x.so")

CKKS_OK = 0
CKKS_ERR_INVALID_ARG = -1
CKKS_ERR_LEVEL_MISMATCH = -2
CKKS_ERR_UNSUPPORTED_PARAMS = -3
CKKS_ERR_WORKSPACE_TOO_SMALL = -4
CKKS_ERR_NO_KEY = -5
CKKS_ERR_HIP = -6

CKKS_OP_KEYSWITCH = 0
CKKS_OP_ROTATE = 1
CKKS_OP_RESCALE = 2
CKKS_OP_CTCT_MUL_RELIN = 3
CKKS_OP_POLY_ACT = 5

HE_CONV_ALIGN_DIRECT = 0
HE_CONV_ALIGN_FOUR_KEYS = 1
HE_CONV_DEFERRED_MODDOWN = 2
HE_CONV_DEFERRED_MERGED = 3
HE_RELAYOUT_DIRECT = 0
HE_RELAYOUT_DEFERRED = 1

EXPORTS = (
    "ckks_ctx_create", "ckks_ctx_destroy", "ckks_last_error_string", "ckks_workspace_bytes",
    "ckks_ntt_fwd", "ckks_ntt_inv", "ckks_key_load", "ckks_key_free", "ckks_galois_element",
    "ckks_keyswitch", "ckks_rotate_hoisted", "ckks_ptct_mac", "ckks_rescale", "ckks_rescale_noalloc", "ckks_ctct_mul_relin",
    "he_conv_workspace_bytes", "he_conv_batched", "he_conv_check_weights", "he_poly_act_deg7", "ckks_f64mod_probe",
    "he_accumulator_workspace_bytes", "he_accumulator_merge", "he_fc_workspace_bytes", "he_fc_batched",
    "he_relayout_workspace_bytes", "he_relayout_two_rotations", "ckks_key_expand_a", "ckks_keyset_stage", "ckks_ctx_set_overlap",
    "ckks_prof_kernel_count", "ckks_prof_kernel_name", "ckks_prof_begin", "ckks_prof_end",
)

_expect_device = "cuda"  # tensors handed to the library must live here


class CkksError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"ckks status {code}: {message}")
        self.code = code


class _Params(C.Structure):
    _fields_ = [("log_n", C.c_uint32), ("num_q", C.c_uint32), ("num_p", C.c_uint32), ("dnum", C.c_uint32),
                ("moduli", C.POINTER(C.c_uint64)), ("psi", C.POINTER(C.c_uint64))]


class _ConvDesc(C.Structure):
    _fields_ = [("c_in", C.c_uint32), ("c_out", C.c_uint32), ("height", C.c_uint32), ("width", C.c_uint32),
                ("batch", C.c_uint32), ("level", C.c_uint32), ("alignment", C.c_uint32), ("weight_bits", C.c_uint32)]


class _FcDesc(C.Structure):
    _fields_ = [("d_in", C.c_uint32), ("d_out", C.c_uint32), ("batch", C.c_uint32), ("level", C.c_uint32), ("base", C.c_uint32)]


def _bind(path: str):
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(path)
    vp, u32, i32, sz = C.c_void_p, C.c_uint32, C.c_int, C.c_size_t
    lib.ckks_ctx_create.argtypes = [C.POINTER(_Params), C.POINTER(vp)]
    lib.ckks_ctx_destroy.argtypes = [vp]
    lib.ckks_ctx_destroy.restype = None
    lib.ckks_last_error_string.argtypes = [vp]
    lib.ckks_last_error_string.restype = C.c_char_p
    lib.ckks_workspace_bytes.argtypes = [vp, i32, u32, u32]
    lib.ckks_workspace_bytes.restype = sz
    for f in (lib.ckks_ntt_fwd, lib.ckks_ntt_inv):
        f.argtypes = [vp, vp, C.POINTER(u32), u32, u32, vp]
    lib.ckks_key_load.argtypes = [vp, vp, u32, C.POINTER(vp)]
    lib.ckks_key_free.argtypes = [vp]
    lib.ckks_key_free.restype = None
    lib.ckks_galois_element.argtypes = [vp, C.c_int32]
    lib.ckks_galois_element.restype = u32
    lib.ckks_keyswitch.argtypes = [vp, vp, u32, vp, vp, vp, sz, vp]
    lib.ckks_rotate_hoisted.argtypes = [vp, vp, u32, C.POINTER(C.c_int32), u32, C.POINTER(vp), C.POINTER(vp), i32, vp, sz, vp]
    lib.ckks_ptct_mac.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), u32, u32, vp, i32, vp]
    lib.ckks_rescale.argtypes = [vp, vp, u32, vp, vp, sz, vp]
    lib.ckks_rescale_noalloc.argtypes = [vp, vp, u32, vp, vp]
    lib.ckks_ctct_mul_relin.argtypes = [vp, vp, vp, u32, vp, vp, vp, sz, vp]
    lib.he_conv_workspace_bytes.argtypes = [vp, C.POINTER(_ConvDesc)]
    lib.he_conv_workspace_bytes.restype = sz
    lib.he_conv_batched.argtypes = [vp, C.POINTER(_ConvDesc), C.POINTER(vp), C.POINTER(vp), vp, vp, C.POINTER(vp), vp, sz, vp]
    lib.he_conv_check_weights.argtypes = [vp, C.POINTER(_ConvDesc), vp, vp]
    lib.ckks_f64mod_probe.argtypes = [i32, vp, vp, vp, C.c_uint64, vp, sz, vp]
    lib.he_poly_act_deg7.argtypes = [vp, C.POINTER(vp), u32, u32, C.POINTER(C.c_int64), vp, i32, C.POINTER(vp), vp, sz, vp]
    lib.he_accumulator_workspace_bytes.argtypes = [vp, u32, u32]
    lib.he_accumulator_workspace_bytes.restype = sz
    lib.he_accumulator_merge.argtypes = [vp, C.POINTER(vp), u32, u32, u32, vp, C.POINTER(vp), vp, vp, sz, vp]
    lib.he_fc_workspace_bytes.argtypes = [vp, C.POINTER(_FcDesc)]
    lib.he_fc_workspace_bytes.restype = sz
    lib.he_fc_batched.argtypes = [vp, C.POINTER(_FcDesc), vp, vp, C.POINTER(vp), C.POINTER(vp), vp, vp, C.POINTER(vp), C.POINTER(vp),
                                  vp, vp, vp, sz, vp]
    lib.he_relayout_workspace_bytes.argtypes = [vp, u32, u32, u32, u32, u32]
    lib.he_relayout_workspace_bytes.restype = sz
    lib.he_relayout_two_rotations.argtypes = [vp, C.POINTER(vp), u32, u32, C.POINTER(C.c_int32), u32, C.POINTER(vp), C.POINTER(C.c_int32),
                                              u32, C.POINTER(vp), C.POINTER(vp), u32, C.POINTER(vp), vp, sz, vp]
    lib.ckks_ctx_set_overlap.argtypes = [vp, i32]
    lib.ckks_key_expand_a.argtypes = [vp, C.c_uint64, vp, vp]
    lib.ckks_keyset_stage.argtypes = [vp, C.POINTER(vp), C.POINTER(C.c_uint64), C.POINTER(vp), u32, vp]
    lib.ckks_prof_kernel_count.restype = u32
    lib.ckks_prof_kernel_name.argtypes = [u32]
    lib.ckks_prof_kernel_name.restype = C.c_char_p
    lib.ckks_prof_begin.argtypes = [vp, u32, u32]
    lib.ckks_prof_end.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_uint64), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
    return lib


_lib = _bind(LIB_PATH)


# --------------------------------------------------------------------------------------- helpers
def from_host(a: np.ndarray) -> torch.Tensor:
    """numpy uint64 array -> int64 tensor with the same bits on the device."""
    a = np.ascontiguousarray(a, dtype=np.uint64)
    return torch.from_numpy(a.view(np.int64)).to(_expect_device)


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().numpy().view(np.uint64)


def empty(*shape) -> torch.Tensor:
    return torch.empty(*shape, dtype=torch.int64, device=_expect_device)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if t.device.type != _expect_device or t.dtype not in (torch.int64, torch.uint64, torch.uint8, torch.float64) or not t.is_contiguous():
        raise ValueError(f"need a contiguous int64 (float64 for the self-test hook) tensor on {_expect_device}")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is not None:
        return int(stream)
    if _expect_device == "cuda":
        return torch.cuda.current_stream().cuda_stream
    return None


def _ptr_array(ptrs: Sequence[Optional[int]]):
    return (C.c_void_p * len(ptrs))(*ptrs)


class Key:
    """Handle of a caller-owned switching key (keeps the tensor alive)."""

    def __init__(self, ctx: "Context", tensor: torch.Tensor, galois_elt: int):
        self.tensor = tensor
        self.galois_elt = galois_elt
        self._ctx = ctx
        h = C.c_void_p()
        ctx._check(_lib.ckks_key_load(ctx.handle, _ptr(tensor), galois_elt, C.byref(h)))
        self.handle = h

    def __del__(self):
        try:
            _lib.ckks_key_free(self.handle)
        except Exception:
            pass


class Context:
    """Owns a ``ckks_ctx`` (immutable tables on the current device)."""

    def __init__(self, params):
        self.log_n, self.num_q, self.num_p, self.dnum = int(params.log_n), int(params.num_q), int(params.num_p), int(params.dnum)
        self.N = 1 << self.log_n
        self.M = self.num_q + self.num_p
        self.moduli = [int(q) for q in params.moduli]
        self._mods = (C.c_uint64 * len(self.moduli))(*self.moduli)
        self._psi = (C.c_uint64 * len(self.moduli))(*[int(x) for x in params.psi])
        p = _Params(self.log_n, self.num_q, self.num_p, self.dnum, self._mods, self._psi)
        h = C.c_void_p()
        rc = _lib.ckks_ctx_create(C.byref(p), C.byref(h))
        if rc != CKKS_OK:
            raise CkksError(rc, _lib.ckks_last_error_string(None).decode())
        self.handle = h
        self._ws: Optional[torch.Tensor] = None

    def __del__(self):
        try:
            _lib.ckks_ctx_destroy(self.handle)
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != CKKS_OK:
            raise CkksError(rc, _lib.ckks_last_error_string(self.handle).decode())

    def workspace(self, nbytes: int) -> torch.Tensor:
        """A cached scratch tensor of at least nbytes (grown on demand, reused across calls)."""
        if self._ws is None or self._ws.numel() * self._ws.element_size() < nbytes:
            self._ws = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=_expect_device)
        return self._ws


# ------------------------------------------------------------------ the C entry points, by name
def ckks_workspace_bytes(ctx: Context, op: int, level: int, count: int = 1) -> int:
    return int(_lib.ckks_workspace_bytes(ctx.handle, op, level, count))


def ckks_galois_element(ctx: Context, offset: int) -> int:
    return int(_lib.ckks_galois_element(ctx.handle, offset))


def ckks_key_load(ctx: Context, key: torch.Tensor, galois_elt: int) -> Key:
    return Key(ctx, key, galois_elt)


def _ntt(fn, ctx, polys, modulus_idx, batch, stream):
    n_limbs = len(modulus_idx)
    if batch is None:
        batch = polys.numel() // (n_limbs * ctx.N)
    if polys.numel() != batch * n_limbs * ctx.N:
        raise ValueError("tensor size does not match batch * n_limbs * N")
    idx = (C.c_uint32 * n_limbs)(*[int(i) for i in modulus_idx])
    ctx._check(fn(ctx.handle, _ptr(polys), idx, n_limbs, batch, _stream(stream)))
    return polys


def ckks_ntt_fwd(ctx: Context, polys: torch.Tensor, modulus_idx: Sequence[int], batch: Optional[int] = None, stream=None):
    """In place on [batch][len(modulus_idx)][N]."""
    return _ntt(_lib.ckks_ntt_fwd, ctx, polys, modulus_idx, batch, stream)


def ckks_ntt_inv(ctx: Context, polys: torch.Tensor, modulus_idx: Sequence[int], batch: Optional[int] = None, stream=None):
    return _ntt(_lib.ckks_ntt_inv, ctx, polys, modulus_idx, batch, stream)


def _ws(ctx: Context, ws: Optional[torch.Tensor], need: int) -> torch.Tensor:
    return ctx.workspace(need) if ws is None else ws


def ckks_keyswitch(ctx: Context, c: torch.Tensor, level: int, key: Key, out: Optional[torch.Tensor] = None,
                   ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if c.numel() != (level + 1) * ctx.N:
        raise ValueError("c must be [level+1][N]")
    if out is None:
        out = empty(2, level + 1, ctx.N)
    ws = _ws(ctx, ws, ckks_workspace_bytes(ctx, CKKS_OP_KEYSWITCH, level))
    ctx._check(_lib.ckks_keyswitch(ctx.handle, _ptr(c), level, key.handle if key else None, _ptr(out), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))
    return out


def ckks_rotate_hoisted(ctx: Context, ct: torch.Tensor, level: int, offsets: Sequence[int], keys: Sequence[Optional[Key]],
                        hoisted: bool = True, outs: Optional[List[torch.Tensor]] = None, ws: Optional[torch.Tensor] = None,
                        stream=None) -> List[torch.Tensor]:
    n = len(offsets)
    if ct.numel() != 2 * (level + 1) * ctx.N or len(keys) != n:
        raise ValueError("ct must be [2][level+1][N] and one key per offset")
    if outs is None:
        outs = [empty(2, level + 1, ctx.N) for _ in range(n)]
    for o in outs:
        if o.numel() != 2 * (level + 1) * ctx.N:
            raise ValueError("each output must be [2][level+1][N]")
    ws = _ws(ctx, ws, ckks_workspace_bytes(ctx, CKKS_OP_ROTATE, level, n))
    offs = (C.c_int32 * n)(*[int(r) for r in offsets])
    ks = _ptr_array([k.handle.value if k is not None else None for k in keys])
    os_ = _ptr_array([_ptr(o) for o in outs])
    ctx._check(_lib.ckks_rotate_hoisted(ctx.handle, _ptr(ct), level, offs, n, ks, os_, int(bool(hoisted)), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))
    return outs


def ckks_ptct_mac(ctx: Context, pts: Sequence[torch.Tensor], cts: Sequence[torch.Tensor], level: int,
                  acc: Optional[torch.Tensor] = None, accumulate: bool = False, stream=None) -> torch.Tensor:
    n = len(pts)
    if len(cts) != n:
        raise ValueError("one plaintext per ciphertext")
    for p_, c_ in zip(pts, cts):
        if p_.numel() != (level + 1) * ctx.N or c_.numel() != 2 * (level + 1) * ctx.N:
            raise ValueError("operands must be [level+1][N] and [2][level+1][N]")
    if acc is None:
        if accumulate:
            raise ValueError("accumulate needs an accumulator")
        acc = empty(2, level + 1, ctx.N)
    elif acc.numel() != 2 * (level + 1) * ctx.N:
        raise ValueError("acc must be [2][level+1][N]")
    pa = _ptr_array([_ptr(p_) for p_ in pts])
    ca = _ptr_array([_ptr(c_) for c_ in cts])
    ctx._check(_lib.ckks_ptct_mac(ctx.handle, pa, ca, n, level, _ptr(acc), int(bool(accumulate)), _stream(stream)))
    return acc


def ckks_rescale(ctx: Context, ct: torch.Tensor, level: int, out: Optional[torch.Tensor] = None,
                 ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if ct.numel() != 2 * (level + 1) * ctx.N:
        raise ValueError("ct must be [2][level+1][N]")
    if out is None:
        out = empty(2, max(level, 1), ctx.N)
    ws = _ws(ctx, ws, ckks_workspace_bytes(ctx, CKKS_OP_RESCALE, level))
    ctx._check(_lib.ckks_rescale(ctx.handle, _ptr(ct), level, _ptr(out), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))
    return out


def ckks_rescale_noalloc(ctx: Context, ct: torch.Tensor, level: int, out: torch.Tensor, stream=None) -> torch.Tensor:
    """ckks_rescale on the library's built-in scratch buffer: no workspace, no allocation (the caller brings `out`)."""
    if ct.numel() != 2 * (level + 1) * ctx.N or out.numel() != 2 * max(level, 1) * ctx.N:
        raise ValueError("ct must be [2][level+1][N] and out [2][level][N]")
    ctx._check(_lib.ckks_rescale_noalloc(ctx.handle, _ptr(ct), level, _ptr(out), _stream(stream)))
    return out


def ckks_ctct_mul_relin(ctx: Context, a: torch.Tensor, b: torch.Tensor, level: int, rlk: Key,
                        out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if a.numel() != 2 * (level + 1) * ctx.N or b.numel() != a.numel():
        raise ValueError("operands must be [2][level+1][N]")
    if out is None:
        out = empty(2, level + 1, ctx.N)
    ws = _ws(ctx, ws, ckks_workspace_bytes(ctx, CKKS_OP_CTCT_MUL_RELIN, level))
    ctx._check(_lib.ckks_ctct_mul_relin(ctx.handle, _ptr(a), _ptr(b), level, rlk.handle if rlk else None, _ptr(out), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))
    return out


def he_conv_workspace_bytes(ctx: Context, c_in: int, c_out: int, height: int, width: int, batch: int, level: int,
                            alignment: int = HE_CONV_ALIGN_DIRECT) -> int:
    d = _ConvDesc(c_in, c_out, height, width, batch, level, int(alignment), 0)
    return int(_lib.he_conv_workspace_bytes(ctx.handle, C.byref(d)))


def conv_weight_bits(w_int) -> int:
    """The smallest weight_bits that holds for these integer weights (host array): |w| < 2^(bits-1)."""
    import numpy as np
    m = int(np.abs(np.asarray(w_int, dtype=np.int64)).max()) if np.size(w_int) else 0
    return m.bit_length() + 1


def he_conv_check_weights(ctx: Context, c_in: int, c_out: int, level: int, w_res: torch.Tensor, weight_bits: int,
                          alignment: int = HE_CONV_ALIGN_DIRECT, stream=None) -> None:
    """Raises CkksError (CKKS_ERR_INVALID_ARG) if a residue of w_res breaks the promise weight_bits.  Waits for the stream."""
    LM = level + 1 + ctx.num_p if alignment in (HE_CONV_DEFERRED_MODDOWN, HE_CONV_DEFERRED_MERGED) else level + 1
    if w_res.numel() != c_out * c_in * 9 * LM:
        raise ValueError("w_res must be [C_out][C_in][9][L], L = %d limbs" % LM)
    d = _ConvDesc(c_in, c_out, 1, 1, 1, level, int(alignment), int(weight_bits))
    ctx._check(_lib.he_conv_check_weights(ctx.handle, C.byref(d), _ptr(w_res), _stream(stream)))


CKKS_F64_MULMOD, CKKS_F64_MULMOD_ANY, CKKS_F64_REDUCE, CKKS_F64_CANONICAL, CKKS_F64_CENTRE, CKKS_F64_DOT8, CKKS_F64_DOT9 = range(7)


def ckks_f64mod_probe(op: int, y: torch.Tensor, w: Optional[torch.Tensor], wq: Optional[torch.Tensor], q: int,
                      out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """y int64[n], w int64[n] (uint64 residues bit for bit) or None, wq float64[n] or None -> float64[n]; the conversion sums
    (CKKS_F64_DOT8, CKKS_F64_DOT9): y int64[n][8 or 9], w int64[8 or 9] -> float64[n]."""
    nd = {CKKS_F64_DOT8: 8, CKKS_F64_DOT9: 9}.get(int(op))
    if nd is not None and (y.dim() != 2 or y.shape[1] != nd or w is None or w.numel() != nd or not y.is_contiguous()):
        raise CkksError(CKKS_ERR_INVALID_ARG, "ckks_f64mod_probe: a conversion sum takes y [n][%d] and %d constants" % (nd, nd))
    n = y.shape[0] if nd is not None else y.numel()
    if out is None:
        out = torch.empty(n, dtype=torch.float64, device=y.device)
    rc = _lib.ckks_f64mod_probe(int(op), _ptr(y), _ptr(w) if w is not None else None, _ptr(wq) if wq is not None else None, int(q), _ptr(out), n,
                                _stream(stream))
    if rc != CKKS_OK:
        raise CkksError(rc, "ckks_f64mod_probe: invalid arguments")
    return out


def he_conv_batched(ctx: Context, height: int, width: int, batch: int, level: int, ins: Sequence[torch.Tensor],
                    rot_keys: Sequence[Optional[Key]], tap_masks: torch.Tensor, w_res: torch.Tensor, c_out: int,
                    outs: Optional[List[torch.Tensor]] = None, ws: Optional[torch.Tensor] = None, stream=None,
                    alignment: int = HE_CONV_ALIGN_DIRECT, weight_bits: int = 0, w_int_host=None,
                    check_weights: bool = False) -> List[torch.Tensor]:
    """weight_bits: 0, or the promise |w| < 2^(weight_bits-1) for every integer weight (see conv_weight_bits).
    A promise is tested before the layer runs when the caller gives the means: w_int_host (the integer weights as a host
    array: compared with the bound here, ValueError) and / or check_weights=True (he_conv_check_weights on w_res: one more
    pass over the device weights and a wait for the stream, CkksError).
    alignment: HE_CONV_ALIGN_DIRECT (eight hoisted rotations), HE_CONV_ALIGN_FOUR_KEYS (the paper's two-stage
    alignment with four keys), HE_CONV_DEFERRED_MODDOWN (one division by P per output channel) or
    HE_CONV_DEFERRED_MERGED (that division merged with the rescale).
    ins: C_in tensors [2][level+1][N]; rot_keys: nine entries in tap order (centre ignored);
    tap_masks [9][L][N]; w_res [C_out][C_in][9][L] residues of the integer weights, L = level+1 limbs
    (level+1+num_p, the extended basis, for the two deferred schedules)."""
    c_in = len(ins)
    L1 = level + 1
    if len(rot_keys) != 9:
        raise ValueError("nine rotation-key entries expected (row-major taps, centre may be None)")
    LM = L1 + ctx.num_p if alignment in (HE_CONV_DEFERRED_MODDOWN, HE_CONV_DEFERRED_MERGED) else L1
    if tap_masks.numel() != 9 * LM * ctx.N or w_res.numel() != c_out * c_in * 9 * LM:
        raise ValueError("tap_masks must be [9][L][N] and w_res [C_out][C_in][9][L], L = %d limbs" % LM)
    for t in ins:
        if t.numel() != 2 * L1 * ctx.N:
            raise ValueError("each input must be [2][level+1][N]")
    if outs is None:
        outs = [empty(2, max(level, 1), ctx.N) for _ in range(c_out)]
    for o in outs:
        if o.numel() != 2 * level * ctx.N:
            raise ValueError("each output must be [2][level][N]")
    if weight_bits and w_int_host is not None and conv_weight_bits(w_int_host) > weight_bits:
        raise ValueError("weight_bits = %d promised, but the weights need %d" % (weight_bits, conv_weight_bits(w_int_host)))
    if weight_bits and check_weights:
        he_conv_check_weights(ctx, c_in, c_out, level, w_res, weight_bits, alignment, stream)
    d = _ConvDesc(c_in, c_out, height, width, batch, level, int(alignment), int(weight_bits))
    ws = _ws(ctx, ws, he_conv_workspace_bytes(ctx, c_in, c_out, height, width, batch, level, alignment))
    ia = _ptr_array([_ptr(t) for t in ins])
    ka = _ptr_array([k.handle.value if k is not None else None for k in rot_keys])
    oa = _ptr_array([_ptr(o) for o in outs])
    ctx._check(_lib.he_conv_batched(ctx.handle, C.byref(d), ia, ka, _ptr(tap_masks), _ptr(w_res), oa, _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))
    return outs


def he_poly_act_deg7(ctx: Context, xs: Sequence[torch.Tensor], level: int, k: Sequence[int], rlk: Key,
                     outs: Optional[List[torch.Tensor]] = None, ws: Optional[torch.Tensor] = None, stream=None,
                     merged: bool = False) -> List[torch.Tensor]:
    """xs: channel ciphertexts [2][level+1][N]; returns one [2][level-3][N] per channel.
    merged: every relinearise-then-rescale pair as one division by P*q_level."""
    n = len(xs)
    if n == 0 or len(k) != 4:
        raise ValueError("need at least one ciphertext and four integers k")
    for x in xs:
        if x.numel() != 2 * (level + 1) * ctx.N:
            raise ValueError("each x must be [2][level+1][N]")
    if outs is None:
        outs = [empty(2, max(level - 3, 1), ctx.N) for _ in range(n)]
    for o in outs:
        if o.numel() != 2 * (level - 3) * ctx.N:
            raise ValueError("each output must be [2][level-3][N]")
    ws = _ws(ctx, ws, ckks_workspace_bytes(ctx, CKKS_OP_POLY_ACT, level, n))
    ka = (C.c_int64 * 4)(*[int(v) for v in k])
    xa = _ptr_array([_ptr(x) for x in xs])
    oa = _ptr_array([_ptr(o) for o in outs])
    ctx._check(_lib.he_poly_act_deg7(ctx.handle, xa, n, level, ka, rlk.handle if rlk else None, int(bool(merged)), oa, _ptr(ws),
                                     ws.numel() * ws.element_size(), _stream(stream)))
    return outs


def he_accumulator_workspace_bytes(ctx: Context, level: int, g: int) -> int:
    return int(_lib.he_accumulator_workspace_bytes(ctx.handle, level, g))


def he_accumulator_merge(ctx: Context, cts: Sequence[torch.Tensor], level: int, sts: int, mask: torch.Tensor,
                         keys: Sequence[Optional[Key]], out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                         stream=None) -> torch.Tensor:
    """cts: g ciphertexts [2][level+1][N] with data in slots [0, sts); mask [level+1][N]; keys[i] = key of offset
    -i*sts (keys[0] ignored).  Returns [2][level][N] with block i in slots [i*sts, (i+1)*sts)."""
    g = len(cts)
    if g == 0 or len(keys) != g:
        raise ValueError("need g >= 1 ciphertexts and g key entries (the first may be None)")
    for t in cts:
        if t.numel() != 2 * (level + 1) * ctx.N:
            raise ValueError("each ciphertext must be [2][level+1][N]")
    if mask.numel() != (level + 1) * ctx.N:
        raise ValueError("mask must be [level+1][N]")
    if out is None:
        out = empty(2, max(level, 1), ctx.N)
    if out.numel() != 2 * level * ctx.N:
        raise ValueError("out must be [2][level][N]")
    ws = _ws(ctx, ws, he_accumulator_workspace_bytes(ctx, level, g))
    ca = _ptr_array([_ptr(t) for t in cts])
    ka = _ptr_array([k.handle.value if k is not None else None for k in keys])
    ctx._check(_lib.he_accumulator_merge(ctx.handle, ca, g, level, sts, _ptr(mask), ka, _ptr(out), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream(stream)))
    return out


def ckks_ctx_set_overlap(ctx: Context, on: bool) -> None:
    """Whether channel batches may run on the context's second stream (default on)."""
    ctx._check(_lib.ckks_ctx_set_overlap(ctx.handle, 1 if on else 0))


def ckks_key_expand_a(ctx: Context, a_seed: int, key: torch.Tensor, stream=None) -> torch.Tensor:
    """Writes the public halves of key ([dnum][2][num_q+num_p][N], device) from the seed; the b halves stay."""
    if key.numel() != ctx.dnum * 2 * ctx.M * ctx.N:
        raise ValueError("key must be [dnum][2][num_q+num_p][N]")
    ctx._check(_lib.ckks_key_expand_a(ctx.handle, C.c_uint64(a_seed), _ptr(key), _stream(stream)))
    return key


def ckks_keyset_stage(ctx: Context, host_b: Sequence[torch.Tensor], a_seeds: Sequence[int], keys: Sequence[torch.Tensor],
                      stream=None) -> None:
    """host_b[i]: CPU tensor [dnum][num_q+num_p][N] (pinned for an asynchronous copy); keys[i]: device [dnum][2][M][N]."""
    n = len(keys)
    if len(host_b) != n or len(a_seeds) != n:
        raise ValueError("one host tensor and one seed per key")
    for hb, k in zip(host_b, keys):
        if hb.device.type != "cpu" or not hb.is_contiguous() or hb.numel() != ctx.dnum * ctx.M * ctx.N or hb.element_size() != 8:
            raise ValueError("host_b must be contiguous 64-bit CPU tensors [dnum][num_q+num_p][N]")
        if k.numel() != ctx.dnum * 2 * ctx.M * ctx.N:
            raise ValueError("keys must be [dnum][2][num_q+num_p][N]")
    hb_arr = (C.c_void_p * n)(*[t.data_ptr() for t in host_b])
    seeds = (C.c_uint64 * n)(*[int(v) for v in a_seeds])
    ctx._check(_lib.ckks_keyset_stage(ctx.handle, hb_arr, seeds, _ptr_array([_ptr(k) for k in keys]), n, _stream(stream)))


def he_relayout_workspace_bytes(ctx: Context, level: int, n_ct: int, n_lo: int, n_hi: int, schedule: int = HE_RELAYOUT_DIRECT) -> int:
    return int(_lib.he_relayout_workspace_bytes(ctx.handle, level, n_ct, n_lo, n_hi, schedule))


def he_relayout_two_rotations(ctx: Context, cts: Sequence[torch.Tensor], level: int, lo: Sequence[int], lo_keys: Sequence[Optional[Key]],
                              hi: Sequence[int], hi_keys: Sequence[Optional[Key]], masks: Sequence[Sequence[Optional[torch.Tensor]]],
                              schedule: int = HE_RELAYOUT_DIRECT, outs: Optional[Sequence[torch.Tensor]] = None,
                              ws: Optional[torch.Tensor] = None, stream=None) -> List[torch.Tensor]:
    """out_b = sum_h Rot(Rescale(sum_l masks[h][l] (.) Rot(cts[b], lo[l])), hi[h]); masks[h][l] is [level+1][N]
    (HE_RELAYOUT_DIRECT) or [level+1+num_p][N] on the extended basis (HE_RELAYOUT_DEFERRED), or None.
    cts[b] [2][level+1][N]; returns [2][level][N] per ciphertext."""
    n_ct, n_lo, n_hi = len(cts), len(lo), len(hi)
    if len(lo_keys) != n_lo or len(hi_keys) != n_hi or len(masks) != n_hi or any(len(row) != n_lo for row in masks):
        raise ValueError("key and mask lists do not match the offsets")
    for t in cts:
        if t.numel() != 2 * (level + 1) * ctx.N:
            raise ValueError("each ciphertext must be [2][level+1][N]")
    mask_limbs = level + 1 + (ctx.num_p if schedule == HE_RELAYOUT_DEFERRED else 0)
    for row in masks:
        for m in row:
            if m is not None and m.numel() != mask_limbs * ctx.N:
                raise ValueError(f"each mask must be [{mask_limbs}][N]")
    if outs is None:
        outs = [empty(2, max(level, 1), ctx.N) for _ in range(n_ct)]
    for t in outs:
        if t.numel() != 2 * level * ctx.N:
            raise ValueError("each output must be [2][level][N]")
    ws = _ws(ctx, ws, he_relayout_workspace_bytes(ctx, level, n_ct, n_lo, n_hi, schedule))
    arr = lambda ks: _ptr_array([k.handle.value if k is not None else None for k in ks])
    i32 = lambda v: (C.c_int32 * len(v))(*[int(x) for x in v])
    ctx._check(_lib.he_relayout_two_rotations(ctx.handle, _ptr_array([_ptr(t) for t in cts]), n_ct, level, i32(lo), n_lo, arr(lo_keys),
                                              i32(hi), n_hi, arr(hi_keys), _ptr_array([_ptr(m) for row in masks for m in row]), schedule,
                                              _ptr_array([_ptr(t) for t in outs]), _ptr(ws), ws.numel() * ws.element_size(),
                                              _stream(stream)))
    return list(outs)


def he_fc_workspace_bytes(ctx: Context, d_in: int, d_out: int, batch: int, level: int, base: int = 0) -> int:
    return int(_lib.he_fc_workspace_bytes(ctx.handle, C.byref(_FcDesc(d_in, d_out, batch, level, base))))


def he_fc_batched(ctx: Context, ct: torch.Tensor, level: int, d_in: int, d_out: int, batch: int, base: int, w_enc: torch.Tensor,
                  merge_mask: torch.Tensor, place_masks: torch.Tensor, bias: torch.Tensor, sum_keys: Sequence[Key],
                  merge_keys: Sequence[Optional[Key]], lo_keys: Sequence[Optional[Key]], hi_keys: Sequence[Optional[Key]],
                  out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """ct [2][level+1][N] with x^(j) in slots [j*d_in, (j+1)*d_in); w_enc [d_out][level+1][N]; merge_mask [level][N];
    place_masks [batch][level-1][N]; bias [level-2][N].  sum_keys[s]: offset 2^s; merge_keys[i]: offset -i;
    lo_keys[l]: offset l*(d_in-d_out); hi_keys[h]: offset h*base*(d_in-d_out) (entries of offset 0 may be None).
    Returns [2][level-2][N] with W x^(j) + bias in slots [j*d_out, (j+1)*d_out)."""
    N = ctx.N
    if level < 3:
        raise ValueError("the layer needs level >= 3")
    n_base = base if base else next(b for b in range(1, batch + 1) if b * b >= batch)
    want = dict(ct=(ct, 2 * (level + 1) * N), w_enc=(w_enc, d_out * (level + 1) * N), merge_mask=(merge_mask, level * N),
                place_masks=(place_masks, batch * (level - 1) * N), bias=(bias, (level - 2) * N))
    for name, (t, n) in want.items():
        if t.numel() != n:
            raise ValueError(f"{name} has {t.numel()} elements, expected {n}")
    if len(sum_keys) != d_in.bit_length() - 1 or len(merge_keys) != d_out or len(lo_keys) != min(n_base, batch) \
            or len(hi_keys) != -(-batch // n_base):
        raise ValueError("key lists do not match the layer's rotations")
    if out is None:
        out = empty(2, level - 2, N)
    if out.numel() != 2 * (level - 2) * N:
        raise ValueError("out must be [2][level-2][N]")
    ws = _ws(ctx, ws, he_fc_workspace_bytes(ctx, d_in, d_out, batch, level, base))
    arr = lambda ks: _ptr_array([k.handle.value if k is not None else None for k in ks])
    ctx._check(_lib.he_fc_batched(ctx.handle, C.byref(_FcDesc(d_in, d_out, batch, level, base)), _ptr(ct), _ptr(w_enc), arr(sum_keys),
                                  arr(merge_keys), _ptr(merge_mask), _ptr(place_masks), arr(lo_keys), arr(hi_keys), _ptr(bias),
                                  _ptr(out), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))
    return out


def ckks_prof_kernel_names() -> List[str]:
    return [_lib.ckks_prof_kernel_name(i).decode() for i in range(_lib.ckks_prof_kernel_count())]


def ckks_prof_begin(ctx: Context, kernels: Optional[Sequence[str]] = None, max_launches: int = 65536) -> None:
    """Start bracketing launches of the named kernel classes (default: all) with HIP events."""
    names = ckks_prof_kernel_names()
    mask = 0
    for k in (names if kernels is None else kernels):
        mask |= 1 << names.index(k)
    ctx._check(_lib.ckks_prof_begin(ctx.handle, mask, max_launches))


def ckks_prof_end(ctx: Context) -> dict:
    """{kernel: dict(ms, launches, bytes, ops)} for the classes that ran, plus the key "dropped"."""
    n = _lib.ckks_prof_kernel_count()
    ms = (C.c_double * n)()
    cnt = (C.c_uint64 * n)()
    nbytes = (C.c_double * n)()
    ops = (C.c_double * n)()
    dropped = C.c_uint64()
    ctx._check(_lib.ckks_prof_end(ctx.handle, ms, cnt, nbytes, ops, C.byref(dropped)))
    out = {name: dict(ms=ms[i], launches=int(cnt[i]), bytes=nbytes[i], ops=ops[i])
           for i, name in enumerate(ckks_prof_kernel_names()) if cnt[i]}
    out["dropped"] = int(dropped.value)
    return out
