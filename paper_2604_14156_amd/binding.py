"""ctypes binding over the C ABI (include/cs.h).

Argument marshalling only: every step of the path runs in the library's kernels.
PyTorch is used for device memory (tensors own the buffers) and for the stream.
The module raises at load time if the shared library is missing: there is no
fallback path.
"""
import ctypes
import os

import torch

from .buildlib import LIB_PATH

CS_OK, CS_EINVAL, CS_EALIGN, CS_EILLPOSED, CS_ENOMEM, CS_EHIP = 0, -1, -2, -3, -4, -5
CS_GAUSS, CS_RADEMACHER, CS_SRHT = 0, 1, 2
CS_F32, CS_BF16 = 0, 1

EXPORTS = ("cs_create", "cs_destroy", "cs_last_error", "cs_set_stream", "cs_set_union_hint", "cs_plan", "cs_plan_drop", "cs_sketch", "cs_sketch_multi",
           "cs_recover_support", "cs_recover_support_multi", "cs_recover_support_iht", "cs_recover_support_inc", "cs_recover_support_inc_carry", "cs_inc_state_words", "cs_block_ffn", "cs_block_ffn_static", "cs_head_attn", "cs_joint_select", "cs_joint_select_coupled", "cs_gather_rows",
           "cs_softmax_entropy", "cs_uds_budget", "cs_stream_read")


class CsOp(ctypes.Structure):
    _fields_ = [("ens", ctypes.c_int32), ("seed", ctypes.c_uint64), ("stream_id", ctypes.c_uint32),
                ("m", ctypes.c_int32), ("n", ctypes.c_int32)]


class CsDict(ctypes.Structure):
    _fields_ = [("psi", ctypes.c_void_p), ("G", ctypes.c_int32), ("b", ctypes.c_int32), ("rb", ctypes.c_int32)]


class CsError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("cs status %d: %s" % (status, message))
        self.status = status


def load_library(path=LIB_PATH):
    if not os.path.exists(path):
        raise ImportError("%s is missing: build it with `python -m paper_2604_14156_amd.buildlib`" % path)
    lib = ctypes.CDLL(path)
    vp, i32, u64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.cs_create.argtypes = [ctypes.POINTER(vp), i32, vp, u64]
    lib.cs_destroy.argtypes = [vp]
    lib.cs_destroy.restype = None
    lib.cs_last_error.argtypes = [vp]
    lib.cs_last_error.restype = ctypes.c_char_p
    lib.cs_set_stream.argtypes = [vp, vp]
    lib.cs_set_union_hint.argtypes = [vp, i32]
    lib.cs_plan.argtypes = [vp, ctypes.POINTER(CsOp), ctypes.POINTER(CsDict)]
    lib.cs_plan_drop.argtypes = lib.cs_plan.argtypes
    lib.cs_sketch.argtypes = [vp, ctypes.POINTER(CsOp), vp, i32, vp]
    lib.cs_sketch_multi.argtypes = [vp, i32, ctypes.POINTER(CsOp), vp, i32, vp]
    lib.cs_recover_support.argtypes = [vp, ctypes.POINTER(CsOp), ctypes.POINTER(CsDict), i32, vp, i32, vp, vp, vp, vp]
    lib.cs_recover_support_multi.argtypes = [vp, i32, ctypes.POINTER(CsOp), ctypes.POINTER(CsDict), i32, vp, i32, vp, vp, vp, vp]
    lib.cs_recover_support_iht.argtypes = [vp, ctypes.POINTER(CsOp), ctypes.POINTER(CsDict), i32, i32, vp, i32, vp, vp, vp, vp]
    lib.cs_recover_support_inc.argtypes = [vp, ctypes.POINTER(CsOp), ctypes.POINTER(CsDict), i32, vp, i32,
                                           vp, vp, ctypes.c_float, i32, vp, vp, vp, vp]
    lib.cs_recover_support_inc_carry.argtypes = [vp, ctypes.POINTER(CsOp), ctypes.POINTER(CsDict), i32, vp, i32,
                                                 vp, i32, vp, vp, vp, vp, vp]
    lib.cs_inc_state_words.argtypes = [i32]
    lib.cs_block_ffn.argtypes = [vp, i32, vp, vp, vp, i32, i32, i32, vp, i32, vp, i32, i32, vp]
    lib.cs_block_ffn_static.argtypes = lib.cs_block_ffn.argtypes
    lib.cs_head_attn.argtypes = [vp, i32, vp, vp, vp, i32, i32, i32, i32, vp, i32, vp]
    lib.cs_joint_select.argtypes = [vp, ctypes.POINTER(CsOp), vp, i32, ctypes.POINTER(CsOp), ctypes.POINTER(CsDict),
                                    vp, i32, vp, vp, vp, vp]
    lib.cs_joint_select_coupled.argtypes = [vp, ctypes.POINTER(CsOp), vp, i32, ctypes.POINTER(CsOp), ctypes.POINTER(CsDict),
                                            vp, i32, vp, vp, vp, vp, vp]
    lib.cs_softmax_entropy.argtypes = [vp, vp, i32, i32, vp]
    lib.cs_uds_budget.argtypes = [ctypes.c_int32, ctypes.c_float, ctypes.c_float, ctypes.c_int32, ctypes.c_int32]
    lib.cs_stream_read.argtypes = [vp, vp, u64, vp]
    lib.cs_gather_rows.argtypes = [vp, i32, vp, i32, i32, vp, i32, vp]
    for name in EXPORTS:
        if name not in ("cs_destroy", "cs_last_error"):
            getattr(lib, name).restype = ctypes.c_int       # cs_status, or the budget of cs_uds_budget
    lib.cs_inc_state_words.restype = ctypes.c_size_t
    return lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t):
    if t.dtype == torch.float32:
        return CS_F32
    if t.dtype == torch.bfloat16:
        return CS_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def make_op(ens, seed, stream_id, m, n):
    return CsOp(int(ens), int(seed), int(stream_id), int(m), int(n))


def make_dict(psi, G, b, rb):
    """psi: device tensor [G][b][rb] or None.  The tensor travels with the struct (attribute `tensor`), so
    that a context which builds a plan from it can keep it alive: plans are found again by address."""
    dct = CsDict(None if psi is None else psi.data_ptr(), int(G), int(b), int(rb))
    dct.tensor = psi
    return dct


class Context:
    """A library context on one device, bound to a torch stream."""

    def __init__(self, device=0, stream=None, scratch_bytes=0):
        self.lib = load_library()
        self.device = torch.device("cuda", device)
        self._h = ctypes.c_void_p()
        sptr = None if stream is None else ctypes.c_void_p(stream.cuda_stream)
        st = self.lib.cs_create(ctypes.byref(self._h), device, sptr, scratch_bytes)
        if st != CS_OK:
            raise CsError(st, "cs_create failed")
        self._keep = {}        # address -> dictionary tensor: dictionaries of cached plans stay alive

    def close(self):
        if self._h:
            self.lib.cs_destroy(self._h)
            self._h = ctypes.c_void_p()

    def _alloc(self, shape, dtype, device):
        """Output buffers the caller did not pass in (tests override this to put guard bands around them)."""
        return torch.empty(shape, dtype=dtype, device=device)

    def _check(self, st):
        if st != CS_OK:
            raise CsError(st, self.lib.cs_last_error(self._h).decode())

    def set_stream(self, stream):
        self._check(self.lib.cs_set_stream(self._h, None if stream is None else ctypes.c_void_p(stream.cuda_stream)))

    def cs_set_union_hint(self, hint):
        """0 auto, 1 the rows' supports cover nearly all units, 2 they share most of their units."""
        self._check(self.lib.cs_set_union_hint(self._h, int(hint)))

    # -- the calls of the C ABI, same names ---------------------------------
    def _retain(self, dct, psi=None):
        """Every call that may build a plan keeps the dictionary's tensor: the plan cache identifies a
        dictionary by its address, which must not be handed to another tensor while the plan lives."""
        for d in (dct if isinstance(dct, (list, tuple)) else [dct]):
            t = psi if psi is not None else getattr(d, "tensor", None)
            if t is not None:
                self._keep[t.data_ptr()] = t

    def cs_plan(self, op, dct, psi=None):
        self._retain(dct, psi)
        self._check(self.lib.cs_plan(self._h, ctypes.byref(op), ctypes.byref(dct)))

    def cs_plan_drop(self, op, dct):
        self._check(self.lib.cs_plan_drop(self._h, ctypes.byref(op), ctypes.byref(dct)))

    def cs_sketch(self, op, z, y=None):
        B = z.shape[0]
        if y is None:
            y = self._alloc((B, op.m), torch.float32, z.device)
        self._check(self.lib.cs_sketch(self._h, ctypes.byref(op), _ptr(z), B, _ptr(y)))
        return y

    def cs_sketch_multi(self, ops, z, y=None):
        """ops: sequence of CsOp (or a ctypes array of them); z [n_ops][B][n] -> y [n_ops][B][m]."""
        n_ops = len(ops)
        arr = ops if isinstance(ops, ctypes.Array) else (CsOp * n_ops)(*ops)
        B = z.shape[1]
        if y is None:
            y = self._alloc((n_ops, B, arr[0].m), torch.float32, z.device)
        self._check(self.lib.cs_sketch_multi(self._h, n_ops, arr, _ptr(z), B, _ptr(y)))
        return y

    def cs_recover_support(self, op, dct, k, y, support=None, coef=None, resid=None, margin=None,
                           want_coef=True, want_resid=True, want_margin=True):
        B = y.shape[0]
        dev = y.device
        self._retain(dct)
        if support is None:
            support = self._alloc((B, k), torch.int32, dev)
        if coef is None and want_coef:
            coef = self._alloc((B, k * dct.rb), torch.float32, dev)
        if resid is None and want_resid:
            resid = self._alloc((B,), torch.float32, dev)
        if margin is None and want_margin:
            margin = self._alloc((B,), torch.float32, dev)
        self._check(self.lib.cs_recover_support(self._h, ctypes.byref(op), ctypes.byref(dct), k, _ptr(y), B,
                                                _ptr(support), _ptr(coef), _ptr(resid), _ptr(margin)))
        return support, coef, resid, margin

    def cs_recover_support_multi(self, ops, dcts, k, y, support=None, coef=None, resid=None, margin=None,
                                 want_coef=True, want_resid=True, want_margin=True):
        """ops, dcts: sequences of n_ops operators / dictionaries (or ctypes arrays); y: [n_ops, B, m]."""
        n_ops, B = y.shape[0], y.shape[1]
        dev = y.device
        if not isinstance(dcts, ctypes.Array):
            self._retain(list(dcts))
        if not isinstance(ops, ctypes.Array):
            ops = (CsOp * n_ops)(*ops)
        if not isinstance(dcts, ctypes.Array):
            dcts = (CsDict * n_ops)(*dcts)
        rb = dcts[0].rb
        if support is None:
            support = self._alloc((n_ops, B, k), torch.int32, dev)
        if coef is None and want_coef:
            coef = self._alloc((n_ops, B, k * rb), torch.float32, dev)
        if resid is None and want_resid:
            resid = self._alloc((n_ops, B), torch.float32, dev)
        if margin is None and want_margin:
            margin = self._alloc((n_ops, B), torch.float32, dev)
        self._check(self.lib.cs_recover_support_multi(self._h, n_ops, ops, dcts, k, _ptr(y), B,
                                                      _ptr(support), _ptr(coef), _ptr(resid), _ptr(margin)))
        return support, coef, resid, margin

    def cs_recover_support_iht(self, op, dct, k, iters, y, support=None, coef=None, resid=None, margin=None,
                               want_coef=True, want_resid=True, want_margin=True):
        B = y.shape[0]
        dev = y.device
        self._retain(dct)
        if support is None:
            support = self._alloc((B, k), torch.int32, dev)
        if coef is None and want_coef:
            coef = self._alloc((B, k * dct.rb), torch.float32, dev)
        if resid is None and want_resid:
            resid = self._alloc((B,), torch.float32, dev)
        if margin is None and want_margin:
            margin = self._alloc((B,), torch.float32, dev)
        self._check(self.lib.cs_recover_support_iht(self._h, ctypes.byref(op), ctypes.byref(dct), k, iters, _ptr(y), B,
                                                    _ptr(support), _ptr(coef), _ptr(resid), _ptr(margin)))
        return support, coef, resid, margin

    def cs_recover_support_inc(self, op, dct, k, y, prev_support, swaps, prev_coef=None, gamma=0.0,
                               support=None, coef=None, resid=None, margin=None, want_coef=True, want_resid=True, want_margin=True):
        B = y.shape[0]
        dev = y.device
        self._retain(dct)
        if support is None:
            support = self._alloc((B, k), torch.int32, dev)
        if coef is None and want_coef:
            coef = self._alloc((B, k * dct.rb), torch.float32, dev)
        if resid is None and want_resid:
            resid = self._alloc((B,), torch.float32, dev)
        if margin is None and want_margin:
            margin = self._alloc((B,), torch.float32, dev)
        self._check(self.lib.cs_recover_support_inc(self._h, ctypes.byref(op), ctypes.byref(dct), k, _ptr(y), B,
                                                    _ptr(prev_support), _ptr(prev_coef), float(gamma), swaps,
                                                    _ptr(support), _ptr(coef), _ptr(resid), _ptr(margin)))
        return support, coef, resid, margin

    def cs_inc_state(self, B, k, device):
        """A zero-filled state buffer for a sequence of cs_recover_support_inc_carry calls on B sketches."""
        words = int(self.lib.cs_inc_state_words(k))
        return torch.zeros((B, words), dtype=torch.int32, device=device)

    def cs_recover_support_inc_carry(self, op, dct, k, y, prev_support, swaps, state,
                                     support=None, coef=None, resid=None, margin=None, want_coef=True, want_resid=True, want_margin=True):
        B = y.shape[0]
        dev = y.device
        self._retain(dct)
        if support is None:
            support = self._alloc((B, k), torch.int32, dev)
        if coef is None and want_coef:
            coef = self._alloc((B, k * dct.rb), torch.float32, dev)
        if resid is None and want_resid:
            resid = self._alloc((B,), torch.float32, dev)
        if margin is None and want_margin:
            margin = self._alloc((B,), torch.float32, dev)
        self._check(self.lib.cs_recover_support_inc_carry(self._h, ctypes.byref(op), ctypes.byref(dct), k, _ptr(y), B,
                                                          _ptr(prev_support), swaps, _ptr(state),
                                                          _ptr(support), _ptr(coef), _ptr(resid), _ptr(margin)))
        return support, coef, resid, margin

    def cs_block_ffn_static(self, Wg, Wu, Wd, x, support, shared, out):
        """The variant that allocates nothing: the caller passes `out`."""
        return self.cs_block_ffn(Wg, Wu, Wd, x, support, shared, out, entry=self.lib.cs_block_ffn_static)

    def cs_block_ffn(self, Wg, Wu, Wd, x, support, shared, out=None, entry=None):
        G, b, d = Wg.shape
        T = x.shape[0]
        k = support.shape[-1]
        if out is None:
            out = self._alloc(tuple(x.shape), x.dtype, x.device)
        self._check((entry or self.lib.cs_block_ffn)(self._h, _dtype_code(x), _ptr(Wg), _ptr(Wu), _ptr(Wd), d, G, b,
                                          _ptr(x), T, _ptr(support), k, 1 if shared else 0, _ptr(out)))
        return out

    def cs_head_attn(self, q, K, V, heads, out=None):
        B, H, L, dh = K.shape
        kh = heads.shape[-1]
        if out is None:
            out = self._alloc(tuple(q.shape), q.dtype, q.device)
        self._check(self.lib.cs_head_attn(self._h, _dtype_code(q), _ptr(q), _ptr(K), _ptr(V), B, H, L, dh,
                                          _ptr(heads), kh, _ptr(out)))
        return out

    def cs_joint_select_coupled(self, tok_op, y_tok, k_tok, ch_op, ch_dict, Y_ch, k_ch):
        dev = y_tok.device
        self._retain(ch_dict)
        tokens = self._alloc((k_tok,), torch.int32, dev)
        support = self._alloc((k_ch,), torch.int32, dev)
        ybar = self._alloc((ch_op.m,), torch.float32, dev)
        resid = self._alloc((1,), torch.float32, dev)
        margin = self._alloc((1,), torch.float32, dev)
        self._check(self.lib.cs_joint_select_coupled(self._h, ctypes.byref(tok_op), _ptr(y_tok), k_tok,
                                                     ctypes.byref(ch_op), ctypes.byref(ch_dict), _ptr(Y_ch), k_ch,
                                                     _ptr(tokens), _ptr(support), _ptr(ybar), _ptr(resid), _ptr(margin)))
        return tokens, support, ybar, resid, margin

    def cs_softmax_entropy(self, logits, entropy=None):
        B, V = logits.shape
        if entropy is None:
            entropy = self._alloc((B,), torch.float32, logits.device)
        self._check(self.lib.cs_softmax_entropy(self._h, _ptr(logits), B, V, _ptr(entropy)))
        return entropy

    def cs_uds_budget(self, m_base, gamma, entropy, m_min, m_max):
        return int(self.lib.cs_uds_budget(int(m_base), float(gamma), float(entropy), int(m_min), int(m_max)))

    def cs_stream_read(self, src, checksum):
        """Diagnostic streaming read of the whole tensor `src`; checksum: uint32/int32 tensor of one element."""
        self._check(self.lib.cs_stream_read(self._h, _ptr(src), src.numel() * src.element_size(), _ptr(checksum)))
        return checksum

    def cs_gather_rows(self, x, tokens, out=None):
        n_rows, d = x.shape
        k_tok = tokens.shape[0]
        if out is None:
            out = self._alloc((k_tok, d), x.dtype, x.device)
        self._check(self.lib.cs_gather_rows(self._h, _dtype_code(x), _ptr(x), n_rows, d, _ptr(tokens), k_tok, _ptr(out)))
        return out

    def cs_joint_select(self, tok_op, y_tok, k_tok, ch_op, ch_dict, y_ch, k_ch):
        dev = y_tok.device
        self._retain(ch_dict)
        tokens = self._alloc((k_tok,), torch.int32, dev)
        support = self._alloc((k_ch,), torch.int32, dev)
        resid = self._alloc((1,), torch.float32, dev)
        margin = self._alloc((1,), torch.float32, dev)
        self._check(self.lib.cs_joint_select(self._h, ctypes.byref(tok_op), _ptr(y_tok), k_tok,
                                             ctypes.byref(ch_op), ctypes.byref(ch_dict), _ptr(y_ch), k_ch,
                                             _ptr(tokens), _ptr(support), _ptr(resid), _ptr(margin)))
        return tokens, support, resid, margin
