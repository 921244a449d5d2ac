"""ctypes binding of libuncomp: argument marshalling only.

Each function takes torch CUDA tensors, passes their device pointers, sizes and
strides to the C entry point of the same name and launches on torch's current
stream.  All arithmetic happens in the HIP kernels; if the shared library has
not been built this module raises at import of the library (there is no
fallback path).
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libuncomp.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4
BF16, F32 = 0, 1
CENTER, TRUNC_RENORM, LAYER_DELTA_INCREASE = 1, 2, 4
DEFAULT_FLAGS = CENTER | TRUNC_RENORM

EXPORTS = (
    "uncomp_create", "uncomp_destroy", "uncomp_workspace_bytes", "uncomp_last_error",
    "uncomp_profile", "uncomp_profile_read", "uncomp_measure_peaks", "uncomp_set_kernel_path", "uncomp_set_overlap", "uncomp_join",
    "uncomp_head_entropy", "uncomp_head_entropy_noalloc", "uncomp_assign_budgets", "uncomp_window_score", "uncomp_select_gather",
    "uncomp_decode_init", "uncomp_decode_step", "uncomp_decode_workspace_bytes",
    "uncomp_hidden_evict", "uncomp_hidden_workspace_bytes",
    "uncomp_matrix_entropy", "uncomp_matrix_workspace_bytes",
    "uncomp_prepare_reset", "uncomp_prepare_accumulate", "uncomp_prepare_finish", "uncomp_budgets_from_labels",
)

_lib = None


class UncompError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"libuncomp status {status}: {msg}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """Loads libuncomp.so from the package directory; raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} not found: build it with `python -m paper_2410_03090_amd.build` "
            "(there is no non-HIP implementation to fall back to)")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i32, i64, u32, f32 = c.c_void_p, c.c_int, c.c_int64, c.c_uint, c.c_float
    lib.uncomp_create.argtypes = [c.POINTER(vp), i32, c.c_size_t]
    lib.uncomp_create.restype = i32
    lib.uncomp_destroy.argtypes = [vp]
    lib.uncomp_destroy.restype = i32
    lib.uncomp_workspace_bytes.argtypes = [i32] * 7
    lib.uncomp_workspace_bytes.restype = c.c_size_t
    lib.uncomp_last_error.argtypes = [vp]
    lib.uncomp_last_error.restype = c.c_char_p
    lib.uncomp_profile.argtypes = [vp, i32]
    lib.uncomp_profile.restype = i32
    lib.uncomp_set_overlap.argtypes = [vp, i32]
    lib.uncomp_set_overlap.restype = i32
    lib.uncomp_join.argtypes = [vp, vp]
    lib.uncomp_join.restype = i32
    lib.uncomp_set_kernel_path.argtypes = [vp, i32]
    lib.uncomp_set_kernel_path.restype = i32
    lib.uncomp_profile_read.argtypes = [vp, i32, c.POINTER(c.c_char_p), c.POINTER(f32)]
    lib.uncomp_profile_read.restype = i32
    lib.uncomp_measure_peaks.argtypes = [vp, vp, c.c_size_t, c.POINTER(c.c_double), c.POINTER(c.c_double),
                                         c.POINTER(c.c_double), vp]
    lib.uncomp_measure_peaks.restype = i32
    lib.uncomp_head_entropy.argtypes = [vp, vp, i32, i32, i32, i32, i64, i64, i32, u32, vp, vp, vp]
    lib.uncomp_head_entropy.restype = i32
    lib.uncomp_head_entropy_noalloc.argtypes = [vp, i32, i32, i32, i32, i64, i64, i32, u32, vp, vp, vp]
    lib.uncomp_head_entropy_noalloc.restype = i32
    lib.uncomp_assign_budgets.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, f32, i32, u32,
                                          vp, vp, vp, vp, vp]
    lib.uncomp_assign_budgets.restype = i32
    lib.uncomp_window_score.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32,
                                        c.POINTER(i64), vp, vp, vp]
    lib.uncomp_window_score.restype = i32
    lib.uncomp_select_gather.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                         c.POINTER(i64), i32, vp, vp, vp, vp, vp]
    lib.uncomp_select_gather.restype = i32
    lib.uncomp_decode_init.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, vp]
    lib.uncomp_decode_init.restype = i32
    lib.uncomp_decode_step.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, i32, i32,
                                       vp, vp, vp, vp, vp, vp, vp, vp]
    lib.uncomp_decode_step.restype = i32
    lib.uncomp_matrix_workspace_bytes.argtypes = [i32, i32]
    lib.uncomp_matrix_workspace_bytes.restype = c.c_size_t
    lib.uncomp_matrix_entropy.argtypes = [vp, vp, i32, i32, i32, i32, i64, i64, i32, u32, i32, vp, vp, vp]
    lib.uncomp_matrix_entropy.restype = i32
    lib.uncomp_prepare_reset.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp]
    lib.uncomp_prepare_reset.restype = i32
    lib.uncomp_prepare_accumulate.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.uncomp_prepare_accumulate.restype = i32
    lib.uncomp_prepare_finish.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.uncomp_prepare_finish.restype = i32
    lib.uncomp_budgets_from_labels.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.uncomp_budgets_from_labels.restype = i32
    lib.uncomp_hidden_workspace_bytes.argtypes = [i32] * 5
    lib.uncomp_hidden_workspace_bytes.restype = c.c_size_t
    lib.uncomp_hidden_evict.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, c.POINTER(i64), vp, i32,
                                        vp, c.POINTER(i64), i32, i32, vp, vp, vp, vp, vp]
    lib.uncomp_hidden_evict.restype = i32
    lib.uncomp_decode_workspace_bytes.argtypes = [i32, i32, i32]
    lib.uncomp_decode_workspace_bytes.restype = c.c_size_t
    _lib = lib
    return lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def head_entropy_noalloc(X: torch.Tensor, k_trunc: int = 32, flags: int = DEFAULT_FLAGS, entropy_out=None, eig_out=None):
    """uncomp_head_entropy_noalloc: X [n_mat, N, D] (last dim contiguous), outputs given by the caller (the call
    itself allocates nothing; without outputs this wrapper makes them first).  Returns (entropy, eig or None)."""
    lib = load_library()
    n_mat, N, D = X.shape
    assert X.stride(2) == 1
    if entropy_out is None:
        entropy_out = torch.empty(n_mat, dtype=torch.float32, device=X.device)
    st = lib.uncomp_head_entropy_noalloc(X.data_ptr(), _dtype_code(X), n_mat, N, D, X.stride(0), X.stride(1), int(k_trunc),
                                         int(flags), entropy_out.data_ptr(), _ptr(eig_out), _stream())
    if st != OK:
        raise UncompError(st, lib.uncomp_last_error(None).decode())
    return entropy_out, eig_out


class Context:
    """Owns one uncomp_ctx (device workspace).  ``workspace_bytes=0`` takes the library default."""

    def __init__(self, device: int = 0, workspace_bytes: int = 0):
        self.lib = load_library()
        h = ctypes.c_void_p()
        st = self.lib.uncomp_create(ctypes.byref(h), int(device), int(workspace_bytes))
        if st != OK:
            raise UncompError(st, "uncomp_create failed")
        self.handle = h
        self.device = device

    @staticmethod
    def workspace_bytes(n_mat: int, N: int, D: int, B: int, H: int, G: int, w: int) -> int:
        return int(load_library().uncomp_workspace_bytes(n_mat, N, D, B, H, G, w))

    @staticmethod
    def decode_workspace_bytes(n_heads: int, G: int, cap: int) -> int:
        return int(load_library().uncomp_decode_workspace_bytes(n_heads, G, cap))

    @staticmethod
    def hidden_workspace_bytes(B: int, H: int, G: int, N: int, w: int) -> int:
        return int(load_library().uncomp_hidden_workspace_bytes(B, H, G, N, w))

    @staticmethod
    def matrix_workspace_bytes(N: int, D: int) -> int:
        return int(load_library().uncomp_matrix_workspace_bytes(N, D))

    def close(self):
        if getattr(self, "handle", None) is not None and self.handle:
            self.lib.uncomp_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != OK:
            raise UncompError(st, self.lib.uncomp_last_error(self.handle).decode())

    def profile(self, on: bool):
        self._check(self.lib.uncomp_profile(self.handle, 1 if on else 0))

    def set_overlap(self, on: bool):
        self._check(self.lib.uncomp_set_overlap(self.handle, 1 if on else 0))

    def join(self):
        self._check(self.lib.uncomp_join(self.handle, _stream()))

    def set_kernel_path(self, plain_alu: bool):
        self._check(self.lib.uncomp_set_kernel_path(self.handle, 1 if plain_alu else 0))

    def measure_peaks(self, buf: torch.Tensor):
        """Streaming-read GB/s over `buf` (any device tensor of at least 64 MiB) and the bf16 MFMA loop's TFLOP/s
        on live and on zero operands.  Synchronises."""
        r, a, z = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        self._check(self.lib.uncomp_measure_peaks(self.handle, buf.data_ptr(), buf.numel() * buf.element_size(),
                                                  ctypes.byref(r), ctypes.byref(a), ctypes.byref(z), _stream()))
        return r.value, a.value, z.value

    def profile_read(self, max_records: int = 1024):
        """(kernel name, ms) of every launch since the last read; synchronise the stream first."""
        names = (ctypes.c_char_p * max_records)()
        ms = (ctypes.c_float * max_records)()
        n = self.lib.uncomp_profile_read(self.handle, max_records, names, ms)
        if n < 0:
            self._check(n)
        return [(names[i].decode(), float(ms[i])) for i in range(n)]

    # -- the four hot calls ------------------------------------------------------------
    def head_entropy(self, X: torch.Tensor, k_trunc: int = 32, flags: int = DEFAULT_FLAGS,
                     want_eig: bool = False, entropy_out=None, eig_out=None):
        """X [n_mat, N, D] (last dim contiguous).  Returns entropy [n_mat] (and eig [n_mat, D])."""
        n_mat, N, D = X.shape
        assert X.stride(2) == 1
        if entropy_out is None:
            entropy_out = torch.empty(n_mat, dtype=torch.float32, device=X.device)
        if want_eig and eig_out is None:
            eig_out = torch.empty(n_mat, D, dtype=torch.float32, device=X.device)
        self._check(self.lib.uncomp_head_entropy(
            self.handle, X.data_ptr(), _dtype_code(X), n_mat, N, D, X.stride(0), X.stride(1),
            int(k_trunc), int(flags), entropy_out.data_ptr(), _ptr(eig_out), _stream()))
        return (entropy_out, eig_out) if want_eig else entropy_out

    def assign_budgets(self, entropy: torch.Tensor, M: int, n_max: int, step: int, N: int, w: int,
                       eps: float = 0.4, delta_n: int = 512, flags: int = DEFAULT_FLAGS, out=None):
        """entropy [L, B, H] float32.  Returns head_budget, head_group [L,B,H], layer_group, layer_tokens [L]."""
        L, B, H = entropy.shape
        assert entropy.is_contiguous() and entropy.dtype == torch.float32
        if out is None:
            kw = dict(dtype=torch.int32, device=entropy.device)
            out = (torch.empty(L, B, H, **kw), torch.empty(L, B, H, **kw),
                   torch.empty(L, **kw), torch.empty(L, **kw))
        hb, hg, lg, lt = out
        self._check(self.lib.uncomp_assign_budgets(
            self.handle, entropy.data_ptr(), L, B, H, int(M), int(n_max), int(step), int(N), int(w),
            float(eps), int(delta_n), int(flags), _ptr(hb), _ptr(hg), _ptr(lg), _ptr(lt), _stream()))
        return hb, hg, lg, lt

    def window_score(self, Qwin: torch.Tensor, K: torch.Tensor, G: int, pool: int = 7, out=None, lse=None):
        """Qwin [B, H*G, w, D] contiguous, K [B, H, N, D] (last dim contiguous).  Returns score [B,H,N-w].
        lse: optional [B, H*G, w] float32 natural-log normalisers of the window rows (skips the library's own
        statistics pass)."""
        B, Hq, w, D = Qwin.shape
        _, H, N, _ = K.shape
        assert Qwin.is_contiguous() and K.stride(3) == 1 and Hq == H * G and Qwin.dtype == K.dtype
        if lse is not None:
            assert lse.shape == (B, Hq, w) and lse.dtype == torch.float32 and lse.is_contiguous()
        if out is None:
            out = torch.empty(B, H, N - w, dtype=torch.float32, device=K.device)
        strides = (ctypes.c_int64 * 3)(K.stride(0), K.stride(1), K.stride(2))
        self._check(self.lib.uncomp_window_score(
            self.handle, Qwin.data_ptr(), K.data_ptr(), _dtype_code(K), B, H, int(G), N, D, w, int(pool),
            strides, _ptr(lse), out.data_ptr(), _stream()))
        return out

    def select_gather(self, score: torch.Tensor, budget: torch.Tensor, K, V, w: int, cap: int, out=None,
                      N: int | None = None):
        """score [B,H,N-w] float32, budget [B,H] int32, K/V [B,H,N,D] or None.
        Returns K_out, V_out [B,H,cap,D] (None without K/V), idx [B,H,cap] int32, len [B,H] int32.
        Fresh outputs are zero-filled (idx with -1) so rows past len are defined."""
        B, H, P = score.shape
        assert score.is_contiguous() and budget.is_contiguous() and budget.dtype == torch.int32
        if K is not None:
            N, D = K.shape[2], K.shape[3]
            assert K.stride() == V.stride() and K.stride(3) == 1 and K.dtype == V.dtype
            strides = (ctypes.c_int64 * 3)(K.stride(0), K.stride(1), K.stride(2))
            code = _dtype_code(K)
        else:
            N, D = (P + w if N is None else N), 128
            strides = None
            code = BF16
        if out is None:
            dev = score.device
            Ko = torch.zeros(B, H, cap, D, dtype=K.dtype, device=dev) if K is not None else None
            Vo = torch.zeros(B, H, cap, D, dtype=V.dtype, device=dev) if K is not None else None
            out = (Ko, Vo, torch.full((B, H, cap), -1, dtype=torch.int32, device=dev),
                   torch.zeros(B, H, dtype=torch.int32, device=dev))
        Ko, Vo, idx, ln = out
        self._check(self.lib.uncomp_select_gather(
            self.handle, score.data_ptr(), budget.data_ptr(), _ptr(K), _ptr(V), code, B, H, N, D, int(w),
            strides, int(cap), _ptr(Ko), _ptr(Vo), idx.data_ptr(), ln.data_ptr(), _stream()))
        return Ko, Vo, idx, ln

    # -- decode-time eviction ------------------------------------------------------------
    def decode_init(self, score: torch.Tensor, idx: torch.Tensor, length: torch.Tensor, N: int, w: int, out=None):
        """score [..., N-w] float32, idx [..., cap] int32, length [...] int32 (leading dims = heads).
        Returns cum [..., cap] float32."""
        cap = idx.shape[-1]
        n_heads = length.numel()
        assert score.is_contiguous() and idx.is_contiguous() and length.is_contiguous()
        assert score.shape[-1] == N - w and score.numel() == n_heads * (N - w) and idx.numel() == n_heads * cap
        if out is None:
            out = torch.empty(idx.shape, dtype=torch.float32, device=idx.device)
        self._check(self.lib.uncomp_decode_init(
            self.handle, score.data_ptr(), idx.data_ptr(), length.data_ptr(), n_heads, int(N), int(w), cap,
            out.data_ptr(), _stream()))
        return out

    def decode_step(self, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor, pos: torch.Tensor,
                    budget: torch.Tensor, w: int, K_c: torch.Tensor, V_c: torch.Tensor, idx: torch.Tensor,
                    cum: torch.Tensor, length: torch.Tensor, out=None, evicted=None, want_out: bool = True):
        """q [n_heads, G, D], k_new / v_new [n_heads, D], pos / budget / length [n_heads] int32,
        K_c / V_c [n_heads, cap, D], idx / cum [n_heads, cap]; the cache tensors are updated in place
        (leading dims may be split, e.g. [B, H, ...]).  Returns out [n_heads, G, D] float32, evicted [n_heads]."""
        n_heads = length.numel()
        G, D = q.shape[-2], q.shape[-1]
        cap = idx.shape[-1]
        for t in (q, k_new, v_new, pos, budget, K_c, V_c, idx, cum, length):
            assert t.is_contiguous()
        assert q.dtype == K_c.dtype == V_c.dtype == k_new.dtype == v_new.dtype
        assert pos.dtype == budget.dtype == length.dtype == idx.dtype == torch.int32 and cum.dtype == torch.float32
        assert q.numel() == n_heads * G * D and K_c.numel() == n_heads * cap * D and k_new.numel() == n_heads * D
        if out is None and want_out:
            out = torch.empty(n_heads, G, D, dtype=torch.float32, device=q.device)
        if evicted is None:
            evicted = torch.empty(n_heads, dtype=torch.int32, device=q.device)
        self._check(self.lib.uncomp_decode_step(
            self.handle, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), _dtype_code(K_c), n_heads, G, D,
            pos.data_ptr(), budget.data_ptr(), int(w), cap, K_c.data_ptr(), V_c.data_ptr(), idx.data_ptr(),
            cum.data_ptr(), length.data_ptr(), _ptr(out), evicted.data_ptr(), _stream()))
        return out, evicted

    # -- stage-1 hidden-state eviction ------------------------------------------------------
    def hidden_evict(self, q_last: torch.Tensor, K: torch.Tensor, G: int, n_keep: torch.Tensor, w: int,
                     Hs, cap: int, want_score: bool = False, out=None):
        """q_last [B, H*G, D] contiguous, K [B, H, N, D] (last dim contiguous), n_keep a one-element int32
        device tensor, Hs [B, N, Dm] (last dim contiguous) or None.
        Returns Hs_out [B, cap, Dm] (None without Hs), idx [B, cap] int32, len [B] int32, score [B, N-w] or None."""
        B, Hq, D = q_last.shape
        _, H, N, _ = K.shape
        assert q_last.is_contiguous() and K.stride(3) == 1 and Hq == H * G and q_last.dtype == K.dtype
        assert n_keep.dtype == torch.int32 and n_keep.numel() >= 1
        ks = (ctypes.c_int64 * 3)(K.stride(0), K.stride(1), K.stride(2))
        dev = K.device
        if Hs is not None:
            assert Hs.stride(2) == 1 and Hs.dtype == K.dtype and Hs.shape[0] == B and Hs.shape[1] == N
            Dm = Hs.shape[2]
            hs = (ctypes.c_int64 * 2)(Hs.stride(0), Hs.stride(1))
        else:
            Dm, hs = 0, None
        if out is None:
            out = (torch.zeros(B, cap, Dm, dtype=K.dtype, device=dev) if Hs is not None else None,
                   torch.full((B, cap), -1, dtype=torch.int32, device=dev),
                   torch.zeros(B, dtype=torch.int32, device=dev))
        Ho, idx, ln = out
        score = torch.empty(B, N - w, dtype=torch.float32, device=dev) if want_score else None
        self._check(self.lib.uncomp_hidden_evict(
            self.handle, q_last.data_ptr(), K.data_ptr(), _dtype_code(K), B, H, int(G), N, D, ks,
            n_keep.data_ptr(), int(w), _ptr(Hs), hs, Dm, int(cap), _ptr(Ho), idx.data_ptr(), ln.data_ptr(),
            _ptr(score), _stream()))
        return Ho, idx, ln, score

    # -- offline preparation ------------------------------------------------------------------
    def prepare_new(self, L: int, H: int, M: int, device="cuda:0"):
        """Fresh running statistics: (erank_sum [L,H] float64, votes [L,H,M] int32, count [1] int32)."""
        st = (torch.empty(L, H, dtype=torch.float64, device=device), torch.empty(L, H, M, dtype=torch.int32, device=device),
              torch.empty(1, dtype=torch.int32, device=device))
        self._check(self.lib.uncomp_prepare_reset(self.handle, L, H, M, st[0].data_ptr(), st[1].data_ptr(),
                                                  st[2].data_ptr(), _stream()))
        return st

    def prepare_accumulate(self, state, entropy: torch.Tensor):
        """entropy [L, B, H] float32 contiguous: adds its B samples to the statistics."""
        L, B, H = entropy.shape
        es, votes, count = state
        assert entropy.is_contiguous() and entropy.dtype == torch.float32 and es.shape == (L, H)
        self._check(self.lib.uncomp_prepare_accumulate(self.handle, entropy.data_ptr(), L, B, H, votes.shape[2],
                                                       es.data_ptr(), votes.data_ptr(), count.data_ptr(), _stream()))

    def prepare_finish(self, state, want_mean: bool = False):
        """Returns labels_mean, labels_vote [L,H] int32 (and the mean erank [L,H] float32)."""
        es, votes, count = state
        L, H, M = votes.shape
        lm = torch.empty(L, H, dtype=torch.int32, device=es.device)
        lv = torch.empty_like(lm)
        mean = torch.empty(L, H, dtype=torch.float32, device=es.device) if want_mean else None
        self._check(self.lib.uncomp_prepare_finish(self.handle, L, H, M, es.data_ptr(), votes.data_ptr(),
                                                   count.data_ptr(), lm.data_ptr(), lv.data_ptr(), _ptr(mean), _stream()))
        return (lm, lv, mean) if want_mean else (lm, lv)

    def budgets_from_labels(self, labels: torch.Tensor, B: int, n_max: int, step: int, N: int, w: int, out=None):
        """labels [L,H] int32 -> head_budget [L,B,H] int32."""
        L, H = labels.shape
        assert labels.is_contiguous() and labels.dtype == torch.int32
        if out is None:
            out = torch.empty(L, B, H, dtype=torch.int32, device=labels.device)
        self._check(self.lib.uncomp_budgets_from_labels(self.handle, labels.data_ptr(), L, int(B), H, int(n_max),
                                                        int(step), int(N), int(w), out.data_ptr(), _stream()))
        return out

    # -- entropy of wide token matrices --------------------------------------------------------
    def matrix_entropy(self, X: torch.Tensor, k_trunc: int = 32, flags: int = DEFAULT_FLAGS, n_iter: int = 8,
                       want_eig: bool = False):
        """X [n_mat, N, D] (last dim contiguous), D a multiple of 128 above 128.
        Returns entropy [n_mat] (and the 128 Ritz values [n_mat, 128] as shares of the trace)."""
        n_mat, N, D = X.shape
        assert X.stride(2) == 1
        ent = torch.empty(n_mat, dtype=torch.float32, device=X.device)
        eig = torch.empty(n_mat, 128, dtype=torch.float32, device=X.device) if want_eig else None
        self._check(self.lib.uncomp_matrix_entropy(
            self.handle, X.data_ptr(), _dtype_code(X), n_mat, N, D, X.stride(0), X.stride(1), int(k_trunc), int(flags),
            int(n_iter), ent.data_ptr(), _ptr(eig), _stream()))
        return (ent, eig) if want_eig else ent
