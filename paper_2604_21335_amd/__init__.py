"""Python binding of libstc (HIP, MI355X): decode attention over a Quest-selected,
group-packed KV cache.  The functions below have the names of the C entry
points in include/stc.h and only marshal arguments; every step of the path runs
in the HIP kernels.  PyTorch is used for device memory and the current stream.

There is no CPU fallback: if libstc.so cannot be loaded the calls raise.
"""
import ctypes
import os

import torch

from . import workloads  # noqa: F401  (seeded synthetic inputs)

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libstc.so")

STC_OK = 0
STC_ERR_NULL, STC_ERR_SHAPE, STC_ERR_ALIGN, STC_ERR_WORKSPACE, STC_ERR_LAUNCH = -1, -2, -3, -4, -5
STC_WS_ROUTE, STC_WS_SELECT, STC_WS_ATTENTION, STC_WS_ATTENTION_TAIL = 1, 2, 3, 4
STC_WS_SELECT_PER_HEAD, STC_WS_ATTENTION_PER_HEAD, STC_WS_STEP, STC_WS_STEP_TAIL = 5, 6, 7, 8
STC_ROUTE_MASK, STC_ROUTE_TOPK, STC_ROUTE_GLOBAL = 0, 1, 2
STC_ROUTE_SHARED = 0x100        # flag: one set of routing inputs per batch element

EXPORTS = ["stc_version", "stc_status_string", "stc_workspace_bytes", "stc_bounds_bytes",
           "stc_build_page_bounds",
           "stc_route_and_pack_values", "stc_select_pages", "stc_score_pages", "stc_decode_attention", "stc_decode_attention_tail", "stc_append_tail",
           "stc_select_pages_per_head", "stc_decode_attention_per_head", "stc_router_logits",
           "stc_union_pages", "stc_decode_attention_union", "stc_flush_tail",
           "stc_compact_tokens", "stc_decode_step", "stc_decode_step_tail",
           "stc_decode_step_static"]


class StcError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, status_string(status)))


class stc_shape_t(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("D", ctypes.c_int32), ("N", ctypes.c_int32), ("P", ctypes.c_int32),
                ("G", ctypes.c_int32), ("N_cap", ctypes.c_int32),
                ("v_cap_groups", ctypes.c_int64)]


def make_shape(B, Hq, Hkv, D, N, G, v_cap_groups, P=16, N_cap=0):
    """N_cap: token capacity (stride) of K, mask, tok_off and bounds; 0 = exactly N."""
    return stc_shape_t(B, Hq, Hkv, D, N, P, G, N_cap, v_cap_groups)


_lib = None


def load_library():
    """dlopen libstc.so from the package directory; build it first only if it is
    absent.  Raises if it can neither be found nor built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from .build import build_library
        build_library()
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    shp = ctypes.POINTER(stc_shape_t)
    lib.stc_version.restype = ctypes.c_int
    lib.stc_version.argtypes = []
    lib.stc_status_string.restype = ctypes.c_char_p
    lib.stc_status_string.argtypes = [ctypes.c_int]
    lib.stc_workspace_bytes.restype = sz
    lib.stc_workspace_bytes.argtypes = [shp, ctypes.c_int, ctypes.c_int]
    lib.stc_bounds_bytes.restype = ctypes.c_size_t
    lib.stc_bounds_bytes.argtypes = [shp]
    lib.stc_build_page_bounds.restype = ctypes.c_int
    lib.stc_build_page_bounds.argtypes = [shp, vp, vp, vp]
    lib.stc_route_and_pack_values.restype = ctypes.c_int
    lib.stc_route_and_pack_values.argtypes = [shp, ctypes.c_int, vp, vp, vp, ctypes.c_int, vp, vp,
                                              vp, vp, vp, vp, sz, vp]
    lib.stc_select_pages.restype = ctypes.c_int
    lib.stc_select_pages.argtypes = [shp, vp, vp, ctypes.c_int, vp, vp, vp, sz, vp]
    lib.stc_score_pages.restype = ctypes.c_int
    lib.stc_score_pages.argtypes = [shp, vp, vp, vp, vp]
    lib.stc_decode_attention.restype = ctypes.c_int
    lib.stc_decode_attention.argtypes = [shp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp, sz, vp]
    lib.stc_select_pages_per_head.restype = ctypes.c_int
    lib.stc_select_pages_per_head.argtypes = lib.stc_select_pages.argtypes
    lib.stc_decode_attention_per_head.restype = ctypes.c_int
    lib.stc_decode_attention_per_head.argtypes = lib.stc_decode_attention.argtypes
    lib.stc_flush_tail.restype = ctypes.c_int
    lib.stc_flush_tail.argtypes = [shp, vp, vp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_int, vp, vp,
                                   ctypes.c_int, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.stc_union_pages.restype = ctypes.c_int
    lib.stc_union_pages.argtypes = [shp, vp, ctypes.c_int, vp, vp, ctypes.c_int, vp]
    lib.stc_decode_attention_union.restype = ctypes.c_int
    lib.stc_decode_attention_union.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp,
                                               sz, vp]
    lib.stc_decode_attention_tail.restype = ctypes.c_int
    lib.stc_decode_attention_tail.argtypes = [shp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp,
                                              ctypes.c_int, ctypes.c_int, vp, vp, sz, vp]
    lib.stc_decode_step.restype = ctypes.c_int
    lib.stc_decode_step.argtypes = [shp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp, vp, sz, vp]
    lib.stc_decode_step_static.restype = ctypes.c_int
    lib.stc_decode_step_static.argtypes = [shp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp, vp]
    lib.stc_decode_step_tail.restype = ctypes.c_int
    lib.stc_decode_step_tail.argtypes = [shp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp,
                                         ctypes.c_int, ctypes.c_int, vp, vp, vp, sz, vp]
    lib.stc_append_tail.restype = ctypes.c_int
    lib.stc_append_tail.argtypes = [shp, vp, vp, vp, vp, ctypes.c_int, ctypes.c_int, vp]
    lib.stc_router_logits.restype = ctypes.c_int
    lib.stc_router_logits.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, i32, vp, vp]
    lib.stc_compact_tokens.restype = ctypes.c_int
    lib.stc_compact_tokens.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]
    _lib = lib
    return lib


def status_string(status):
    return load_library().stc_status_string(int(status)).decode()


def _ptr(t, dtype=None, name="tensor"):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a CUDA tensor" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise TypeError("%s has dtype %s" % (name, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _check(status, where):
    if status != STC_OK:
        raise StcError(status, where)


_U16 = (torch.int16, torch.uint16)
_U32 = (torch.int32, torch.uint32)


def stc_version():
    return load_library().stc_version()


def stc_workspace_bytes(shape, which_call, k_pages=0):
    return int(load_library().stc_workspace_bytes(ctypes.byref(shape), which_call, k_pages))


def stc_bounds_bytes(shape):
    return int(load_library().stc_bounds_bytes(ctypes.byref(shape)))


def bounds_rows(bounds, shape):
    """The tiled bounds buffer as a [B, Hkv, NP, 2, D] tensor (row 0 = minima, row 1 = maxima):
    a pure re-ordering of its elements, for inspection and tests."""
    B, Hkv, D = shape.B, shape.Hkv, shape.D
    NP = (shape.N + shape.P - 1) // shape.P
    cap = shape.N_cap or shape.N
    nt = ((cap + shape.P - 1) // shape.P + 7) // 8          # tiles per stream in memory
    # dwords [s][t][j][g][e][col][w], each (min, max)
    t = bounds.reshape(B, Hkv, nt, D // 32, 2, 8, 4, 4, 2)
    # -> [B, Hkv, t, g, col, (min|max), e, j, w]
    t = t.permute(0, 1, 2, 4, 6, 8, 5, 3, 7)
    return t.reshape(B, Hkv, nt * 8, 2, D)[:, :, :NP].contiguous()


def stc_build_page_bounds(shape, K, bounds):
    _check(load_library().stc_build_page_bounds(
        ctypes.byref(shape), _ptr(K, torch.bfloat16, "K"), _ptr(bounds, torch.bfloat16, "bounds"),
        _stream()), "stc_build_page_bounds")


def stc_route_and_pack_values(shape, mode, V, logits, kcount, fixed_k, mask_in, mask, tok_off,
                              vpacked, dev_status, ws):
    _check(load_library().stc_route_and_pack_values(
        ctypes.byref(shape), mode, _ptr(V, torch.bfloat16, "V"),
        _ptr(logits, torch.float32, "logits"), _ptr(kcount, torch.uint8, "kcount"), int(fixed_k),
        _ptr(mask_in, _U16, "mask_in"), _ptr(mask, _U16, "mask"), _ptr(tok_off, _U32, "tok_off"),
        _ptr(vpacked, torch.bfloat16, "vpacked"), _ptr(dev_status, torch.int32, "dev_status"),
        _ptr(ws, None, "ws"), _nbytes(ws), _stream()), "stc_route_and_pack_values")


def stc_select_pages(shape, q, bounds, k_pages, page_idx, page_score, ws):
    _check(load_library().stc_select_pages(
        ctypes.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(bounds, torch.bfloat16, "bounds"),
        int(k_pages), _ptr(page_idx, torch.int32, "page_idx"),
        _ptr(page_score, torch.float32, "page_score"), _ptr(ws, None, "ws"), _nbytes(ws),
        _stream()), "stc_select_pages")


def stc_score_pages(shape, q, bounds, page_score):
    _check(load_library().stc_score_pages(
        ctypes.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(bounds, torch.bfloat16, "bounds"),
        _ptr(page_score, torch.float32, "page_score"), _stream()), "stc_score_pages")


def stc_decode_attention(shape, q, K, vpacked, mask, tok_off, page_idx, k_pages, out, ws):
    _check(load_library().stc_decode_attention(
        ctypes.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(K, torch.bfloat16, "K"),
        _ptr(vpacked, torch.bfloat16, "vpacked"), _ptr(mask, _U16, "mask"),
        _ptr(tok_off, _U32, "tok_off"), _ptr(page_idx, torch.int32, "page_idx"), int(k_pages),
        _ptr(out, torch.float32, "out"), _ptr(ws, None, "ws"), _nbytes(ws), _stream()),
        "stc_decode_attention")


def stc_select_pages_per_head(shape, q, bounds, k_pages, page_idx, page_score, ws):
    _check(load_library().stc_select_pages_per_head(
        ctypes.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(bounds, torch.bfloat16, "bounds"),
        int(k_pages), _ptr(page_idx, torch.int32, "page_idx"),
        _ptr(page_score, torch.float32, "page_score"), _ptr(ws, None, "ws"), _nbytes(ws),
        _stream()), "stc_select_pages_per_head")


def stc_decode_attention_per_head(shape, q, K, vpacked, mask, tok_off, page_idx, k_pages, out, ws):
    _check(load_library().stc_decode_attention_per_head(
        ctypes.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(K, torch.bfloat16, "K"),
        _ptr(vpacked, torch.bfloat16, "vpacked"), _ptr(mask, _U16, "mask"),
        _ptr(tok_off, _U32, "tok_off"), _ptr(page_idx, torch.int32, "page_idx"), int(k_pages),
        _ptr(out, torch.float32, "out"), _ptr(ws, None, "ws"), _nbytes(ws), _stream()),
        "stc_decode_attention_per_head")


def stc_flush_tail(shape, K_tail, V_tail, n_flush, n_tail, tail_cap, mode, logits, kcount, fixed_k, mask_in,
                   K, bounds, mask, tok_off, vpacked, dev_status):
    _check(load_library().stc_flush_tail(
        ctypes.byref(shape), _ptr(K_tail, torch.bfloat16, "K_tail"),
        _ptr(V_tail, torch.bfloat16, "V_tail"), int(n_flush), int(n_tail), int(tail_cap), int(mode),
        _ptr(logits, torch.float32, "logits"), _ptr(kcount, torch.uint8, "kcount"), int(fixed_k),
        _ptr(mask_in, _U16, "mask_in"), _ptr(K, torch.bfloat16, "K"),
        _ptr(bounds, torch.bfloat16, "bounds"), _ptr(mask, _U16, "mask"),
        _ptr(tok_off, _U32, "tok_off"), _ptr(vpacked, torch.bfloat16, "vpacked"),
        _ptr(dev_status, torch.int32, "dev_status"), _stream()), "stc_flush_tail")


def stc_union_pages(shape, page_idx_per_head, k_pages, union_idx, union_heads):
    _check(load_library().stc_union_pages(
        ctypes.byref(shape), _ptr(page_idx_per_head, torch.int32, "page_idx_per_head"),
        int(k_pages), _ptr(union_idx, torch.int32, "union_idx"),
        _ptr(union_heads, _U16, "union_heads"), int(union_idx.shape[-1]), _stream()),
        "stc_union_pages")


def stc_decode_attention_union(shape, q, K, vpacked, mask, tok_off, union_idx, union_heads, out,
                               ws):
    _check(load_library().stc_decode_attention_union(
        ctypes.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(K, torch.bfloat16, "K"),
        _ptr(vpacked, torch.bfloat16, "vpacked"), _ptr(mask, _U16, "mask"),
        _ptr(tok_off, _U32, "tok_off"), _ptr(union_idx, torch.int32, "union_idx"),
        _ptr(union_heads, _U16, "union_heads"), int(union_idx.shape[-1]),
        _ptr(out, torch.float32, "out"), _ptr(ws, None, "ws"), _nbytes(ws), _stream()),
        "stc_decode_attention_union")


def stc_decode_step(shape, q, bounds, K, vpacked, mask, tok_off, k_pages, page_idx, out, ws):
    _check(load_library().stc_decode_step(
        ctypes.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(bounds, torch.bfloat16, "bounds"),
        _ptr(K, torch.bfloat16, "K"), _ptr(vpacked, torch.bfloat16, "vpacked"),
        _ptr(mask, _U16, "mask"), _ptr(tok_off, _U32, "tok_off"), int(k_pages),
        _ptr(page_idx, torch.int32, "page_idx"), _ptr(out, torch.float32, "out"),
        _ptr(ws, None, "ws"), _nbytes(ws), _stream()), "stc_decode_step")


STC_STATIC_SCRATCH_BYTES = 8 * 1024 * 1024


def stc_decode_step_static(shape, q, bounds, K, vpacked, mask, tok_off, k_pages, page_idx, out):
    """stc_decode_step over the library's own static scratch array: no workspace argument."""
    _check(load_library().stc_decode_step_static(
        ctypes.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(bounds, torch.bfloat16, "bounds"),
        _ptr(K, torch.bfloat16, "K"), _ptr(vpacked, torch.bfloat16, "vpacked"),
        _ptr(mask, _U16, "mask"), _ptr(tok_off, _U32, "tok_off"), int(k_pages),
        _ptr(page_idx, torch.int32, "page_idx"), _ptr(out, torch.float32, "out"), _stream()),
        "stc_decode_step_static")


def stc_decode_step_tail(shape, q, bounds, K, vpacked, mask, tok_off, k_pages, K_tail, V_tail,
                         n_tail, tail_cap, page_idx, out, ws):
    _check(load_library().stc_decode_step_tail(
        ctypes.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(bounds, torch.bfloat16, "bounds"),
        _ptr(K, torch.bfloat16, "K"), _ptr(vpacked, torch.bfloat16, "vpacked"),
        _ptr(mask, _U16, "mask"), _ptr(tok_off, _U32, "tok_off"), int(k_pages),
        _ptr(K_tail, torch.bfloat16, "K_tail"), _ptr(V_tail, torch.bfloat16, "V_tail"),
        int(n_tail), int(tail_cap), _ptr(page_idx, torch.int32, "page_idx"),
        _ptr(out, torch.float32, "out"), _ptr(ws, None, "ws"), _nbytes(ws), _stream()),
        "stc_decode_step_tail")


def stc_decode_attention_tail(shape, q, K, vpacked, mask, tok_off, page_idx, k_pages, K_tail,
                              V_tail, n_tail, tail_cap, out, ws):
    _check(load_library().stc_decode_attention_tail(
        ctypes.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(K, torch.bfloat16, "K"),
        _ptr(vpacked, torch.bfloat16, "vpacked"), _ptr(mask, _U16, "mask"),
        _ptr(tok_off, _U32, "tok_off"), _ptr(page_idx, torch.int32, "page_idx"), int(k_pages),
        _ptr(K_tail, torch.bfloat16, "K_tail"), _ptr(V_tail, torch.bfloat16, "V_tail"),
        int(n_tail), int(tail_cap), _ptr(out, torch.float32, "out"), _ptr(ws, None, "ws"),
        _nbytes(ws), _stream()), "stc_decode_attention_tail")


def stc_append_tail(shape, k_new, v_new, K_tail, V_tail, n_tail, tail_cap):
    _check(load_library().stc_append_tail(
        ctypes.byref(shape), _ptr(k_new, torch.bfloat16, "k_new"),
        _ptr(v_new, torch.bfloat16, "v_new"), _ptr(K_tail, torch.bfloat16, "K_tail"),
        _ptr(V_tail, torch.bfloat16, "V_tail"), int(n_tail), int(tail_cap), _stream()),
        "stc_append_tail")


def stc_router_logits(h, W, bias, logits, Hkv):
    """h [B, N, d_model] bf16, W [G, d_model] bf16, bias [G] or [B, G] float32 or None ->
    logits [B, Hkv, N, G] float32 (the same for every KV head).  A [B, G] bias is one vector
    per batch element (the query term of a query-conditioned router)."""
    B, N, dm = h.shape
    G = W.shape[0]
    per_batch = 0
    if bias is not None and bias.dim() == 2:
        if tuple(bias.shape) != (B, G):
            raise ValueError("a per-element bias must be [B, G]")
        per_batch = 1
    _check(load_library().stc_router_logits(
        B, Hkv, N, dm, G, _ptr(h, torch.bfloat16, "h"), _ptr(W, torch.bfloat16, "W"),
        _ptr(bias, torch.float32, "bias"), per_batch, _ptr(logits, torch.float32, "logits"),
        _stream()), "stc_router_logits")


def stc_compact_tokens(src, token_idx, dst, B, Hkv, N_src, n_keep, D, dev_status=None):
    _check(load_library().stc_compact_tokens(
        _ptr(src, torch.bfloat16, "src"), _ptr(token_idx, torch.int32, "token_idx"),
        _ptr(dst, torch.bfloat16, "dst"), B, Hkv, N_src, n_keep, D,
        _ptr(dev_status, torch.int32, "dev_status"), _stream()), "stc_compact_tokens")


class RoutedCache:
    """Device buffers of one layer's compressed cache plus per-step outputs.

    Allocation (through torch, all of it in the constructor, sized for the token capacity) and
    nothing else: every computation is one of the stc_* calls above.
    """

    def __init__(self, B, Hq, Hkv, D, N, G, k_pages, v_cap_groups=None, device="cuda:0",
                 keep_scores=True, tail_cap=0, n_cap=0):
        """n_cap > N: room for n_cap tokens, so that tail tokens can be moved into the cache
        (flush); the cache then keeps its own copy of K."""
        self.device = torch.device(device)
        self.B, self.Hq, self.Hkv, self.D, self.N, self.G = B, Hq, Hkv, D, N, G
        self.n_cap = n_cap
        self.keep_scores = keep_scores
        self.k_pages = k_pages
        cap = (n_cap or N) * G if v_cap_groups is None else v_cap_groups
        self.shape = make_shape(B, Hq, Hkv, D, N, G, cap, N_cap=n_cap)
        dev = self.device
        Nc = n_cap or N                     # strides of mask and tok_off; most tokens ever held
        NPc = (Nc + 15) // 16
        k_max = min(k_pages, NPc)
        tail_pages = (tail_cap + 15) // 16
        self.bounds = torch.empty(stc_bounds_bytes(self.shape) // 2, dtype=torch.bfloat16,
                                  device=dev)
        self.mask = torch.empty(B, Hkv, Nc, dtype=torch.int16, device=dev)
        self.tok_off = torch.empty(B, Hkv, Nc + 1, dtype=torch.int32, device=dev)
        self.vpacked = torch.empty(B, Hkv, cap, D // G, dtype=torch.bfloat16, device=dev)
        self.dev_status = torch.zeros(1, dtype=torch.int32, device=dev)
        self._page_idx_buf = torch.empty(B * Hkv * k_max, dtype=torch.int32, device=dev)
        self.out = torch.empty(B, Hq, D, dtype=torch.float32, device=dev)
        self.K = (torch.empty(B, Hkv, n_cap, D, dtype=torch.bfloat16, device=dev)
                  if n_cap else None)
        # uncompressed tail of recent tokens (tail_cap = 0: none)
        self.tail_cap, self.n_tail = tail_cap, 0
        if tail_cap:
            self.K_tail = torch.empty(B, Hkv, tail_cap, D, dtype=torch.bfloat16, device=dev)
            self.V_tail = torch.empty_like(self.K_tail)
        # workspaces for the largest shape the cache can reach (sizes grow with N and k)
        big = make_shape(B, Hq, Hkv, D, Nc, G, cap, N_cap=n_cap)

        def ws(which, k):
            return torch.empty(max(stc_workspace_bytes(big, which, k), 16), dtype=torch.uint8,
                               device=dev)
        self._ws_route = ws(STC_WS_ROUTE, 0)
        self._ws_select = ws(STC_WS_SELECT, 1)
        self._ws_attn = ws(STC_WS_ATTENTION_TAIL if tail_cap else STC_WS_ATTENTION,
                           k_max + tail_pages)
        self._ws_step = ws(STC_WS_STEP_TAIL, k_max + tail_pages)
        self._scores_all = (torch.empty(B * Hkv * NPc, dtype=torch.float32, device=dev)
                            if keep_scores else None)    # scores when every page is kept
        self._resize()

    def _resize(self):
        """Views for the current token count (no allocation): page list, page scores."""
        self.NP = (self.N + 15) // 16
        self.k_eff = min(self.k_pages, self.NP)
        B, Hkv = self.B, self.Hkv
        self.page_idx = self._page_idx_buf[:B * Hkv * self.k_eff].view(B, Hkv, self.k_eff)
        if self.k_pages >= self.NP:      # every page is kept: the list is 0 .. NP-1
            stc_select_pages(self.shape, None, None, self.k_pages, self.page_idx, None, None)
        self._step_cache = None
        # the page scores sit at the front of the workspace of stc_decode_step: page_score is a
        # view of them, so that both forms of step() leave the scores there
        self.page_score = None
        if self.keep_scores:
            n = B * Hkv * self.NP
            if self.k_pages < self.NP or self.tail_cap:
                src = self._ws_step[:4 * n].view(torch.float32)
            else:
                src = self._scores_all[:n]
            self.page_score = src.view(B, Hkv, self.NP)

    def build(self, K, V, logits=None, kcount=None, fixed_k=0, mask_in=None, global_k=None,
              shared=False):
        """Cache construction: page bounds of K, routing mask + packed store of V.  The mask
        comes from mask_in, from a global budget of N*global_k token-group pairs per stream,
        or from the per-token top kcount[t] / fixed_k of the logits.  shared: the routing
        inputs are [B, 1, ...], one set per batch element for all its KV heads."""
        if self.n_cap:
            self.K[:, :, :self.N].copy_(K)
        else:
            self.K = K
        self._step_cache = None
        stc_build_page_bounds(self.shape, self.K, self.bounds)
        mode = STC_ROUTE_MASK if mask_in is not None else STC_ROUTE_TOPK
        if global_k is not None:
            mode, fixed_k, kcount = STC_ROUTE_GLOBAL, int(global_k), None
        if shared:
            mode |= STC_ROUTE_SHARED
        stc_route_and_pack_values(self.shape, mode, V, logits, kcount, fixed_k, mask_in, self.mask,
                                  self.tok_off, self.vpacked, self.dev_status, self._ws_route)

    def bounds_rows(self):
        return bounds_rows(self.bounds, self.shape)

    def select(self, q):
        stc_select_pages(self.shape, q, self.bounds, self.k_pages, self.page_idx, self.page_score,
                         self._ws_select)

    def score(self, q, page_score):
        stc_score_pages(self.shape, q, self.bounds, page_score)

    def append(self, k_new, v_new):
        """New token of every stream ([B, Hkv, D] each) into the uncompressed tail."""
        stc_append_tail(self.shape, k_new, v_new, self.K_tail, self.V_tail, self.n_tail,
                        self.tail_cap)
        self.n_tail += 1

    def flush(self, n, logits=None, kcount=None, fixed_k=0, mask_in=None):
        """Move the oldest n tail tokens into the compressed cache (routing them by mask_in,
        or by the top kcount[t] / fixed_k of logits); the call moves the rest of the tail to
        its front."""
        mode = STC_ROUTE_MASK if mask_in is not None else STC_ROUTE_TOPK
        stc_flush_tail(self.shape, self.K_tail, self.V_tail, n, self.n_tail, self.tail_cap, mode,
                       logits, kcount, fixed_k, mask_in, self.K, self.bounds, self.mask,
                       self.tok_off, self.vpacked, self.dev_status)
        self.n_tail -= n
        self.N += n
        self.shape.N = self.N
        self._resize()

    def attend(self, q):
        page_idx = self.page_idx if self.k_pages < self.NP else None
        if self.tail_cap:
            stc_decode_attention_tail(self.shape, q, self.K, self.vpacked, self.mask, self.tok_off,
                                      page_idx, self.k_eff, self.K_tail, self.V_tail,
                                      self.n_tail, self.tail_cap, self.out, self._ws_attn)
            return
        stc_decode_attention(self.shape, q, self.K, self.vpacked, self.mask, self.tok_off,
                             page_idx, self.k_eff, self.out, self._ws_attn)

    def _step_args(self):
        """C arguments of the one-call step for this cache's own tensors, validated once;
        step() fills in the query, the tail length and the stream."""
        if self._step_cache is None:
            fixed = [ctypes.byref(self.shape), None, _ptr(self.bounds, torch.bfloat16, "bounds"),
                     _ptr(self.K, torch.bfloat16, "K"), _ptr(self.vpacked, torch.bfloat16, "vpacked"),
                     _ptr(self.mask, _U16, "mask"), _ptr(self.tok_off, _U32, "tok_off"),
                     int(self.k_eff)]
            if self.tail_cap:
                fixed += [_ptr(self.K_tail, torch.bfloat16, "K_tail"),
                          _ptr(self.V_tail, torch.bfloat16, "V_tail"), 0, int(self.tail_cap)]
            fixed += [_ptr(self.page_idx, torch.int32, "page_idx"),
                      _ptr(self.out, torch.float32, "out"), _ptr(self._ws_step, None, "ws"),
                      _nbytes(self._ws_step), None]
            lib = load_library()
            self._step_cache = (lib.stc_decode_step_tail if self.tail_cap else lib.stc_decode_step,
                                fixed)
        return self._step_cache

    def step(self, q, one_call=True):
        """One decode step: page selection, then routed attention.  When every page is kept
        there is nothing to select: the attention call takes "all pages" as a missing list.
        one_call: through stc_decode_step (the page scores then stay in its workspace)
        instead of stc_select_pages + stc_decode_attention."""
        if self.k_pages < self.NP:
            if one_call:
                fn, args = self._step_args()
                args[1] = _ptr(q, torch.bfloat16, "q")
                if self.tail_cap:
                    args[10] = int(self.n_tail)
                args[-1] = _stream()
                _check(fn(*args), "stc_decode_step")
                return self.out
            self.select(q)
        self.attend(q)
        return self.out
