"""ctypes binding of include/molret.h.  Argument marshalling only: every step of the retrieval path runs in
the HIP kernels of libmolret.so; torch provides device memory and the current stream.  There is no fallback:
if the library is missing, loading raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

HINDEXER_EXACT = 0
HINDEXER_PAPER = 1
HINDEXER_FORCE_REDO = 0x100
HINDEXER_DEFER_REDO = 0x200
PACK_BORROW_STAGE1 = 1
PACK_BORROW_EMBS = 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = (
    "mol_corpus_pack", "mol_corpus_free", "hindexer_workspace_bytes", "mol_workspace_bytes",
    "hindexer_default_lambda", "hindexer_topk", "mol_score", "mol_topk", "mol_last_error",
    "mol_profile_enable", "mol_profile_read", "mol_quantize_int8", "mol_gather_items",
    "mol_topk_static", "mol_static_init", "mol_topk_static_max_bytes",
    "mol_bench_stream_read", "mol_bench_gather",
)

PROF_SLOTS = ("sample_scores", "threshold", "scan_filter", "select", "user_gate", "mol_score", "final_topk", "spare")


class MolError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"molret status {status}: {message}")
        self.status = status


class _Config(C.Structure):
    _fields_ = [
        ("N", C.c_int64), ("d1", C.c_int32), ("stage1_dtype", C.c_int32),
        ("k_u", C.c_int32), ("k_x", C.c_int32), ("d_p", C.c_int32),
        ("d_gu", C.c_int32), ("d_gx", C.c_int32), ("H", C.c_int32),
        ("act", C.c_int32), ("logit_scale", C.c_float),
        ("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p),
        ("flags", C.c_uint32),
        ("gate_form", C.c_int32), ("d_hu", C.c_int32), ("d_hx", C.c_int32),
        ("Wu1", C.c_void_p), ("bu1", C.c_void_p), ("Wu2", C.c_void_p), ("bu2", C.c_void_p),
        ("Wx1", C.c_void_p), ("bx1", C.c_void_p), ("Wx2", C.c_void_p), ("bx2", C.c_void_p),
        ("mol_dtype", C.c_int32),
        ("k_x_gen", C.c_int32), ("d_s", C.c_int32), ("d_hg", C.c_int32),
        ("item_seed", C.c_void_p), ("Wg1", C.c_void_p), ("bg1", C.c_void_p), ("Wg2", C.c_void_p), ("bg2", C.c_void_p),
    ]


def lib_path() -> str:
    return os.path.join(_HERE, "libmolret.so")


def load_library() -> C.CDLL:
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` at the repo root")
    lib = C.CDLL(path)
    vp, i32, i64, u64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_uint64, C.c_size_t
    lib.mol_corpus_pack.argtypes = [C.POINTER(_Config), vp, vp, vp, vp, C.POINTER(vp)]
    lib.mol_corpus_pack.restype = i32
    lib.mol_corpus_free.argtypes = [vp]
    lib.mol_corpus_free.restype = i32
    lib.hindexer_workspace_bytes.argtypes = [vp, i32, i32, i64]
    lib.hindexer_workspace_bytes.restype = sz
    lib.mol_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.mol_workspace_bytes.restype = sz
    lib.hindexer_default_lambda.argtypes = [vp, i32]
    lib.hindexer_default_lambda.restype = i64
    lib.hindexer_topk.argtypes = [vp, vp, i32, i32, vp, i64, u64, i32, vp, vp, vp, vp, sz, vp]
    lib.hindexer_topk.restype = i32
    lib.mol_score.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp, sz, vp]
    lib.mol_score.restype = i32
    lib.mol_topk.argtypes = [vp, vp, vp, i32, vp, vp, i32, i32, vp, vp, vp, sz, vp]
    lib.mol_topk.restype = i32
    lib.mol_topk_static.argtypes = [vp, vp, vp, i32, vp, vp, i32, i32, vp, vp, vp]
    lib.mol_topk_static.restype = i32
    lib.mol_static_init.argtypes = []
    lib.mol_static_init.restype = i32
    lib.mol_topk_static_max_bytes.argtypes = []
    lib.mol_topk_static_max_bytes.restype = sz
    lib.mol_bench_stream_read.argtypes = [vp, sz, i32, vp, vp]
    lib.mol_bench_stream_read.restype = i32
    lib.mol_bench_gather.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    lib.mol_bench_gather.restype = i32
    lib.mol_profile_enable.argtypes = [i32]
    lib.mol_profile_enable.restype = i32
    lib.mol_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int)]
    lib.mol_profile_read.restype = i32
    lib.mol_quantize_int8.argtypes = [vp, i32, i64, C.c_float, vp, vp]
    lib.mol_quantize_int8.restype = i32
    lib.mol_gather_items.argtypes = [vp, vp, i32, i32, vp, vp]
    lib.mol_gather_items.restype = i32
    lib.mol_last_error.argtypes = []
    lib.mol_last_error.restype = C.c_char_p
    _LIB = lib
    return lib


def _check(status: int):
    if status != 0:
        raise MolError(status, load_library().mol_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Corpus:
    """Owns a mol_corpus_t handle (and references to borrowed tensors)."""

    def __init__(self, handle: int, N: int, d1: int, stage1_dtype, k_u: int, k_x: int, d_p: int, H: int, d_gu: int,
                 keep, mol_dtype=torch.bfloat16):
        self.mol_dtype = mol_dtype
        self.handle = handle
        self.N, self.d1, self.stage1_dtype = N, d1, stage1_dtype
        self.k_u, self.k_x, self.d_p, self.H, self.d_gu = k_u, k_x, d_p, H, d_gu
        self._keep = keep

    def free(self):
        if self.handle:
            load_library().mol_corpus_free(self.handle)
            self.handle = None
            self._keep = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def mol_corpus_pack(stage1_items: Optional[torch.Tensor], item_embs: torch.Tensor, item_gate: torch.Tensor,
                    W1: torch.Tensor, b1: Optional[torch.Tensor], W2: torch.Tensor, b2: Optional[torch.Tensor],
                    k_u: int, logit_scale: float = 1.0, act: str = "relu", borrow: bool = False,
                    user_mlp=None, item_mlp=None, item_seed: Optional[torch.Tensor] = None, gen_mlp=None) -> Corpus:
    """user_mlp / item_mlp = (Wa bf16 [d_h, d_in], ba f32 [d_h] or None, Wb bf16 [P, d_h], bb f32 [P] or None) select
    Algorithm 1's decomposed gate; W1 [H, P], b1, W2 [P, H], b2 are then the cross MLP.
    item_seed bf16 [N, d_s] and gen_mlp = (Wg1 [d_hg, d_s], bg1, Wg2 [k_g * d_p, d_hg], bg2): the last k_g item-side
    embeddings are generated on the fly (Section 3.1); item_embs then holds the cached k_x - k_g."""
    lib = load_library()
    decomposed = user_mlp is not None or item_mlp is not None
    if decomposed and (user_mlp is None or item_mlp is None):
        raise ValueError("the decomposed gate needs both user_mlp and item_mlp")
    N, k_x, d_p = item_embs.shape
    k_g = 0
    if gen_mlp is not None:
        if item_seed is None:
            raise ValueError("gen_mlp needs item_seed")
        k_g = gen_mlp[2].shape[0] // d_p
        k_x += k_g                     # item_embs holds the cached embeddings only
    t16 = item_embs.dtype
    if t16 not in (torch.bfloat16, torch.float16):
        raise ValueError("item_embs must be bfloat16 or float16")
    _dev(item_embs, t16, "item_embs")
    _dev(item_gate, t16, "item_gate")
    _dev(W1, t16, "W1")
    _dev(W2, t16, "W2")
    if b1 is not None:
        _dev(b1, torch.float32, "b1")
    if b2 is not None:
        _dev(b2, torch.float32, "b2")
    P, H = W2.shape
    d_gx = item_gate.shape[1]
    if decomposed:
        for name, mlp, d_in in (("user_mlp", user_mlp, None), ("item_mlp", item_mlp, d_gx)):
            Wa, ba, Wb, bb = mlp
            _dev(Wa, t16, name + " Wa")
            _dev(Wb, t16, name + " Wb")
            for bias in (ba, bb):
                if bias is not None:
                    _dev(bias, torch.float32, name + " bias")
            if Wb.shape != (P, Wa.shape[0]) or (d_in is not None and Wa.shape[1] != d_in):
                raise ValueError(f"inconsistent {name} shapes")
        d_gu = user_mlp[0].shape[1]
        if W1.shape != (H, P):
            raise ValueError("decomposed gate: W1 must be [H, P]")
    else:
        d_gu = W1.shape[1] - P - d_gx
    if P != k_u * k_x or W1.shape[0] != H or d_gu < 1 or item_gate.shape[0] != N:
        raise ValueError("inconsistent model shapes")
    cfg = _Config()
    cfg.mol_dtype = 3 if t16 == torch.float16 else 1
    if k_g:
        Wg1, bg1, Wg2, bg2 = gen_mlp
        _dev(item_seed, t16, "item_seed")
        _dev(Wg1, t16, "Wg1")
        _dev(Wg2, t16, "Wg2")
        for bias in (bg1, bg2):
            if bias is not None:
                _dev(bias, torch.float32, "generator bias")
        if item_seed.shape[0] != N or Wg1.shape[1] != item_seed.shape[1] or Wg2.shape != (k_g * d_p, Wg1.shape[0]):
            raise ValueError("inconsistent generator shapes")
        cfg.k_x_gen, cfg.d_s, cfg.d_hg = k_g, item_seed.shape[1], Wg1.shape[0]
        cfg.item_seed, cfg.Wg1, cfg.bg1, cfg.Wg2, cfg.bg2 = _ptr(item_seed), _ptr(Wg1), _ptr(bg1), _ptr(Wg2), _ptr(bg2)
    if decomposed:
        cfg.gate_form = 1
        cfg.d_hu, cfg.d_hx = user_mlp[0].shape[0], item_mlp[0].shape[0]
        cfg.Wu1, cfg.bu1, cfg.Wu2, cfg.bu2 = (_ptr(t) for t in user_mlp)
        cfg.Wx1, cfg.bx1, cfg.Wx2, cfg.bx2 = (_ptr(t) for t in item_mlp)
    cfg.N = N
    if stage1_items is not None:
        if stage1_items.dtype not in (torch.float32, torch.bfloat16, torch.int8):
            raise ValueError("stage1_items must be float32, bfloat16 or int8")
        _dev(stage1_items, stage1_items.dtype, "stage1_items")
        if stage1_items.shape[0] != N:
            raise ValueError("stage1_items rows != N")
        cfg.d1 = stage1_items.shape[1]
        cfg.stage1_dtype = {torch.float32: 0, torch.bfloat16: 1, torch.int8: 2}[stage1_items.dtype]
    else:
        cfg.d1 = 0
        cfg.stage1_dtype = 1
    cfg.k_u, cfg.k_x, cfg.d_p = k_u, k_x, d_p
    cfg.d_gu, cfg.d_gx, cfg.H = d_gu, d_gx, H
    cfg.act = {"relu": 0, "silu": 1}[act]
    cfg.logit_scale = logit_scale
    cfg.W1, cfg.b1, cfg.W2, cfg.b2 = _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2)
    cfg.flags = (PACK_BORROW_STAGE1 | PACK_BORROW_EMBS) if borrow else 0
    out = C.c_void_p()
    _check(lib.mol_corpus_pack(C.byref(cfg), _ptr(stage1_items), _ptr(item_embs), _ptr(item_gate), _stream(),
                               C.byref(out)))
    keep = (stage1_items, item_embs) if borrow else None
    corpus = Corpus(out.value, N, cfg.d1, None if stage1_items is None else stage1_items.dtype, k_u, k_x, d_p, H, d_gu,
                    keep, t16)
    corpus.k_g = k_g
    return corpus


def quantize_int8(src: torch.Tensor, scale: float, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """dst = clamp(rint(src * scale), -127, 127) as int8, same shape (Section 4.1.1)."""
    if src.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("src must be float32 or bfloat16")
    _dev(src, src.dtype, "src")
    if out is None:
        out = torch.empty(src.shape, dtype=torch.int8, device=src.device)
    _dev(out, torch.int8, "out")
    _check(load_library().mol_quantize_int8(_ptr(src), 0 if src.dtype == torch.float32 else 1, src.numel(), float(scale),
                                            _ptr(out), _stream()))
    return out


def hindexer_default_lambda(corpus: Corpus, Kp: int) -> int:
    return int(load_library().hindexer_default_lambda(corpus.handle, Kp))


def hindexer_workspace_bytes(corpus: Corpus, B: int, Kp: int, lam: int = 0) -> int:
    return int(load_library().hindexer_workspace_bytes(corpus.handle, B, Kp, lam))


def mol_workspace_bytes(corpus: Corpus, B: int, Kp: int, k: int) -> int:
    return int(load_library().mol_workspace_bytes(corpus.handle, B, Kp, k))


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor]) -> torch.Tensor:
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    return workspace


def hindexer_topk(corpus: Corpus, q1: torch.Tensor, Kp: int, lam: int = 0, seed: int = 0, mode: int = HINDEXER_EXACT,
                  sample_idx: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                  out: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None
                  ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    lib = load_library()
    _dev(q1, corpus.stage1_dtype, "q1")
    B = q1.shape[0]
    if q1.shape[1] != corpus.d1:
        raise ValueError("q1 width != d1")
    if sample_idx is not None:
        _dev(sample_idx, torch.int32, "sample_idx")
        lam = sample_idx.numel()
    if out is None:
        out = (torch.empty(B, Kp, dtype=torch.int32, device=q1.device),
               torch.empty(B, Kp, dtype=torch.float32, device=q1.device),
               torch.empty(B, dtype=torch.int32, device=q1.device))
    ci, cs, cc = out
    need = lib.hindexer_workspace_bytes(corpus.handle, B, Kp, lam)
    ws = _workspace(need, q1.device, workspace)
    _check(lib.hindexer_topk(corpus.handle, _ptr(q1), B, Kp, _ptr(sample_idx), lam, seed, mode, _ptr(ci), _ptr(cs),
                             _ptr(cc), _ptr(ws), ws.numel(), _stream()))
    return ci, cs, cc


def gather_items(corpus: Corpus, cand_idx: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """bf16 [B, Kp, k_x, d_p]: the item embeddings of the candidates (zeros for padding), Section 4.1.3."""
    _dev(cand_idx, torch.int32, "cand_idx")
    B, Kp = cand_idx.shape
    if out is None:
        out = torch.empty(B, Kp, corpus.k_x - getattr(corpus, "k_g", 0), corpus.d_p, dtype=corpus.mol_dtype,
                          device=cand_idx.device)
    _dev(out, corpus.mol_dtype, "out")
    _check(load_library().mol_gather_items(corpus.handle, _ptr(cand_idx), B, Kp, _ptr(out), _stream()))
    return out


def mol_score(corpus: Corpus, user_embs: torch.Tensor, user_gate: torch.Tensor,
              cand_idx: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
              out: Optional[torch.Tensor] = None) -> torch.Tensor:
    lib = load_library()
    _dev(user_embs, corpus.mol_dtype, "user_embs")
    _dev(user_gate, corpus.mol_dtype, "user_gate")
    B = user_embs.shape[0]
    if tuple(user_embs.shape[1:]) != (corpus.k_u, corpus.d_p) or tuple(user_gate.shape) != (B, corpus.d_gu):
        raise ValueError("user tensor shapes do not match the corpus")
    Kp = 0
    if cand_idx is not None:
        _dev(cand_idx, torch.int32, "cand_idx")
        Kp = cand_idx.shape[1]
    row = Kp if cand_idx is not None else corpus.N
    if out is None:
        out = torch.empty(B, row, dtype=torch.float32, device=user_embs.device)
    ws = _workspace(lib.mol_workspace_bytes(corpus.handle, B, 1, 1), user_embs.device, workspace)
    _check(lib.mol_score(corpus.handle, _ptr(user_embs), _ptr(user_gate), B, _ptr(cand_idx), Kp, _ptr(out), _ptr(ws),
                         ws.numel(), _stream()))
    return out


def mol_topk(corpus: Corpus, user_embs: torch.Tensor, user_gate: torch.Tensor, cand_idx: Optional[torch.Tensor],
             k: int, workspace: Optional[torch.Tensor] = None,
             out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None,
             cand_count: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    lib = load_library()
    _dev(user_embs, corpus.mol_dtype, "user_embs")
    _dev(user_gate, corpus.mol_dtype, "user_gate")
    B = user_embs.shape[0]
    if tuple(user_embs.shape[1:]) != (corpus.k_u, corpus.d_p) or tuple(user_gate.shape) != (B, corpus.d_gu):
        raise ValueError("user tensor shapes do not match the corpus")
    Kp = 0
    if cand_idx is not None:
        _dev(cand_idx, torch.int32, "cand_idx")
        Kp = cand_idx.shape[1]
    if out is None:
        out = (torch.empty(B, k, dtype=torch.int32, device=user_embs.device),
               torch.empty(B, k, dtype=torch.float32, device=user_embs.device))
    ws = _workspace(lib.mol_workspace_bytes(corpus.handle, B, Kp, k), user_embs.device, workspace)
    if cand_count is not None:
        _dev(cand_count, torch.int32, "cand_count")
        if cand_count.numel() != B:
            raise ValueError("cand_count must have B entries")
    _check(lib.mol_topk(corpus.handle, _ptr(user_embs), _ptr(user_gate), B, _ptr(cand_idx), _ptr(cand_count), Kp, k,
                        _ptr(out[0]), _ptr(out[1]), _ptr(ws), ws.numel(), _stream()))
    return out


def static_init() -> None:
    _check(load_library().mol_static_init())


def topk_static_max_bytes() -> int:
    return int(load_library().mol_topk_static_max_bytes())


def mol_topk_static(corpus: Corpus, user_embs: torch.Tensor, user_gate: torch.Tensor, cand_idx: Optional[torch.Tensor],
                    k: int, out: Tuple[torch.Tensor, torch.Tensor], cand_count: Optional[torch.Tensor] = None
                    ) -> Tuple[torch.Tensor, torch.Tensor]:
    """mol_topk on the library's static workspace: the caller brings the outputs, nothing is allocated here or below."""
    lib = load_library()
    _dev(user_embs, corpus.mol_dtype, "user_embs")
    _dev(user_gate, corpus.mol_dtype, "user_gate")
    B = user_embs.shape[0]
    if tuple(user_embs.shape[1:]) != (corpus.k_u, corpus.d_p) or tuple(user_gate.shape) != (B, corpus.d_gu):
        raise ValueError("user tensor shapes do not match the corpus")
    Kp = 0
    if cand_idx is not None:
        _dev(cand_idx, torch.int32, "cand_idx")
        Kp = cand_idx.shape[1]
    if cand_count is not None:
        _dev(cand_count, torch.int32, "cand_count")
    _dev(out[0], torch.int32, "out_idx")
    _dev(out[1], torch.float32, "out_score")
    if tuple(out[0].shape) != (B, k) or tuple(out[1].shape) != (B, k):
        raise ValueError("out tensors must be [B, k]")
    _check(lib.mol_topk_static(corpus.handle, _ptr(user_embs), _ptr(user_gate), B, _ptr(cand_idx), _ptr(cand_count), Kp, k,
                               _ptr(out[0]), _ptr(out[1]), _stream()))
    return out


def bench_stream_read(t: torch.Tensor, blocks: int, sink: torch.Tensor) -> None:
    """Read-only sweep over t's bytes (benchmark ceiling of the corpus scan)."""
    nbytes = t.numel() * t.element_size() // 16 * 16
    _check(load_library().mol_bench_stream_read(_ptr(t), nbytes, blocks, _ptr(sink), _stream()))


def bench_gather(corpus: Corpus, cand_idx: torch.Tensor, blocks: int, sink: torch.Tensor) -> None:
    """Bare gather with the scoring kernel's access pattern (benchmark ceiling of mol_score)."""
    _dev(cand_idx, torch.int32, "cand_idx")
    B, Kp = cand_idx.shape
    _check(load_library().mol_bench_gather(corpus.handle, _ptr(cand_idx), B, Kp, blocks, _ptr(sink), _stream()))


def profile_enable(on, slots=None) -> None:
    """on = False/True: no / every slot; slots = iterable of PROF_SLOTS names: only those."""
    if slots is not None:
        mask = 0
        for name in slots:
            mask |= 1 << PROF_SLOTS.index(name)
        _check(load_library().mol_profile_enable(2 * mask))
    else:
        _check(load_library().mol_profile_enable(1 if on else 0))


def profile_read() -> dict:
    """{slot name: (total ms, launches)} of the kernels launched since the last read."""
    ms = (C.c_double * len(PROF_SLOTS))()
    n = (C.c_int * len(PROF_SLOTS))()
    _check(load_library().mol_profile_read(ms, n))
    return {name: (ms[i], n[i]) for i, name in enumerate(PROF_SLOTS)}
