"""ctypes binding of liblvlm.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; this module turns
torch tensors (used for device memory and streams) into the pointers, strides
and plain structs of include/lvlm.h and raises on any non-zero status.  There
is no fallback: if the shared library is missing the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
# the in-tree build, or another build of the same sources named by LVLM_LIBRARY (e.g. one with a sanitized host side)
LIB_PATH = os.environ.get("LVLM_LIBRARY") or os.path.join(HERE, "liblvlm.so")

# ---- enums (include/lvlm.h) ----
BF16, F32, I32 = 0, 1, 2
OP_SCORE, OP_MERGE, OP_KV_COMPRESS, OP_DECODE_ATTN, OP_MERGE_SIMILAR, OP_SCORE_PROBS, OP_PREFILL_ATTN = 0, 1, 2, 3, 4, 5, 6
MERGE_LINEAR_RANK, MERGE_PAIRWISE, MERGE_LINEAR_RAW = 0, 1, 2
RULE_WEIGHTED, RULE_TOP = 0, 1
KV_THRESHOLD, KV_BUDGET = 0, 1
ORDER_STABLE, ORDER_FILL = 0, 1
KIND_PROTECTED, KIND_IMAGE, KIND_GENERATED = 0, 1, 2
MAX_PLANES = 8
STATUS = {0: "LVLM_OK", 1: "LVLM_ERR_INVALID_ARG", 2: "LVLM_ERR_UNSUPPORTED", 3: "LVLM_ERR_WORKSPACE",
          4: "LVLM_ERR_HIP"}

_DTYPE = {torch.bfloat16: BF16, torch.float32: F32, torch.int32: I32}


class ScoreDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("B", C.c_int32), ("N", C.c_int32), ("T", C.c_int32),
                ("q_pos0", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("hd", C.c_int32),
                ("img_begin", C.c_int32), ("n_img", C.c_int32), ("causal", C.c_int32), ("scale", C.c_float),
                ("q_stride_b", C.c_int64), ("q_stride_t", C.c_int64), ("q_stride_h", C.c_int64),
                ("k_stride_b", C.c_int64), ("k_stride_n", C.c_int64), ("k_stride_h", C.c_int64),
                ("sh_stride_b", C.c_int64), ("sh_stride_h", C.c_int64)]


class ProbsDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("B", C.c_int32), ("N", C.c_int32), ("T", C.c_int32),
                ("Hq", C.c_int32), ("Hkv", C.c_int32), ("img_begin", C.c_int32), ("n_img", C.c_int32),
                ("p_stride_b", C.c_int64), ("p_stride_h", C.c_int64), ("p_stride_t", C.c_int64),
                ("sh_stride_b", C.c_int64), ("sh_stride_h", C.c_int64)]


class PrefillDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("B", C.c_int32), ("N", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32),
                ("hd", C.c_int32), ("causal", C.c_int32), ("scale", C.c_float), ("T", C.c_int32),
                ("img_begin", C.c_int32), ("n_img", C.c_int32),
                ("q_stride_b", C.c_int64), ("q_stride_n", C.c_int64), ("q_stride_h", C.c_int64),
                ("k_stride_b", C.c_int64), ("k_stride_n", C.c_int64), ("k_stride_h", C.c_int64),
                ("v_stride_b", C.c_int64), ("v_stride_n", C.c_int64), ("v_stride_h", C.c_int64),
                ("o_stride_b", C.c_int64), ("o_stride_n", C.c_int64), ("o_stride_h", C.c_int64),
                ("sh_stride_b", C.c_int64), ("sh_stride_h", C.c_int64)]


class Plane(C.Structure):
    _fields_ = [("src", C.c_void_p), ("dst", C.c_void_p), ("src_stride_b", C.c_int64),
                ("dst_stride_b", C.c_int64), ("row_elems", C.c_int32), ("dtype", C.c_int32),
                ("merge_rule", C.c_int32), ("reserved", C.c_int32)]


class MergeDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("N", C.c_int32), ("img_begin", C.c_int32), ("n_img", C.c_int32),
                ("n_keep", C.c_int32), ("n_planes", C.c_int32)]


class MergeQuery(C.Structure):
    _fields_ = [("desc", C.POINTER(MergeDesc)), ("planes", C.POINTER(Plane))]


class KvDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("B", C.c_int32), ("Hkv", C.c_int32), ("hd", C.c_int32),
                ("Lmax", C.c_int32), ("len_bound", C.c_int32), ("mode", C.c_int32), ("order", C.c_int32),
                ("budget", C.c_int32), ("n_recent", C.c_int32), ("beta", C.c_double)]


class AttnDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32),
                ("hd", C.c_int32), ("Lmax", C.c_int32), ("len_bound", C.c_int32), ("new_kind", C.c_int32),
                ("new_pos", C.c_int32), ("scale", C.c_float), ("score_decay", C.c_float),
                ("evict_budget", C.c_int32), ("evict_recent", C.c_int32)]


class ProfileEntry(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("calls", C.c_int32), ("total_ms", C.c_float), ("min_ms", C.c_float),
                ("max_ms", C.c_float)]


class LvlmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(the HIP library is the only implementation; there is no fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32p, f32p = C.c_void_p, C.c_void_p, C.c_void_p
    lib.lvlm_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
    lib.lvlm_destroy.argtypes = [C.c_void_p]
    lib.lvlm_last_error.argtypes = [C.c_void_p]
    lib.lvlm_last_error.restype = C.c_char_p
    lib.lvlm_workspace_bytes.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.POINTER(C.c_size_t)]
    lib.lvlm_set_workspace.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
    lib.lvlm_schedule.argtypes = [C.c_int, C.c_double, C.c_int, C.POINTER(C.c_int)]
    lib.lvlm_merge_weights.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_float)]
    lib.lvlm_score_tokens.argtypes = [vp, vp, C.POINTER(ScoreDesc), vp, vp, f32p, f32p, f32p]
    lib.lvlm_score_plan.argtypes = [vp, C.POINTER(ScoreDesc), C.POINTER(C.c_int32)]
    lib.lvlm_score_from_probs.argtypes = [vp, vp, C.POINTER(ProbsDesc), vp, f32p, f32p]
    lib.lvlm_prefill_attn.argtypes = [vp, vp, C.POINTER(PrefillDesc), vp, vp, vp, vp, f32p, f32p, f32p]
    lib.lvlm_merge_compact.argtypes = [vp, vp, C.POINTER(MergeDesc), f32p, f32p, C.POINTER(Plane), i32p, i32p]
    lib.lvlm_merge_similar.argtypes = [vp, vp, C.POINTER(MergeDesc), f32p, C.POINTER(Plane), f32p, f32p, i32p, i32p]
    lib.lvlm_kv_compress.argtypes = [vp, vp, C.POINTER(KvDesc), vp, vp, f32p, vp, i32p, i32p, i32p]
    lib.lvlm_decode_attn.argtypes = [vp, vp, C.POINTER(AttnDesc), vp, vp, vp, vp, vp, f32p, vp, i32p, i32p, vp]
    lib.lvlm_decode_attn_static.argtypes = lib.lvlm_decode_attn.argtypes
    lib.lvlm_decode_plan.argtypes = [vp, C.POINTER(AttnDesc), C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.lvlm_stream_probe.argtypes = [vp, vp, vp, C.c_size_t, C.c_int32, vp]
    lib.lvlm_profile.argtypes = [C.c_void_p, C.c_int]
    lib.lvlm_profile_read.argtypes = [C.c_void_p, C.POINTER(ProfileEntry), C.c_int, C.POINTER(C.c_int)]
    for name in ("lvlm_profile", "lvlm_profile_read", "lvlm_create", "lvlm_destroy", "lvlm_workspace_bytes", "lvlm_set_workspace", "lvlm_schedule",
                 "lvlm_merge_weights", "lvlm_score_tokens", "lvlm_score_plan", "lvlm_score_from_probs", "lvlm_prefill_attn", "lvlm_merge_compact",
                 "lvlm_merge_similar",
                 "lvlm_kv_compress",
                 "lvlm_decode_attn", "lvlm_decode_attn_static", "lvlm_decode_plan", "lvlm_stream_probe"):
        getattr(lib, name).restype = C.c_int
    return lib


lib = _load()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def schedule(n_img: int, final_keep: float, n_stages: int = 3):
    out = (C.c_int * n_stages)()
    st = lib.lvlm_schedule(n_img, float(final_keep), n_stages, out)
    if st:
        raise LvlmError(st, "lvlm_schedule")
    return list(out)


def merge_weights(mode: int, m: int) -> torch.Tensor:
    out = (C.c_float * m)()
    st = lib.lvlm_merge_weights(mode, m, out)
    if st:
        raise LvlmError(st, "lvlm_merge_weights")
    return torch.tensor(list(out), dtype=torch.float32)


class Context:
    """One lvlm_ctx plus a grow-only workspace tensor (device memory via torch)."""

    def __init__(self, device: int = 0):
        self._h = C.c_void_p()
        st = lib.lvlm_create(C.byref(self._h), device)
        if st:
            raise LvlmError(st, "lvlm_create")
        self.device = device
        self._ws: Optional[torch.Tensor] = None

    def close(self):
        if self._h:
            lib.lvlm_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st:
            raise LvlmError(st, lib.lvlm_last_error(self._h).decode())

    def workspace_bytes(self, op: int, desc) -> int:
        n = C.c_size_t()
        self._check(lib.lvlm_workspace_bytes(self._h, op, C.byref(desc), C.byref(n)))
        return n.value

    def reserve(self, nbytes: int):
        """Grows the attached workspace (never shrinks); call outside graph capture."""
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=f"cuda:{self.device}")
            self._check(lib.lvlm_set_workspace(self._h, _ptr(self._ws), self._ws.numel()))

    def set_workspace(self, ws: Optional[torch.Tensor]):
        self._ws = ws
        self._check(lib.lvlm_set_workspace(self._h, _ptr(ws), 0 if ws is None else ws.numel()))

    def stream_probe(self, src: torch.Tensor, n_workgroups: int, sink: torch.Tensor):
        """lvlm_stream_probe: a read-only pass over src (diagnostic)."""
        self._check(lib.lvlm_stream_probe(self._h, _stream(), _ptr(src), src.numel() * src.element_size(), n_workgroups,
                                          _ptr(sink)))

    def profile(self, enable: bool):
        """lvlm_profile: bracket every kernel launch with HIP events (eager mode only)."""
        self._check(lib.lvlm_profile(self._h, int(enable)))

    def profile_read(self):
        """lvlm_profile_read -> {kernel name: (calls, total_ms, min_ms, max_ms)}; clears the record."""
        arr = (ProfileEntry * 64)()
        n = C.c_int()
        self._check(lib.lvlm_profile_read(self._h, arr, 64, C.byref(n)))
        return {arr[i].name.decode(): (arr[i].calls, arr[i].total_ms, arr[i].min_ms, arr[i].max_ms)
                for i in range(n.value)}

    # ---- step 1 ----
    def score_desc(self, q, k, *, q_pos0, img_begin, n_img, scale=None, causal=True, score_head=None) -> ScoreDesc:
        B, T, Hq, hd = q.shape
        _, N, Hkv, _ = k.shape
        assert q.stride(3) == 1 and k.stride(3) == 1, "head dimension must be contiguous"
        return ScoreDesc(_DTYPE[q.dtype], B, N, T, q_pos0, Hq, Hkv, hd, img_begin, n_img, int(causal),
                         float(hd ** -0.5 if scale is None else scale),
                         q.stride(0), q.stride(1), q.stride(2), k.stride(0), k.stride(1), k.stride(2),
                         0 if score_head is None else score_head.stride(0),
                         0 if score_head is None else score_head.stride(1))

    def score_plan(self, desc: ScoreDesc) -> int:
        """lvlm_score_plan: 0 = two-pass kernels, 1 = one launch (a chunk per workgroup), 2 = one launch (shared tiles),
        3 = the shared-tile kernel with the keys cut into runs (one launch per sweep)."""
        form = C.c_int32()
        self._check(lib.lvlm_score_plan(self._h, C.byref(desc), C.byref(form)))
        return form.value

    def score_tokens(self, q, k, *, q_pos0, img_begin, n_img, scale=None, causal=True, row_lse=None,
                     score_head=None, score_mean=None, reserve=True):
        """lvlm_score_tokens.  q [B,T,Hq,d], k [B,N,Hkv,d] -> (score_head [B,Hkv,n_img], score_mean [B,n_img])."""
        d = self.score_desc(q, k, q_pos0=q_pos0, img_begin=img_begin, n_img=n_img, scale=scale, causal=causal,
                            score_head=score_head)
        if score_head is None:
            score_head = torch.empty(d.B, d.Hkv, n_img, dtype=torch.float32, device=q.device)
        if score_mean is None:
            score_mean = torch.empty(d.B, n_img, dtype=torch.float32, device=q.device)
        if reserve:
            self.reserve(self.workspace_bytes(OP_SCORE, d))
        self._check(lib.lvlm_score_tokens(self._h, _stream(), C.byref(d), _ptr(q), _ptr(k), _ptr(row_lse),
                                          _ptr(score_head), _ptr(score_mean)))
        return score_head, score_mean

    def score_from_probs(self, probs, *, n_kv_heads, img_begin, n_img, score_head=None, score_mean=None, reserve=True):
        """lvlm_score_from_probs.  probs [B,Hq,T,N] (softmax rows of the query rows to be summed) ->
        (score_head [B,Hkv,n_img], score_mean [B,n_img])."""
        B, Hq, T, N = probs.shape
        assert probs.stride(3) == 1, "the key axis must be contiguous"
        d = ProbsDesc(_DTYPE[probs.dtype], B, N, T, Hq, n_kv_heads, img_begin, n_img,
                      probs.stride(0), probs.stride(1), probs.stride(2),
                      0 if score_head is None else score_head.stride(0),
                      0 if score_head is None else score_head.stride(1))
        if score_head is None:
            score_head = torch.empty(B, n_kv_heads, n_img, dtype=torch.float32, device=probs.device)
        if score_mean is None:
            score_mean = torch.empty(B, n_img, dtype=torch.float32, device=probs.device)
        if reserve:
            self.reserve(self.workspace_bytes(OP_SCORE_PROBS, d))
        self._check(lib.lvlm_score_from_probs(self._h, _stream(), C.byref(d), _ptr(probs), _ptr(score_head),
                                              _ptr(score_mean)))
        return score_head, score_mean

    def prefill_attn(self, q, k, v, *, scale=None, causal=True, n_text=0, img_begin=0, n_img=0, out=None, row_lse=None,
                     score_head=None, score_mean=None, reserve=True):
        """lvlm_prefill_attn.  q [B,N,Hq,d], k, v [B,N,Hkv,d] (any strides with a contiguous head vector) ->
        (out [B,N,Hq,d], row_lse [B,Hq,N], score_head, score_mean); the scores (of the last n_text rows over
        the image keys) only when n_text > 0, else None."""
        B, N, Hq, hd = q.shape
        Hkv = k.shape[2]
        assert k.shape == (B, N, Hkv, hd) and v.shape == (B, N, Hkv, hd)
        assert q.stride(3) == 1 and k.stride(3) == 1 and v.stride(3) == 1
        if out is None:
            out = torch.empty(B, N, Hq, hd, dtype=q.dtype, device=q.device)
        if row_lse is None:
            row_lse = torch.empty(B, Hq, N, dtype=torch.float32, device=q.device)
        assert out.stride(3) == 1 and row_lse.is_contiguous()
        if n_text > 0:
            if score_head is None:
                score_head = torch.empty(B, Hkv, n_img, dtype=torch.float32, device=q.device)
            if score_mean is None:
                score_mean = torch.empty(B, n_img, dtype=torch.float32, device=q.device)
        dense = score_head is None or score_head.is_contiguous()
        d = PrefillDesc(_DTYPE[q.dtype], B, N, Hq, Hkv, hd, int(causal), float(scale if scale is not None else hd ** -0.5),
                        n_text, img_begin, n_img, q.stride(0), q.stride(1), q.stride(2), k.stride(0), k.stride(1),
                        k.stride(2), v.stride(0), v.stride(1), v.stride(2), out.stride(0), out.stride(1), out.stride(2),
                        0 if dense else score_head.stride(0), 0 if dense else score_head.stride(1))
        if reserve:
            self.reserve(self.workspace_bytes(OP_PREFILL_ATTN, d))
        self._check(lib.lvlm_prefill_attn(self._h, _stream(), C.byref(d), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(row_lse),
                                          _ptr(score_head), _ptr(score_mean)))
        return out, row_lse, score_head, score_mean

    # ---- steps 2-4 ----
    @staticmethod
    def _planes(planes: Sequence[torch.Tensor], outs: Sequence[torch.Tensor], rules: Sequence[int]):
        arr = (Plane * len(planes))()
        for i, (src, dst, rule) in enumerate(zip(planes, outs, rules)):
            assert src.dim() == 3 and src.stride(2) == 1 and src.stride(1) == src.shape[2]
            assert dst.stride(2) == 1 and dst.stride(1) == dst.shape[2]
            arr[i] = Plane(src.data_ptr(), dst.data_ptr(), src.stride(0), dst.stride(0), src.shape[2],
                           _DTYPE[src.dtype], rule, 0)
        return arr

    def merge_compact(self, planes, score_mean, *, img_begin, n_img, n_keep, w=None, rules=None, outs=None,
                      keep_idx=None, merged_idx=None, reserve=True):
        """lvlm_merge_compact.  planes: list of [B,N,row] tensors -> (outs, keep_idx, merged_idx)."""
        B, N = planes[0].shape[0], planes[0].shape[1]
        r = n_img - n_keep
        rules = list(rules) if rules is not None else [RULE_WEIGHTED] * len(planes)
        if outs is None:
            outs = [torch.empty(B, N - r, p.shape[2], dtype=p.dtype, device=p.device) for p in planes]
        dev = planes[0].device
        if keep_idx is None:
            keep_idx = torch.empty(B, max(n_keep - 1, 0) if r > 0 else n_img, dtype=torch.int32, device=dev)
        if merged_idx is None:
            merged_idx = torch.empty(B, r + 1 if r > 0 else 0, dtype=torch.int32, device=dev)
        d = MergeDesc(B, N, img_begin, n_img, n_keep, len(planes))
        arr = self._planes(planes, outs, rules)
        if reserve:
            self.reserve(self.workspace_bytes(OP_MERGE, MergeQuery(C.pointer(d), arr)))
        self._check(lib.lvlm_merge_compact(self._h, _stream(), C.byref(d), _ptr(score_mean), _ptr(w), arr,
                                           _ptr(keep_idx) if keep_idx.numel() else None,
                                           _ptr(merged_idx) if merged_idx.numel() else None))
        return outs, keep_idx, merged_idx

    # ---- step 3b ----
    def merge_similar(self, planes, score_mean, *, img_begin, n_img, n_keep, size=None, rules=None, outs=None,
                      size_out=None, keep_idx=None, assign=None, reserve=True):
        """lvlm_merge_similar.  planes: list of [B,N,row] tensors -> (outs, keep_idx, assign, size_out)."""
        B, N = planes[0].shape[0], planes[0].shape[1]
        r = n_img - n_keep
        rules = list(rules) if rules is not None else [RULE_WEIGHTED] * len(planes)
        dev = planes[0].device
        if outs is None:
            outs = [torch.empty(B, N - r, p.shape[2], dtype=p.dtype, device=p.device) for p in planes]
        if keep_idx is None:
            keep_idx = torch.empty(B, n_keep, dtype=torch.int32, device=dev)
        if assign is None:
            assign = torch.empty(B, n_img, dtype=torch.int32, device=dev)
        if size_out is None:
            size_out = torch.empty(B, n_keep, dtype=torch.float32, device=dev)
        d = MergeDesc(B, N, img_begin, n_img, n_keep, len(planes))
        arr = self._planes(planes, outs, rules)
        if reserve:
            self.reserve(self.workspace_bytes(OP_MERGE_SIMILAR, MergeQuery(C.pointer(d), arr)))
        self._check(lib.lvlm_merge_similar(self._h, _stream(), C.byref(d), _ptr(score_mean), arr, _ptr(size),
                                           _ptr(size_out), _ptr(keep_idx), _ptr(assign)))
        return outs, keep_idx, assign, size_out

    # ---- step 5 ----
    def kv_compress(self, k_cache, v_cache, score, kind, orig_pos, length, *, mode, order=ORDER_STABLE,
                    beta=0.995, budget=0, n_recent=0, len_bound=0, n_evicted=None, reserve=True, want_evicted=True):
        """lvlm_kv_compress (in place).  Caches [B,Hkv,Lmax,d]; returns n_evicted [B,Hkv] (None if not wanted)."""
        B, Hkv, Lmax, hd = k_cache.shape
        assert k_cache.is_contiguous() and v_cache.is_contiguous() and score.is_contiguous()
        d = KvDesc(_DTYPE[k_cache.dtype], B, Hkv, hd, Lmax, len_bound, mode, order, budget, n_recent, float(beta))
        if n_evicted is None and want_evicted:
            n_evicted = torch.empty(B, Hkv, dtype=torch.int32, device=k_cache.device)
        if reserve:
            self.reserve(self.workspace_bytes(OP_KV_COMPRESS, d))
        self._check(lib.lvlm_kv_compress(self._h, _stream(), C.byref(d), _ptr(k_cache), _ptr(v_cache), _ptr(score),
                                         _ptr(kind), _ptr(orig_pos), _ptr(length), _ptr(n_evicted)))
        return n_evicted

    # ---- step 6 ----
    def decode_plan(self, desc: AttnDesc):
        """lvlm_decode_plan: (n_split, split_len, form); form 0 = one tile per wave, 1 = some wave has a second tile,
        2 = whole 128-entry splits plus one entry taken by one wave."""
        n, sl, form = C.c_int32(), C.c_int32(), C.c_int32()
        self._check(lib.lvlm_decode_plan(self._h, C.byref(desc), C.byref(n), C.byref(sl), C.byref(form)))
        return n.value, sl.value, form.value

    def decode_attn(self, q, k_new, v_new, k_cache, v_cache, score, kind, orig_pos, length, *, scale=None,
                    score_decay=1.0, new_kind=KIND_GENERATED, new_pos=0, len_bound=0, evict_budget=0, evict_recent=0,
                    out=None, reserve=True, static_scratch=False):
        """lvlm_decode_attn.  q [B,Hq,d], k_new/v_new [B,Hkv,d] or None -> out [B,Hq,d].
        static_scratch: lvlm_decode_attn_static instead (the library's own fixed scratch array, no workspace)."""
        B, Hq, hd = q.shape
        _, Hkv, Lmax, _ = k_cache.shape
        assert q.is_contiguous() and k_cache.is_contiguous() and v_cache.is_contiguous()
        d = AttnDesc(_DTYPE[q.dtype], B, Hq, Hkv, hd, Lmax, len_bound, new_kind, new_pos,
                     float(hd ** -0.5 if scale is None else scale), float(score_decay), evict_budget, evict_recent)
        if out is None:
            out = torch.empty_like(q)
        if reserve and not static_scratch:
            self.reserve(self.workspace_bytes(OP_DECODE_ATTN, d))
        call = lib.lvlm_decode_attn_static if static_scratch else lib.lvlm_decode_attn
        self._check(call(self._h, _stream(), C.byref(d), _ptr(q), _ptr(k_new), _ptr(v_new),
                        _ptr(k_cache), _ptr(v_cache), _ptr(score), _ptr(kind), _ptr(orig_pos), _ptr(length), _ptr(out)))
        return out
