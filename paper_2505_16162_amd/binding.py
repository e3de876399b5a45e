"""Thin ctypes binding of libknnssd.so: argument marshalling only.

Every step of the decode path runs in the library's HIP kernels. PyTorch is used
here for two things: owning device memory (weights, KV cache, workspace, anchor
table) and naming the HIP stream the kernels are put on. There is no CPU or
PyTorch fallback: if the library is missing or a call fails, an exception is
raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libknnssd.so")

KNNSSD_MAX_ROWS = 16
_DT = {"fp32": 0, "bf16": 1}

EXPORTS = [
    "knnssd_workspace_bytes", "knnssd_kvcache_bytes", "knnssd_create", "knnssd_destroy",
    "knnssd_pack_supported", "knnssd_pack_matrix",
    "knnssd_set_anchors", "knnssd_prefill", "knnssd_select_skipset", "knnssd_set_skipset", "knnssd_last_selection", "knnssd_knn_topk", "knnssd_route_static",
    "knnssd_draft_step", "knnssd_verify", "knnssd_generate", "knnssd_profile_pass", "knnssd_get_logits", "knnssd_read_kv",
    "knnssd_strerror", "knnssd_stream_next_domain",
]


class ModelCfg(ctypes.Structure):
    _fields_ = [("n_blocks", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("d_ffn", ctypes.c_int32),
                ("vocab", ctypes.c_int32), ("max_seq", ctypes.c_int32), ("max_anchors", ctypes.c_int32),
                ("rope_base", ctypes.c_float), ("rms_eps", ctypes.c_float),
                ("weight_dtype", ctypes.c_int32), ("kv_dtype", ctypes.c_int32), ("weights_packed", ctypes.c_int32),
                ("prefill_mode", ctypes.c_int32), ("verify_attn", ctypes.c_int32), ("attn_merge", ctypes.c_int32)]


class Weights(ctypes.Structure):
    _fields_ = [("embed", ctypes.c_void_p), ("lm_head", ctypes.c_void_p), ("final_norm", ctypes.c_void_p),
                ("attn_norm", ctypes.c_void_p), ("wqkv", ctypes.c_void_p), ("wo", ctypes.c_void_p),
                ("mlp_norm", ctypes.c_void_p), ("wgu", ctypes.c_void_p), ("wdown", ctypes.c_void_p)]


class GenCfg(ctypes.Structure):
    _fields_ = [("max_new", ctypes.c_int32), ("max_draft", ctypes.c_int32), ("conf_threshold", ctypes.c_float),
                ("keep_mask", ctypes.c_int32)]


class Stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in
                ("rounds", "drafted", "accepted", "emitted", "ns_prefill", "ns_knn", "ns_draft", "ns_verify",
                 "ns_total", "draft_passes", "verify_passes")]

    def as_dict(self) -> Dict[str, int]:
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class KnnSsdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"knnssd error {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the built library; fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2505_16162_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
    lib.knnssd_workspace_bytes.restype = ctypes.c_size_t
    lib.knnssd_workspace_bytes.argtypes = [ctypes.POINTER(ModelCfg)]
    lib.knnssd_kvcache_bytes.restype = ctypes.c_size_t
    lib.knnssd_kvcache_bytes.argtypes = [ctypes.POINTER(ModelCfg)]
    lib.knnssd_create.restype = i32
    lib.knnssd_create.argtypes = [ctypes.POINTER(ModelCfg), ctypes.POINTER(Weights), vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp,
                                  ctypes.POINTER(vp)]
    lib.knnssd_pack_supported.restype = i32
    lib.knnssd_pack_supported.argtypes = [ctypes.POINTER(ModelCfg)]
    lib.knnssd_pack_matrix.restype = i32
    lib.knnssd_pack_matrix.argtypes = [ctypes.POINTER(ModelCfg), i32, vp, vp, vp]
    lib.knnssd_destroy.restype = i32
    lib.knnssd_destroy.argtypes = [vp]
    lib.knnssd_set_anchors.restype = i32
    lib.knnssd_set_anchors.argtypes = [vp, vp, i32, vp, i32, i32, vp, i32, i32]
    lib.knnssd_prefill.restype = i32
    lib.knnssd_prefill.argtypes = [vp, vp, i32, vp, ctypes.POINTER(i32)]
    lib.knnssd_select_skipset.restype = i32
    lib.knnssd_select_skipset.argtypes = [vp, vp, ctypes.POINTER(i32), ctypes.POINTER(i32), vp]
    lib.knnssd_set_skipset.restype = i32
    lib.knnssd_set_skipset.argtypes = [vp, vp]
    lib.knnssd_knn_topk.restype = i32
    lib.knnssd_knn_topk.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    lib.knnssd_route_static.restype = i32
    lib.knnssd_route_static.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.knnssd_last_selection.restype = i32
    lib.knnssd_last_selection.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.knnssd_draft_step.restype = i32
    lib.knnssd_draft_step.argtypes = [vp, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(f32)]
    lib.knnssd_verify.restype = i32
    lib.knnssd_verify.argtypes = [vp, vp, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.knnssd_generate.restype = i32
    lib.knnssd_generate.argtypes = [vp, vp, i32, vp, ctypes.POINTER(GenCfg), vp, ctypes.POINTER(i32), ctypes.POINTER(Stats)]
    lib.knnssd_profile_pass.restype = i32
    lib.knnssd_profile_pass.argtypes = [vp, i32, vp, i32, i32] + [ctypes.POINTER(ctypes.c_int64)] * 4
    lib.knnssd_get_logits.restype = i32
    lib.knnssd_get_logits.argtypes = [vp, i32, vp]
    lib.knnssd_read_kv.restype = i32
    lib.knnssd_read_kv.argtypes = [vp, i32, i32, vp, vp]
    lib.knnssd_stream_next_domain.restype = i32
    lib.knnssd_stream_next_domain.argtypes = [i32, i32, ctypes.c_double, ctypes.c_double, ctypes.c_double]
    lib.knnssd_strerror.restype = ctypes.c_char_p
    lib.knnssd_strerror.argtypes = [i32]
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise KnnSsdError(rc, load_library().knnssd_strerror(rc).decode())


def make_cfg(shape, max_anchors: int = 0) -> ModelCfg:
    return ModelCfg(shape.n_blocks, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                    shape.vocab, shape.max_seq, max_anchors, float(shape.rope_base), float(shape.rms_eps),
                    _DT[shape.weight_dtype], _DT[shape.kv_dtype], 0, 0, 0, 0)


def _i32_array(values: Sequence[int]):
    arr = (ctypes.c_int32 * len(values))(*[int(v) for v in values])
    return arr


def knnssd_route_static(query: torch.Tensor, anchors: torch.Tensor, labels: torch.Tensor, result: torch.Tensor,
                        stream: Optional[torch.cuda.Stream] = None) -> None:
    """Routing without a context or a workspace (argument marshalling only; the caller owns every tensor, result
    included: int32[4] on the device, filled in stream order)."""
    lib = load_library()
    s = stream if stream is not None else torch.cuda.current_stream(query.device)
    _check(lib.knnssd_route_static(query.data_ptr(), anchors.data_ptr(), labels.data_ptr(), anchors.shape[0], anchors.shape[1],
                                   ctypes.c_void_p(s.cuda_stream), result.data_ptr()))


def knnssd_stream_next_domain(current: int, n_domains: int, mix_ratio: float, u_switch: float, u_pick: float) -> int:
    """Eq. 8 transition (host-only call of the library; argument marshalling only)."""
    rc = load_library().knnssd_stream_next_domain(int(current), int(n_domains), float(mix_ratio), float(u_switch), float(u_pick))
    if rc < 0:
        _check(rc)
    return int(rc)


class KnnSsd:
    """A library context over torch-owned device memory. Method names follow the C ABI."""

    def __init__(self, shape, weights: Dict, max_anchors: int = 0, device="cuda:0", stream: Optional[torch.cuda.Stream] = None,
                 generic_kernels: bool = False, chunked_prefill: bool = False, verify_attn: str = "mfma",
                 separate_merge: bool = False):
        """generic_kernels: keep the matrices row-major and run the any-shape kernels (cfg.weights_packed = 0);
        chunked_prefill: cfg.prefill_mode = KNNSSD_PREFILL_CHUNKED; verify_attn: "mfma" | "valu" (cfg.verify_attn)."""
        self.lib = load_library()
        self.shape = shape
        self.device = torch.device(device)
        if self.device.type != "cuda":
            raise ValueError("the decode path runs on the GPU only")
        self.cfg = make_cfg(shape, max_anchors)
        if self.lib.knnssd_workspace_bytes(ctypes.byref(self.cfg)) == 0:
            raise KnnSsdError(-2, "shape not supported")
        self._keep: List = []
        dev = self.device

        def on_dev(t: torch.Tensor) -> torch.Tensor:
            t = t.to(dev).contiguous()
            self._keep.append(t)
            return t

        nb = shape.n_blocks
        self.stream = stream if stream is not None else torch.cuda.current_stream(dev)
        # Stream order: shapes the tuned kernels support get every matrix repacked once by the library
        self.packed = bool(self.lib.knnssd_pack_supported(ctypes.byref(self.cfg))) and not generic_kernels
        self.cfg.weights_packed = 1 if self.packed else 0
        self.cfg.prefill_mode = 1 if chunked_prefill else 0
        self.cfg.verify_attn = {"mfma": 0, "valu": 1}[verify_attn]
        self.cfg.attn_merge = 1 if separate_merge else 0
        # sizes of the caller-owned buffers, asked for with the final cfg (they depend on weights_packed)
        ws_bytes = self.lib.knnssd_workspace_bytes(ctypes.byref(self.cfg))
        kv_bytes = self.lib.knnssd_kvcache_bytes(ctypes.byref(self.cfg))
        if ws_bytes == 0 or kv_bytes == 0:
            raise KnnSsdError(-2, "shape not supported")

        def matrix(t: torch.Tensor, which: int) -> torch.Tensor:
            t = t.to(dev).contiguous()
            if self.packed:
                dst = torch.empty_like(t)
                _check(self.lib.knnssd_pack_matrix(ctypes.byref(self.cfg), which, t.data_ptr(), dst.data_ptr(),
                                                   ctypes.c_void_p(self.stream.cuda_stream)))
                torch.cuda.synchronize(dev)     # the row-major copy may be freed once the pack kernel is done
                t = dst
            self._keep.append(t)
            return t

        # fused row-major matrices the ABI asks for: [q;k;v] and [gate;up] stacked along rows
        blocks = weights["blocks"]
        wqkv, wo, wgu, wdown, an, mn = [], [], [], [], [], []
        for b in blocks:
            wqkv.append(matrix(torch.cat([b["wq"].to(dev), b["wk"].to(dev), b["wv"].to(dev)], 0), 0))
            wo.append(matrix(b["wo"], 1))
            wgu.append(matrix(torch.cat([b["wg"].to(dev), b["wu"].to(dev)], 0), 2))
            wdown.append(matrix(b["wd"], 3))
            an.append(on_dev(b["attn_norm"].float()))
            mn.append(on_dev(b["mlp_norm"].float()))
        self.embed = on_dev(weights["embed"])
        self.lm_head = matrix(weights["lm_head"], 4)
        self.final_norm = on_dev(weights["final_norm"].float())

        def ptr_array(ts):
            arr = (ctypes.c_void_p * max(nb, 1))(*[t.data_ptr() for t in ts])
            self._keep.append(arr)
            return ctypes.cast(arr, ctypes.c_void_p)

        self.w = Weights(self.embed.data_ptr(), self.lm_head.data_ptr(), self.final_norm.data_ptr(),
                         ptr_array(an), ptr_array(wqkv), ptr_array(wo), ptr_array(mn), ptr_array(wgu), ptr_array(wdown))
        self.kv = torch.zeros(kv_bytes, dtype=torch.uint8, device=dev)
        self.ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=dev)
        h = ctypes.c_void_p()
        torch.cuda.synchronize(dev)
        _check(self.lib.knnssd_create(ctypes.byref(self.cfg), ctypes.byref(self.w), self.kv.data_ptr(), kv_bytes,
                                      self.ws.data_ptr(), ws_bytes, ctypes.c_void_p(self.stream.cuda_stream), ctypes.byref(h)))
        self.h = h
        self.weight_bytes = sum(t.numel() * t.element_size() for t in wqkv + wo + wgu + wdown) + \
            self.lm_head.numel() * self.lm_head.element_size()

    def close(self):
        if getattr(self, "h", None):
            self.lib.knnssd_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the calls of the C ABI, same names -------------------------------------------------
    def knnssd_set_anchors(self, anchors: torch.Tensor, labels: torch.Tensor, masks: torch.Tensor):
        """anchors: fp32 or bf16 [n][d_model] (stored as given: a bf16 table is scanned as bf16)."""
        dt = torch.bfloat16 if anchors.dtype == torch.bfloat16 else torch.float32
        self.anchors = anchors.to(self.device, dt).contiguous()
        self.labels = labels.to(self.device, torch.int32).contiguous()
        m = masks.to("cpu", torch.uint8).contiguous()
        if m.dim() != 2:
            raise ValueError("masks must be [n_domains][2*n_blocks]")
        self._masks_host = m
        _check(self.lib.knnssd_set_anchors(self.h, self.anchors.data_ptr(), _DT["bf16" if dt == torch.bfloat16 else "fp32"],
                                           self.labels.data_ptr(), self.anchors.shape[0], self.anchors.shape[1],
                                           m.data_ptr(), m.shape[0], m.shape[1]))

    def knnssd_prefill(self, tokens: Sequence[int], want_hidden: bool = True):
        toks = _i32_array(tokens)
        hidden = torch.empty(self.shape.d_model, dtype=torch.float32, device=self.device) if want_hidden else None
        first = ctypes.c_int32()
        _check(self.lib.knnssd_prefill(self.h, toks, len(tokens), hidden.data_ptr() if want_hidden else None,
                                       ctypes.byref(first)))
        return int(first.value), hidden

    def knnssd_select_skipset(self, query: torch.Tensor):
        q = query.to(self.device, torch.float32).contiguous()
        idx, dom = ctypes.c_int32(), ctypes.c_int32()
        mask = (ctypes.c_uint8 * (2 * self.shape.n_blocks))()
        _check(self.lib.knnssd_select_skipset(self.h, q.data_ptr(), ctypes.byref(idx), ctypes.byref(dom), mask))
        return int(idx.value), int(dom.value), list(mask)

    def knnssd_set_skipset(self, mask: Optional[Sequence[int]]):
        if mask is None:
            _check(self.lib.knnssd_set_skipset(self.h, None))
        else:
            arr = (ctypes.c_uint8 * len(mask))(*[int(v) for v in mask])
            if len(mask) != 2 * self.shape.n_blocks:
                raise ValueError("mask must have 2*n_blocks entries")
            _check(self.lib.knnssd_set_skipset(self.h, arr))

    def knnssd_draft_step(self, token_in: int, pos: int):
        tok, p = ctypes.c_int32(), ctypes.c_float()
        _check(self.lib.knnssd_draft_step(self.h, int(token_in), int(pos), ctypes.byref(tok), ctypes.byref(p)))
        return int(tok.value), float(p.value)

    def knnssd_verify(self, tokens: Sequence[int], start_pos: int):
        toks = _i32_array(tokens)
        j, nxt, new_len = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
        _check(self.lib.knnssd_verify(self.h, toks, len(tokens), int(start_pos), ctypes.byref(j), ctypes.byref(nxt),
                                      ctypes.byref(new_len)))
        return int(j.value), int(nxt.value), int(new_len.value)

    def knnssd_knn_topk(self, queries: torch.Tensor, k: int):
        """K nearest anchors and the majority domain for each row of `queries` ([n][d_model])."""
        q = queries.to(self.device, torch.float32).contiguous()
        if q.dim() == 1:
            q = q[None, :]
        n = q.shape[0]
        idx = (ctypes.c_int32 * (n * k))()
        cos = (ctypes.c_float * (n * k))()
        dom = (ctypes.c_int32 * n)()
        _check(self.lib.knnssd_knn_topk(self.h, q.data_ptr(), n, int(k), idx, cos, dom))
        return ([list(idx[i * k:(i + 1) * k]) for i in range(n)], [list(cos[i * k:(i + 1) * k]) for i in range(n)], list(dom))

    def knnssd_last_selection(self):
        idx, dom = ctypes.c_int32(), ctypes.c_int32()
        _check(self.lib.knnssd_last_selection(self.h, ctypes.byref(idx), ctypes.byref(dom)))
        return int(idx.value), int(dom.value)

    def last_domain(self) -> int:
        return self.knnssd_last_selection()[1]

    def knnssd_generate(self, prompt: Sequence[int], max_new: int, max_draft: int, conf_threshold: float = 0.0,
                        query: Optional[torch.Tensor] = None, route: bool = True):
        toks = _i32_array(prompt)
        gen = GenCfg(int(max_new), int(max_draft), float(conf_threshold), 0 if route else 1)
        out = (ctypes.c_int32 * max(int(max_new), 1))()
        n_out = ctypes.c_int32()
        st = Stats()
        q = None
        if query is not None:
            q = query.to(self.device, torch.float32).contiguous()
        _check(self.lib.knnssd_generate(self.h, toks, len(prompt), q.data_ptr() if q is not None else None,
                                        ctypes.byref(gen), out, ctypes.byref(n_out), ctypes.byref(st)))
        return list(out[:n_out.value]), st.as_dict()

    def knnssd_profile_pass(self, kind: int, tokens: Sequence[int], start_pos: int):
        toks = _i32_array(tokens)
        out = [ctypes.c_int64() for _ in range(4)]
        _check(self.lib.knnssd_profile_pass(self.h, int(kind), toks, len(tokens), int(start_pos),
                                            *[ctypes.byref(o) for o in out]))
        return dict(n_launches=out[0].value, gemm_ns=out[1].value, gemm_bytes=out[2].value, pass_ns=out[3].value)

    def knnssd_get_logits(self, row: int = 0) -> torch.Tensor:
        out = torch.empty(self.shape.vocab, dtype=torch.float32)
        _check(self.lib.knnssd_get_logits(self.h, int(row), out.data_ptr()))
        return out

    def knnssd_read_kv(self, block: int, pos: int):
        kvd = self.shape.n_kv_heads * self.shape.head_dim
        k = torch.empty(kvd, dtype=torch.float32)
        v = torch.empty(kvd, dtype=torch.float32)
        _check(self.lib.knnssd_read_kv(self.h, int(block), int(pos), k.data_ptr(), v.data_ptr()))
        return k, v
