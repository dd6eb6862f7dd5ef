"""ctypes binding of libvvs.so: the same entry points as include/vvs.h, taking torch CUDA tensors.

Argument marshalling only - every step of the verify pass runs inside the HIP library.  PyTorch is
used for device memory and the current stream.  There is no fallback: importing this module on a
machine where the library has not been built raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# VVS_LIBRARY: another build of the same library (for comparing builds); default: the in-tree one
LIB_PATH = os.environ.get("VVS_LIBRARY") or os.path.join(_HERE, "libvvs.so")

VVS_OK, VVS_EINVAL, VVS_ESTATE, VVS_ESIZE, VVS_EHIP = 0, -1, -2, -3, -4
VVS_FP32, VVS_BF16 = 0, 1
VVS_STRICT, VVS_RELAXED = 0, 1
VVS_NORM_AUTO, VVS_NORM_SEPARATE = 0, 1
VVS_MAX_T = 64
VVS_K_GEMM, VVS_K_ATTENTION, VVS_K_ACCEPT, VVS_K_ELEMENTWISE, VVS_K_COMMIT = range(5)


class VvsConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "d_ff", "vocab", "logit_lo", "logit_hi",
                                         "grid_h", "grid_w", "prefix_len", "prefix_kind", "n_classes", "n_prompts",
                                         "max_nodes", "dtype")] + \
               [("cfg_scale", C.c_float), ("rms_eps", C.c_float), ("rope_base", C.c_float),
                ("relax_k", C.c_int32), ("relax_delta", C.c_float),
                ("feature_slots", C.c_int32), ("feature_pre_norm", C.c_int32), ("draft_input", C.c_int32),
                ("norm_mode", C.c_int32)]


class VvsError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"vvs status {status}: {msg}")
        self.status = status


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2511_13587_amd.build); "
                          "there is no CPU or PyTorch fallback for the verify pass")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    sigs = {
        "vvs_query_sizes": (i32, [C.POINTER(VvsConfig), C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]),
        "vvs_create": (i32, [C.POINTER(VvsConfig), vp, vp, vp, C.POINTER(vp)]),
        "vvs_destroy": (None, [vp]),
        "vvs_last_error": (C.c_char_p, [vp]),
        "vvs_num_weight_tensors": (i32, [C.POINTER(VvsConfig)]),
        "vvs_load_weights": (i32, [vp, C.POINTER(vp), i32, vp]),
        "vvs_set_neighbors": (i32, [vp, vp]),
        "vvs_check_tree": (i32, [i32, vp, vp, vp, vp]),
        "vvs_plan_is_fused": (i32, [vp, i32]),
        "vvs_prefill": (i32, [vp, vp, vp, i32, vp, vp, vp, vp]),
        "vvs_verify": (i32, [vp, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]),
        "vvs_verify_post": (i32, [vp, i32, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]),
        "vvs_read_features": (i32, [vp, vp, vp, vp]),
        "vvs_select_unverified": (i32, [i32, vp, vp, C.c_float, vp, C.POINTER(i32)]),
        "vvs_skip_uniform": (i32, [i32, i32]),
        "vvs_skip_dynamic": (i32, [C.c_float, C.c_float, i32]),
        "vvs_set_codebook": (i32, [vp, vp, i32]),
        "vvs_path_similarity": (i32, [vp, i32, vp, vp, vp, C.c_float, i32, vp, vp]),
        "vvs_draft": (i32, [vp, vp, i32, vp, vp, i32, vp, i32, vp, vp, vp, vp]),
        "vvs_accept_from_logits": (i32, [vp, i32, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]),
        "vvs_accept_from_logits_noalloc": (i32, [vp, i32, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]),
        "vvs_kv_commit": (i32, [vp, vp]),
        "vvs_read_state": (i32, [vp, vp, vp]),
        "vvs_set_state": (i32, [vp, vp, vp]),
        "vvs_timing_enable": (i32, [vp, i32]),
        "vvs_timing_read": (i32, [vp, i32, C.POINTER(i32), C.POINTER(C.c_float)]),
        "vvs_debug_logits": (i32, [vp, vp, vp, vp, vp]),
        "vvs_debug_kv": (i32, [vp, i32, i32, i32, vp, vp, vp]),
        "vvs_debug_gemm_scratch_bytes": (sz, [vp, i32, i32, i32]),
        "vvs_debug_gemm": (i32, [vp, i32, i32, i32, vp, vp, vp, vp, vp]),
        "vvs_debug_copy": (i32, [vp, vp, vp, sz, vp]),
        "vvs_debug_fill_probe": (i32, [vp, vp, sz, sz, i32, i32, i32, i32, vp, vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib, list(sigs)


lib, EXPORTS = _load()


def make_config(shape, max_nodes: Optional[int] = None, feature_slots: int = 5, feature_pre_norm: int = 0,
                draft_input: int = 0, norm_mode: int = 0) -> VvsConfig:
    """vvs_config from a synth.Shape-like object."""
    return VvsConfig(shape.n_layers, shape.d_model, shape.n_heads, shape.d_ff, shape.vocab, shape.logit_lo,
                     shape.logit_hi, shape.grid_h, shape.grid_w, shape.prefix_len, shape.prefix_kind,
                     shape.n_classes, shape.n_prompts, shape.n_nodes if max_nodes is None else max_nodes,
                     shape.dtype, shape.cfg_scale, shape.rms_eps, shape.rope_base, shape.relax_k, shape.relax_delta,
                     feature_slots, feature_pre_norm, draft_input, norm_mode)


def vvs_query_sizes(cfg: VvsConfig):
    kv, ws, pw = C.c_size_t(), C.c_size_t(), C.c_size_t()
    st = lib.vvs_query_sizes(C.byref(cfg), C.byref(kv), C.byref(ws), C.byref(pw))
    if st != VVS_OK:
        raise VvsError(st, (lib.vvs_last_error(None) or b"").decode())
    return kv.value, ws.value, pw.value


def vvs_check_tree(n_nodes: int, parent: Optional[np.ndarray], mask: Optional[np.ndarray]):
    """Host-only topology check; returns (status, depth[T], parent[N])."""
    depth = np.zeros(max(n_nodes, 0) + 1, dtype=np.int32)
    pout = np.zeros(max(n_nodes, 1), dtype=np.int32)
    p = None if parent is None else np.ascontiguousarray(parent, dtype=np.int32)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    st = lib.vvs_check_tree(n_nodes, None if p is None else p.ctypes.data, None if m is None else m.ctypes.data,
                            depth.ctypes.data, pout.ctypes.data)
    return st, depth, pout[:max(n_nodes, 0)]


def vvs_select_unverified(n_nodes: int, parent: Optional[np.ndarray], mask: Optional[np.ndarray], u: float):
    """Host-only: (status, kept node ids) of the uniformly drawn, truncated candidate path."""
    nodes = np.zeros(VVS_MAX_T, dtype=np.int32)
    kept = C.c_int32()
    p = None if parent is None else np.ascontiguousarray(parent, dtype=np.int32)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    st = lib.vvs_select_unverified(n_nodes, None if p is None else p.ctypes.data, None if m is None else m.ctypes.data,
                                   float(u), nodes.ctypes.data, C.byref(kept))
    return st, nodes[:max(kept.value, 0)].copy()


def vvs_skip_uniform(step_index: int, interval: int) -> bool:
    return bool(lib.vvs_skip_uniform(step_index, interval))


def vvs_skip_dynamic(similarity: float, threshold: float, last_step_verified: bool) -> bool:
    return bool(lib.vvs_skip_dynamic(float(similarity), float(threshold), 1 if last_step_verified else 0))


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def to_device(a: np.ndarray, dtype: int) -> torch.Tensor:
    """Model-dtype host array (float32 values) -> device tensor (bf16 bits as int16, or float32)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == VVS_BF16:
        u = a.view(np.uint32)
        bits = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)
        return torch.from_numpy(bits.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


class Context:
    """Owns the three device buffers and the vvs_ctx; methods mirror the C entry points."""

    def __init__(self, cfg: VvsConfig, device: str = "cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("libvvs needs a HIP device; there is no CPU path")
        self.cfg = cfg
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.kv_bytes, self.ws_bytes, self.pw_bytes = vvs_query_sizes(cfg)
        self.kv = torch.empty(self.kv_bytes, dtype=torch.uint8, device=self.device)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.device)
        self.pw = torch.empty(self.pw_bytes, dtype=torch.uint8, device=self.device)
        torch.cuda.synchronize()
        h = C.c_void_p()
        st = lib.vvs_create(C.byref(cfg), self.kv.data_ptr(), self.ws.data_ptr(), self.pw.data_ptr(), C.byref(h))
        if st != VVS_OK:
            raise VvsError(st, (lib.vvs_last_error(None) or b"").decode())
        self.h = h
        self.B = cfg.n_prompts
        self.R = 2 * cfg.n_prompts
        self.veff = cfg.logit_hi - cfg.logit_lo
        self._nbr = None
        self.last_T = 0

    def close(self):
        if getattr(self, "h", None):
            torch.cuda.synchronize()
            lib.vvs_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != VVS_OK:
            raise VvsError(st, (lib.vvs_last_error(self.h) or b"").decode())

    # -- weights -------------------------------------------------------------------------------
    def vvs_load_weights(self, tensors: Sequence[Optional[torch.Tensor]]):
        arr = (C.c_void_p * len(tensors))(*[_ptr(t) for t in tensors])
        self._check(lib.vvs_load_weights(self.h, arr, len(tensors), _stream()))

    def load_weights_from_host(self, weights: Dict[str, np.ndarray], names: Sequence[str]):
        """Uploads float32 host arrays in canonical order (converted to the model dtype) and packs."""
        dev = [to_device(weights[n], self.cfg.dtype) for n in names]
        self.vvs_load_weights(dev)
        torch.cuda.synchronize()
        del dev

    def vvs_set_neighbors(self, nbr: torch.Tensor):
        assert nbr.dtype == torch.int32
        self._nbr = nbr
        self._check(lib.vvs_set_neighbors(self.h, _ptr(nbr)))

    # -- the three calls of the hot path ---------------------------------------------------------
    def vvs_prefill(self, prefix_cond: torch.Tensor, prefix_uncond: Optional[torch.Tensor], forced: Optional[torch.Tensor],
                    uniform: torch.Tensor, first_token: torch.Tensor):
        n_forced = 0 if forced is None else int(forced.shape[1])
        self._check(lib.vvs_prefill(self.h, _ptr(prefix_cond), _ptr(prefix_uncond), n_forced, _ptr(forced),
                                    _ptr(uniform), _ptr(first_token), _stream()))
        self.last_T = 1

    def vvs_verify(self, n_nodes: int, parent: Optional[np.ndarray], tree_mask: Optional[np.ndarray],
                   draft_tokens: Optional[torch.Tensor], draft_probs: Optional[torch.Tensor], uniforms: torch.Tensor,
                   mode: int, accept_len: torch.Tensor, path: torch.Tensor, next_token: torch.Tensor):
        p = None if parent is None else np.ascontiguousarray(parent, dtype=np.int32)
        m = None if tree_mask is None else np.ascontiguousarray(tree_mask, dtype=np.uint8)
        self._check(lib.vvs_verify(self.h, n_nodes, None if p is None else p.ctypes.data,
                                   None if m is None else m.ctypes.data, _ptr(draft_tokens), _ptr(draft_probs),
                                   _ptr(uniforms), mode, _ptr(accept_len), _ptr(path), _ptr(next_token), _stream()))
        self.last_T = n_nodes + 1

    def vvs_verify_post(self, n_nodes: int, n_post: int, parent: Optional[np.ndarray], tree_mask: Optional[np.ndarray],
                        draft_tokens: Optional[torch.Tensor], draft_probs: Optional[torch.Tensor], uniforms: torch.Tensor,
                        mode: int, accept_len: torch.Tensor, path: torch.Tensor, next_token: torch.Tensor):
        p = None if parent is None else np.ascontiguousarray(parent, dtype=np.int32)
        m = None if tree_mask is None else np.ascontiguousarray(tree_mask, dtype=np.uint8)
        self._check(lib.vvs_verify_post(self.h, n_nodes, n_post, None if p is None else p.ctypes.data,
                                        None if m is None else m.ctypes.data, _ptr(draft_tokens), _ptr(draft_probs),
                                        _ptr(uniforms), mode, _ptr(accept_len), _ptr(path), _ptr(next_token), _stream()))
        self.last_T = n_nodes + 1

    def vvs_set_codebook(self, embed: torch.Tensor):
        assert embed.dtype == torch.float32 and embed.dim() == 2
        self._codebook = embed                      # kept by reference in the library
        self._check(lib.vvs_set_codebook(self.h, _ptr(embed), int(embed.shape[1])))

    def vvs_path_similarity(self, n_nodes: int, parent, tree_mask, draft_tokens: Optional[torch.Tensor], alpha: float, stride: int = 2):
        p = None if parent is None else np.ascontiguousarray(parent, dtype=np.int32)
        m = None if tree_mask is None else np.ascontiguousarray(tree_mask, dtype=np.uint8)
        out = torch.empty((self.B,), dtype=torch.float32, device=self.device)
        self._check(lib.vvs_path_similarity(self.h, n_nodes, None if p is None else p.ctypes.data,
                                            None if m is None else m.ctypes.data, _ptr(draft_tokens), float(alpha), int(stride),
                                            _ptr(out), _stream()))
        return out

    def vvs_read_features(self):
        """(features float32 [R, feature_slots, d] oldest first, count int32 [B])."""
        feats = torch.empty((self.R, self.cfg.feature_slots, self.cfg.d_model), dtype=torch.float32, device=self.device)
        count = torch.empty((self.B,), dtype=torch.int32, device=self.device)
        self._check(lib.vvs_read_features(self.h, _ptr(feats), _ptr(count), _stream()))
        return feats.cpu().numpy(), count.cpu().numpy()

    def vvs_draft(self, target: "Context", n_nodes: int, parent, tree_mask, n_ctx: int, recent_tokens: torch.Tensor,
                  n_unverified: int, given_tokens: Optional[torch.Tensor], draft_tokens: torch.Tensor, draft_probs: torch.Tensor):
        """self is the drafter context (draft_input = 1)."""
        p = None if parent is None else np.ascontiguousarray(parent, dtype=np.int32)
        m = None if tree_mask is None else np.ascontiguousarray(tree_mask, dtype=np.uint8)
        assert recent_tokens.dtype == torch.int32 and draft_tokens.dtype == torch.int32 and draft_probs.dtype == torch.float32
        self._check(lib.vvs_draft(self.h, target.h, n_nodes, None if p is None else p.ctypes.data,
                                  None if m is None else m.ctypes.data, n_ctx, _ptr(recent_tokens), n_unverified,
                                  _ptr(given_tokens), _ptr(draft_tokens), _ptr(draft_probs), _stream()))
        internal = 0 if p is None else len(set(int(v) for v in p if v > 0))
        self.last_T = n_ctx + (n_nodes - 1 if p is None else internal)

    def vvs_accept_from_logits(self, n_nodes: int, parent, tree_mask, raw_logits: torch.Tensor, draft_tokens, draft_probs,
                               uniforms, mode, accept_len, path, next_token):
        p = None if parent is None else np.ascontiguousarray(parent, dtype=np.int32)
        m = None if tree_mask is None else np.ascontiguousarray(tree_mask, dtype=np.uint8)
        self._check(lib.vvs_accept_from_logits(self.h, n_nodes, None if p is None else p.ctypes.data,
                                               None if m is None else m.ctypes.data, _ptr(raw_logits), _ptr(draft_tokens),
                                               _ptr(draft_probs), _ptr(uniforms), mode, _ptr(accept_len), _ptr(path),
                                               _ptr(next_token), _stream()))

    def vvs_accept_from_logits_noalloc(self, n_nodes: int, parent, tree_mask, raw_logits: torch.Tensor, draft_tokens, draft_probs,
                                       uniforms, mode, accept_len, path, next_token):
        p = None if parent is None else np.ascontiguousarray(parent, dtype=np.int32)
        m = None if tree_mask is None else np.ascontiguousarray(tree_mask, dtype=np.uint8)
        self._check(lib.vvs_accept_from_logits_noalloc(self.h, n_nodes, None if p is None else p.ctypes.data,
                                                       None if m is None else m.ctypes.data, _ptr(raw_logits), _ptr(draft_tokens),
                                                       _ptr(draft_probs), _ptr(uniforms), mode, _ptr(accept_len), _ptr(path),
                                                       _ptr(next_token), _stream()))

    def vvs_kv_commit(self):
        self._check(lib.vvs_kv_commit(self.h, _stream()))

    # -- inspection ----------------------------------------------------------------------------
    def vvs_plan_is_fused(self, n_tokens: int) -> bool:
        return bool(lib.vvs_plan_is_fused(self.h, n_tokens))

    def vvs_read_state(self) -> np.ndarray:
        out = torch.empty((3, self.B), dtype=torch.int32, device=self.device)
        self._check(lib.vvs_read_state(self.h, _ptr(out), _stream()))
        return out.cpu().numpy()

    def vvs_set_state(self, state: torch.Tensor):
        assert state.dtype == torch.int32 and state.numel() == 3 * self.B
        self._check(lib.vvs_set_state(self.h, _ptr(state), _stream()))

    def vvs_timing_enable(self, on: bool):
        self._check(lib.vvs_timing_enable(self.h, 1 if on else 0))

    def vvs_timing_read(self, kernel_class: int):
        n, ms = C.c_int32(), C.c_float()
        self._check(lib.vvs_timing_read(self.h, kernel_class, C.byref(n), C.byref(ms)))
        return n.value, ms.value

    def vvs_debug_logits(self):
        T = self.last_T
        raw = torch.empty((self.R, T, self.veff), dtype=torch.float32, device=self.device)
        mixed = torch.empty((self.B, T, self.veff), dtype=torch.float32, device=self.device)
        probs = torch.empty((self.B, T, self.veff), dtype=torch.float32, device=self.device)
        self._check(lib.vvs_debug_logits(self.h, _ptr(raw), _ptr(mixed), _ptr(probs), _stream()))
        return raw, mixed, probs

    def vvs_debug_kv(self, layer: int, row: int, n_slots: int):
        d = self.cfg.d_model
        k = torch.empty((n_slots, d), dtype=torch.float32, device=self.device)
        v = torch.empty((n_slots, d), dtype=torch.float32, device=self.device)
        self._check(lib.vvs_debug_kv(self.h, layer, row, n_slots, _ptr(k), _ptr(v), _stream()))
        return k, v

    def vvs_debug_copy(self, dst: torch.Tensor, src: torch.Tensor):
        nbytes = src.numel() * src.element_size()
        assert dst.numel() * dst.element_size() == nbytes
        self._check(lib.vvs_debug_copy(self.h, _ptr(dst), _ptr(src), nbytes, _stream()))

    def vvs_debug_fill_probe(self, src: torch.Tensor, reps: int, mode: int, n_workgroups: int, waves: int,
                             region_bytes: int = 0, wg_stride_bytes: int = 0) -> torch.Tensor:
        """region_bytes 0: the whole of src, read by every workgroup; else workgroup w reads region_bytes at w * wg_stride_bytes"""
        total = src.numel() * src.element_size()
        region = region_bytes or total
        assert (n_workgroups - 1) * wg_stride_bytes + region <= total
        sink = torch.zeros(n_workgroups, dtype=torch.int32, device=self.device)
        self._check(lib.vvs_debug_fill_probe(self.h, _ptr(src), region, wg_stride_bytes, reps, mode, n_workgroups, waves,
                                             _ptr(sink), _stream()))
        return sink

    def vvs_debug_gemm(self, a: torch.Tensor, w: torch.Tensor, m: int, n: int, k: int) -> torch.Tensor:
        nbytes = lib.vvs_debug_gemm_scratch_bytes(self.h, m, n, k)
        scratch = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        out = torch.empty((m, n), dtype=torch.float32, device=self.device)
        self._check(lib.vvs_debug_gemm(self.h, m, n, k, _ptr(a), _ptr(w), _ptr(scratch), _ptr(out), _stream()))
        torch.cuda.synchronize()
        return out
