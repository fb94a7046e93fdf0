"""ctypes binding of libspecverify.so: argument marshalling only.

Every step of the verification pass runs in the library's HIP kernels; torch is
used here for device allocations and the stream.  The function names mirror
include/specverify.h.  Importing this module fails loudly if the library has
not been built (python -m paper_2511_16193_amd.build).
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecverify.so")

SV_FP32, SV_BF16 = 0, 1
SV_GREEDY, SV_STOCHASTIC, SV_MATCH = 0, 1, 2
SV_INVERSE_CDF, SV_EXP_RACE = 0, 1
SV_OPT_GEMM_VARIANT, SV_OPT_ATTN_GENERIC, SV_OPT_ATTN_MIN_ROW_TILES, SV_OPT_ATTN_CHUNK_KEYS, SV_OPT_ATTN_MAX_ROW_TILES, SV_OPT_GRAPH, SV_OPT_GEMM_TILE = 1, 2, 3, 4, 5, 6, 7
SV_PROF_GEMM, SV_PROF_ATTENTION, SV_PROF_SAMPLER, SV_PROF_ROLLBACK, SV_PROF_MOE = 0, 1, 2, 3, 4

EXPORTS = [
    "verify_kv_pool_bytes", "verify_workspace_bytes", "verify_init", "verify_destroy", "verify_last_error",
    "verify_seq_add", "verify_seq_remove", "verify_seq_set_len", "verify_seq_len", "verify_kv_write",
    "verify_kv_read", "verify_prefill", "verify_prefill_batch", "verify_step",
    "sv_op_gemm_bf16", "sv_op_gemm_bf16_ws", "sv_op_gemm_plan", "sv_op_pack_rows", "sv_op_pack_weight", "sv_op_sample_scratch_bytes", "sv_op_sample", "sv_op_sample_static", "sv_op_moe_scratch_bytes", "sv_op_moe_ffn", "sv_op_attention", "sv_op_layer", "sv_op_rollback", "sv_set_option", "sv_seq_set_lens", "sv_profile_enable",
    "sv_profile_read", "sv_probe_mfma_bf16", "sv_probe_hbm_copy", "sv_probe_hbm_read", "sv_probe_mfma_valu",
    "sv_plan_accept_prob", "sv_plan_tau", "sv_plan_decoupled", "sv_plan_best_window", "sv_fit_affine",
]


class SvModel(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ff",
                                         "vocab", "n_experts", "top_k", "d_expert", "dtype")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class SvWeights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("ln1", "wqkv", "wo", "ln2", "w_gate_up", "w_down", "w_router")] + \
               [("packed", C.c_int32)]


class SvRuntime(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("max_batch", "max_k", "max_chains", "max_seqs", "page_size", "num_pages",
                                         "max_pages_per_seq", "verify_mode", "sample_mode")] + \
               [("temperature", C.c_float), ("kv_pool", C.c_void_p), ("kv_pool_bytes", C.c_size_t),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


class SvBatch(C.Structure):
    _fields_ = [("B", C.c_int32), ("k", C.c_int32), ("N", C.c_int32), ("seq_ids", C.POINTER(C.c_int32)),
                ("last_tokens", C.c_void_p), ("draft_lens", C.c_void_p)]


class SvAffine(C.Structure):
    _fields_ = [("slope", C.c_double), ("icpt", C.c_double)]


class SvPlanInput(C.Structure):
    _fields_ = [("B", C.c_int), ("G", C.c_int), ("p", C.c_double), ("n_configs", C.c_int), ("g_v", C.POINTER(C.c_int)),
                ("W", C.c_int), ("D", C.POINTER(SvAffine)), ("V", C.POINTER(SvAffine))]


class SvPlan(C.Structure):
    _fields_ = [("g_d", C.c_int), ("g_v", C.c_int), ("w", C.c_int), ("b", C.c_int), ("tgs", C.c_double)]


class SvOut(C.Structure):
    _fields_ = [("accepted_len", C.c_void_p), ("out_tokens", C.c_void_p), ("best_chain", C.c_void_p),
                ("logits", C.c_void_p)]


def load_library() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_16193_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    lib.verify_kv_pool_bytes.restype = C.c_size_t
    lib.verify_kv_pool_bytes.argtypes = [C.POINTER(SvModel), C.POINTER(SvRuntime)]
    lib.verify_workspace_bytes.restype = C.c_size_t
    lib.verify_workspace_bytes.argtypes = [C.POINTER(SvModel), C.POINTER(SvRuntime)]
    lib.verify_init.argtypes = [C.POINTER(SvModel), C.POINTER(SvWeights), C.POINTER(SvRuntime), C.c_void_p,
                                C.POINTER(C.c_void_p)]
    lib.verify_destroy.argtypes = [C.c_void_p]
    lib.verify_destroy.restype = None
    lib.verify_last_error.argtypes = [C.c_void_p]
    lib.verify_last_error.restype = C.c_char_p
    lib.verify_seq_add.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    lib.verify_seq_remove.argtypes = [C.c_void_p, C.c_int32]
    lib.verify_seq_set_len.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    lib.verify_seq_len.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]
    lib.verify_kv_write.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.verify_kv_read.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.verify_prefill.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
    lib.verify_prefill_batch.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_void_p, C.c_int32,
                                         C.POINTER(C.c_int32), C.c_void_p]
    lib.verify_step.argtypes = [C.c_void_p, C.POINTER(SvBatch), C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(SvOut)]
    lib.sv_op_gemm_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                    C.c_void_p]
    lib.sv_op_pack_weight.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    lib.sv_op_pack_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    lib.sv_op_gemm_bf16_ws.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                       C.c_void_p]
    lib.sv_op_gemm_plan.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.sv_op_sample_scratch_bytes.restype = C.c_size_t
    lib.sv_op_sample_scratch_bytes.argtypes = [C.c_int, C.c_int, C.c_int]
    lib.sv_op_sample.argtypes = [C.c_void_p] * 5 + [C.c_int] * 6 + [C.c_float] + [C.c_void_p] * 5
    lib.sv_op_sample_static.argtypes = [C.c_void_p] * 5 + [C.c_int] * 6 + [C.c_float] + [C.c_void_p] * 4
    lib.sv_op_moe_scratch_bytes.restype = C.c_size_t
    lib.sv_op_moe_scratch_bytes.argtypes = [C.c_int] * 5
    lib.sv_op_moe_ffn.argtypes = [C.c_void_p] * 4 + [C.c_int] * 5 + [C.c_void_p, C.c_size_t] + [C.c_void_p] * 4
    lib.sv_op_attention.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                    C.c_void_p]
    lib.sv_op_layer.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.c_void_p]
    lib.sv_op_rollback.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int]
    lib.sv_seq_set_lens.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int]
    lib.sv_profile_enable.argtypes = [C.c_void_p, C.c_uint]
    lib.sv_profile_read.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int)]
    lib.sv_probe_mfma_bf16.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_int, C.c_void_p, C.POINTER(C.c_double)]
    lib.sv_probe_hbm_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.POINTER(C.c_double)]
    lib.sv_probe_hbm_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
    lib.sv_probe_mfma_valu.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_double)]
    lib.sv_set_option.argtypes = [C.c_void_p, C.c_int, C.c_int]
    lib.sv_plan_accept_prob.restype = C.c_double
    lib.sv_plan_accept_prob.argtypes = [C.c_double, C.c_int, C.c_int]
    lib.sv_plan_tau.restype = C.c_double
    lib.sv_plan_tau.argtypes = [C.c_double, C.c_int]
    lib.sv_plan_decoupled.argtypes = [C.POINTER(SvPlanInput), C.POINTER(SvPlan)]
    lib.sv_plan_best_window.argtypes = [C.c_double, SvAffine, C.POINTER(SvAffine), C.c_int, C.c_double,
                                        C.POINTER(C.c_int), C.POINTER(C.c_double)]
    lib.sv_fit_affine.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int, C.POINTER(SvAffine)]
    return lib


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = load_library()
    return _lib


class SvError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"specverify error {code}: {msg}")
        self.code = code


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_ptr():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Verifier:
    """Owns the device buffers a context borrows and forwards calls to the C ABI."""

    def __init__(self, model: dict, weights: dict, *, max_batch: int, max_k: int, max_chains: int = 1,
                 max_seqs: int | None = None, page_size: int = 64, num_pages: int, max_pages_per_seq: int,
                 verify_mode: int = SV_STOCHASTIC, sample_mode: int = SV_EXP_RACE, temperature: float = 1.0,
                 packed: bool = False, device="cuda:0"):
        self.lib = lib()
        self.device = torch.device(device)
        self.model = dict(model)
        dt = SV_BF16 if model["dtype"] == "bf16" else SV_FP32
        self.torch_dtype = torch.bfloat16 if dt == SV_BF16 else torch.float32
        self.m = SvModel(model["n_layers"], model["d_model"], model["n_q_heads"], model["n_kv_heads"],
                         model["head_dim"], model["d_ff"], model["vocab"], model.get("n_experts", 0),
                         model.get("top_k", 0), model.get("d_expert", 0), dt, model["rope_theta"], model["rms_eps"])
        self.rt = SvRuntime(max_batch, max_k, max_chains, max_seqs or max_batch, page_size, num_pages,
                            max_pages_per_seq, verify_mode, sample_mode, temperature, None, 0, None, 0)
        pool_bytes = self.lib.verify_kv_pool_bytes(C.byref(self.m), C.byref(self.rt))
        ws_bytes = self.lib.verify_workspace_bytes(C.byref(self.m), C.byref(self.rt))
        if pool_bytes == 0 or ws_bytes == 0:
            raise SvError(-1, "invalid model / runtime description")
        self.kv_pool = torch.empty(pool_bytes, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=self.device)
        self.rt.kv_pool, self.rt.kv_pool_bytes = self.kv_pool.data_ptr(), pool_bytes
        self.rt.workspace, self.rt.workspace_bytes = self.workspace.data_ptr(), ws_bytes

        self._keep = weights                       # borrowed by the context: keep alive
        nl = model["n_layers"]

        def arr(name):
            if name not in weights["layers"][0]:
                return None
            a = (C.c_void_p * nl)()
            for l in range(nl):
                t = weights["layers"][l][name]
                assert t.is_cuda and t.is_contiguous() and t.dtype == self.torch_dtype, name
                a[l] = t.data_ptr()
            return a

        self._arrs = {n: arr(n) for n in ("ln1", "wqkv", "wo", "ln2", "w_gate_up", "w_down", "w_router")}
        w = SvWeights(weights["embed"].data_ptr(), weights["lm_head"].data_ptr(), weights["final_norm"].data_ptr(),
                      *[self._arrs[n] if self._arrs[n] is not None else None
                        for n in ("ln1", "wqkv", "wo", "ln2", "w_gate_up", "w_down", "w_router")], 1 if packed else 0)
        ctx = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = self.lib.verify_init(C.byref(self.m), C.byref(w), C.byref(self.rt), _stream_ptr(), C.byref(ctx))
        if rc != 0:
            raise SvError(rc, "verify_init failed")
        self.ctx = ctx
        self.vocab = model["vocab"]

    # -- plumbing --
    def _check(self, rc: int):
        if rc != 0:
            raise SvError(rc, self.lib.verify_last_error(self.ctx).decode())

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.verify_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- sequences --
    def seq_add(self, seq_id: int, cached_len: int):
        self._check(self.lib.verify_seq_add(self.ctx, seq_id, cached_len))

    def seq_remove(self, seq_id: int):
        self._check(self.lib.verify_seq_remove(self.ctx, seq_id))

    def seq_set_len(self, seq_id: int, length: int):
        self._check(self.lib.verify_seq_set_len(self.ctx, seq_id, length))

    def seq_len(self, seq_id: int) -> int:
        out = C.c_int32()
        self._check(self.lib.verify_seq_len(self.ctx, seq_id, C.byref(out)))
        return out.value

    def kv_write(self, seq_id: int, layer: int, pos0: int, k: torch.Tensor, v: torch.Tensor):
        assert k.dtype == self.torch_dtype and k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
        self._check(self.lib.verify_kv_write(self.ctx, seq_id, layer, pos0, k.shape[0], _ptr(k), _ptr(v)))

    def kv_read(self, seq_id: int, layer: int, pos0: int, n: int):
        shape = (n, self.model["n_kv_heads"], self.model["head_dim"])
        k = torch.empty(shape, dtype=self.torch_dtype, device=self.device)
        v = torch.empty(shape, dtype=self.torch_dtype, device=self.device)
        self._check(self.lib.verify_kv_read(self.ctx, seq_id, layer, pos0, n, _ptr(k), _ptr(v)))
        return k, v

    def prefill(self, seq_id: int, tokens: torch.Tensor, want_logits: bool = True):
        tokens = tokens.to(device=self.device, dtype=torch.int32).contiguous()
        out = torch.empty(self.vocab, dtype=torch.float32, device=self.device) if want_logits else None
        self._check(self.lib.verify_prefill(self.ctx, seq_id, _ptr(tokens), tokens.numel(), _ptr(out)))
        return out

    def prefill_batch(self, seq_ids, tokens: torch.Tensor, lens, want_logits: bool = True):
        """tokens int32 [B, ld] (row b = prompt of seq_ids[b], lens[b] tokens long); any order: the rows are
        handed over longest first and the logits returned in the caller's order."""
        B = len(seq_ids)
        order = sorted(range(B), key=lambda b: -int(lens[b]))
        tokens = tokens.to(device=self.device, dtype=torch.int32)
        tok = tokens[torch.as_tensor(order, device=self.device)].contiguous()
        ids = (C.c_int32 * B)(*[int(seq_ids[b]) for b in order])
        n = (C.c_int32 * B)(*[int(lens[b]) for b in order])
        out = torch.empty((B, self.vocab), dtype=torch.float32, device=self.device) if want_logits else None
        self._check(self.lib.verify_prefill_batch(self.ctx, ids, B, _ptr(tok), tok.shape[1], n, _ptr(out)))
        if out is None:
            return None
        inv = torch.empty(B, dtype=torch.long)
        inv[torch.as_tensor(order)] = torch.arange(B)
        return out[inv.to(self.device)]

    # -- the step --
    def step(self, seq_ids, last_tokens: torch.Tensor, drafts: torch.Tensor | None, draft_probs: torch.Tensor | None,
             uniforms: torch.Tensor | None, *, draft_lens: torch.Tensor | None = None, want_logits: bool = False,
             out: dict | None = None):
        """drafts int32 [B,N,k]; draft_probs fp32 [B,N,k,V] or None; uniforms fp32 [B,N,k+1]."""
        B = len(seq_ids)
        if drafts is None:
            N, k = 1, 0
        else:
            assert drafts.dtype == torch.int32 and drafts.is_contiguous() and drafts.shape[0] == B
            N, k = drafts.shape[1], drafts.shape[2]
        assert last_tokens.dtype == torch.int32 and last_tokens.numel() == B
        if draft_probs is not None:
            assert draft_probs.dtype == torch.float32 and draft_probs.is_contiguous()
            assert tuple(draft_probs.shape) == (B, N, k, self.vocab)
        if uniforms is not None:
            assert uniforms.dtype == torch.float32 and uniforms.is_contiguous() and tuple(uniforms.shape) == (B, N, k + 1)
        ids = (C.c_int32 * B)(*[int(s) for s in seq_ids])
        if out is None:
            out = {
                "accepted_len": torch.empty(B, dtype=torch.int32, device=self.device),
                "out_tokens": torch.empty((B, k + 1), dtype=torch.int32, device=self.device),
                "best_chain": torch.empty(B, dtype=torch.int32, device=self.device),
            }
            if want_logits:
                out["logits"] = torch.empty((B, 1 + N * k, self.vocab), dtype=torch.float32, device=self.device)
        batch = SvBatch(B, k, N, ids, last_tokens.data_ptr(), None if draft_lens is None else draft_lens.data_ptr())
        o = SvOut(out["accepted_len"].data_ptr(), out["out_tokens"].data_ptr(), out["best_chain"].data_ptr(),
                  out["logits"].data_ptr() if "logits" in out else None)
        self._check(self.lib.verify_step(self.ctx, C.byref(batch), _ptr(drafts), _ptr(draft_probs), _ptr(uniforms),
                                         C.byref(o)))
        return out

    def op_attention(self, seq_ids, n: int, k: int, layer: int, q: torch.Tensor) -> torch.Tensor:
        """q [B*n, n_q_heads, head_dim] storage type -> [B*n, n_q_heads*head_dim]."""
        B = len(seq_ids)
        assert q.dtype == self.torch_dtype and q.is_contiguous() and q.shape[0] == B * n
        out = torch.empty((B * n, q.shape[1] * q.shape[2]), dtype=self.torch_dtype, device=self.device)
        ids = (C.c_int32 * B)(*[int(s) for s in seq_ids])
        self._check(self.lib.sv_op_attention(self.ctx, ids, B, n, k, layer, _ptr(q), _ptr(out)))
        return out

    def op_layer(self, seq_ids, n: int, k: int, layer: int, h: torch.Tensor, want_routing: bool = False):
        """h fp32 [B*n, d_model] entering `layer` -> the residual stream after it (and, for mixture-of-experts
        models with want_routing, the rows' expert ids [B*n, top_k] and weights)."""
        B = len(seq_ids)
        assert h.dtype == torch.float32 and h.is_contiguous() and tuple(h.shape) == (B * n, self.model["d_model"])
        out = torch.empty_like(h)
        ids = (C.c_int32 * B)(*[int(s) for s in seq_ids])
        top_ids = top_w = None
        if want_routing and self.model.get("n_experts", 0):
            top_ids = torch.empty((B * n, self.model["top_k"]), dtype=torch.int32, device=self.device)
            top_w = torch.empty((B * n, self.model["top_k"]), dtype=torch.float32, device=self.device)
        self._check(self.lib.sv_op_layer(self.ctx, ids, B, n, k, layer, _ptr(h), _ptr(out), _ptr(top_ids), _ptr(top_w)))
        return (out, top_ids, top_w) if want_routing else out

    def op_rollback(self, seq_ids, N: int, k: int, accepted_len: torch.Tensor, best_chain: torch.Tensor, commit: bool = True):
        """The rollback stage alone on given verdicts (int32 device tensors [B])."""
        B = len(seq_ids)
        assert accepted_len.dtype == torch.int32 and best_chain.dtype == torch.int32 and accepted_len.numel() == B == best_chain.numel()
        ids = (C.c_int32 * B)(*[int(s) for s in seq_ids])
        self._check(self.lib.sv_op_rollback(self.ctx, ids, B, N, k, _ptr(accepted_len), _ptr(best_chain), 1 if commit else 0))

    def seq_set_lens(self, seq_ids, lens):
        n = len(seq_ids)
        ids = (C.c_int32 * n)(*[int(s) for s in seq_ids])
        ln = (C.c_int32 * n)(*[int(x) for x in lens])
        self._check(self.lib.sv_seq_set_lens(self.ctx, ids, ln, n))

    def profile_enable(self, kind_mask: int):
        self._check(self.lib.sv_profile_enable(self.ctx, kind_mask))

    def profile_read(self, kind: int):
        """-> (total milliseconds, number of timed launch groups) since the last read; synchronises."""
        ms, n = C.c_double(), C.c_int()
        self._check(self.lib.sv_profile_read(self.ctx, kind, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def set_option(self, option: int, value: int):
        self._check(self.lib.sv_set_option(self.ctx, option, value))


# ---- single operations ----

def op_pack_weight(w: torch.Tensor) -> torch.Tensor:
    """Row-major bf16 [N,K] (or a stack [E,N,K]) -> same shape, fragment order of the projection kernels."""
    assert w.dtype == torch.bfloat16 and w.is_contiguous() and w.is_cuda
    out = torch.empty_like(w)
    if w.shape[-2] % 128 == 0:          # whole 128-row panels per matrix: a stack packs as one tall matrix
        mats = w.reshape(1, -1, w.shape[-1])
        outs = out.reshape(1, -1, w.shape[-1])
    else:
        mats = w.reshape(-1, w.shape[-2], w.shape[-1])
        outs = out.reshape(-1, w.shape[-2], w.shape[-1])
    for i in range(mats.shape[0]):
        rc = lib().sv_op_pack_weight(_ptr(mats[i]), _ptr(outs[i]), mats.shape[1], mats.shape[2], _stream_ptr())
        if rc != 0:
            raise SvError(rc, "sv_op_pack_weight")
    return out


def op_pack_rows(a: torch.Tensor) -> torch.Tensor:
    """Row-major bf16 activations [M,K] -> packed order, ceil(M/32)*32 rows (padding rows zero)."""
    assert a.dtype == torch.bfloat16 and a.is_contiguous() and a.is_cuda
    M, K = a.shape
    out = torch.empty(((M + 31) // 32 * 32, K), dtype=torch.bfloat16, device=a.device)
    rc = lib().sv_op_pack_rows(_ptr(a), _ptr(out), M, K, _stream_ptr())
    if rc != 0:
        raise SvError(rc, "sv_op_pack_rows")
    return out


def op_gemm_bf16_ws(a_packed: torch.Tensor, w_packed: torch.Tensor, M: int, splits: int = 1, wide: bool = True,
                    row_tiles: int = 0) -> torch.Tensor:
    """Weight-streaming projection on packed operands -> [splits, M, N] fp32 partial products."""
    K = a_packed.shape[1]
    N = w_packed.shape[0]
    out = torch.empty((splits, M, N), dtype=torch.float32, device=a_packed.device)
    rc = lib().sv_op_gemm_bf16_ws(_ptr(a_packed), _ptr(w_packed), _ptr(out), M, N, K, splits, 1 if wide else 0, row_tiles, _stream_ptr())
    if rc != 0:
        raise SvError(rc, "sv_op_gemm_bf16_ws")
    return out


def op_gemm_plan(M: int, N: int, K: int) -> dict:
    """The launch shape the step would give this projection: {"splits", "wide", "row_tiles"}."""
    s, w, t = C.c_int(), C.c_int(), C.c_int()
    rc = lib().sv_op_gemm_plan(M, N, K, C.byref(s), C.byref(w), C.byref(t))
    if rc != 0:
        raise SvError(rc, "sv_op_gemm_plan")
    return {"splits": s.value, "wide": bool(w.value), "row_tiles": t.value}


def op_moe_ffn(a: torch.Tensor, w_router: torch.Tensor, w_gate_up: torch.Tensor, w_down: torch.Tensor, top_k: int):
    """Mixture-of-experts FFN of bf16 rows a [T,d]; w_router [E,d], w_gate_up [E,2F,d], w_down [E,d,F], all bf16
    row-major (packed here).  -> (out [T,d] fp32, expert ids [T,top_k] int32, weights [T,top_k] fp32)."""
    T, d = a.shape
    E, F = w_router.shape[0], w_down.shape[2]
    ap, gp, dp = op_pack_rows(a), op_pack_weight(w_gate_up), op_pack_weight(w_down)
    nbytes = lib().sv_op_moe_scratch_bytes(T, d, E, top_k, F)
    if nbytes == 0:
        raise SvError(-4, "sv_op_moe_scratch_bytes")
    scratch = torch.empty(nbytes, dtype=torch.uint8, device=a.device)
    out = torch.empty((T, d), dtype=torch.float32, device=a.device)
    ids = torch.empty((T, top_k), dtype=torch.int32, device=a.device)
    wts = torch.empty((T, top_k), dtype=torch.float32, device=a.device)
    rc = lib().sv_op_moe_ffn(_ptr(ap), _ptr(w_router.contiguous()), _ptr(gp), _ptr(dp), T, d, E, top_k, F, _ptr(scratch),
                             nbytes, _ptr(out), _ptr(ids), _ptr(wts), _stream_ptr())
    if rc != 0:
        raise SvError(rc, "sv_op_moe_ffn")
    return out, ids, wts


def pack_weights(weights: dict) -> dict:
    """Packed copies of the projection matrices of a weight dict (embed and gains shared)."""
    names = ("wqkv", "wo", "w_gate_up", "w_down")
    out = {k: v for k, v in weights.items() if k != "layers"}
    out["lm_head"] = op_pack_weight(weights["lm_head"])
    out["layers"] = [{k: (op_pack_weight(v) if k in names else v) for k, v in lw.items()} for lw in weights["layers"]]
    return out


def op_gemm_bf16(a: torch.Tensor, w: torch.Tensor, splits: int = 1, variant: int = 0) -> torch.Tensor:
    """a [M,K] bf16, w [N,K] bf16, both row-major -> [splits, M, N] fp32 partial products."""
    assert a.dtype == torch.bfloat16 and w.dtype == torch.bfloat16 and a.is_contiguous() and w.is_contiguous()
    M, K = a.shape
    N = w.shape[0]
    out = torch.empty((splits, M, N), dtype=torch.float32, device=a.device)
    rc = lib().sv_op_gemm_bf16(_ptr(a), _ptr(w), _ptr(out), M, N, K, splits, variant, _stream_ptr())
    if rc != 0:
        raise SvError(rc, "sv_op_gemm_bf16")
    return out


def op_sample(logits: torch.Tensor, drafts: torch.Tensor, draft_probs, uniforms, *, verify_mode: int,
              sample_mode: int = SV_EXP_RACE, temperature: float = 1.0, draft_lens=None):
    """logits fp32 [B, 1+N*k, V]; drafts int32 [B,N,k]."""
    B, N, k = drafts.shape
    V = logits.shape[-1]
    assert logits.dtype == torch.float32 and logits.is_contiguous() and logits.shape[1] == 1 + N * k
    dev = logits.device
    scratch = torch.empty(lib().sv_op_sample_scratch_bytes(B, N, k), dtype=torch.uint8, device=dev)
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    toks = torch.empty((B, k + 1), dtype=torch.int32, device=dev)
    best = torch.empty(B, dtype=torch.int32, device=dev)
    rc = lib().sv_op_sample(_ptr(logits), _ptr(drafts), _ptr(draft_probs), _ptr(uniforms), _ptr(draft_lens), B, N, k, V,
                            verify_mode, sample_mode, temperature, _ptr(scratch), _ptr(acc), _ptr(toks), _ptr(best),
                            _stream_ptr())
    if rc != 0:
        raise SvError(rc, "sv_op_sample")
    return acc, toks, best


def op_sample_static(logits: torch.Tensor, drafts: torch.Tensor, draft_probs, uniforms, acc: torch.Tensor,
                     toks: torch.Tensor, best: torch.Tensor, *, verify_mode: int, sample_mode: int = SV_EXP_RACE,
                     temperature: float = 1.0, draft_lens=None):
    """sv_op_sample on the library's static scratch: the caller brings the outputs too (acc int32 [B], toks int32
    [B,k+1], best int32 [B]), so that nothing at all is allocated between the call and its kernels."""
    B, N, k = drafts.shape
    V = logits.shape[-1]
    assert logits.dtype == torch.float32 and logits.is_contiguous() and logits.shape[1] == 1 + N * k
    rc = lib().sv_op_sample_static(_ptr(logits), _ptr(drafts), _ptr(draft_probs), _ptr(uniforms), _ptr(draft_lens), B, N, k,
                                   V, verify_mode, sample_mode, temperature, _ptr(acc), _ptr(toks), _ptr(best),
                                   _stream_ptr())
    if rc != 0:
        raise SvError(rc, "sv_op_sample_static")
    return acc, toks, best


def probe_peaks(device="cuda:0", mfma_iters: int = 60000, copy_bytes: int = 1 << 30, copy_reps: int = 5) -> dict:
    """The two micro-benchmarked rooflines of this GPU: dense bf16 MFMA rate on random operands (and on zeros),
    and the rate of a plain device copy."""
    dev = torch.device(device)
    out = {}
    sink = torch.empty(256 * 256, dtype=torch.float32, device=dev)
    for name, ops in (("mfma_bf16_tflops_random_operands", torch.randn(256 * 256 * 64, device=dev).to(torch.bfloat16)),
                      ("mfma_bf16_tflops_zero_operands", torch.zeros(256 * 256 * 64, dtype=torch.bfloat16, device=dev))):
        best = 0.0
        for _ in range(3):                      # the clock takes a few milliseconds of load to settle: best of three runs
            v = C.c_double()
            rc = lib().sv_probe_mfma_bf16(_ptr(ops), ops.numel() * 2, _ptr(sink), mfma_iters, _stream_ptr(), C.byref(v))
            if rc != 0:
                raise SvError(rc, "sv_probe_mfma_bf16")
            best = max(best, v.value)
        out[name] = best
    out["hbm_copy_gbs_read_plus_write"] = 2.0 * probe_copy(copy_bytes, copy_reps, dev)
    src = torch.ones(copy_bytes // 4, dtype=torch.float32, device=dev)
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    v = C.c_double()
    rc = lib().sv_probe_hbm_read(_ptr(src), copy_bytes, copy_reps, _ptr(flag), _stream_ptr(), C.byref(v))
    if rc != 0:
        raise SvError(rc, "sv_probe_hbm_read")
    out["hbm_read_gbs"] = v.value
    return out


def probe_mfma_valu(iters: int = 20000, device="cuda:0") -> dict:
    """Do matrix and vector instructions of a SIMD overlap?  Times (ms) of `iters` rounds of eight 16x16x32 bf16 MFMAs,
    of 8 * NV FMAs, and of both woven, for NV in (2, 4, 6) and one or two waves per SIMD."""
    dev = torch.device(device)
    sink = torch.empty(256 * 512, dtype=torch.float32, device=dev)
    out = {}
    for waves in (1, 2):
        for nv in (2, 4, 6):
            ms = (C.c_double * 3)()
            rc = lib().sv_probe_mfma_valu(_ptr(sink), iters, nv, waves, _stream_ptr(), ms)
            if rc != 0:
                raise SvError(rc, "sv_probe_mfma_valu")
            out[f"waves_per_simd_{waves}_fma_per_mfma_{nv}"] = {"mfma_ms": ms[0], "fma_ms": ms[1], "woven_ms": ms[2]}
    return out


def probe_copy(nbytes: int = 1 << 30, reps: int = 1, device="cuda:0") -> float:
    """`reps` plain device copies of nbytes (after one untimed warm-up copy); GB/s copied (as much read as written)."""
    dev = torch.device(device)
    src = torch.ones(nbytes // 4, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    v = C.c_double()
    rc = lib().sv_probe_hbm_copy(_ptr(src), _ptr(dst), nbytes, reps, _stream_ptr(), C.byref(v))
    if rc != 0:
        raise SvError(rc, "sv_probe_hbm_copy")
    return v.value


# ---- planner (host-only entry points of specverify_plan.h) ----

def plan_accept_prob(p: float, a: int, w: int) -> float:
    return lib().sv_plan_accept_prob(p, a, w)


def plan_tau(p: float, w: int) -> float:
    return lib().sv_plan_tau(p, w)


def fit_affine(bs, ts):
    """(slope, icpt) of the least-squares line through the points."""
    n = len(bs)
    out = SvAffine()
    rc = lib().sv_fit_affine((C.c_double * n)(*bs), (C.c_double * n)(*ts), n, C.byref(out))
    if rc != 0:
        raise SvError(rc, "sv_fit_affine: need two or more points with distinct batch sizes")
    return out.slope, out.icpt


def plan_decoupled(B: int, G: int, p: float, g_v, D, V, W: int) -> dict:
    """Algorithm 1.  g_v: verifier configurations; D[g-1] = (slope, icpt) for g = 1..max(g_v);
    V[c][w-1] = (slope, icpt) for configuration c and window w = 1..W."""
    nc = len(g_v)
    if len(D) < max(g_v) or len(V) != nc or any(len(v) != W for v in V):
        raise ValueError("D needs max(g_v) entries, V one row of W entries per configuration")
    inp = SvPlanInput(B, G, p, nc, (C.c_int * nc)(*g_v), W, (SvAffine * len(D))(*[SvAffine(*d) for d in D]),
                      (SvAffine * (nc * W))(*[SvAffine(*x) for v in V for x in v]))
    out = SvPlan()
    rc = lib().sv_plan_decoupled(C.byref(inp), C.byref(out))
    if rc != 0:
        raise SvError(rc, "sv_plan_decoupled: invalid arguments")
    return {"g_d": out.g_d, "g_v": out.g_v, "w": out.w, "b": out.b, "tgs": out.tgs}


def plan_best_window(p: float, D, V, b: float):
    W = len(V)
    w, t = C.c_int(), C.c_double()
    rc = lib().sv_plan_best_window(p, SvAffine(*D), (SvAffine * W)(*[SvAffine(*x) for x in V]), W, b, C.byref(w), C.byref(t))
    if rc != 0:
        raise SvError(rc, "sv_plan_best_window: invalid arguments")
    return w.value, t.value
