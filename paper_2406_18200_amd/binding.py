"""ctypes binding for libseed_verify.so -- same names and argument meaning as include/seed_verify.h."""
import ctypes as C
import os
from dataclasses import dataclass

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

SEED_KIND_LOGITS, SEED_KIND_PROBS = 0, 1
SEED_STEP_PREFILL_SHARED, SEED_STEP_GREEDY, SEED_STEP_COMMIT_ALL = 1, 2, 4
ERROR_NAMES = {-1: "SEED_E_INVALID_ARG", -2: "SEED_E_SHAPE", -3: "SEED_E_CAPACITY", -4: "SEED_E_NULL_PTR",
               -5: "SEED_E_UNSUPPORTED_DTYPE", -6: "SEED_E_NOT_INIT", -7: "SEED_E_HIP"}


class SeedError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{ERROR_NAMES.get(code, code)}: {msg}")
        self.code = code


class ModelCfgC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ff", "vocab", "dtype")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("max_branches", "max_rows_per_branch", "max_shared", "max_private")]


class LayerWC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "norm_attn", "norm_ffn",
                                          "sq", "sk", "sv", "so", "sgate", "sup", "sdown")]


class WeightsC(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("norm_final", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(LayerWC)), ("lm_head_scale", C.c_void_p)]


class TreeC(C.Structure):
    _fields_ = [("depth", C.c_int32), ("k_config", C.POINTER(C.c_int32))]


def _tree_struct(k_config):
    """seed_tree for a k_config tuple (None -> NULL); returns (pointer or None, keep-alive objects)."""
    if k_config is None:
        return None, None
    arr = (C.c_int32 * len(k_config))(*[int(k) for k in k_config])
    t = TreeC(len(k_config), arr)
    return C.pointer(t), (arr, t)


def tree_sizes(k_config):
    """(n_nodes incl. the root, n_par = nodes that have children) of a k_config tree in level order."""
    level, n, n_par = 1, 1, 1
    for j, k in enumerate(k_config):
        level *= int(k)
        if j:
            n_par = n
        n += level
    return n, (n - level)


class AcceptArgsC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_branches", "gamma", "n_target_rows", "vocab", "probs_kind", "greedy")] + \
               [("temperature", C.c_float)] + \
               [(n, C.c_void_p) for n in ("p_or_logits", "q", "draft_tok", "u_acc", "u_res", "accept_len",
                                          "out_tok", "n_out", "p_tok", "private_len")] + \
               [("tree", C.POINTER(TreeC)), ("path_node", C.c_void_p)]


class StepArgsC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_branches", "rows_per_branch", "flags", "shared_len")] + \
               [("row_tok", C.c_void_p), ("private_len", C.c_void_p), ("logits_out", C.c_void_p),
                ("accept", C.POINTER(AcceptArgsC)), ("branch_slot", C.c_void_p), ("tree", C.POINTER(TreeC))]


class DraftArgsC(C.Structure):
    _fields_ = [("n_branches", C.c_int32), ("flags", C.c_int32), ("shared_len", C.c_int32),
                ("temperature", C.c_float), ("row_tok", C.c_void_p), ("private_len", C.c_void_p),
                ("u", C.c_void_p), ("q_out", C.c_void_p), ("q_stride", C.c_int64), ("tok_out", C.c_void_p),
                ("tok_stride", C.c_int64), ("logits_out", C.c_void_p), ("branch_slot", C.c_void_p)]


class SchedStatsC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("units", "draft_steps", "drafted", "accepted", "emitted")] + \
               [("wall_ms", C.c_double)]


class SchedArgsC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_branches", "gamma", "max_new", "unit_branches", "shared_len_target",
                                         "shared_len_draft")] + \
               [("temperature", C.c_float), ("first_tok", C.c_void_p), ("u_draft", C.c_void_p),
                ("u_acc", C.c_void_p), ("u_res", C.c_void_p), ("u_stride", C.c_int32),
                ("target_private_len", C.c_void_p), ("draft_private_len", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t), ("out_tok", C.c_void_p), ("out_len", C.c_void_p),
                ("stats", C.POINTER(SchedStatsC))]


EXPORTS = ("seed_verify_workspace_bytes", "seed_verify_init", "seed_verify_step", "seed_draft_step",
           "seed_accept_resample", "seed_accept_resample_static", "seed_sample_probs", "seed_uniform_philox", "seed_kv_load", "seed_verify_status",
           "seed_verify_profile_enable", "seed_verify_profile_read", "seed_verify_profile_overhead", "seed_hbm_read_probe",
           "seed_verify_destroy", "seed_last_error",
           "seed_sched_workspace_bytes", "seed_sched_run")


def library_path():
    return os.path.join(HERE, "libseed_verify.so")


def load_library():
    """Loads the HIP library; raises (never falls back) if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2406_18200_amd.build`")
    lib = C.CDLL(path)
    lib.seed_last_error.restype = C.c_char_p
    lib.seed_verify_workspace_bytes.restype = C.c_size_t
    lib.seed_verify_workspace_bytes.argtypes = [C.POINTER(ModelCfgC)]
    lib.seed_verify_init.argtypes = [C.POINTER(C.c_void_p), C.POINTER(ModelCfgC), C.POINTER(WeightsC), C.c_void_p,
                                     C.c_size_t, C.c_void_p]
    lib.seed_verify_step.argtypes = [C.c_void_p, C.POINTER(StepArgsC)]
    lib.seed_draft_step.argtypes = [C.c_void_p, C.POINTER(DraftArgsC)]
    lib.seed_accept_resample.argtypes = [C.POINTER(AcceptArgsC), C.c_void_p]
    lib.seed_accept_resample_static.argtypes = [C.POINTER(AcceptArgsC), C.c_void_p]
    lib.seed_sample_probs.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    lib.seed_uniform_philox.argtypes = [C.c_uint32, C.c_uint32, C.c_void_p, C.c_int64, C.c_void_p]
    lib.seed_kv_load.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                 C.c_int32, C.c_int32]
    lib.seed_verify_status.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
    lib.seed_verify_profile_enable.argtypes = [C.c_void_p, C.c_int32]
    lib.seed_verify_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_double),
                                             C.POINTER(C.c_double)]
    lib.seed_verify_profile_overhead.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double)]
    lib.seed_hbm_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.seed_verify_destroy.argtypes = [C.c_void_p]
    lib.seed_verify_destroy.restype = None
    lib.seed_sched_workspace_bytes.restype = C.c_size_t
    lib.seed_sched_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
    lib.seed_sched_run.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(SchedArgsC)]
    _LIB = lib
    return lib


def _check(rc):
    if rc != 0:
        raise SeedError(rc, load_library().seed_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_handle():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


@dataclass
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    dtype: str                    # "fp32" | "bf16" | "bf16w8" (projection matrices as e4m3 codes + row scales) | "bf16w4" (MXFP4 codes + block scales)
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    max_branches: int = 16
    max_rows_per_branch: int = 8
    max_shared: int = 4096
    max_private: int = 256

    def to_c(self):
        return ModelCfgC(self.n_layers, self.d_model, self.n_heads, self.head_dim, self.d_ff, self.vocab,
                         {"fp32": 0, "bf16": 1, "bf16w8": 2, "bf16w4": 3}[self.dtype], self.rms_eps, self.rope_theta, self.max_branches,
                         self.max_rows_per_branch, self.max_shared, self.max_private)


def _accept_struct(n_branches, gamma, n_target_rows, vocab, probs_kind, greedy, temperature, p_or_logits, q,
                   draft_tok, u_acc, u_res, accept_len, out_tok, n_out, p_tok, private_len, tree=None, path_node=None):
    return AcceptArgsC(n_branches, gamma, n_target_rows, vocab, probs_kind, int(greedy), float(temperature),
                       _ptr(p_or_logits), _ptr(q), _ptr(draft_tok), _ptr(u_acc), _ptr(u_res), _ptr(accept_len),
                       _ptr(out_tok), _ptr(n_out), _ptr(p_tok), _ptr(private_len), tree, _ptr(path_node))


def _accept_outputs(N, gamma, device, want_p_tok=True, n_drafts=None):
    import torch
    return (torch.empty(N, dtype=torch.int32, device=device),
            torch.empty((N, gamma + 1), dtype=torch.int32, device=device),
            torch.empty(N, dtype=torch.int32, device=device),
            torch.empty((N, gamma if n_drafts is None else n_drafts), dtype=torch.float32, device=device)
            if want_p_tok else None)


def accept_resample(p_or_logits, q, draft_tok, u_acc, u_res, *, kind="probs", temperature=1.0, greedy=False,
                    private_len=None, static_scratch=False, outs=None, k_config=None):
    """seed_accept_resample: p_or_logits float32 [N][Tp][V], q float32 [N][gamma][V], draft_tok int32
    [N][gamma], u_acc float32 [N][gamma], u_res float32 [N] (device tensors).  Returns device tensors
    (accept_len, out_tok, n_out, p_tok).  static_scratch: call seed_accept_resample_static instead (the entry
    point that allocates nothing; pass `outs`, four preallocated output tensors, to allocate nothing here either)."""
    import torch
    lib = load_library()
    N, Tp, V = p_or_logits.shape
    for t in (p_or_logits, q, draft_tok, u_acc, u_res):
        assert t is None or t.is_contiguous()
    tree, keep = _tree_struct(k_config)
    if k_config is None:
        gamma, path = draft_tok.shape[1], None
    else:
        # candidate tree: draft_tok / u_acc are [N][n_nodes - 1]; a fifth output holds the accepted nodes
        gamma = len(k_config)
        assert draft_tok.shape[1] == tree_sizes(k_config)[0] - 1
        path = torch.empty((N, gamma), dtype=torch.int32, device=p_or_logits.device)
    if outs is None:
        outs = _accept_outputs(N, gamma, p_or_logits.device, n_drafts=draft_tok.shape[1])
    a = _accept_struct(N, gamma, Tp, V, SEED_KIND_LOGITS if kind == "logits" else SEED_KIND_PROBS, greedy,
                       temperature, p_or_logits, q, draft_tok, u_acc, u_res, *outs[:4], private_len, tree, path)
    fn = lib.seed_accept_resample_static if static_scratch else lib.seed_accept_resample
    _check(fn(C.byref(a), _stream_handle()))
    del keep
    return outs if path is None else tuple(outs[:4]) + (path,)


def sample_probs(probs, u):
    """seed_sample_probs: probs float32 [n][V] (row stride = probs.stride(0)), u float32 [n] -> int32 [n]."""
    import torch
    lib = load_library()
    n, V = probs.shape
    assert probs.stride(1) == 1
    out = torch.empty(n, dtype=torch.int32, device=probs.device)
    _check(lib.seed_sample_probs(_ptr(probs), probs.stride(0), _ptr(u), _ptr(out), n, V, _stream_handle()))
    return out


def uniform_philox(seed, shape, stream=0, device="cuda:0"):
    """seed_uniform_philox: float32 uniforms on the 2^-24 grid, element i a pure function of (seed, stream, i)."""
    import torch
    lib = load_library()
    out = torch.empty(shape, dtype=torch.float32, device=device)
    _check(lib.seed_uniform_philox(int(seed) & 0xFFFFFFFF, int(stream) & 0xFFFFFFFF, _ptr(out), out.numel(), _stream_handle()))
    return out


def hbm_read_probe(buf):
    """seed_hbm_read_probe: one streaming read of the device tensor `buf` on the current stream."""
    lib = load_library()
    _check(lib.seed_hbm_read_probe(_ptr(buf), buf.numel() * buf.element_size() // 16 * 16, None, _stream_handle()))


class VerifyContext:
    """seed_verify_init / seed_verify_step / seed_draft_step / seed_kv_load on one model instance.

    `weights` is a dict: tok_emb, norm_final, lm_head (device tensors in the model dtype) and layers =
    list of dicts with wq, wk, wv, wo, wgate, wup, wdown, norm_attn, norm_ffn.  They are repacked into the
    context's workspace at construction and may be released afterwards.
    """

    def __init__(self, shape, weights, device="cuda:0"):
        import torch
        self.lib = load_library()
        self.shape = shape
        self.device = torch.device(device)
        self.cfg = shape.to_c()
        nbytes = self.lib.seed_verify_workspace_bytes(C.byref(self.cfg))
        if nbytes == 0:
            _check(-1 if not self.lib.seed_last_error() else self._cfg_error())
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        layers = (LayerWC * shape.n_layers)()
        for l, lw in enumerate(weights["layers"]):
            layers[l] = LayerWC(*[_ptr(lw.get(n)) for n in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown",
                                                              "norm_attn", "norm_ffn", "sq", "sk", "sv", "so",
                                                              "sgate", "sup", "sdown")])
        w = WeightsC(_ptr(weights["tok_emb"]), _ptr(weights["norm_final"]), _ptr(weights["lm_head"]), layers,
                     _ptr(weights.get("lm_head_scale")))
        self.handle = C.c_void_p()
        self.stream = torch.cuda.current_stream(self.device)
        _check(self.lib.seed_verify_init(C.byref(self.handle), C.byref(self.cfg), C.byref(w),
                                         _ptr(self.workspace), nbytes, C.c_void_p(self.stream.cuda_stream)))
        self.stream.synchronize()

    def _cfg_error(self):
        # re-run validation through init's path to get the precise code
        h = C.c_void_p()
        return self.lib.seed_verify_init(C.byref(h), C.byref(self.cfg), None, None, 0, None)

    def close(self):
        if getattr(self, "handle", None) and self.handle.value:
            self.lib.seed_verify_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def kv_load(self, layer, k_shared, v_shared, k_private=None, v_private=None):
        """k_shared / v_shared [H][S][dh]; k_private / v_private [N][H][R][dh] (model dtype, device)."""
        S = 0 if k_shared is None else k_shared.shape[1]
        n_b, R = (0, 0) if k_private is None else (k_private.shape[0], k_private.shape[2])
        _check(self.lib.seed_kv_load(self.handle, layer, _ptr(k_shared), _ptr(v_shared), S, _ptr(k_private),
                                     _ptr(v_private), n_b, R))

    def step(self, row_tok, shared_len, private_len=None, *, flags=0, logits_out=None, accept=None,
             branch_slot=None, k_config=None):
        """seed_verify_step.  row_tok int32 [N][T].  `accept` = dict(q, draft_tok, u_acc, u_res, temperature,
        greedy=False) -> returns (accept_len, out_tok, n_out, p_tok); otherwise returns None.  branch_slot:
        int32 [N] cache slots of the call's branches (private_len is then indexed by slot).  k_config: the rows of
        every branch are the first T nodes of that candidate tree (seed_tree); draft_tok / u_acc are then
        [N][n_nodes - 1], q is [N][n_par][V], and a fifth output holds the accepted node of every depth."""
        import torch
        N, T = row_tok.shape
        acc_c, outs = None, None
        tree, keep = _tree_struct(k_config)
        if accept is not None:
            n_drafts = accept["draft_tok"].shape[1]
            gamma = n_drafts if k_config is None else len(k_config)
            outs = _accept_outputs(N, gamma, row_tok.device, n_drafts=n_drafts)
            path = None if k_config is None else torch.empty((N, gamma), dtype=torch.int32, device=row_tok.device)
            acc_c = _accept_struct(N, gamma, T, self.shape.vocab, SEED_KIND_LOGITS, accept.get("greedy", False),
                                   accept.get("temperature", 1.0), None, accept.get("q"), accept["draft_tok"],
                                   accept.get("u_acc"), accept.get("u_res"), *outs, None, tree, path)
            if path is not None:
                outs = tuple(outs) + (path,)
        a = StepArgsC(N, T, flags, int(shared_len), _ptr(row_tok), _ptr(private_len), _ptr(logits_out),
                      C.pointer(acc_c) if acc_c is not None else None, _ptr(branch_slot), tree)
        _check(self.lib.seed_verify_step(self.handle, C.byref(a)))
        del keep
        return outs

    def prefill_shared(self, tokens, shared_len=0):
        """Appends prefix tokens (int32 device tensor [S]) to the shared KV cache in chunks; returns new length."""
        cap = self.shape.max_branches * self.shape.max_rows_per_branch
        pos = int(shared_len)
        for lo in range(0, tokens.numel(), cap):
            chunk = tokens[lo:lo + cap].contiguous().view(1, -1)
            self.step(chunk, pos, None, flags=SEED_STEP_PREFILL_SHARED)
            pos += chunk.shape[1]
        return pos

    def draft_step(self, row_tok, shared_len, private_len, u, temperature, *, q_out=None, tok_out=None,
                   q_stride=None, tok_stride=1, flags=0, logits_out=None, branch_slot=None):
        """seed_draft_step: one autoregressive token per branch.  q_out / tok_out may be views into
        q[N][gamma][V] / draft_tok[N][gamma] columns (pass the strides of the branch dimension)."""
        import torch
        N = row_tok.numel()
        if tok_out is None:
            tok_out = torch.empty(N, dtype=torch.int32, device=row_tok.device)
        if q_out is not None and q_stride is None:
            q_stride = q_out.stride(0)
        a = DraftArgsC(N, flags, int(shared_len), float(temperature), _ptr(row_tok), _ptr(private_len), _ptr(u),
                       _ptr(q_out), int(q_stride or 0), _ptr(tok_out), int(tok_stride), _ptr(logits_out),
                       _ptr(branch_slot))
        _check(self.lib.seed_draft_step(self.handle, C.byref(a)))
        return tok_out

    def profile_enable(self, on):
        _check(self.lib.seed_verify_profile_enable(self.handle, int(bool(on))))

    def profile_read(self):
        """(launches, total milliseconds, weight bytes) of the projection launches since the last read."""
        n, ms, by = C.c_int64(0), C.c_double(0), C.c_double(0)
        _check(self.lib.seed_verify_profile_read(self.handle, C.byref(n), C.byref(ms), C.byref(by)))
        return n.value, ms.value, by.value

    def profile_overhead(self, n_pairs=200):
        """seed_verify_profile_overhead: milliseconds a pair of timing events adds around a launch."""
        ms = C.c_double(0)
        _check(self.lib.seed_verify_profile_overhead(self.handle, int(n_pairs), C.byref(ms)))
        return ms.value

    def status(self):
        s = C.c_int32(0)
        _check(self.lib.seed_verify_status(self.handle, C.byref(s)))
        return s.value


def sched_run(target, draft, first_tok, u_draft, u_acc, u_res, target_private_len, draft_private_len, *, gamma,
              max_new, temperature, shared_len_target, shared_len_draft, unit_branches=0):
    """seed_sched_run: Algorithm 1 over a target and a draft VerifyContext (create them on two different
    torch streams for overlap).  first_tok: int sequence [n] (host); u_*: float32 device tensors [n][stride];
    *_private_len: int32 device tensors over the contexts' slots.  Returns (tokens int32 numpy [n][max_new],
    lengths [n], stats dict)."""
    import numpy as np
    import torch
    lib = load_library()
    n = len(first_tok)
    V = target.shape.vocab
    nbytes = lib.seed_sched_workspace_bytes(n, int(gamma), V)
    if nbytes == 0:
        raise SeedError(-1, "seed_sched_workspace_bytes: invalid n_branches / gamma / vocab")
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=u_draft.device)
    base = (ws.data_ptr() + 255) // 256 * 256
    first = np.ascontiguousarray(first_tok, dtype=np.int32)
    out_tok = np.full((n, max_new), -1, np.int32)
    out_len = np.zeros(n, np.int32)
    stats = SchedStatsC()
    a = SchedArgsC(n, int(gamma), int(max_new), int(unit_branches), int(shared_len_target), int(shared_len_draft),
                   float(temperature), first.ctypes.data, _ptr(u_draft), _ptr(u_acc), _ptr(u_res),
                   int(u_draft.stride(0)), _ptr(target_private_len), _ptr(draft_private_len), C.c_void_p(base),
                   nbytes, out_tok.ctypes.data, out_len.ctypes.data, C.pointer(stats))
    torch.cuda.synchronize()
    _check(lib.seed_sched_run(target.handle, draft.handle, C.byref(a)))
    return out_tok, out_len, {f: getattr(stats, f) for f, _ in SchedStatsC._fields_}
