"""ctypes binding of libposs.so: argument marshalling only.

Same names as include/poss.h.  PyTorch appears only as the owner of device
memory (weights, workspace, optional output buffers) and of the stream.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libposs.so")

POSS_OK, E_INVALID_ARG, E_BAD_STATE, E_CAPACITY, E_BAD_TREE, E_HIP = 0, -1, -2, -3, -4, -5
MAX_ROWS, MASK_WORDS, MAX_DEPTH = 128, 2, 16

EXPORTS = ["poss_workspace_bytes", "poss_load", "poss_reset", "poss_prefill", "poss_draft_tree",
           "poss_verify_tree", "poss_accept_and_commit", "poss_get_stats", "poss_get_tokens",
           "poss_prefill_seq", "poss_get_tree_seq", "poss_get_commit_seq", "poss_get_tokens_seq", "poss_set_uniforms_seq", "poss_reset_seq", "poss_set_active",
           "poss_last_error", "poss_free", "poss_profile_gemm", "poss_gemm_profile", "poss_set_tuning", "poss_set_launch_rows", "poss_set_sampling", "poss_set_draft_sampling",
           "poss_debug_build_tree", "poss_debug_set_taps", "poss_debug_read_kv", "poss_debug_draft_logits",
           "poss_debug_gemm_scratch_bytes", "poss_debug_gemm", "poss_gemm_static"]

c_i32, c_f32, c_vp = ctypes.c_int32, ctypes.c_float, ctypes.c_void_p


class PossConfig(ctypes.Structure):
    _fields_ = [(n, c_i32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rms_eps", c_f32), ("rope_theta", c_f32), ("dtype", c_i32)] + \
               [(n, c_i32) for n in ("n_specialists", "positions_per_specialist", "fc_bias", "top_k", "depth",
                                     "total_tokens", "max_seq", "kv_page_tokens", "kv_page_order", "batch")]


class PossWeights(ctypes.Structure):
    _fields_ = [("embed", c_vp), ("lm_head", c_vp), ("final_norm", c_vp),
                ("layer", ctypes.POINTER(c_vp)), ("spec", ctypes.POINTER(c_vp))]


class PossTree(ctypes.Structure):
    _fields_ = [("n_nodes", c_i32), ("token", ctypes.POINTER(c_i32)), ("parent", ctypes.POINTER(c_i32)),
                ("depth", ctypes.POINTER(c_i32)), ("pos", ctypes.POINTER(c_i32)),
                ("mask", ctypes.POINTER(ctypes.c_uint64)), ("score", ctypes.POINTER(c_f32))]


class PossStats(ctypes.Structure):
    _fields_ = [("rounds", ctypes.c_int64), ("committed_tokens", ctypes.c_int64),
                ("c", ctypes.c_int64 * (MAX_DEPTH + 1)),
                ("ms_draft", ctypes.c_double), ("ms_verify", ctypes.c_double), ("ms_commit", ctypes.c_double)]


class PossError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("poss error %d: %s" % (code, msg))
        self.code = code


_lib = None


def load_library():
    """dlopen libposs.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libposs.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER
    lib.poss_workspace_bytes.restype = ctypes.c_size_t
    lib.poss_workspace_bytes.argtypes = [P(PossConfig)]
    lib.poss_load.argtypes = [P(PossConfig), P(PossWeights), c_vp, ctypes.c_size_t, c_vp, P(c_vp)]
    lib.poss_reset.argtypes = [c_vp]
    lib.poss_reset_seq.argtypes = [c_vp, c_i32]
    lib.poss_set_active.argtypes = [c_vp, c_i32, c_i32]
    lib.poss_prefill.argtypes = [c_vp, P(c_i32), c_i32, P(c_i32)]
    lib.poss_draft_tree.argtypes = [c_vp, P(PossTree)]
    lib.poss_verify_tree.argtypes = [c_vp, P(PossTree), P(c_i32), c_vp, c_vp]
    lib.poss_accept_and_commit.argtypes = [c_vp, P(c_i32), P(c_i32), P(c_i32), P(c_i32)]
    lib.poss_get_stats.argtypes = [c_vp, P(PossStats)]
    lib.poss_get_tokens.argtypes = [c_vp, P(c_i32), c_i32, P(c_i32)]
    lib.poss_prefill_seq.argtypes = [c_vp, c_i32, P(c_i32), c_i32, P(c_i32)]
    lib.poss_get_tree_seq.argtypes = [c_vp, c_i32, P(PossTree)]
    lib.poss_get_commit_seq.argtypes = [c_vp, c_i32, P(c_i32), P(c_i32), P(c_i32), P(c_i32)]
    lib.poss_get_tokens_seq.argtypes = [c_vp, c_i32, P(c_i32), c_i32, P(c_i32)]
    lib.poss_last_error.restype = ctypes.c_char_p
    lib.poss_last_error.argtypes = [c_vp]
    lib.poss_free.restype = None
    lib.poss_free.argtypes = [c_vp]
    lib.poss_profile_gemm.argtypes = [c_vp, c_i32]
    lib.poss_gemm_profile.argtypes = [c_vp, P(ctypes.c_int64), P(ctypes.c_double), P(ctypes.c_double)]
    lib.poss_set_tuning.argtypes = [c_vp, c_i32, c_i32]
    lib.poss_set_launch_rows.argtypes = [c_vp, c_i32]
    lib.poss_set_sampling.argtypes = [c_vp, c_f32, ctypes.POINTER(c_f32), c_i32]
    lib.poss_set_uniforms_seq.argtypes = [c_vp, c_i32, ctypes.POINTER(c_f32), c_i32]
    lib.poss_set_draft_sampling.argtypes = [c_vp, c_i32, ctypes.POINTER(c_f32), ctypes.POINTER(c_f32)]
    lib.poss_debug_build_tree.argtypes = [c_vp, P(c_i32), P(c_f32), P(PossTree)]
    lib.poss_debug_set_taps.argtypes = [c_vp, c_vp]
    lib.poss_debug_draft_logits.argtypes = [c_vp, c_i32, c_i32, c_vp]
    lib.poss_debug_read_kv.argtypes = [c_vp, c_i32, c_i32, c_i32, c_i32, P(c_f32), P(c_f32)]
    lib.poss_debug_gemm_scratch_bytes.restype = ctypes.c_size_t
    lib.poss_debug_gemm_scratch_bytes.argtypes = [c_i32, c_i32, c_i32, c_i32]
    lib.poss_debug_gemm.argtypes = [c_i32, c_vp, c_vp, c_vp, c_i32, c_i32, c_i32, c_i32, c_vp, c_vp, c_i32, P(c_f32)]
    lib.poss_gemm_static.argtypes = [c_i32, c_vp, c_vp, c_vp, c_i32, c_i32, c_i32, c_i32, c_vp]
    _lib = lib
    return lib


def make_config(cfg, **over):
    """PossConfig from any object with the fields of include/poss.h (e.g. synth.ModelConfig)."""
    c = PossConfig()
    for name, _ in PossConfig._fields_:
        v = over.get(name, getattr(cfg, name, 0))
        setattr(c, name, v)
    return c


def _iptr(a):
    return a.ctypes.data_as(ctypes.POINTER(c_i32))


class TreeArrays:
    """Host arrays of a poss_tree (capacity rows)."""

    def __init__(self, capacity=MAX_ROWS):
        self.token = np.zeros(capacity, np.int32)
        self.parent = np.zeros(capacity, np.int32)
        self.depth = np.zeros(capacity, np.int32)
        self.pos = np.zeros(capacity, np.int32)
        self.mask = np.zeros((capacity, MASK_WORDS), np.uint64)
        self.score = np.zeros(capacity, np.float32)
        self.c = PossTree(0, _iptr(self.token), _iptr(self.parent), _iptr(self.depth), _iptr(self.pos),
                          self.mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                          self.score.ctypes.data_as(ctypes.POINTER(c_f32)))

    @classmethod
    def from_lists(cls, token, parent):
        tr = cls(max(len(token), 1))
        tr.c.n_nodes = len(token)
        tr.token[:len(token)] = token
        tr.parent[:len(parent)] = parent
        return tr

    @property
    def n(self):
        return int(self.c.n_nodes)

    def as_dict(self):
        n = self.n
        return dict(n=n, token=self.token[:n].tolist(), parent=self.parent[:n].tolist(),
                    depth=self.depth[:n].tolist(), pos=self.pos[:n].tolist(),
                    mask=[int(self.mask[i, 0]) | (int(self.mask[i, 1]) << 64) for i in range(n)],
                    score=self.score[:n].copy())


class Poss:
    """One context.  `weights`: dict name -> torch tensor on the GPU (names of synth.tensor_specs);
    the workspace is a torch uint8 tensor this object keeps alive."""

    def __init__(self, cfg, weights, stream=None, **over):
        import torch
        self.lib = load_library()
        self.cfg = cfg
        self.c_cfg = make_config(cfg, **over)
        need = self.lib.poss_workspace_bytes(ctypes.byref(self.c_cfg))
        if need == 0:
            raise PossError(E_INVALID_ARG, "configuration rejected by poss_workspace_bytes")
        self.workspace = torch.empty(need, dtype=torch.uint8, device="cuda")
        names = ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")
        lay = (c_vp * (cfg.n_layers * 9))(*[weights[f"layer{l}.{n}"].data_ptr()
                                           for l in range(cfg.n_layers) for n in names])
        sp = (c_vp * (cfg.n_specialists * 11))(*[weights[f"spec{s}.{n}"].data_ptr()
                                               for s in range(cfg.n_specialists)
                                               for n in ("fc_w", "fc_b") + names])
        w = PossWeights(weights["embed"].data_ptr(), weights["lm_head"].data_ptr(),
                        weights["final_norm"].data_ptr(), lay, sp)
        self._keep = (lay, sp, w)
        self.stream = stream
        sh = c_vp(stream.cuda_stream) if stream is not None else c_vp(0)
        h = c_vp()
        rc = self.lib.poss_load(ctypes.byref(self.c_cfg), ctypes.byref(w), c_vp(self.workspace.data_ptr()),
                                need, sh, ctypes.byref(h))
        if rc != POSS_OK:
            raise PossError(rc, self.lib.poss_last_error(None).decode())
        self.h = h
        self.workspace_bytes = need

    # -- helpers
    def _check(self, rc):
        if rc != POSS_OK:
            raise PossError(rc, self.lib.poss_last_error(self.h).decode())

    def close(self):
        if getattr(self, "h", None):
            self.lib.poss_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the five calls
    def reset(self, seq=None):
        """Forget every sequence (and the statistics), or one sequence of a batch."""
        self._check(self.lib.poss_reset(self.h) if seq is None else self.lib.poss_reset_seq(self.h, seq))

    def set_active(self, seq, active):
        """Set a sequence of a batch aside (False) or take it back into the rounds (True)."""
        self._check(self.lib.poss_set_active(self.h, seq, 1 if active else 0))

    def prefill(self, prompt, seq=0):
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        first = c_i32()
        self._check(self.lib.poss_prefill_seq(self.h, seq, _iptr(p), len(p), ctypes.byref(first)))
        return int(first.value)

    def get_tree(self, seq):
        tr = TreeArrays()
        self._check(self.lib.poss_get_tree_seq(self.h, seq, ctypes.byref(tr.c)))
        return tr

    def commit_result(self, seq):
        """(path, n_accepted, committed tokens) of the last accept_and_commit for one sequence of the batch."""
        path = np.zeros(MAX_DEPTH + 1, np.int32)
        toks = np.zeros(MAX_DEPTH + 1, np.int32)
        m, nc = c_i32(), c_i32()
        self._check(self.lib.poss_get_commit_seq(self.h, seq, _iptr(path), ctypes.byref(m), _iptr(toks), ctypes.byref(nc)))
        return path[:m.value + 1].tolist(), int(m.value), toks[:nc.value].tolist()

    def draft_tree(self, want_tree=True):
        tr = TreeArrays() if want_tree else None
        self._check(self.lib.poss_draft_tree(self.h, ctypes.byref(tr.c) if tr else None))
        return tr

    def verify_tree(self, tree=None, logits_out=None, feat_out=None, want_argmax=True):
        """tree: None (the drafted trees), one TreeArrays (batch 1) or a list with one TreeArrays per sequence."""
        g = np.zeros(MAX_ROWS, np.int32) if want_argmax else None
        batch = max(1, int(self.c_cfg.batch))
        if tree is None:
            tp = None
        else:
            trees = list(tree) if isinstance(tree, (list, tuple)) else [tree]
            if len(trees) != batch:
                raise ValueError("verify_tree needs one tree per sequence (%d), got %d" % (batch, len(trees)))
            arr = (PossTree * batch)(*[t.c for t in trees])
            self._keep_trees = (arr, trees)
            tp = ctypes.cast(arr, ctypes.POINTER(PossTree))
        self._check(self.lib.poss_verify_tree(
            self.h, tp, _iptr(g) if g is not None else None,
            c_vp(logits_out.data_ptr()) if logits_out is not None else None,
            c_vp(feat_out.data_ptr()) if feat_out is not None else None))
        return g

    def accept_and_commit(self):
        path = np.zeros(MAX_DEPTH + 1, np.int32)
        toks = np.zeros(MAX_DEPTH + 1, np.int32)
        m, nc = c_i32(), c_i32()
        self._check(self.lib.poss_accept_and_commit(self.h, _iptr(path), ctypes.byref(m), _iptr(toks),
                                                    ctypes.byref(nc)))
        return path[:m.value + 1].tolist(), int(m.value), toks[:nc.value].tolist()

    # -- the rest
    def stats(self):
        s = PossStats()
        self._check(self.lib.poss_get_stats(self.h, ctypes.byref(s)))
        return s

    def tokens(self, seq=0):
        n = c_i32()
        self._check(self.lib.poss_get_tokens_seq(self.h, seq, None, 0, ctypes.byref(n)))
        out = np.zeros(n.value, np.int32)
        self._check(self.lib.poss_get_tokens_seq(self.h, seq, _iptr(out), n.value, ctypes.byref(n)))
        return out.tolist()

    def profile_gemm(self, enable):
        self._check(self.lib.poss_profile_gemm(self.h, 1 if enable else 0))

    def gemm_profile(self):
        n, ms, b = ctypes.c_int64(), ctypes.c_double(), ctypes.c_double()
        self._check(self.lib.poss_gemm_profile(self.h, ctypes.byref(n), ctypes.byref(ms), ctypes.byref(b)))
        return int(n.value), float(ms.value), float(b.value)

    def set_sampling(self, temperature, u=None):
        """temperature 0: greedy verification.  Otherwise u = one uniform number in [0, 1) per tree depth."""
        if u is None:
            self._check(self.lib.poss_set_sampling(self.h, float(temperature), None, 0))
            return
        u = np.ascontiguousarray(u, dtype=np.float32)
        self._check(self.lib.poss_set_sampling(self.h, float(temperature), u.ctypes.data_as(ctypes.POINTER(c_f32)), len(u)))

    def set_draft_sampling(self, u_draft=None, u_accept=None):
        """Drawn children and the rejection rule (needs a temperature from set_sampling).  u_draft [depth][k][k], u_accept
        [depth + 1][k + 1], all in [0, 1); both None: back to the deterministic tree."""
        if u_draft is None:
            self._check(self.lib.poss_set_draft_sampling(self.h, 0, None, None))
            return
        cfg = self.cfg
        ud = np.ascontiguousarray(u_draft, dtype=np.float32).reshape(cfg.depth, cfg.top_k, cfg.top_k)
        ua = np.ascontiguousarray(u_accept, dtype=np.float32).reshape(cfg.depth + 1, cfg.top_k + 1)
        fp = ctypes.POINTER(c_f32)
        self._check(self.lib.poss_set_draft_sampling(self.h, 1, ud.ctypes.data_as(fp), ua.ctypes.data_as(fp)))

    def set_uniforms(self, seq, u):
        """Uniform numbers of one sequence of a batch (set_sampling gives all sequences the same ones)."""
        u = np.ascontiguousarray(u, dtype=np.float32)
        self._check(self.lib.poss_set_uniforms_seq(self.h, seq, u.ctypes.data_as(ctypes.POINTER(c_f32)), len(u)))

    def set_tuning(self, gemm_target_workgroups=0, attn_keys_per_split=0):
        self._check(self.lib.poss_set_tuning(self.h, gemm_target_workgroups, attn_keys_per_split))

    def set_launch_rows(self, rows):
        """Rows one launch of a batch's pass carries at most (128..256)."""
        self._check(self.lib.poss_set_launch_rows(self.h, rows))

    def debug_build_tree(self, ids, logp):
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        logp = np.ascontiguousarray(logp, dtype=np.float32)
        tr = TreeArrays()
        self._check(self.lib.poss_debug_build_tree(self.h, _iptr(ids), logp.ctypes.data_as(ctypes.POINTER(c_f32)),
                                                   ctypes.byref(tr.c)))
        return tr

    def debug_set_taps(self, taps):
        self._check(self.lib.poss_debug_set_taps(self.h, c_vp(taps.data_ptr()) if taps is not None else None))

    def debug_draft_logits(self, row0, n):
        """Drafter logits of expanded nodes row0 .. row0+n-1 of a tree drafted with drawn children: GPU tensor [n, vocab]."""
        import torch
        out = torch.empty(n, self.cfg.vocab, dtype=torch.float32, device="cuda")
        self._check(self.lib.poss_debug_draft_logits(self.h, row0, n, c_vp(out.data_ptr())))
        return out

    def debug_read_kv(self, which, layer, slot0, n):
        cfg = self.cfg
        k = np.zeros((n, cfg.n_kv_heads, cfg.head_dim), np.float32)
        v = np.zeros_like(k)
        fp = ctypes.POINTER(c_f32)
        self._check(self.lib.poss_debug_read_kv(self.h, which, layer, slot0, n, k.ctypes.data_as(fp), v.ctypes.data_as(fp)))
        return k, v


def debug_gemm(dtype, x, w, target_workgroups=0, repeats=1, stream=None):
    """Y = X W^T through the library's GEMM path; x [M,K], w [N,K] torch GPU tensors of `dtype`."""
    import torch
    lib = load_library()
    M, K = x.shape
    N = w.shape[0]
    nb = lib.poss_debug_gemm_scratch_bytes(dtype, M, N, K)
    if nb == 0:
        raise PossError(E_INVALID_ARG, "shape rejected")
    scratch = torch.empty(nb, dtype=torch.uint8, device="cuda")
    y = torch.empty(M, N, dtype=torch.float32, device="cuda")
    ms = c_f32()
    rc = lib.poss_debug_gemm(dtype, c_vp(x.data_ptr()), c_vp(w.data_ptr()), c_vp(y.data_ptr()), M, N, K,
                             target_workgroups, c_vp(scratch.data_ptr()),
                             c_vp(stream.cuda_stream) if stream is not None else c_vp(0), repeats, ctypes.byref(ms))
    if rc != POSS_OK:
        raise PossError(rc, lib.poss_last_error(None).decode())
    return y, float(ms.value)


GEMM_STATIC_BYTES = 32 << 20


def gemm_static(dtype, x, w, y, target_workgroups=0, stream=None):
    """Y = X W^T with the library's own static scratch array: allocates nothing, enqueues and returns.
    x [M,K], w [N,K] torch GPU tensors of `dtype`; y [M,N] float32 GPU tensor the caller allocated."""
    lib = load_library()
    M, K = x.shape
    N = w.shape[0]
    rc = lib.poss_gemm_static(dtype, c_vp(x.data_ptr()), c_vp(w.data_ptr()), c_vp(y.data_ptr()), M, N, K,
                              target_workgroups, c_vp(stream.cuda_stream) if stream is not None else c_vp(0))
    if rc != POSS_OK:
        raise PossError(rc, lib.poss_last_error(None).decode())
