"""ctypes binding of libchimera.so: the same names as include/chimera.h,
argument marshalling only.  Device memory and streams come from PyTorch-ROCm;
every computation runs inside the library."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libchimera.so")

OK, EINVAL, ENOMEM, ESTATE, EDEVICE = 0, -1, -2, -3, -4
F32, BF16 = 0, 1
DIRECT, GPIPE, ONE_F_ONE_B, DOUBLING, HALVING = 0, 1, 2, 3, 4
OP_F, OP_B, OP_F2, OP_BH0, OP_BH1 = 0, 1, 2, 3, 4
OPT_CAUSAL, OPT_GELU, OPT_KERNELS, OPT_OVERLAP, OPT_KEEP = 0, 1, 2, 3, 4
EPI_NONE, EPI_BIAS, EPI_BIAS_GELU, EPI_BIAS_RESIDUAL, EPI_DGELU, EPI_ACCUM_F32 = range(6)


class ChimeraError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("chimera error %d: %s" % (code, text))
        self.code = code


class chimera_op(C.Structure):
    _fields_ = [("kind", C.c_int32), ("pipe", C.c_int32), ("mb", C.c_int32), ("stage", C.c_int32),
                ("slot", C.c_int32), ("start", C.c_int32), ("last_of_stage", C.c_int32)]

    def astuple(self):
        return (self.kind, self.pipe, self.mb, self.stage)


_p, _i, _sz = C.c_void_p, C.c_int, C.c_size_t
_SIGNATURES = {
    "chimera_last_error": (C.c_char_p, []),
    "chimera_schedule": (_i, [_i, _i, _i, _i, C.POINTER(chimera_op), _sz, C.POINTER(_sz)]),
    "chimera_schedule_stats": (_i, [_i, _i, _i, _i, _i, C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                    C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "chimera_schedule_pipes": (_i, [_i, _i, _i, _i, _i, C.POINTER(chimera_op), _sz, C.POINTER(_sz)]),
    "chimera_schedule_stats_costs": (_i, [_i, _i, _i, _i, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                          C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "chimera_pipe_worker": (_i, [_i, _i, _i, _i]),
    "chimera_model_iteration_time": (_i, [_i, _i, _i, _i, _i] + [C.c_double] * 6 + [_i, C.POINTER(C.c_double)]),
    "chimera_stage_create": (_p, [_i] * 6),
    "chimera_stage_set_option": (_i, [_p, _i, _i]),
    "chimera_stage_destroy": (None, [_p]),
    "chimera_stage_weight_bytes": (_sz, [_p]),
    "chimera_stage_grad_bytes": (_sz, [_p]),
    "chimera_stage_stash_slot_bytes": (_sz, [_p]),
    "chimera_stage_workspace_bytes": (_sz, [_p]),
    "chimera_stage_bind": (_i, [_p, _p, _p, _p, _i, _p, _p]),
    "chimera_stage_set_io": (_i, [_p, _i, _p, _p, _p, _p]),
    "chimera_fwd": (_i, [_p, _i]),
    "chimera_fwd_slot": (_i, [_p, _i, _i]),
    "chimera_bwd": (_i, [_p, _i]),
    "chimera_bwd_half": (_i, [_p, _i, _i]),
    "chimera_worker_bind_pipes": (_i, [_p, _i]),
    "chimera_worker_bind_doubling": (_i, [_p, _p]),
    "chimera_run_worker_pipes": (_i, [_i, _i, _i, _i, _i]),
    "chimera_stage_in_flight": (_i, [_p]),
    "chimera_stage_zero_grads": (_i, [_p]),
    "chimera_stage_read_grads": (_i, [_p, _p, _sz]),
    "chimera_worker_bind": (_i, [_p, _p]),
    "chimera_run_worker": (_i, [_i, _i, _i]),
    "chimera_run_worker_algo": (_i, [_i, _i, _i, _i]),
    "chimera_worker_set_timing": (_i, [_i]),
    "chimera_worker_last_timing": (_i, [C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(_i), C.POINTER(_i)]),
    "chimera_profile_enable": (_i, [_i]),
    "chimera_profile_reset": (_i, []),
    "chimera_profile_read": (_i, [_i, C.POINTER(C.c_double), C.POINTER(C.c_longlong), C.POINTER(C.c_double)]),
    "chimera_model_select": (_i, [_i, _i, C.c_int64, C.c_double, C.c_double, C.c_double, _i, _i, _p, _p, _p]),
    "chimera_worker_last_enqueue_ms": (_i, [_p]),
    "chimera_op_gemm_workspace_bytes": (_sz, [_i, _i, _i]),
    "chimera_op_gemm_tuning": (_i, [_i, _i, _i, _i]),
    "chimera_op_gemm_group_last_kernel": (C.c_char_p, []),
    "chimera_op_gemm": (_i, [_i] * 7 + [_p, _i, _i, _p, _i, _i, _p, _p, _p, _p, _p, _sz, _p]),
    "chimera_op_gemm_group_accumulate": (_i, [_i, _p, _p, _i, _p, _p, _p, _p, _p, _p, _i, _p]),
    "chimera_op_layernorm_fwd": (_i, [_i, _i, _i, _p, _p, _p, _p, _p, _p, _p]),
    "chimera_op_layernorm_bwd_scratch_floats": (_sz, [_i, _i]),
    "chimera_op_layernorm_bwd": (_i, [_i, _i, _i] + [_p] * 11),
    "chimera_op_layernorm_bwd_noalloc_max_scratch_floats": (_sz, []),
    "chimera_op_layernorm_bwd_noalloc": (_i, [_i, _i, _i] + [_p] * 10),
    "chimera_op_colsum_scratch_floats": (_sz, [_i, _i]),
    "chimera_op_colsum": (_i, [_i, _i, _i, _p, _p, _p, _p]),
    "chimera_op_attention_fwd": (_i, [_i] * 7 + [_p, _p, _p, _p]),
    "chimera_op_attention_bwd": (_i, [_i] * 7 + [_p] * 7),
    "chimera_op_embedding_fwd": (_i, [_i] * 5 + [_p, _p, _p, _p, _p]),
    "chimera_op_embedding_bwd": (_i, [_i] * 5 + [_p, _p, _p, _p, _p]),
    "chimera_op_softmax_xent": (_i, [_i, _i, _i, _p, _p, C.c_float, _p, _p, _p]),
    "chimera_head_workspace_bytes": (_sz, [_i, _i, _i, _i]),
    "chimera_head_loss": (_i, [_i] * 4 + [_p] * 5 + [C.c_float] + [_p] * 6 + [_sz, _p]),
    "chimera_probe_mfma_bf16": (_i, [_p, _i, C.POINTER(C.c_double), _p]),
    "chimera_probe_copy": (_i, [_p, _p, _sz, C.POINTER(C.c_double), _p]),
}

_lib = None


def lib():
    """The loaded library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -m paper_2107_06925_amd.build` "
                              "(there is no CPU fallback)" % LIB_PATH)
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def last_error():
    return lib().chimera_last_error().decode()


def check(code):
    if code != OK:
        raise ChimeraError(code, last_error())
    return code


# ------------------------------------------------------------------ schedule
def chimera_schedule(algo, D, N, rank):
    n = _sz(0)
    cap = 3 * max(N, 1)            # backward halving lists three ops per micro-batch
    buf = (chimera_op * cap)()
    check(lib().chimera_schedule(algo, D, N, rank, buf, cap, C.byref(n)))
    return list(buf[:n.value])


def chimera_schedule_pipes(algo, D, N, f, rank):
    n = _sz(0)
    cap = 3 * max(N, 1)
    buf = (chimera_op * cap)()
    check(lib().chimera_schedule_pipes(algo, D, N, f, rank, buf, cap, C.byref(n)))
    return list(buf[:n.value])


def chimera_schedule_stats_costs(algo, D, N, f, costs):
    """costs: one integer per op kind (F, B, F2, BH0, BH1)."""
    mk = C.c_int64(0)
    bub = (C.c_int64 * max(D, 1))()
    peak = (C.c_int32 * max(D, 1))()
    crit = (C.c_int32 * 2)()
    check(lib().chimera_schedule_stats_costs(algo, D, N, f, (C.c_int64 * 5)(*costs), C.byref(mk), bub, peak, crit))
    return {"makespan": mk.value, "bubbles": list(bub[:D]), "stash_peak_halves": list(peak[:D]), "critical": (crit[0], crit[1])}


def chimera_pipe_worker(D, f, pipe, stage):
    w = lib().chimera_pipe_worker(D, f, pipe, stage)
    if w < 0:
        check(w)
    return w


def chimera_model_iteration_time(algo, D, N, f, W, f_t, b_t, alpha, beta, act_words, grad_words, eager=True):
    out = (C.c_double * 7)()
    check(lib().chimera_model_iteration_time(algo, D, N, f, W, f_t, b_t, alpha, beta, act_words, grad_words, int(eager), out))
    return {"T": out[0], "compute": out[1], "p2p": out[2], "allreduce": out[3], "unoverlapped": out[4],
            "c_f": int(out[5]), "c_b": int(out[6])}


class Candidate(C.Structure):
    _fields_ = [("D", C.c_int32), ("W", C.c_int32), ("B", C.c_int32), ("recompute", C.c_int32), ("f_t", C.c_double),
                ("b_t", C.c_double), ("act_words", C.c_double), ("grad_words", C.c_double), ("weight_bytes", C.c_double),
                ("act_bytes", C.c_double)]


class CandidateEval(C.Structure):
    _fields_ = [("valid", C.c_int32), ("N", C.c_int32), ("fits", C.c_int32), ("chosen", C.c_int32), ("c_f", C.c_int32),
                ("c_b", C.c_int32), ("mem_bytes", C.c_double), ("T", C.c_double), ("throughput", C.c_double)]


def chimera_model_select(algo, f, minibatch, capacity_bytes, alpha, beta, candidates, eager=True):
    """candidates: dicts with the fields of chimera_candidate (b_t None or <= 0: modelled).
    Returns (list of evaluation dicts, None for an invalid candidate; best index or None)."""
    n = len(candidates)
    arr = (Candidate * max(n, 1))()
    for a, c in zip(arr, candidates):
        a.D, a.W, a.B, a.recompute = c["D"], c["W"], c["B"], int(bool(c.get("recompute", False)))
        a.f_t, a.b_t = c["f_t"], (c.get("b_t") or 0.0)
        a.act_words, a.grad_words, a.weight_bytes, a.act_bytes = c["act_words"], c["grad_words"], c["weight_bytes"], c["act_bytes"]
    ev = (CandidateEval * max(n, 1))()
    best = C.c_int(-1)
    check(lib().chimera_model_select(algo, f, minibatch, capacity_bytes, alpha, beta, int(eager), n, arr, ev, C.byref(best)))
    out = [None if not e.valid else dict(N=e.N, mem_bytes=e.mem_bytes, fits=bool(e.fits), chosen=bool(e.chosen), T=e.T,
                                          throughput=e.throughput, c_f=e.c_f, c_b=e.c_b) for e in ev[:n]]
    return out, (None if best.value < 0 else best.value)


def chimera_schedule_stats(algo, D, N, cost_f=1, cost_b=1):
    mk = C.c_int64(0)
    bub = (C.c_int64 * max(D, 1))()
    peak = (C.c_int32 * max(D, 1))()
    crit = (C.c_int32 * 2)()
    check(lib().chimera_schedule_stats(algo, D, N, cost_f, cost_b, C.byref(mk), bub, peak, crit))
    return dict(makespan=mk.value, bubbles=list(bub), stash_peak=list(peak), critical=(crit[0], crit[1]))


# --------------------------------------------------------------------- stage
def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Stage:
    """Owns the device buffers (torch tensors) a chimera_stage borrows."""

    def __init__(self, layers, hidden, heads, seq, microbatch, dtype, causal=True, gelu_erf=False,
                 reference_kernels=False, stash_slots=1, stream=None, device="cuda:0", overlap=True, keep=True,
                 share_weights_of=None):
        """keep=False: forward-only stage (activation recomputation).  share_weights_of: another
        Stage whose weight and gradient buffers this one binds to instead of owning its own."""
        import torch
        self.torch = torch
        self.handle = lib().chimera_stage_create(layers, hidden, heads, seq, microbatch, dtype)
        if not self.handle:
            raise ChimeraError(EINVAL, last_error())
        self.layers, self.hidden, self.heads, self.seq, self.microbatch, self.dtype = layers, hidden, heads, seq, microbatch, dtype
        check(lib().chimera_stage_set_option(self.handle, OPT_CAUSAL, int(bool(causal))))
        check(lib().chimera_stage_set_option(self.handle, OPT_GELU, int(bool(gelu_erf))))
        check(lib().chimera_stage_set_option(self.handle, OPT_KERNELS, int(bool(reference_kernels))))
        check(lib().chimera_stage_set_option(self.handle, OPT_OVERLAP, int(bool(overlap))))
        check(lib().chimera_stage_set_option(self.handle, OPT_KEEP, int(bool(keep))))
        self.tdtype = torch.float32 if dtype == F32 else torch.bfloat16
        esz = 4 if dtype == F32 else 2
        L = lib()
        dev = torch.device(device)
        self.device = dev
        if share_weights_of is not None:
            self.weights, self.grads = share_weights_of.weights, share_weights_of.grads
            assert self.weights.numel() == L.chimera_stage_weight_bytes(self.handle) // esz
        else:
            self.weights = torch.empty(L.chimera_stage_weight_bytes(self.handle) // esz, dtype=self.tdtype, device=dev)
            self.grads = torch.zeros(L.chimera_stage_grad_bytes(self.handle) // 4, dtype=torch.float32, device=dev)
        self.slot_bytes = L.chimera_stage_stash_slot_bytes(self.handle)
        self.stash = torch.empty(self.slot_bytes * stash_slots, dtype=torch.uint8, device=dev)
        self.workspace = torch.empty(L.chimera_stage_workspace_bytes(self.handle), dtype=torch.uint8, device=dev)
        self.stash_slots = stash_slots
        self.stream = stream if stream is not None else torch.cuda.current_stream(dev)
        check(L.chimera_stage_bind(self.handle, _ptr(self.weights), _ptr(self.grads), _ptr(self.stash), stash_slots,
                                   _ptr(self.workspace), C.c_void_p(self.stream.cuda_stream)))
        self.io = {}

    def set_weights(self, flat_f32):
        """flat_f32: numpy float32 vector in the flat parameter order."""
        t = self.torch.from_numpy(flat_f32).to(self.device).to(self.tdtype)
        assert t.numel() == self.weights.numel(), (t.numel(), self.weights.numel())
        self.weights.copy_(t)

    def set_io(self, mb, x, dy):
        """x, dy: torch tensors [M, H] of the stage dtype on the device; allocates y and dx."""
        y = self.torch.empty_like(x)
        dx = self.torch.empty_like(x)
        self.io[mb] = (x, y, dy, dx)
        check(lib().chimera_stage_set_io(self.handle, mb, _ptr(x), _ptr(y), _ptr(dy), _ptr(dx)))
        return y, dx

    def fwd(self, mb):
        check(lib().chimera_fwd(self.handle, mb))

    def bwd(self, mb):
        check(lib().chimera_bwd(self.handle, mb))

    def bwd_half(self, mb, half):
        check(lib().chimera_bwd_half(self.handle, mb, half))

    def zero_grads(self):
        check(lib().chimera_stage_zero_grads(self.handle))

    def read_grads(self):
        import numpy as np
        out = np.empty(self.grads.numel(), dtype=np.float32)
        check(lib().chimera_stage_read_grads(self.handle, out.ctypes.data_as(C.c_void_p), out.nbytes))
        return out

    def close(self):
        if self.handle:
            lib().chimera_stage_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def chimera_worker_bind(down, up):
    check(lib().chimera_worker_bind(down.handle, up.handle if up is not None else None))


def chimera_worker_bind_pipes(stages):
    arr = (C.c_void_p * len(stages))(*[None if st is None else st.handle for st in stages])
    check(lib().chimera_worker_bind_pipes(arr, len(stages)))


def chimera_worker_bind_doubling(down2, up2):
    check(lib().chimera_worker_bind_doubling(down2.handle, up2.handle))


def chimera_run_worker_pipes(algo, rank, D, N, f=1):
    check(lib().chimera_run_worker_pipes(algo, rank, D, N, f))


def chimera_run_worker(rank, D, N):
    check(lib().chimera_run_worker(rank, D, N))


def chimera_run_worker_algo(algo, rank, D, N):
    check(lib().chimera_run_worker_algo(algo, rank, D, N))


def chimera_worker_set_timing(on):
    check(lib().chimera_worker_set_timing(int(on)))


def chimera_worker_last_timing():
    f, b, nf, nb = C.c_double(), C.c_double(), C.c_int(), C.c_int()
    check(lib().chimera_worker_last_timing(C.byref(f), C.byref(b), C.byref(nf), C.byref(nb)))
    return dict(fwd_ms=f.value, bwd_ms=b.value, n_fwd=nf.value, n_bwd=nb.value)


def chimera_worker_last_enqueue_ms():
    v = C.c_double()
    check(lib().chimera_worker_last_enqueue_ms(C.byref(v)))
    return v.value


PROFILE_CLASSES = ("gemm_fwd", "gemm_dgrad", "gemm_wgrad", "attn_fwd", "attn_bwd", "ln_fwd", "ln_bwd", "colsum", "gemm_wgrad_tail")


def chimera_profile_enable(on):
    check(lib().chimera_profile_enable(int(on)))


def chimera_profile_reset():
    check(lib().chimera_profile_reset())


def chimera_profile_read():
    """{class name: dict(ms, launches, work)}; work is flop (gemm, attention) or bytes."""
    out = {}
    for i, name in enumerate(PROFILE_CLASSES):
        ms, n, w = C.c_double(), C.c_longlong(), C.c_double()
        check(lib().chimera_profile_read(i, C.byref(ms), C.byref(n), C.byref(w)))
        out[name] = dict(ms=ms.value, launches=n.value, work=w.value)
    return out


def stash_slots_needed_pipes(algo, D, N, f, rank):
    """Stash slots every pipeline's stage needs on worker `rank` (index = pipeline)."""
    ops = chimera_schedule_pipes(algo, D, N, f, rank)
    need = [0] * (2 * f)
    for o in ops:
        need[o.pipe] = max(need[o.pipe], o.slot + 1)
    if any(o.kind == OP_F2 for o in ops):
        need = [n + 1 for n in need]              # the recomputing backwards take one more
    return need


def stash_slots_needed(algo, D, N, rank):
    """Slots each of the worker's two stages needs: (down, up)."""
    need = [0, 0]
    for op in chimera_schedule(algo, D, N, rank):
        need[op.pipe] = max(need[op.pipe], op.slot + 1)
    return tuple(need)


# ---------------------------------------------------------- single operators
def _stream(t):
    import torch
    return C.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _dt(t):
    import torch
    return F32 if t.dtype == torch.float32 else BF16


_gemm_ws = {}


def gemm_workspace(m, n, k, device):
    """A zero-initialised split-K workspace for this shape (cached per size), or None."""
    import torch
    need = lib().chimera_op_gemm_workspace_bytes(m, n, k)
    if not need:
        return None
    if need not in _gemm_ws:
        _gemm_ws[need] = torch.zeros(need, dtype=torch.uint8, device=device)
    return _gemm_ws[need]


def chimera_op_gemm(a, b, c, m, n, k, a_kc, b_kc, epilogue=EPI_NONE, bias=None, r=None, c2=None, impl=0,
                    gelu_erf=False, lda=None, ldb=None, workspace="auto"):
    lda = lda if lda is not None else (k if a_kc else m)
    ldb = ldb if ldb is not None else (k if b_kc else n)
    ws = gemm_workspace(m, n, k, a.device) if isinstance(workspace, str) else workspace
    check(lib().chimera_op_gemm(_dt(a), impl, epilogue, int(gelu_erf), m, n, k, _ptr(a), lda, int(a_kc), _ptr(b), ldb,
                                int(b_kc), _ptr(bias), _ptr(r), _ptr(c), _ptr(c2), _ptr(ws),
                                ws.numel() if ws is not None else 0, _stream(a)))


def chimera_op_gemm_group_accumulate(problems, k, bsums=None, overwrite=False):
    """problems: list of (a [k, m] bf16, b [k, n] bf16, c [m, n] float32) device tensors;
    bsums: optional list of float32 [n] tensors (or None) receiving += column sums of b."""
    cnt = len(problems)
    ints = lambda v: (C.c_int * cnt)(*v)
    ptrs = lambda v: (C.c_void_p * cnt)(*[t.data_ptr() for t in v])
    a, b, c = zip(*problems) if cnt else ((), (), ())
    m = [t.shape[1] for t in a]
    n = [t.shape[1] for t in b]
    check(lib().chimera_op_gemm_group_accumulate(cnt, ints(m), ints(n), k, ptrs(a), ints([t.stride(0) for t in a]), ptrs(b),
                                                 ints([t.stride(0) for t in b]), ptrs(c),
                                                 None if bsums is None else (C.c_void_p * cnt)(
                                                     *[None if t is None else t.data_ptr() for t in bsums]),
                                                 int(overwrite), _stream(a[0]) if cnt else None))


def chimera_op_layernorm_fwd(x, gamma, beta, y, mean, rstd):
    rows, cols = x.shape
    check(lib().chimera_op_layernorm_fwd(_dt(x), rows, cols, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(mean),
                                         _ptr(rstd), _stream(x)))


def chimera_op_layernorm_bwd(dy, x, mean, rstd, gamma, res, dx, dgamma, dbeta):
    import torch
    rows, cols = x.shape
    scratch = torch.empty(lib().chimera_op_layernorm_bwd_scratch_floats(rows, cols), dtype=torch.float32, device=x.device)
    check(lib().chimera_op_layernorm_bwd(_dt(x), rows, cols, _ptr(dy), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gamma),
                                         _ptr(res), _ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(scratch), _stream(x)))


def chimera_op_layernorm_bwd_noalloc(dy, x, mean, rstd, gamma, res, dx, dgamma, dbeta):
    rows, cols = x.shape
    check(lib().chimera_op_layernorm_bwd_noalloc(_dt(x), rows, cols, _ptr(dy), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gamma),
                                                 _ptr(res), _ptr(dx), _ptr(dgamma), _ptr(dbeta), _stream(x)))


def chimera_op_colsum(x, out):
    import torch
    rows, cols = x.shape
    scratch = torch.empty(lib().chimera_op_colsum_scratch_floats(rows, cols), dtype=torch.float32, device=x.device)
    check(lib().chimera_op_colsum(_dt(x), rows, cols, _ptr(x), _ptr(out), _ptr(scratch), _stream(x)))


def chimera_op_attention_fwd(qkv, ctx, lse, batch, seq, heads, head_dim, causal, impl=0):
    check(lib().chimera_op_attention_fwd(_dt(qkv), impl, batch, seq, heads, head_dim, int(causal), _ptr(qkv), _ptr(ctx),
                                         _ptr(lse), _stream(qkv)))


def chimera_op_attention_bwd(qkv, ctx, lse, dctx, dqkv, delta, batch, seq, heads, head_dim, causal, impl=0):
    check(lib().chimera_op_attention_bwd(_dt(qkv), impl, batch, seq, heads, head_dim, int(causal), _ptr(qkv), _ptr(ctx),
                                         _ptr(lse), _ptr(dctx), _ptr(dqkv), _ptr(delta), _stream(qkv)))


def chimera_probe_mfma_bf16(sink, iters=2000):
    out = C.c_double(0)
    check(lib().chimera_probe_mfma_bf16(_ptr(sink), iters, C.byref(out), _stream(sink)))
    return out.value


def chimera_probe_copy(src, dst):
    out = C.c_double(0)
    check(lib().chimera_probe_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), C.byref(out), _stream(src)))
    return out.value


def chimera_op_embedding_fwd(tokens, seq, wte, wpe, x):
    check(lib().chimera_op_embedding_fwd(_dt(wte), tokens.numel(), seq, wte.shape[1], wte.shape[0], _ptr(tokens), _ptr(wte),
                                         _ptr(wpe), _ptr(x), _stream(x)))


def chimera_op_embedding_bwd(tokens, seq, dx, dwte, dwpe):
    check(lib().chimera_op_embedding_bwd(_dt(dx), tokens.numel(), seq, dx.shape[1], dwte.shape[0], _ptr(tokens), _ptr(dx),
                                         _ptr(dwte), _ptr(dwpe), _stream(dx)))


def chimera_op_softmax_xent(logits, targets, scale, loss_rows, loss):
    check(lib().chimera_op_softmax_xent(_dt(logits), logits.shape[0], logits.shape[1], _ptr(logits), _ptr(targets), scale,
                                        _ptr(loss_rows), _ptr(loss), _stream(logits)))


def chimera_head_loss(y, targets, lnf_g, lnf_b, w_head, scale, dy, dlnf_g, dlnf_b, dw_head, loss, workspace=None):
    """w_head [hidden, vocab]; allocates the workspace (a torch uint8 tensor) unless one is given."""
    import torch
    need = lib().chimera_head_workspace_bytes(_dt(y), y.shape[0], y.shape[1], w_head.shape[1])
    ws = workspace if workspace is not None else torch.empty(need, dtype=torch.uint8, device=y.device)
    check(lib().chimera_head_loss(_dt(y), y.shape[0], y.shape[1], w_head.shape[1], _ptr(y), _ptr(targets), _ptr(lnf_g),
                                  _ptr(lnf_b), _ptr(w_head), scale, _ptr(dy), _ptr(dlnf_g), _ptr(dlnf_b), _ptr(dw_head),
                                  _ptr(loss), _ptr(ws), ws.numel(), _stream(y)))
    return ws
