"""ctypes binding with the same names as the C ABI in include/bls.h (argument marshalling only)."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))

MODEL_MLP, MODEL_RESNET_CIFAR, MODEL_WRN, MODEL_ENCODER = 0, 1, 2, 3
ACT_DTYPES = {"f32": 0, "bf16": 1}
AGG_NORMALISE, AGG_BROADCAST = 1, 2

DECLARED_SYMBOLS = (
    "bls_ctx_create", "bls_ctx_destroy", "bls_last_error", "bls_ctx_synchronize", "bls_model_create",
    "bls_model_destroy", "bls_model_num_params", "bls_model_num_buffers", "bls_model_workspace_bytes", "bls_model_num_tensors",
    "bls_model_tensor_layout", "score_losses", "topk_by_loss", "local_step", "weighted_aggregate",
    "bls_weights_from_tau", "bls_profile_begin", "bls_profile_end", "bls_epoch_allocation", "bls_worker_share",
    "sample_epoch", "sample_epoch_variant", "communication_round", "bls_ctx_set_lanes", "topk_by_loss_static",
    "train_epochs", "bls_sum_limits",
)
ROUND_UNIFORM_WEIGHTS, ROUND_SEQUENTIAL = 1, 2
TOPK_STATIC_MAX_N = 1 << 20
SAMPLING_SCHEMES = {"separated": 0, "unified": 1}
HIGH_LOSS_TO = {"fast": 0, "slow": 1, "none": 2}
PROFILE_CLASSES = ("conv_fwd", "conv_dgrad", "conv_wgrad", "norm", "head", "gemm", "update", "gather", "topk",
                   "aggregate", "wgrad_reduce")


class BlsError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("bls status %d: %s" % (code, message))
        self.code = code


class _ModelDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("classes", C.c_int32), ("image_hw", C.c_int32), ("in_channels", C.c_int32),
                ("hidden", C.c_int32), ("widths", C.c_int32 * 3), ("blocks", C.c_int32), ("act_dtype", C.c_int32)]


class _TensorInfo(C.Structure):
    _fields_ = [("name", C.c_char * 56), ("offset", C.c_int64), ("ndim", C.c_int32), ("shape", C.c_int32 * 4),
                ("is_buffer", C.c_int32)]


class _Sgd(C.Structure):
    _fields_ = [("lr", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float)]


class _EpochPlan(C.Structure):
    _fields_ = [("epochs", C.c_int64), ("tau_f", C.c_int64), ("tau_s", C.c_int64), ("P_f", C.c_int32), ("P_s", C.c_int32),
                ("lam", C.c_double), ("scheme", C.c_int32), ("high_loss_to", C.c_int32), ("round_flags", C.c_int32),
                ("n_milestones", C.c_int32), ("batch", C.c_int64), ("opt", _Sgd), ("lr_gamma", C.c_float),
                ("milestones", C.POINTER(C.c_int64))]


def library_path():
    return os.path.join(_HERE, "libbls.so")


def _load():
    path = library_path()
    if not os.path.exists(path):
        raise ImportError("libbls.so is not built: run `python -m paper_2508_08540_amd.build` (needs hipcc)")
    L = C.CDLL(path)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int32
    L.bls_ctx_create.argtypes = [C.POINTER(vp), C.c_int, vp]
    L.bls_ctx_destroy.argtypes = [vp]
    L.bls_ctx_destroy.restype = None
    L.bls_last_error.argtypes = [vp]
    L.bls_last_error.restype = C.c_char_p
    L.bls_ctx_synchronize.argtypes = [vp]
    L.bls_model_create.argtypes = [C.POINTER(_ModelDesc), C.POINTER(vp)]
    L.bls_model_destroy.argtypes = [vp]
    L.bls_model_destroy.restype = None
    for f in (L.bls_model_num_params, L.bls_model_num_buffers):
        f.argtypes = [vp]
        f.restype = i64
    L.bls_model_workspace_bytes.argtypes = [vp, i64, C.c_int]
    L.bls_model_workspace_bytes.restype = i64
    L.bls_model_num_tensors.argtypes = [vp]
    L.bls_model_num_tensors.restype = i32
    L.bls_model_tensor_layout.argtypes = [vp, C.POINTER(_TensorInfo), i32]
    L.score_losses.argtypes = [vp, vp, vp, vp, vp, vp, i64, vp]
    L.topk_by_loss.argtypes = [vp, vp, i64, i64, vp, vp]
    L.topk_by_loss_static.argtypes = [vp, vp, i64, i64, vp, vp]
    L.local_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, vp, i64, i64, i64, C.POINTER(_Sgd), vp]
    L.bls_epoch_allocation.argtypes = [i64, i64, C.c_int, i64, C.c_int, C.c_double, C.POINTER(i64), C.POINTER(i64),
                                       C.POINTER(i64)]
    L.bls_worker_share.argtypes = [i64, C.c_int, C.c_int, C.POINTER(i64), C.POINTER(i64)]
    L.sample_epoch.argtypes = [vp, vp, vp, vp, i64, i64, C.c_int, i64, C.c_int, C.c_double, vp, vp]
    L.bls_ctx_set_lanes.argtypes = [vp, C.c_int]
    L.communication_round.argtypes = [vp, vp, vp, vp, vp, C.c_int, vp, vp, i64, i64, vp, vp, C.c_int]
    L.train_epochs.argtypes = [vp, vp, C.POINTER(_EpochPlan), vp, vp, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp, C.POINTER(i64)]
    L.sample_epoch_variant.argtypes = [vp, vp, vp, vp, i64, i64, C.c_int, i64, C.c_int, C.c_double, C.c_int, C.c_int, vp, vp]
    L.weighted_aggregate.argtypes = [vp, C.POINTER(vp), C.POINTER(C.c_float), C.c_int, i64, vp, C.c_int]
    L.bls_weights_from_tau.argtypes = [C.POINTER(i64), C.c_int, C.POINTER(C.c_float)]
    L.bls_profile_begin.argtypes = [vp]
    L.bls_profile_end.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64), C.c_int]
    return L


lib = _load()


def _ptr(t):
    """Device (or host) address of a torch tensor / None."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors passed to the library must be contiguous")
    return C.c_void_p(t.data_ptr())


class Context:
    """A device, the HIP stream work is enqueued on (torch's current stream by default) and scratch memory."""

    def __init__(self, device=0, stream=None):
        import torch
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
        h = C.c_void_p()
        rc = lib.bls_ctx_create(C.byref(h), int(device), C.c_void_p(stream))
        if rc != 0:
            raise BlsError(rc, "bls_ctx_create failed (is a GPU visible?)")
        self.handle, self.device = h, device

    def check(self, rc):
        if rc != 0:
            raise BlsError(rc, lib.bls_last_error(self.handle).decode())

    def synchronize(self):
        self.check(lib.bls_ctx_synchronize(self.handle))

    def profile_begin(self):
        self.check(lib.bls_profile_begin(self.handle))

    def set_lanes(self, lanes):
        """Workers that communication_round runs side by side (library-owned streams and scratch)."""
        self.check(lib.bls_ctx_set_lanes(self.handle, lanes))

    def profile_end(self):
        """{class: (milliseconds, bracketed launch groups)} since profile_begin."""
        n = len(PROFILE_CLASSES)
        ms, cnt = (C.c_double * n)(), (C.c_int64 * n)()
        got = lib.bls_profile_end(self.handle, ms, cnt, n)
        if got < 0:
            self.check(got)
        return {name: (ms[i], cnt[i]) for i, name in enumerate(PROFILE_CLASSES)}

    def close(self):
        if self.handle:
            lib.bls_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Model:
    """Architecture description and flat layout; host only."""

    def __init__(self, kind, classes=10, image_hw=32, in_channels=3, hidden=128, widths=(16, 32, 64), blocks=3,
                 act_dtype="f32"):
        desc = _ModelDesc(kind, classes, image_hw, in_channels, hidden, (C.c_int32 * 3)(*widths), blocks,
                          ACT_DTYPES[act_dtype])
        self.act_dtype = act_dtype
        h = C.c_void_p()
        rc = lib.bls_model_create(C.byref(desc), C.byref(h))
        if rc != 0:
            raise BlsError(rc, "bls_model_create rejected the description")
        self.handle = h
        self.num_params = lib.bls_model_num_params(h)
        self.num_buffers = lib.bls_model_num_buffers(h)
        n = lib.bls_model_num_tensors(h)
        arr = (_TensorInfo * n)()
        got = lib.bls_model_tensor_layout(h, arr, n)
        assert got == n
        self.tensors = [dict(name=t.name.decode(), offset=t.offset, shape=tuple(t.shape[:t.ndim]),
                             is_buffer=bool(t.is_buffer)) for t in arr]

    def workspace_bytes(self, n, training):
        """Device scratch the context grows to for local_step at batch size n (training) or score_losses over n samples."""
        got = lib.bls_model_workspace_bytes(self.handle, int(n), 1 if training else 0)
        if got < 0:
            raise BlsError(int(got), "bls_model_workspace_bytes rejected the arguments")
        return int(got)

    @classmethod
    def mlp(cls, d_hw=32, in_channels=3, hidden=128, classes=10):
        return cls(MODEL_MLP, classes, d_hw, in_channels, hidden)

    @classmethod
    def resnet_cifar(cls, widths=(16, 32, 64), blocks=3, classes=10, image_hw=32, in_channels=3, act_dtype="f32"):
        """act_dtype "bf16": activations and the kernels' weight copies in bf16, everything else fp32."""
        return cls(MODEL_RESNET_CIFAR, classes, image_hw, in_channels, 0, widths, blocks, act_dtype)

    @classmethod
    def wide_resnet(cls, widths=(128, 256, 512), blocks=2, classes=100, image_hw=32, in_channels=3, stem=16, act_dtype="f32"):
        """Pre-activation wide residual network; the defaults are WRN-16-8."""
        return cls(MODEL_WRN, classes, image_hw, in_channels, stem, widths, blocks, act_dtype)

    @classmethod
    def transformer(cls, vocab=32000, seq_len=128, d_model=512, heads=8, d_ff=2048, layers=6, act_dtype="f32"):
        """Post-layer-norm transformer encoder language model; samples are int32 token sequences [N, seq_len].
        act_dtype "bf16": operands of every matrix product rounded to bf16, sums and storage fp32."""
        return cls(MODEL_ENCODER, vocab, seq_len, 0, d_model, (heads, d_ff, 0), layers, act_dtype)

    def pack(self, tensors, buffers=False):
        """dict name -> array  =>  flat float32 numpy vector in the library's layout."""
        out = np.zeros(self.num_buffers if buffers else self.num_params, dtype=np.float32)
        for t in self.tensors:
            if t["is_buffer"] == buffers:
                a = np.asarray(tensors[t["name"]], dtype=np.float32)
                assert a.shape == t["shape"], (t["name"], a.shape, t["shape"])
                out[t["offset"]:t["offset"] + a.size] = a.reshape(-1)
        return out

    def unpack(self, flat, buffers=False):
        flat = np.asarray(flat)
        return {t["name"]: flat[t["offset"]:t["offset"] + int(np.prod(t["shape"]))].reshape(t["shape"])
                for t in self.tensors if t["is_buffer"] == buffers}

    def __del__(self):
        try:
            if self.handle:
                lib.bls_model_destroy(self.handle)
                self.handle = None
        except Exception:
            pass


def score_losses(ctx, model, params, buffers, x, y, losses_out):
    ctx.check(lib.score_losses(ctx.handle, model.handle, _ptr(params), _ptr(buffers), _ptr(x), _ptr(y),
                               x.shape[0], _ptr(losses_out)))
    return losses_out


def topk_by_loss(ctx, losses, k, idx_out, val_out=None):
    ctx.check(lib.topk_by_loss(ctx.handle, _ptr(losses), losses.shape[0], k, _ptr(idx_out), _ptr(val_out)))
    return idx_out


def topk_by_loss_static(ctx, losses, k, idx_out, val_out=None):
    """topk_by_loss on the library's fixed device array: no allocation, N <= TOPK_STATIC_MAX_N."""
    ctx.check(lib.topk_by_loss_static(ctx.handle, _ptr(losses), losses.shape[0], k, _ptr(idx_out), _ptr(val_out)))
    return idx_out


def local_step(ctx, model, params, buffers, momentum, x_pool, y_pool, sel_idx, batch, tau, lr, mu=0.0,
               weight_decay=0.0, step_losses_out=None, k=None):
    opt = _Sgd(lr, mu, weight_decay)
    ctx.check(lib.local_step(ctx.handle, model.handle, _ptr(params), _ptr(buffers), _ptr(momentum), _ptr(x_pool),
                             _ptr(y_pool), x_pool.shape[0], _ptr(sel_idx), sel_idx.shape[0] if k is None else k,
                             batch, tau, C.byref(opt), _ptr(step_losses_out)))


def weighted_aggregate(ctx, replicas, weights, out, flags=0):
    P = len(replicas)
    d = out.numel()
    ptrs = (C.c_void_p * P)(*[r.data_ptr() for r in replicas])
    w = (C.c_float * P)(*[float(v) for v in weights])
    ctx.check(lib.weighted_aggregate(ctx.handle, ptrs, w, P, d, _ptr(out), flags))
    return out


def epoch_allocation(N, tau_f, P_f, tau_s, P_s, lam):
    """(N_F, k, N_S) of one epoch (host arithmetic)."""
    nf, k, ns = C.c_int64(), C.c_int64(), C.c_int64()
    rc = lib.bls_epoch_allocation(N, tau_f, P_f, tau_s, P_s, lam, C.byref(nf), C.byref(k), C.byref(ns))
    if rc != 0:
        raise BlsError(rc, "bls_epoch_allocation rejected the arguments")
    return nf.value, k.value, ns.value


def worker_share(n, P, p):
    """(offset, count) of worker p's segment in a worker-major list of n items."""
    off, cnt = C.c_int64(), C.c_int64()
    rc = lib.bls_worker_share(n, P, p, C.byref(off), C.byref(cnt))
    if rc != 0:
        raise BlsError(rc, "bls_worker_share rejected the arguments")
    return off.value, cnt.value


def sample_epoch(ctx, losses, u_fast, u_slow, tau_f, P_f, tau_s, P_s, lam, fast_idx_out, slow_idx_out, scheme=None,
                 high_loss_to=None):
    """scheme / high_loss_to given: the appendix's variants through sample_epoch_variant."""
    if scheme is None and high_loss_to is None:
        ctx.check(lib.sample_epoch(ctx.handle, _ptr(losses), _ptr(u_fast), _ptr(u_slow), losses.shape[0], tau_f, P_f, tau_s,
                                   P_s, lam, _ptr(fast_idx_out), _ptr(slow_idx_out)))
    else:
        ctx.check(lib.sample_epoch_variant(ctx.handle, _ptr(losses), _ptr(u_fast), _ptr(u_slow), losses.shape[0], tau_f, P_f,
                                           tau_s, P_s, lam, SAMPLING_SCHEMES[scheme or "separated"],
                                           HIGH_LOSS_TO[high_loss_to or "fast"], _ptr(fast_idx_out), _ptr(slow_idx_out)))


class _Worker(C.Structure):
    _fields_ = [("tau", C.c_int64), ("idx", C.c_void_p), ("n_idx", C.c_int64), ("params", C.c_void_p), ("buffers", C.c_void_p),
                ("momentum", C.c_void_p)]


def communication_round(ctx, model, global_params, global_buffers, workers, x_pool, y_pool, batch, lr, mu=0.0, weight_decay=0.0,
                        loss_table=None, flags=0):
    """workers: list of dict(tau, idx, params, buffers, momentum) of device tensors (buffers may be None)."""
    arr = (_Worker * len(workers))()
    for i, w in enumerate(workers):
        addr = lambda t: None if t is None else _ptr(t).value
        arr[i] = _Worker(int(w["tau"]), addr(w["idx"]), w["idx"].shape[0], addr(w["params"]), addr(w.get("buffers")), addr(w["momentum"]))
    opt = _Sgd(lr, mu, weight_decay)
    ctx.check(lib.communication_round(ctx.handle, model.handle, _ptr(global_params), _ptr(global_buffers), arr, len(workers),
                                      _ptr(x_pool), _ptr(y_pool), x_pool.shape[0], batch, C.byref(opt), _ptr(loss_table), flags))


def train_epochs(ctx, model, global_params, global_buffers, worker_params, worker_buffers, worker_momentum, x_pool, y_pool, u_fast, u_slow,
                 loss_table, idx_work, epochs, tau_f, P_f, tau_s, P_s, lam, batch, lr, mu=0.0, weight_decay=0.0, milestones=(), lr_gamma=0.1,
                 scheme="separated", high_loss_to="fast", round_flags=0):
    """The outer loop of Algorithm 1 on device tensors; returns the number of communication rounds that were run."""
    ms = (C.c_int64 * max(len(milestones), 1))(*[int(m) for m in milestones])
    plan = _EpochPlan(int(epochs), int(tau_f), int(tau_s), int(P_f), int(P_s), float(lam), SAMPLING_SCHEMES[scheme], HIGH_LOSS_TO[high_loss_to],
                      int(round_flags), len(milestones), int(batch), _Sgd(lr, mu, weight_decay), float(lr_gamma), ms)
    rounds = C.c_int64()
    ctx.check(lib.train_epochs(ctx.handle, model.handle, C.byref(plan), _ptr(global_params), _ptr(global_buffers), _ptr(worker_params),
                               _ptr(worker_buffers), _ptr(worker_momentum), _ptr(x_pool), _ptr(y_pool), x_pool.shape[0], _ptr(u_fast),
                               _ptr(u_slow), _ptr(loss_table), _ptr(idx_work), C.byref(rounds)))
    return rounds.value


def sum_limits():
    """(forward, backward, weight-gradient) bound of one workgroup's contribution to a fixed-point batch sum."""
    f, b, w = C.c_double(), C.c_double(), C.c_double()
    lib.bls_sum_limits.argtypes = [C.POINTER(C.c_double)] * 3
    lib.bls_sum_limits(C.byref(f), C.byref(b), C.byref(w))
    return f.value, b.value, w.value


def weights_from_tau(tau):
    P = len(tau)
    t = (C.c_int64 * P)(*[int(v) for v in tau])
    w = (C.c_float * P)()
    rc = lib.bls_weights_from_tau(t, P, w)
    if rc != 0:
        raise BlsError(rc, "bls_weights_from_tau rejected the step counts")
    return np.array(list(w), dtype=np.float32)
