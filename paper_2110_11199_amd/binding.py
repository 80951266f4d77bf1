"""ctypes binding of libadpsgd.so: the same entry points as include/adpsgd.h.

Argument marshalling only; every step of the iteration runs in the HIP library.
PyTorch is used for device memory (the workspace and the caller's batches) and
for the stream handle.  There is no fallback: if the library has not been built
the import of this module fails.
"""
import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  -- first: the library must bind to the HIP runtime that PyTorch has loaded,
#                              or its device pointers and streams would belong to another runtime instance

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadpsgd.so")

if not os.path.exists(LIB_PATH):
    raise ImportError("libadpsgd.so is not built: run `python -m paper_2110_11199_amd.build` "
                      "(needs hipcc; there is no CPU fallback)")
_lib = C.CDLL(LIB_PATH)

OK, EINVAL, ENOMEM, EHIP = 0, -1, -2, -3
FIXED_RING, RANDOM_RING, D1D, SDPSGD = 0, 1, 2, 3
MIX_DEFAULT, MIX_PAIR, MIX_TRI, MIX_ALL, MIX_HYBRID_PAIR, MIX_HYBRID_TRI = -1, 0, 1, 2, 3, 4
FP32, BF16_GEMM = 0, 1
MAX_LEARNERS = 128


class ModelShape(C.Structure):
    _fields_ = [("input_dim", C.c_int32), ("hidden", C.c_int32), ("layers", C.c_int32),
                ("bidirectional", C.c_int32), ("bottleneck", C.c_int32), ("classes", C.c_int32),
                ("batch", C.c_int32), ("frames", C.c_int32), ("flat_params", C.c_int64)]


class Config(C.Structure):
    _fields_ = [("L", C.c_int32), ("shape", ModelShape), ("pattern", C.c_int32), ("mix", C.c_int32),
                ("tau", C.c_int32), ("precision", C.c_int32), ("seed", C.c_uint64),
                ("straggler_p", C.c_float), ("init_scale", C.c_float), ("group_size", C.c_int32)]


_vp, _i64, _i32p = C.c_void_p, C.c_int64, C.POINTER(C.c_int32)
_lib.adpsgd_workspace_bytes.argtypes = [C.POINTER(Config), C.POINTER(C.c_size_t)]
_lib.adpsgd_create.argtypes = [C.POINTER(Config), _vp, C.c_size_t, _vp, C.POINTER(_vp)]
_lib.adpsgd_step.argtypes = [_vp, C.POINTER(_vp), C.c_float]
_lib.adpsgd_step_masked.argtypes = [_vp, C.POINTER(_vp), C.c_float, _i32p]
_lib.adpsgd_delay.argtypes = [C.c_uint64, _vp]
_lib.adpsgd_capture_begin.argtypes = [_vp]
_lib.adpsgd_capture_end.argtypes = [_vp, C.POINTER(_vp)]
_lib.adpsgd_graph_replay.argtypes = [_vp]
_lib.adpsgd_graph_steps.argtypes = [_vp]
_lib.adpsgd_graph_steps.restype = _i64
_lib.adpsgd_graph_destroy.argtypes = [_vp]
_lib.adpsgd_graph_destroy.restype = None
_lib.adpsgd_params.argtypes = [_vp, C.c_int]
_lib.adpsgd_params.restype = _vp
_lib.adpsgd_set_params.argtypes = [_vp, C.c_int, _vp]
_lib.adpsgd_grads.argtypes = [_vp, C.c_int]
_lib.adpsgd_grads.restype = _vp
_lib.adpsgd_losses.argtypes = [_vp, C.POINTER(C.c_float)]
_lib.adpsgd_param_count.argtypes = [_vp]
_lib.adpsgd_param_count.restype = _i64
_lib.adpsgd_layout_count.argtypes = [_vp]
_lib.adpsgd_layout.argtypes = [_vp, C.c_int, C.POINTER(_i64), C.POINTER(_i64), C.POINTER(_i64)]
_lib.adpsgd_schedule.argtypes = [_vp, _i64, _i32p, _i32p, _i32p]
_lib.adpsgd_schedule_of.argtypes = [C.c_int32, C.c_uint64, C.c_float, C.c_int32, _i64, _i32p, _i32p, _i32p]
_lib.adpsgd_lr_at_epoch.argtypes = [C.c_int32, C.c_float, C.c_float, C.c_int32, C.c_int32, C.POINTER(C.c_float)]
_lib.adpsgd_iteration.argtypes = [_vp]
_lib.adpsgd_iteration.restype = _i64
_lib.adpsgd_average.argtypes = [_vp, _vp]
_lib.adpsgd_consensus.argtypes = [_vp, C.POINTER(C.c_double)]
_lib.adpsgd_consensus_static.argtypes = [_vp, _i64, C.c_int32, _i64, _vp, _vp]
_lib.adpsgd_set_profiling.argtypes = [_vp, C.c_int]
_lib.adpsgd_profile.argtypes = [_vp, C.POINTER(C.c_float), _i32p, C.POINTER(C.c_double), C.POINTER(C.c_double)]
_lib.adpsgd_destroy.argtypes = [_vp]
_lib.adpsgd_destroy.restype = None
_lib.adpsgd_last_error.restype = C.c_char_p
_lib.adpsgd_gemm.argtypes = [C.c_int] * 7 + [_vp, _i64, _i64, _vp, _i64, _i64, _vp, _i64, _i64, _vp, _i64,
                                             C.c_int, C.c_int, _vp]
_lib.adpsgd_set_tuning.argtypes = [_vp, C.c_int, C.c_int]
_lib.adpsgd_probe_mfma.argtypes = [_vp, C.c_int, C.c_int, _vp]
_lib.adpsgd_probe_stream.argtypes = [C.c_int, C.c_int, C.c_int, _vp, _i64, _i64, _vp]
_lib.adpsgd_status.argtypes = [_vp]

EXPORTS = ["adpsgd_workspace_bytes", "adpsgd_create", "adpsgd_step", "adpsgd_params", "adpsgd_set_params",
           "adpsgd_grads", "adpsgd_losses", "adpsgd_param_count", "adpsgd_layout_count", "adpsgd_layout",
           "adpsgd_schedule", "adpsgd_schedule_of", "adpsgd_iteration", "adpsgd_average", "adpsgd_destroy",
           "adpsgd_last_error", "adpsgd_gemm", "adpsgd_set_profiling", "adpsgd_profile",
           "adpsgd_set_tuning", "adpsgd_consensus", "adpsgd_status", "adpsgd_consensus_static", "adpsgd_lr_at_epoch",
           "adpsgd_probe_mfma", "adpsgd_probe_stream", "adpsgd_step_masked", "adpsgd_delay",
           "adpsgd_capture_begin", "adpsgd_capture_end", "adpsgd_graph_replay", "adpsgd_graph_steps", "adpsgd_graph_destroy"]
STATIC_MAX_ELEMENTS = 1 << 34
TUNE_GEMM_TILE, TUNE_REC_DIRECT, TUNE_REC_FWD_GROUPS, TUNE_REC_PERSISTENT, TUNE_REC_WAIT_US, TUNE_MEAN_CHUNK = 0, 1, 2, 3, 4, 5
TUNE_TRI_SEGMENT, TUNE_PAIR_SPLIT, TUNE_SYNC_SEGMENT = 6, 7, 8
PHASES = ["stage_cast", "batched_gemm", "recurrent_fwd", "recurrent_bwd", "softmax_ce", "bias_colsum", "mix_update"]


class AdpsgdError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("adpsgd error %d: %s" % (code, text))
        self.code = code


def adpsgd_last_error():
    return _lib.adpsgd_last_error().decode()


def _check(rc):
    if rc != 0:
        raise AdpsgdError(rc, adpsgd_last_error())


def make_config(L, pattern, seed=0, input_dim=0, hidden=0, layers=0, bidirectional=0, bottleneck=0,
                classes=0, batch=0, frames=0, flat_params=0, mix=MIX_DEFAULT, tau=-1, precision=FP32,
                straggler_p=0.0, init_scale=0.0, group_size=0):
    return Config(L, ModelShape(input_dim, hidden, layers, bidirectional, bottleneck, classes, batch, frames,
                                flat_params), pattern, mix, tau, precision, seed, straggler_p, init_scale, group_size)


def adpsgd_workspace_bytes(cfg):
    n = C.c_size_t(0)
    _check(_lib.adpsgd_workspace_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def adpsgd_create(cfg, dev_workspace_ptr, nbytes, stream_ptr):
    h = _vp()
    _check(_lib.adpsgd_create(C.byref(cfg), dev_workspace_ptr, nbytes, stream_ptr, C.byref(h)))
    return h


def adpsgd_step(h, batch_ptrs, lr):
    arr = (_vp * len(batch_ptrs))(*batch_ptrs)
    _check(_lib.adpsgd_step(h, arr, lr))


def adpsgd_step_masked(h, batch_ptrs, lr, active):
    arr = (_vp * len(batch_ptrs))(*batch_ptrs)
    act = (C.c_int32 * len(active))(*[int(a) for a in active])
    _check(_lib.adpsgd_step_masked(h, arr, lr, act))


def adpsgd_delay(microseconds, stream_ptr):
    _check(_lib.adpsgd_delay(int(microseconds), stream_ptr))


def adpsgd_capture_begin(h):
    _check(_lib.adpsgd_capture_begin(h))


def adpsgd_capture_end(h):
    g = _vp()
    _check(_lib.adpsgd_capture_end(h, C.byref(g)))
    return g


def adpsgd_graph_replay(g):
    _check(_lib.adpsgd_graph_replay(g))


def adpsgd_graph_steps(g):
    return _lib.adpsgd_graph_steps(g)


def adpsgd_graph_destroy(g):
    _lib.adpsgd_graph_destroy(g)


def adpsgd_params(h, i):
    return _lib.adpsgd_params(h, i)


def adpsgd_set_params(h, i, dev_src_ptr):
    _check(_lib.adpsgd_set_params(h, i, dev_src_ptr))


def adpsgd_grads(h, i):
    return _lib.adpsgd_grads(h, i)


def adpsgd_losses(h, L):
    out = (C.c_float * L)()
    _check(_lib.adpsgd_losses(h, out))
    return np.array(out[:], dtype=np.float32)


def adpsgd_param_count(h):
    return _lib.adpsgd_param_count(h)


def adpsgd_layout(h):
    out = []
    for idx in range(_lib.adpsgd_layout_count(h)):
        o, r, c = _i64(), _i64(), _i64()
        _check(_lib.adpsgd_layout(h, idx, C.byref(o), C.byref(r), C.byref(c)))
        out.append((o.value, r.value, c.value))
    return out


def adpsgd_schedule(h, k, L):
    o, p, a = (C.c_int32 * L)(), (C.c_int32 * L)(), (C.c_int32 * L)()
    _check(_lib.adpsgd_schedule(h, k, o, p, a))
    return list(o), list(p), list(a)


def adpsgd_schedule_of(pattern, seed, straggler_p, L, k):
    o, p, a = (C.c_int32 * L)(), (C.c_int32 * L)(), (C.c_int32 * L)()
    _check(_lib.adpsgd_schedule_of(pattern, seed, straggler_p, L, k, o, p, a))
    return list(o), list(p), list(a)


def adpsgd_lr_at_epoch(epoch, peak_lr, start_lr=0.0, warmup_epochs=0, hold_until_epoch=10):
    out = C.c_float(0.0)
    _check(_lib.adpsgd_lr_at_epoch(epoch, peak_lr, start_lr, warmup_epochs, hold_until_epoch, C.byref(out)))
    return out.value


def adpsgd_iteration(h):
    return _lib.adpsgd_iteration(h)


def adpsgd_average(h, dev_out_ptr):
    _check(_lib.adpsgd_average(h, dev_out_ptr))


def adpsgd_consensus(h):
    out = C.c_double(0.0)
    _check(_lib.adpsgd_consensus(h, C.byref(out)))
    return out.value


def adpsgd_consensus_static(dev_x_ptr, stride, L, P, dev_out_ptr, stream_ptr):
    _check(_lib.adpsgd_consensus_static(dev_x_ptr, stride, L, P, dev_out_ptr, stream_ptr))


def adpsgd_set_profiling(h, enable):
    _check(_lib.adpsgd_set_profiling(h, int(enable)))


def adpsgd_profile(h):
    n = len(PHASES)
    ms, cnt, work, nbytes = (C.c_float * n)(), (C.c_int32 * n)(), (C.c_double * n)(), (C.c_double * n)()
    _check(_lib.adpsgd_profile(h, ms, cnt, work, nbytes))
    return {PHASES[i]: {"ms": ms[i], "launches": cnt[i], "work": work[i], "bytes": nbytes[i]} for i in range(n)}


def adpsgd_set_tuning(h, key, value):
    _check(_lib.adpsgd_set_tuning(h, int(key), int(value)))


def adpsgd_probe_mfma(dev_out_ptr, blocks, iters, stream_ptr):
    _check(_lib.adpsgd_probe_mfma(dev_out_ptr, blocks, iters, stream_ptr))


def adpsgd_probe_stream(reads, writes_f32, writes_bf16, dev_buf_ptr, pitch_bytes, elems, stream_ptr):
    _check(_lib.adpsgd_probe_stream(reads, writes_f32, writes_bf16, dev_buf_ptr, pitch_bytes, elems, stream_ptr))


def adpsgd_status(h):
    _check(_lib.adpsgd_status(h))


def adpsgd_destroy(h):
    _lib.adpsgd_destroy(h)


def adpsgd_gemm(precision, a_kmajor, b_kmajor, c_is_elem, M, N, K, A, lda, strideA, B, ldb, strideB,
                Cp, ldc, strideC, bias, strideBias, groups, stream_ptr, tile_config=-1):
    _check(_lib.adpsgd_gemm(precision, a_kmajor, b_kmajor, c_is_elem, M, N, K, A, lda, strideA, B, ldb,
                            strideB, Cp, ldc, strideC, bias, strideBias, groups, tile_config, stream_ptr))


class Adpsgd:
    """Convenience owner of a handle and its torch-allocated workspace."""

    def __init__(self, cfg, device="cuda:0"):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.L = cfg.L
        self.device = torch.device(device)
        nbytes = adpsgd_workspace_bytes(cfg)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        self._off = (-base) % 256
        self.stream = torch.cuda.current_stream(self.device)
        self.h = adpsgd_create(cfg, base + self._off, nbytes, self.stream.cuda_stream)
        self.P = adpsgd_param_count(self.h)

    def _view(self, ptr, n):
        off = ptr - self.workspace.data_ptr()
        return self.workspace[off:off + 4 * n].view(self.torch.float32)

    def step(self, batch_tensors, lr, active=None):
        """batch_tensors: model mode [(feats, labels)] per learner; flat mode [grad] per learner.
        An entry may be None (a straggler's batch is not read)."""
        ptrs = []
        for b in batch_tensors:
            if isinstance(b, (tuple, list)):
                ptrs += [b[0].data_ptr() if b[0] is not None else None, b[1].data_ptr() if b[1] is not None else None]
            else:
                ptrs.append(b.data_ptr() if b is not None else None)
        if active is None:
            adpsgd_step(self.h, ptrs, lr)
        else:
            adpsgd_step_masked(self.h, ptrs, lr, active)

    def params(self, i):
        return self._view(adpsgd_params(self.h, i), self.P)

    def grads(self, i):
        return self._view(adpsgd_grads(self.h, i), self.P)

    def set_params(self, i, src):
        assert src.dtype == self.torch.float32 and src.numel() == self.P and src.is_contiguous()
        adpsgd_set_params(self.h, i, src.data_ptr())

    def losses(self):
        return adpsgd_losses(self.h, self.L)

    def schedule(self, k):
        return adpsgd_schedule(self.h, k, self.L)

    def average(self):
        out = self.torch.empty(self.P, dtype=self.torch.float32, device=self.device)
        adpsgd_average(self.h, out.data_ptr())
        return out

    def consensus(self):
        return adpsgd_consensus(self.h)

    def status(self):
        adpsgd_status(self.h)

    def tune(self, key, value):
        adpsgd_set_tuning(self.h, key, value)

    def capture_begin(self):
        adpsgd_capture_begin(self.h)

    def capture_end(self):
        """Returns the recording; replay it with adpsgd_graph_replay, free it with adpsgd_graph_destroy
        before close()."""
        return adpsgd_capture_end(self.h)

    def close(self):
        if self.h is not None:
            adpsgd_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
