"""Thin ctypes binding of libasd.so: same names as include/asd.h (the sampling
boundary) and include/asd_testing.h (test / profiling hooks), argument
marshalling only.  Every step of the sampling path runs in the HIP library;
PyTorch is used for device memory and streams."""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libasd.so")

ASD_OK, ASD_EINVAL, ASD_ENOMEM, ASD_EDEVICE, ASD_ESTATE, ASD_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
ASD_DEN_GMM, ASD_DEN_MLP = 1, 2
PROF = dict(MODEL=0, PLAN=1, GMM_ROWWISE=2, GMM_LOGITS=3, GMM_SOFTMAX=4, GMM_COMBINE=5, MLP_PACK=6, MLP_GEMM_IN=7,
            MLP_GEMM_BLK=8, MLP_GEMM_OUT=9, DRAFT=10, ACCEPT=11, GMM_SCREEN=12, GMM_CERT=13, ACCEPT_EARLY=14)


class AsdError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (status_string(status), message))
        self.status = status


class asd_schedule(C.Structure):
    _fields_ = [("K", C.c_int32), ("c_x", C.c_void_p), ("c_0", C.c_void_p), ("sigma", C.c_void_p),
                ("tau", C.c_void_p)]


class asd_denoiser(C.Structure):
    _fields_ = [("kind", C.c_int32), ("d", C.c_int32), ("n_tau", C.c_int32),
                ("C", C.c_int32), ("means", C.c_void_p), ("log_w", C.c_void_p), ("var", C.c_float),
                ("abar", C.c_void_p), ("sl_time", C.c_void_p),
                ("width", C.c_int32), ("n_blocks", C.c_int32), ("linears_per_block", C.c_int32),
                ("temb_dim", C.c_int32), ("out_clip", C.c_float), ("predict_eps", C.c_int32),
                ("act_terms", C.c_int32),
                ("w_in", C.c_void_p), ("w_blk", C.c_void_p), ("w_out", C.c_void_p),
                ("b_in", C.c_void_p), ("b_blk", C.c_void_p), ("b_out", C.c_void_p), ("temb", C.c_void_p)]


class asd_config(C.Structure):
    _fields_ = [("sched", asd_schedule), ("den", asd_denoiser), ("L", C.c_int32), ("chains", C.c_int32),
                ("seed", C.c_uint64)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libasd.so is not built: run `python -m paper_2505_03983_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32, u32, u64 = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64
        sig = {
            "asd_init": (i32, [C.POINTER(asd_config), C.POINTER(vp)]),
            "asd_destroy": (i32, [vp]),
            "asd_set_seed": (i32, [vp, u64]),
            "asd_draft": (i32, [vp, vp, vp, vp]),
            "asd_verify": (i32, [vp, vp, vp, vp, vp]),
            "asd_accept": (i32, [vp, vp, vp, vp, vp, vp, vp]),
            "asd_sample": (i32, [vp, vp, vp, vp, vp]),
            "asd_sample_noalloc": (i32, [vp, vp, vp, vp, vp]),
            "asd_sample_sequential": (i32, [vp, vp, vp, vp]),
            "asd_last_round_count": (i32, [vp]),
            "asd_use_graphs": (i32, [vp, i32]),
            "asd_use_resident": (i32, [vp, i32]),
            "asd_use_call_reuse": (i32, [vp, i32]),
            "asd_use_sparse_combine": (i32, [vp, i32]),
            "asd_use_logit_screen": (i32, [vp, i32]),
            "asd_logit_screen_active": (i32, [vp]),
            "asd_profile_model_work": (i32, [vp, vp, vp, vp, vp, vp, vp, vp]),
            "asd_use_tall_tiles": (i32, [vp, i32]),
            "asd_tall_tiles_active": (i32, [vp]),
            "asd_use_early_accept": (i32, [vp, i32]),
            "asd_early_accept_active": (i32, [vp]),
            "asd_profile_early_accept": (i32, [vp, vp, vp, vp, vp]),
            "asd_use_onehot_certificate": (i32, [vp, i32]),
            "asd_onehot_certificate_active": (i32, [vp]),
            "asd_use_adaptive_window": (i32, [vp, i32]),
            "asd_resident_active": (i32, [vp]),
            "asd_use_split_gemm": (i32, [vp, i32]),
            "asd_split_gemm_active": (i32, [vp]),
            "asd_denoise": (i32, [vp, vp, vp, i32, vp, vp]),
            "asd_profile_enable": (i32, [vp, i32]),
            "asd_profile_select": (i32, [vp, C.c_uint32]),
            "asd_profile_read": (i32, [vp, i32, i32, vp, vp]),
            "asd_profile_rows": (i32, [vp, vp, vp]),
            "asd_profile_accept_rows": (i32, [vp, vp, vp]),
            "asd_debug_philox": (i32, [u64, u32, u32, u32, i32, vp, vp]),
            "asd_debug_randoms": (i32, [u64, u32, u32, i32, vp, vp, vp]),
            "asd_schedule_ddpm_linear": (i32, [i32, C.c_double, C.c_double, vp, vp, vp, vp, vp]),
            "asd_schedule_from_abar": (i32, [i32, vp, vp, vp, vp, vp, vp]),
            "asd_abar_cosine": (i32, [i32, C.c_double, C.c_double, vp]),
            "asd_schedule_sl_euler": (i32, [i32, vp, vp, vp, vp, vp, vp]),
            "asd_status_string": (C.c_char_p, [i32]),
            "asd_last_error": (C.c_char_p, []),
        }
        for name, (res, args) in sig.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def status_string(s):
    return lib().asd_status_string(int(s)).decode()


def last_error():
    return lib().asd_last_error().decode()


def _check(s):
    if s != ASD_OK:
        raise AsdError(s, last_error())


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous()
        return t.data_ptr()
    if isinstance(t, np.ndarray):
        assert t.flags["C_CONTIGUOUS"]
        return t.ctypes.data
    return int(t)


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def asd_schedule_ddpm_linear(K, beta_min=1e-4, beta_max=0.02):
    """Host tables of the library: dict(c_x, c_0, sigma [K] f32; tau [K] i32; abar [K+1] f32)."""
    n = max(int(K), 0)
    out = dict(c_x=np.zeros(n, np.float32), c_0=np.zeros(n, np.float32), sigma=np.zeros(n, np.float32),
               tau=np.zeros(n, np.int32), abar=np.zeros(n + 1, np.float32))
    _check(lib().asd_schedule_ddpm_linear(int(K), float(beta_min), float(beta_max), _ptr(out["c_x"]),
                                          _ptr(out["c_0"]), _ptr(out["sigma"]), _ptr(out["tau"]),
                                          _ptr(out["abar"])))
    return out


def asd_schedule_from_abar(abar):
    """Host tables for a variance-preserving schedule given by abar[0..K] (float64)."""
    abar = np.ascontiguousarray(abar, dtype=np.float64)
    n = len(abar) - 1
    out = dict(c_x=np.zeros(max(n, 0), np.float32), c_0=np.zeros(max(n, 0), np.float32),
               sigma=np.zeros(max(n, 0), np.float32), tau=np.zeros(max(n, 0), np.int32),
               abar=np.zeros(max(n, 0) + 1, np.float32))
    _check(lib().asd_schedule_from_abar(n, _ptr(abar), _ptr(out["c_x"]), _ptr(out["c_0"]), _ptr(out["sigma"]),
                                        _ptr(out["tau"]), _ptr(out["abar"])))
    return out


def asd_schedule_sl_euler(t):
    """Host tables of the Euler chain on the SL process over times t[0..K] (float64); 'sl_time' is the fp32 copy."""
    t = np.ascontiguousarray(t, dtype=np.float64)
    n = max(len(t) - 1, 0)
    out = dict(c_x=np.zeros(n, np.float32), c_0=np.zeros(n, np.float32), sigma=np.zeros(n, np.float32),
               tau=np.zeros(n, np.int32), sl_time=np.zeros(n + 1, np.float32))
    _check(lib().asd_schedule_sl_euler(n, _ptr(t), _ptr(out["c_x"]), _ptr(out["c_0"]), _ptr(out["sigma"]),
                                       _ptr(out["tau"]), _ptr(out["sl_time"])))
    return out


def asd_abar_cosine(K, s=0.008, beta_clip=0.999):
    abar = np.zeros(max(int(K), 0) + 1, np.float64)
    _check(lib().asd_abar_cosine(int(K), float(s), float(beta_clip), _ptr(abar)))
    return abar


def make_config(sched, den, L, chains, seed):
    """sched: dict of host numpy tables; den: dict with 'kind' and parameters
    (device torch tensors for DEV fields, numpy for HOST fields).  Returns
    (asd_config, keepalive list)."""
    keep = []

    def host(a, dt):
        a = np.ascontiguousarray(a, dtype=dt)
        keep.append(a)
        return a.ctypes.data

    cfg = asd_config()
    cfg.sched.K = int(sched["K"]) if "K" in sched else len(sched["c_x"])
    cfg.sched.c_x = host(sched["c_x"], np.float32)
    cfg.sched.c_0 = host(sched["c_0"], np.float32)
    cfg.sched.sigma = host(sched["sigma"], np.float32)
    cfg.sched.tau = host(sched["tau"], np.int32)
    cfg.den.kind = ASD_DEN_GMM if den["kind"] == "gmm" else ASD_DEN_MLP if den["kind"] == "mlp" else int(den["kind"])
    cfg.den.d = int(den["d"])
    cfg.den.n_tau = int(den["n_tau"])
    if den["kind"] == "gmm":
        cfg.den.C = int(den["C"])
        cfg.den.means = _ptr(den["means"])
        cfg.den.log_w = _ptr(den["log_w"])
        cfg.den.var = float(den["var"])
        cfg.den.abar = host(den["abar"], np.float32) if den.get("abar") is not None else None
        cfg.den.sl_time = host(den["sl_time"], np.float32) if den.get("sl_time") is not None else None
    elif den["kind"] == "mlp":
        cfg.den.width = int(den["width"])
        cfg.den.n_blocks = int(den["n_blocks"])
        cfg.den.linears_per_block = int(den.get("linears_per_block", 1))
        cfg.den.temb_dim = int(den["temb_dim"])
        cfg.den.out_clip = float(den.get("out_clip", 0.0))
        cfg.den.predict_eps = int(bool(den.get("predict_eps", False)))
        cfg.den.act_terms = int(den.get("act_terms", 1))
        cfg.den.abar = host(den["abar"], np.float32) if den.get("abar") is not None else None
        for k in ("w_in", "w_blk", "w_out", "b_in", "b_blk", "b_out", "temb"):
            setattr(cfg.den, k, _ptr(den.get(k)))
    keep.append(den)
    cfg.L = int(L)
    cfg.chains = int(chains)
    cfg.seed = int(seed)
    return cfg, keep


class Ctx:
    """Owns an asd_ctx*; methods are the C entry points."""

    def __init__(self, sched, den, L, chains, seed=0):
        self.cfg, self._keep = make_config(sched, den, L, chains, seed)
        h = C.c_void_p()
        self._destroy = lib().asd_destroy
        _check(lib().asd_init(C.byref(self.cfg), C.byref(h)))
        self.h = h
        self.K, self.L, self.chains, self.d = self.cfg.sched.K, int(L), int(chains), self.cfg.den.d

    def close(self):
        h, self.h = getattr(self, "h", None), None
        if h:
            self._destroy(h)

    def __del__(self):
        # at interpreter exit module globals may already be gone: the destroy function was captured at
        # construction, and whatever still fails then is of no consequence
        try:
            self.close()
        except Exception:
            pass

    def use_graphs(self, on=True):
        _check(lib().asd_use_graphs(self.h, int(bool(on))))

    def use_adaptive_window(self, on=True):
        _check(lib().asd_use_adaptive_window(self.h, int(bool(on))))

    def use_call_reuse(self, on=True):
        _check(lib().asd_use_call_reuse(self.h, int(bool(on))))

    def use_sparse_combine(self, on=True):
        _check(lib().asd_use_sparse_combine(self.h, int(bool(on))))

    def use_logit_screen(self, mode=1):
        _check(lib().asd_use_logit_screen(self.h, int(mode)))

    def logit_screen_active(self):
        return int(lib().asd_logit_screen_active(self.h))

    def use_tall_tiles(self, on=True):
        _check(lib().asd_use_tall_tiles(self.h, int(bool(on))))

    def tall_tiles_active(self):
        return bool(lib().asd_tall_tiles_active(self.h))

    def use_early_accept(self, on=True):
        _check(lib().asd_use_early_accept(self.h, int(bool(on))))

    def early_accept_active(self):
        return bool(lib().asd_early_accept_active(self.h))

    def profile_early_accept(self):
        """(model rows the early accept kernel formed itself, chain-rounds it committed, rows of their windows, rows
        it resampled) since profile_enable."""
        v = [C.c_int64(0) for _ in range(4)]
        _check(lib().asd_profile_early_accept(self.h, *[C.addressof(x) for x in v]))
        return tuple(x.value for x in v)

    def use_onehot_certificate(self, on=True):
        _check(lib().asd_use_onehot_certificate(self.h, int(bool(on))))

    def onehot_certificate_active(self):
        return bool(lib().asd_onehot_certificate_active(self.h))

    def use_resident(self, on=True):
        _check(lib().asd_use_resident(self.h, int(bool(on))))

    def resident_active(self):
        return bool(lib().asd_resident_active(self.h))

    def use_split_gemm(self, on=True):
        _check(lib().asd_use_split_gemm(self.h, int(bool(on))))

    def split_gemm_active(self):
        return bool(lib().asd_split_gemm_active(self.h))

    def split_gemm_products(self):
        """16-bit matrix-core products per fp32 product of the split-operand kernels: 3 (fp16 terms), 6 (bf16), 0 (off)."""
        return int(lib().asd_split_gemm_active(self.h))

    def set_seed(self, seed):
        _check(lib().asd_set_seed(self.h, int(seed)))

    def draft(self, traj, a, stream=None):
        _check(lib().asd_draft(self.h, _ptr(traj), _ptr(a), _stream(stream)))

    def verify(self, traj, a, x0hat, stream=None):
        _check(lib().asd_verify(self.h, _ptr(traj), _ptr(a), _ptr(x0hat), _stream(stream)))

    def accept(self, traj, a, x0hat, accepted=None, stats=None, stream=None):
        _check(lib().asd_accept(self.h, _ptr(traj), _ptr(a), _ptr(x0hat), _ptr(accepted), _ptr(stats),
                                _stream(stream)))

    def sample(self, traj, rounds=None, y0=None, stream=None):
        _check(lib().asd_sample(self.h, _ptr(y0), _ptr(traj), _ptr(rounds), _stream(stream)))
        return lib().asd_last_round_count(self.h)

    def sample_noalloc(self, traj, rounds=None, y0=None, stream=None):
        _check(lib().asd_sample_noalloc(self.h, _ptr(y0), _ptr(traj), _ptr(rounds), _stream(stream)))
        return lib().asd_last_round_count(self.h)

    def sample_sequential(self, traj, y0=None, stream=None):
        _check(lib().asd_sample_sequential(self.h, _ptr(y0), _ptr(traj), _stream(stream)))

    def profile_enable(self, on=True):
        """on: False / True (the denoisers' kernels, draft, accept) / 2 (also whole model calls and row planning)."""
        _check(lib().asd_profile_enable(self.h, int(on)))

    def profile_select(self, slots=None):
        """slots: the scopes timed while profiling is on, as "KIND/draft" or "KIND/verify" with KIND from PROF
        (None: all)."""
        mask = 0xFFFFFFFF
        if slots is not None:
            mask = 0
            for s in slots:
                kind, call = s.split("/")
                mask |= 1 << (PROF[kind] + 16 * {"draft": 0, "verify": 1}[call])
        _check(lib().asd_profile_select(self.h, mask))

    def profile_read(self, kernel, call=0):
        n, ms = C.c_int64(0), C.c_double(0.0)
        _check(lib().asd_profile_read(self.h, int(kernel), int(call), C.addressof(n), C.addressof(ms)))
        return n.value, ms.value

    def profile_rows(self):
        a, b = C.c_int64(0), C.c_int64(0)
        _check(lib().asd_profile_rows(self.h, C.addressof(a), C.addressof(b)))
        return a.value, b.value

    def profile_model_work(self):
        """(logit tiles computed, logit tiles, combine slabs visited, combine slabs, logit tiles of screened calls,
        row tiles written in closed form, row tiles certified one-hot before any matrix work) of the verify calls."""
        v = [C.c_int64(0) for _ in range(7)]
        _check(lib().asd_profile_model_work(self.h, *[C.addressof(x) for x in v]))
        return tuple(x.value for x in v)

    def profile_accept_rows(self):
        a, b = C.c_int64(0), C.c_int64(0)
        _check(lib().asd_profile_accept_rows(self.h, C.addressof(a), C.addressof(b)))
        return a.value, b.value

    def denoise(self, x, tau, out, stream=None):
        _check(lib().asd_denoise(self.h, _ptr(x), _ptr(tau), int(x.shape[0]), _ptr(out), _stream(stream)))


def asd_debug_philox(seed, chain, step, stream_id, nblk, out, stream=None):
    _check(lib().asd_debug_philox(int(seed), int(chain), int(step), int(stream_id), int(nblk), _ptr(out),
                                  _stream(stream)))


def asd_debug_randoms(seed, chain, step, d, xi, u, stream=None):
    _check(lib().asd_debug_randoms(int(seed), int(chain), int(step), int(d), _ptr(xi), _ptr(u), _stream(stream)))
