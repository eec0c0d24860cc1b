"""ctypes binding of libpoplar (include/poplar.h).  Argument marshalling only.

Functions carry the C names without the `poplar_` prefix.  Device arguments
are torch tensors on the GPU (only their data_ptr() is handed over) or raw
integer addresses; host arguments are Python numbers and lists.  A non-zero
status raises PoplarError with the library's message.  The library must have
been built (python -m paper_2408_12596_amd.build); there is no fallback.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpoplar.so")

OK, ERR_INVALID, ERR_OOM, ERR_HIP, ERR_UNIMPLEMENTED = 0, -1, -2, -3, -4
ARCH_GPT, ARCH_LLAMA = 0, 1
GEMM_NT, GEMM_NN, GEMM_TN = 0, 1, 2
F32, BF16 = 0, 1
(T_G1, T_B1, T_WQKV, T_BQKV, T_WO, T_BO, T_G2, T_B2, T_W1, T_BM1, T_W2, T_BM2) = range(12)
T_WTE, T_WPE, T_GF, T_BF, T_WHEAD = 100, 101, 102, 103, 104


class PoplarError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"poplar status {status}: {msg}")
        self.status = status


class OutOfMemory(PoplarError):
    pass


class ModelCfg(C.Structure):
    _fields_ = [("arch", C.c_int32), ("n_layer", C.c_int32), ("hidden", C.c_int32), ("n_head", C.c_int32),
                ("ffn", C.c_int32), ("seq", C.c_int32), ("vocab", C.c_int32), ("dtype", C.c_int32),
                ("world", C.c_int32), ("rank", C.c_int32), ("zero_stage", C.c_int32), ("causal", C.c_int32),
                ("cap_bytes", C.c_int64), ("checkpoint", C.c_int32), ("deterministic", C.c_int32)]


class State(C.Structure):
    _fields_ = [("params", C.c_void_p), ("own_shard", C.c_void_p), ("master", C.c_void_p), ("m", C.c_void_p),
                ("v", C.c_void_p), ("grads", C.c_void_p), ("master_len", C.c_int64), ("grads_len", C.c_int64), ("own_len", C.c_int64),
                ("tokens", C.c_void_p), ("max_batch", C.c_int32),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_int64), ("loss", C.c_void_p),
                ("adam_t", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("targets", C.c_void_p)]


class Profile(C.Structure):
    _fields_ = [("stage", C.c_int32), ("batch", C.c_int32), ("t_fwd", C.c_double), ("t_bwd", C.c_double),
                ("t_gather_fwd", C.c_double), ("t_gather_bwd", C.c_double), ("t_reduce_bwd", C.c_double),
                ("t_adam", C.c_double), ("t_consumed", C.c_double), ("accounted_bytes", C.c_int64),
                ("flops", C.c_double), ("loss", C.c_float), ("t_gemm", C.c_double), ("gemm_flops", C.c_double),
                ("t_attn", C.c_double), ("attn_flops", C.c_double), ("n_gemm", C.c_int32), ("n_attn", C.c_int32),
                ("measured_bytes", C.c_int64), ("n_gemm_kernels", C.c_int32), ("reduce_elems", C.c_int64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_void_p, C.c_int64)
RELEASE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)
BYTES_FN = C.CFUNCTYPE(C.c_int64, C.c_void_p)


class MemHooks(C.Structure):
    _fields_ = [("user", C.c_void_p), ("alloc", ALLOC_FN), ("release", RELEASE_FN), ("bytes_now", BYTES_FN), ("bytes_total", BYTES_FN)]


class Curve(C.Structure):
    _fields_ = [("n_pts", C.c_int32), ("batch", C.POINTER(C.c_int32)), ("time", C.POINTER(C.c_double)), ("mbs", C.c_int32)]


class Alloc(C.Structure):
    _fields_ = [("gmbs", C.POINTER(C.c_int32)), ("b", C.POINTER(C.c_int32)), ("gas", C.POINTER(C.c_int32)),
                ("lbs", C.POINTER(C.c_int32)), ("T", C.c_double), ("t", C.c_double), ("T_steps", C.c_double)]


EXPORTS = [
    "poplar_last_error", "poplar_create", "poplar_destroy", "poplar_layer_param_count", "poplar_model_param_count",
    "poplar_param_offset", "poplar_shard_range", "poplar_layer_saved_bytes", "poplar_layer_workspace_bytes",
    "poplar_layer_fwd", "poplar_layer_bwd", "poplar_embed_fwd", "poplar_embed_bwd", "poplar_head_workspace_bytes",
    "poplar_head_loss_fwd_bwd", "poplar_adam_shard", "poplar_zero2_reduce_local", "poplar_zero3_gather_local",
    "poplar_bind_state", "poplar_step_workspace_bytes", "poplar_step_accounted_bytes", "poplar_profile_step",
    "poplar_accum_step", "poplar_search_mbs", "poplar_search_stage", "poplar_comm_model", "poplar_speed_curve", "poplar_allocate", "poplar_set_kernel_timing", "poplar_device_info",
    "poplar_gemm", "poplar_set_sampling", "poplar_set_mem_hooks", "poplar_step_forward_bytes",
    "poplar_layer_bwd_static", "poplar_static_scratch_bytes",
]

_lib = None


def lib():
    """The loaded library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2408_12596_amd.build`")
        _lib = C.CDLL(LIB_PATH)
        _declare(_lib)
    return _lib


def _declare(L):
    """Argument types of every entry point, so that 64-bit values and pointers are never truncated."""
    vp, i32, i64, f32, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_double
    cfgp, p64 = C.POINTER(ModelCfg), C.POINTER(C.c_int64)
    sig = {
        "poplar_create": [cfgp, vp, C.POINTER(vp)],
        "poplar_destroy": [vp],
        "poplar_layer_param_count": [cfgp, p64],
        "poplar_model_param_count": [cfgp, p64],
        "poplar_param_offset": [cfgp, i32, i32, p64, p64, p64],
        "poplar_shard_range": [i64, i32, i32, p64, p64, p64],
        "poplar_layer_saved_bytes": [cfgp, i32, p64],
        "poplar_layer_workspace_bytes": [cfgp, i32, p64],
        "poplar_layer_fwd": [vp, i32, vp, vp, vp, vp, vp, i64],
        "poplar_layer_bwd": [vp, i32, vp, vp, vp, vp, vp, vp, i32, vp, i64],
        "poplar_layer_bwd_static": [vp, i32, vp, vp, vp, vp, vp, vp, i32],
        "poplar_static_scratch_bytes": [p64],
        "poplar_embed_fwd": [vp, i32, vp, vp, vp, vp],
        "poplar_embed_bwd": [vp, i32, vp, vp, vp, vp, i32],
        "poplar_head_workspace_bytes": [cfgp, i32, p64],
        "poplar_head_loss_fwd_bwd": [vp, i32, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, i32, vp, i64],
        "poplar_adam_shard": [vp, vp, vp, vp, vp, vp, i64, i32, f32, f32, f32, f32],
        "poplar_zero2_reduce_local": [vp, vp, vp, i64, i64, i64, i64],
        "poplar_zero3_gather_local": [vp, vp, vp, vp, i64, i64, i64, i64],
        "poplar_bind_state": [vp, C.POINTER(State)],
        "poplar_step_workspace_bytes": [cfgp, i32, i32, p64],
        "poplar_step_accounted_bytes": [cfgp, i32, i32, i32, p64],
        "poplar_step_forward_bytes": [cfgp, i32, i32, p64],
        "poplar_profile_step": [vp, i32, i32, C.POINTER(Profile)],
        "poplar_accum_step": [vp, i32, i32, C.POINTER(i32), i32, C.POINTER(Profile)],
        "poplar_search_mbs": [vp, i32, C.POINTER(i32), C.POINTER(Profile), i32, C.POINTER(i32)],
        "poplar_search_stage": [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(Profile), i32, C.POINTER(i32)],
        "poplar_set_kernel_timing": [vp, i32],
        "poplar_set_sampling": [vp, i32, i32],
        "poplar_set_mem_hooks": [vp, C.POINTER(MemHooks)],
        "poplar_device_info": [C.POINTER(i32), C.POINTER(i32), C.POINTER(i64)],
        "poplar_gemm": [vp, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, f32],
        "poplar_comm_model": [i64, i32, i32, f64, f64, f64] + [C.POINTER(f64)] * 5,
        "poplar_speed_curve": [C.POINTER(Curve), C.POINTER(f64)],
        "poplar_allocate": [i32, i32, C.POINTER(Curve), i64, f64, f64, C.POINTER(Alloc)],
    }
    L.poplar_last_error.restype = C.c_char_p
    L.poplar_last_error.argtypes = []
    for name, args in sig.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = C.c_int


def _check(status):
    if status != OK:
        msg = lib().poplar_last_error().decode()
        raise (OutOfMemory if status == ERR_OOM else PoplarError)(status, msg)


def _ptr(t):
    """Device address of a torch tensor, a raw address, or NULL."""
    if t is None:
        return C.c_void_p(0)
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def make_cfg(arch="gpt", L=1, H=256, nh=4, F=1024, S=128, V=1, dtype="bf16", world=1, rank=0, zero_stage=1,
             causal=True, cap_bytes=0, checkpoint=False, deterministic=False):
    return ModelCfg(ARCH_GPT if arch == "gpt" else ARCH_LLAMA, L, H, nh, F, S, V, BF16 if dtype == "bf16" else F32,
                    world, rank, zero_stage, int(causal), cap_bytes, int(checkpoint), int(deterministic))


# ---- host-only queries --------------------------------------------------------
def layer_param_count(cfg):
    n = C.c_int64()
    _check(lib().poplar_layer_param_count(C.byref(cfg), C.byref(n)))
    return n.value


def model_param_count(cfg):
    n = C.c_int64()
    _check(lib().poplar_model_param_count(C.byref(cfg), C.byref(n)))
    return n.value


def param_offset(cfg, layer, tensor_id):
    off, r, c = C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib().poplar_param_offset(C.byref(cfg), layer, tensor_id, C.byref(off), C.byref(r), C.byref(c)))
    return off.value, r.value, c.value


_GPT_LAYER = [("g1", T_G1), ("b1", T_B1), ("Wqkv", T_WQKV), ("bqkv", T_BQKV), ("Wo", T_WO), ("bo", T_BO),
              ("g2", T_G2), ("b2", T_B2), ("W1", T_W1), ("bm1", T_BM1), ("W2", T_W2), ("bm2", T_BM2)]
_LLAMA_LAYER = [("g1", T_G1), ("Wqkv", T_WQKV), ("Wo", T_WO), ("g2", T_G2), ("Wgu", T_W1), ("Wd", T_W2)]


def model_spec(cfg):
    """[(name, shape, offset)] of every tensor in flat order, from the library's own layout."""
    gpt = cfg.arch == ARCH_GPT
    out = []

    def add(name, layer, tid):
        off, r, c = param_offset(cfg, layer, tid)
        out.append((name, (r,) if c == 1 and tid not in (T_WQKV, T_WO, T_W1, T_W2, T_WTE, T_WPE, T_WHEAD) else (r, c), off))

    add("wte", 0, T_WTE)
    if gpt:
        add("wpe", 0, T_WPE)
    for l in range(cfg.n_layer):
        for name, tid in (_GPT_LAYER if gpt else _LLAMA_LAYER):
            add(f"l{l}.{name}", l, tid)
    add("gf", 0, T_GF)
    if gpt:
        add("bf", 0, T_BF)
    else:
        add("Whead", 0, T_WHEAD)
    return out


def shard_range(P, N, r):
    off, ln, valid = C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib().poplar_shard_range(P, N, r, C.byref(off), C.byref(ln), C.byref(valid)))
    return off.value, ln.value, valid.value


def _bytes_query(fn, cfg, *args):
    n = C.c_int64()
    _check(fn(C.byref(cfg), *args, C.byref(n)))
    return n.value


def layer_saved_bytes(cfg, B):
    return _bytes_query(lib().poplar_layer_saved_bytes, cfg, B)


def layer_workspace_bytes(cfg, B):
    return _bytes_query(lib().poplar_layer_workspace_bytes, cfg, B)


def head_workspace_bytes(cfg, B):
    return _bytes_query(lib().poplar_head_workspace_bytes, cfg, B)


def step_workspace_bytes(cfg, stage, B):
    return _bytes_query(lib().poplar_step_workspace_bytes, cfg, stage, B)


def step_forward_bytes(cfg, stage, B):
    return _bytes_query(lib().poplar_step_forward_bytes, cfg, stage, B)


def step_accounted_bytes(cfg, stage, B, forward_only=False):
    return _bytes_query(lib().poplar_step_accounted_bytes, cfg, stage, B, int(forward_only))


def static_scratch_bytes():
    n = C.c_int64()
    _check(lib().poplar_static_scratch_bytes(C.byref(n)))
    return n.value


def device_info():
    cu, khz, mem = C.c_int32(), C.c_int32(), C.c_int64()
    _check(lib().poplar_device_info(C.byref(cu), C.byref(khz), C.byref(mem)))
    return dict(compute_units=cu.value, clock_khz=khz.value, memory_bytes=mem.value)


def comm_model(P, world, stage, param_bytes, grad_bytes, bytes_per_second):
    out = [C.c_double() for _ in range(5)]
    _check(lib().poplar_comm_model(P, world, stage, param_bytes, grad_bytes, bytes_per_second, *[C.byref(x) for x in out]))
    keys = ("micro_bytes", "step_bytes", "total_micro_elements", "t_micro", "t_step")
    return {k: x.value for k, x in zip(keys, out)}


def speed_curve(batches, times, mbs):
    n = len(batches)
    b = (C.c_int32 * n)(*batches)
    t = (C.c_double * n)(*times)
    out = (C.c_double * (mbs + 1))()
    cv = Curve(n, b, t, mbs)
    _check(lib().poplar_speed_curve(C.byref(cv), out))
    return list(out)


def allocate(stage, gbs, curves, time_communication=0.0, peak_frac=0.95):
    """curves: list of (batches, times, mbs).  Returns dict(gmbs, b, gas, lbs, T, t, T_steps)."""
    n = len(curves)
    keep = []
    arr = (Curve * n)()
    for i, (bs, ts, mbs) in enumerate(curves):
        b = (C.c_int32 * len(bs))(*bs)
        t = (C.c_double * len(ts))(*ts)
        keep += [b, t]
        arr[i] = Curve(len(bs), b, t, mbs)
    outs = [(C.c_int32 * n)() for _ in range(4)]
    al = Alloc(*outs, 0.0, 0.0, 0.0)
    _check(lib().poplar_allocate(stage, n, arr, C.c_int64(gbs), C.c_double(time_communication), C.c_double(peak_frac), C.byref(al)))
    return dict(gmbs=list(outs[0]), b=list(outs[1]), gas=list(outs[2]), lbs=list(outs[3]), T=al.T, t=al.t, T_steps=al.T_steps)


# ---- context ---------------------------------------------------------------------
class Context:
    """poplar_ctx bound to a HIP stream (an integer handle; 0 = default stream)."""

    def __init__(self, cfg, stream=0):
        self.cfg = cfg
        self._h = C.c_void_p()
        _check(lib().poplar_create(C.byref(cfg), C.c_void_p(stream), C.byref(self._h)))
        self._state_refs = None

    def close(self):
        if self._h:
            lib().poplar_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def layer_fwd(self, B, x_in, params, x_out, saved, workspace=None, workspace_bytes=0):
        _check(lib().poplar_layer_fwd(self._h, B, _ptr(x_in), _ptr(params), _ptr(x_out), _ptr(saved), _ptr(workspace), C.c_int64(workspace_bytes)))

    def layer_bwd(self, B, x_in, dy, params, saved, dx, grads, accumulate, workspace, workspace_bytes):
        _check(lib().poplar_layer_bwd(self._h, B, _ptr(x_in), _ptr(dy), _ptr(params), _ptr(saved), _ptr(dx), _ptr(grads),
                                      int(accumulate), _ptr(workspace), C.c_int64(workspace_bytes)))

    def layer_bwd_static(self, B, x_in, dy, params, saved, dx, grads, accumulate):
        _check(lib().poplar_layer_bwd_static(self._h, B, _ptr(x_in), _ptr(dy), _ptr(params), _ptr(saved), _ptr(dx), _ptr(grads),
                                             int(accumulate)))

    def gemm(self, layout, M, N, K, A, lda, B, ldb, C, ldc, c_float=False, beta=0.0):
        _check(lib().poplar_gemm(self._h, layout, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, int(c_float), beta))

    def embed_fwd(self, B, tokens, wte, wpe, x):
        _check(lib().poplar_embed_fwd(self._h, B, _ptr(tokens), _ptr(wte), _ptr(wpe), _ptr(x)))

    def embed_bwd(self, B, tokens, dx, dwte, dwpe, accumulate):
        _check(lib().poplar_embed_bwd(self._h, B, _ptr(tokens), _ptr(dx), _ptr(dwte), _ptr(dwpe), int(accumulate)))

    def head_loss_fwd_bwd(self, B, x, targets, gf, bf, whead, loss_scale, loss, dx, d_gf, d_bf, d_whead, accumulate,
                          workspace, workspace_bytes):
        _check(lib().poplar_head_loss_fwd_bwd(self._h, B, _ptr(x), _ptr(targets), _ptr(gf), _ptr(bf), _ptr(whead),
                                              C.c_float(loss_scale), _ptr(loss), _ptr(dx), _ptr(d_gf), _ptr(d_bf), _ptr(d_whead),
                                              int(accumulate), _ptr(workspace), C.c_int64(workspace_bytes)))

    def adam_shard(self, p32, m, v, g, p_lowp, n, step_t, lr, b1, b2, eps):
        _check(lib().poplar_adam_shard(self._h, _ptr(p32), _ptr(m), _ptr(v), _ptr(g), _ptr(p_lowp), C.c_int64(n), step_t,
                                       C.c_float(lr), C.c_float(b1), C.c_float(b2), C.c_float(eps)))

    def zero2_reduce_local(self, gshard, g_unit, unit_lo, unit_hi, shard_off, shard_len):
        _check(lib().poplar_zero2_reduce_local(self._h, _ptr(gshard), _ptr(g_unit), C.c_int64(unit_lo), C.c_int64(unit_hi),
                                               C.c_int64(shard_off), C.c_int64(shard_len)))

    def zero3_gather_local(self, out, own_shard, peers, lo, hi, shard_off, shard_len):
        _check(lib().poplar_zero3_gather_local(self._h, _ptr(out), _ptr(own_shard), _ptr(peers), C.c_int64(lo), C.c_int64(hi),
                                               C.c_int64(shard_off), C.c_int64(shard_len)))

    def bind_state(self, params, master, m, v, grads, tokens, max_batch, workspace, workspace_bytes, loss,
                   own_shard=None, adam_t=1, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, targets=None,
                   master_len=None, grads_len=None, own_len=None):
        """master_len / grads_len / own_len: elements allocated; read off the tensors when not given (raw addresses need them)."""
        def count(t, given):
            if given is not None:
                return given
            if t is None:
                return 0
            if isinstance(t, int):
                raise ValueError("a raw address needs its element count")
            return t.numel()
        mlen = min(count(master, master_len), count(m, master_len), count(v, master_len))
        st = State(_ptr(params), _ptr(own_shard), _ptr(master), _ptr(m), _ptr(v), _ptr(grads), mlen, count(grads, grads_len),
                   count(own_shard, own_len), _ptr(tokens), max_batch,
                   _ptr(workspace), workspace_bytes, _ptr(loss), adam_t, lr, beta1, beta2, eps, _ptr(targets))
        _check(lib().poplar_bind_state(self._h, C.byref(st)))
        self._state_refs = (params, master, m, v, grads, tokens, workspace, loss, own_shard, targets)  # keep the tensors alive

    def set_sampling(self, warmup, repeats):
        _check(lib().poplar_set_sampling(self._h, int(warmup), int(repeats)))

    def set_mem_hooks(self, alloc=None, release=None, bytes_now=None, bytes_total=None):
        """Python callables alloc(bytes) -> address or 0, release(address), bytes_now() -> int, bytes_total() -> int;
        all None removes the hooks."""
        if alloc is None:
            _check(lib().poplar_set_mem_hooks(self._h, None))
            self._hooks = None
            return
        hooks = MemHooks(None, ALLOC_FN(lambda user, n: alloc(n) or None), RELEASE_FN(lambda user, p: release(p)),
                         BYTES_FN(lambda user: bytes_now()), BYTES_FN(lambda user: bytes_total()))
        _check(lib().poplar_set_mem_hooks(self._h, C.byref(hooks)))
        self._hooks = hooks   # the callbacks must outlive their use

    def set_kernel_timing(self, on):
        _check(lib().poplar_set_kernel_timing(self._h, int(on)))

    def profile_step(self, stage, local_batch):
        out = Profile()
        _check(lib().poplar_profile_step(self._h, stage, local_batch, C.byref(out)))
        return out.as_dict()

    def accum_step(self, stage, micro_batches, loss_batch):
        arr = (C.c_int32 * len(micro_batches))(*micro_batches)
        out = Profile()
        _check(lib().poplar_accum_step(self._h, stage, len(micro_batches), arr, loss_batch, C.byref(out)))
        return out.as_dict()

    def search_stage(self, first_stage, max_samples=64):
        stage, mbs, n = C.c_int32(), C.c_int32(), C.c_int32()
        arr = (Profile * max_samples)()
        _check(lib().poplar_search_stage(self._h, first_stage, C.byref(stage), C.byref(mbs), arr, max_samples, C.byref(n)))
        return stage.value, mbs.value, [arr[i].as_dict() for i in range(n.value)]

    def search_mbs(self, stage, max_samples=64):
        mbs, n = C.c_int32(), C.c_int32()
        arr = (Profile * max_samples)()
        _check(lib().poplar_search_mbs(self._h, stage, C.byref(mbs), arr, max_samples, C.byref(n)))
        return mbs.value, [arr[i].as_dict() for i in range(n.value)]
