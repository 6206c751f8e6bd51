"""ctypes binding of libdeer (see include/deer.h).  Argument marshalling only: every step of the
path runs in the library's HIP kernels.  torch is used for device memory and the stream."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libdeer.so")

DEER_TARGET, DEER_DRAFTER = 0, 1
DEER_F32, DEER_BF16 = 0, 1
TENSOR_IDS = {"embed": 1, "lm_head": 2, "wq": 3, "wk": 4, "wv": 5, "wo": 6, "wg": 7, "wu": 8, "wd": 9, "router": 10}
STATUS = {0: "DEER_OK", -1: "DEER_EINVAL", -2: "DEER_ESTATE", -3: "DEER_ECAPACITY", -4: "DEER_EHIP", -5: "DEER_EVERSION"}
EXPORTS = ["deer_query_sizes", "deer_init_models", "deer_load_tensor", "deer_prefill", "deer_set_prefilled",
           "deer_draft_block", "deer_verify_block", "deer_accept_and_commit", "deer_accept_and_commit_static", "deer_destroy", "deer_last_error",
           "deer_debug_get_logits", "deer_get_lengths", "deer_get_kv_layout", "deer_debug_profile",
           "deer_debug_profile_read", "deer_debug_force_commit", "deer_debug_load_kv", "deer_set_bonus_token",
           "deer_draft_block_multipass", "deer_debug_gemm_tiled",
           "deer_debug_gemm_stamps", "deer_debug_experts_streamed", "deer_debug_route_spread",
           "deer_debug_stream_read"]


class DeerError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status


class ModelCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ff", "vocab",
                                          "n_experts", "top_k", "d_ff_expert")] + [("rope_base", C.c_float), ("rms_eps", C.c_float)]


class InitParams(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("abi_version", C.c_uint32), ("target", ModelCfg), ("drafter", ModelCfg),
                ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("max_k", C.c_int32), ("mask_token_id", C.c_int32),
                ("eos_token_id", C.c_int32), ("keep_logits", C.c_int32), ("device", C.c_int32), ("hip_stream", C.c_void_p)]


class Sizes(C.Structure):
    _fields_ = [("weights", C.c_size_t * 2), ("kv", C.c_size_t * 2), ("workspace", C.c_size_t), ("staging", C.c_size_t)]


class Buffers(C.Structure):
    _fields_ = [("weights", C.c_void_p * 2), ("kv", C.c_void_p * 2), ("workspace", C.c_void_p)]


class KvLayout(C.Structure):
    _fields_ = [("k_base", C.c_size_t), ("v_base", C.c_size_t), ("layer_stride", C.c_size_t), ("seq_stride", C.c_size_t),
                ("head_stride", C.c_size_t), ("max_seq", C.c_int32), ("head_dim", C.c_int32)]


_lib = None


def load_library(path: str = LIB_PATH):
    """Loads libdeer.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2512_15176_amd.build` "
                                "(there is no CPU or PyTorch fallback)")
    lib = C.CDLL(path)
    for name in EXPORTS:
        getattr(lib, name)
    lib.deer_last_error.restype = C.c_char_p
    lib.deer_last_error.argtypes = [C.c_void_p]
    lib.deer_query_sizes.argtypes = [C.POINTER(InitParams), C.POINTER(Sizes)]
    lib.deer_init_models.argtypes = [C.POINTER(InitParams), C.POINTER(Buffers), C.POINTER(Sizes), C.POINTER(C.c_void_p)]
    lib.deer_load_tensor.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int64, C.c_int64]
    lib.deer_prefill.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.deer_set_prefilled.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.deer_draft_block.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_uint64, C.c_void_p]
    lib.deer_draft_block_multipass.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_uint64, C.c_int32, C.c_void_p]
    lib.deer_verify_block.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_void_p]
    lib.deer_accept_and_commit.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.deer_accept_and_commit_static.argtypes = lib.deer_accept_and_commit.argtypes
    lib.deer_destroy.argtypes = [C.c_void_p]
    lib.deer_debug_route_spread.argtypes = [C.c_void_p, C.c_int]
    lib.deer_debug_experts_streamed.argtypes = [C.c_void_p, C.c_void_p]
    lib.deer_debug_stream_read.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_float)]
    lib.deer_debug_gemm_stamps.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int32, C.c_void_p]
    lib.deer_set_bonus_token.argtypes = [C.c_void_p, C.c_int]
    lib.deer_debug_get_logits.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_size_t]
    lib.deer_get_lengths.argtypes = [C.c_void_p, C.c_void_p]
    lib.deer_get_kv_layout.argtypes = [C.c_void_p, C.c_int, C.POINTER(KvLayout)]
    lib.deer_debug_profile.argtypes = [C.c_void_p, C.c_int]
    lib.deer_debug_force_commit.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
    lib.deer_debug_load_kv.argtypes = [C.c_void_p, C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.deer_debug_gemm_tiled.argtypes = [C.c_void_p, C.c_int]
    lib.deer_debug_profile_read.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    _lib = lib
    return lib


def model_cfg(shape) -> ModelCfg:
    """shape: any object with the ModelShape fields (see deer_inputs.ModelShape)."""
    return ModelCfg(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff,
                    shape.vocab, shape.n_experts, shape.top_k, shape.d_ff_expert, shape.rope_base, shape.rms_eps)


def init_params(target, drafter, max_batch, max_seq, max_k, mask_token_id, eos_token_id=-1, keep_logits=False,
                device=0, stream=0) -> InitParams:
    return InitParams(C.sizeof(InitParams), 1, model_cfg(target), model_cfg(drafter), max_batch, max_seq, max_k,
                      mask_token_id, eos_token_id, int(keep_logits), device, stream)


def query_sizes(params: InitParams) -> Sizes:
    lib = load_library()
    s = Sizes()
    rc = lib.deer_query_sizes(C.byref(params), C.byref(s))
    if rc:
        raise DeerError(rc, lib.deer_last_error(None).decode())
    return s


class DeerEngine:
    """Owns the device buffers (torch tensors) and a libdeer context.  Method names follow the C ABI."""

    def __init__(self, target, drafter, max_batch, max_seq, max_k, mask_token_id, eos_token_id=-1, keep_logits=False,
                 device=0):
        import torch
        self.torch = torch
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("DeerEngine needs a GPU: libdeer has no CPU path")
        self.device = torch.device("cuda", device)
        torch.cuda.set_device(self.device)
        self.target, self.drafter = target, drafter
        self.max_batch, self.max_seq, self.max_k = max_batch, max_seq, max_k
        stream = torch.cuda.current_stream(self.device).cuda_stream
        self.params = init_params(target, drafter, max_batch, max_seq, max_k, mask_token_id, eos_token_id, keep_logits,
                                  device, stream)
        self.sizes = query_sizes(self.params)
        alloc = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device=self.device)
        self._weights = [alloc(self.sizes.weights[i]) for i in range(2)]
        self._kv = [alloc(self.sizes.kv[i]) for i in range(2)]
        self._workspace = alloc(self.sizes.workspace)
        bufs = Buffers((C.c_void_p * 2)(*[t.data_ptr() for t in self._weights]),
                       (C.c_void_p * 2)(*[t.data_ptr() for t in self._kv]), self._workspace.data_ptr())
        ctx = C.c_void_p()
        rc = self.lib.deer_init_models(C.byref(self.params), C.byref(bufs), C.byref(self.sizes), C.byref(ctx))
        if rc:
            raise DeerError(rc, self.lib.deer_last_error(None).decode())
        self.ctx = ctx
        self.batch = 0
        self.bonus = 0
        self._draft = torch.zeros(max_batch * 32, dtype=torch.int32, device=self.device)

    # -- helpers ---------------------------------------------------------------------------------
    def _check(self, rc):
        if rc:
            raise DeerError(rc, self.lib.deer_last_error(self.ctx).decode())

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.deer_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights ---------------------------------------------------------------------------------
    def load_tensor(self, model, name, layer, expert, array):
        """array: numpy float32 (canonical values) or uint16 (bf16 bit patterns), [rows][cols]; or a
        contiguous torch device tensor (float32 / bfloat16) that is already resident."""
        torch = self.torch
        if isinstance(array, torch.Tensor):
            assert array.is_cuda and array.is_contiguous() and array.dim() == 2
            dt = {torch.float32: DEER_F32, torch.bfloat16: DEER_BF16}[array.dtype]
            self._check(self.lib.deer_load_tensor(self.ctx, model, TENSOR_IDS[name], layer, expert, array.data_ptr(), dt,
                                                  array.shape[0], array.shape[1]))
            torch.cuda.current_stream(self.device).synchronize()
            return
        a = np.ascontiguousarray(array)
        if a.dtype == np.uint16:
            dev = torch.from_numpy(a.view(np.int16)).to(self.device)
            dt = DEER_BF16
        elif a.dtype == np.float32:
            dev = torch.from_numpy(a).to(self.device)
            dt = DEER_F32
        else:
            raise TypeError("weights must be float32 values or uint16 bf16 bit patterns")
        self._check(self.lib.deer_load_tensor(self.ctx, model, TENSOR_IDS[name], layer, expert, dev.data_ptr(), dt,
                                              a.shape[0], a.shape[1]))
        torch.cuda.current_stream(self.device).synchronize()   # dev is freed on return

    def load_model(self, model, shape, provider):
        """provider(name, layer, expert) -> numpy array as accepted by load_tensor."""
        self.load_tensor(model, "embed", -1, -1, provider("embed", -1, -1))
        self.load_tensor(model, "lm_head", -1, -1, provider("lm_head", -1, -1))
        for l in range(shape.n_layers):
            for name in ("wq", "wk", "wv", "wo"):
                self.load_tensor(model, name, l, -1, provider(name, l, -1))
            if shape.n_experts:
                self.load_tensor(model, "router", l, -1, provider("router", l, -1))
            for e in (range(shape.n_experts) if shape.n_experts else [-1]):
                for name in ("wg", "wu", "wd"):
                    self.load_tensor(model, name, l, e, provider(name, l, e))

    # -- the path --------------------------------------------------------------------------------
    def prefill(self, prompts):
        lens = np.array([len(p) for p in prompts], dtype=np.int32)
        ids = np.ascontiguousarray(np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts]))
        self._check(self.lib.deer_prefill(self.ctx, len(prompts), ids.ctypes.data, lens.ctypes.data))
        self.batch = len(prompts)

    def set_prefilled(self, lens, last_tokens):
        lens = np.ascontiguousarray(lens, dtype=np.int32)
        last = np.ascontiguousarray(last_tokens, dtype=np.int32)
        self._check(self.lib.deer_set_prefilled(self.ctx, len(lens), lens.ctypes.data, last.ctypes.data))
        self.batch = len(lens)

    def draft_block(self, k, T=0.0, seed=0):
        """Returns the device tensor [batch][k] (int32) of drafted tokens."""
        self._check(self.lib.deer_draft_block(self.ctx, k, T, seed, self._draft.data_ptr()))
        return self._draft[: self.batch * k].view(self.batch, k)

    def draft_block_multipass(self, k, T=0.0, seed=0, n_passes=1):
        """As draft_block, in n_passes drafter passes over a block that is filled in from the left."""
        self._check(self.lib.deer_draft_block_multipass(self.ctx, k, T, seed, n_passes, self._draft.data_ptr()))
        return self._draft[: self.batch * k].view(self.batch, k)

    def verify_block(self, k, T, draft_dev):
        assert draft_dev.is_cuda and draft_dev.dtype == self.torch.int32 and draft_dev.is_contiguous()
        self._verify_arg = draft_dev   # keep alive until accept
        self._check(self.lib.deer_verify_block(self.ctx, k, T, draft_dev.data_ptr()))

    def set_bonus_token(self, enable):
        self._check(self.lib.deer_set_bonus_token(self.ctx, int(bool(enable))))
        self.bonus = int(bool(enable))

    def accept_and_commit(self, k, T=0.0, seed=0, static=False):
        """static=True: the entry point whose kernel scratch is the library's static device array."""
        acc = np.zeros(self.batch, dtype=np.int32)
        ncom = np.zeros(self.batch, dtype=np.int32)
        com = np.zeros((self.batch, k + self.bonus), dtype=np.int32)
        fn = self.lib.deer_accept_and_commit_static if static else self.lib.deer_accept_and_commit
        self._check(fn(self.ctx, k, T, seed, acc.ctypes.data, com.ctypes.data, ncom.ctypes.data))
        return acc, [com[b, : ncom[b]].tolist() for b in range(self.batch)], ncom

    # -- inspection ------------------------------------------------------------------------------
    def debug_get_logits(self, model, k):
        out = np.empty((self.batch, k, self.target.vocab), dtype=np.float32)
        self._check(self.lib.deer_debug_get_logits(self.ctx, model, out.ctypes.data, out.size))
        return out

    def debug_profile(self, enable):
        self._check(self.lib.deer_debug_profile(self.ctx, int(enable)))

    def debug_profile_read(self, kernel_class):
        """(total_ms, launches, algorithmic_bytes) of the recorded launches of one kernel class."""
        ms, n, by = C.c_double(), C.c_int64(), C.c_double()
        self._check(self.lib.deer_debug_profile_read(self.ctx, kernel_class, C.byref(ms), C.byref(n), C.byref(by)))
        return ms.value, n.value, by.value

    def debug_gemm_stamps(self, model, launch):
        """Returns the stamps recorded so far as an int64 array [workgroups][8] (or None), then selects the
        streaming-GEMM launch (index within a pass of `model`, < 0: off) that records from now on."""
        nb = C.c_int32(0)
        buf = np.zeros((32768, 8), dtype=np.uint64)
        self._check(self.lib.deer_debug_gemm_stamps(self.ctx, model, -1 if launch is None else launch, buf.ctypes.data,
                                                    buf.shape[0], C.byref(nb)))
        return buf[: nb.value].astype(np.int64) if nb.value > 0 else None

    def debug_route_spread(self, enable):
        self._check(self.lib.deer_debug_route_spread(self.ctx, int(bool(enable))))

    def debug_stream_read(self, buf, nbytes, workgroups, nontemporal, reps):
        """Mean milliseconds per launch of a plain read of the first nbytes of the device tensor buf."""
        if not buf.is_cuda or not buf.is_contiguous() or nbytes > buf.numel() * buf.element_size():
            raise ValueError("debug_stream_read needs a contiguous device tensor of at least nbytes")
        ms = C.c_float(0.0)
        self._check(self.lib.deer_debug_stream_read(self.ctx, C.c_void_p(buf.data_ptr()), nbytes, workgroups, int(bool(nontemporal)),
                                                    reps, C.byref(ms)))
        return ms.value

    def debug_experts_streamed(self):
        n = C.c_int64(0)
        self._check(self.lib.deer_debug_experts_streamed(self.ctx, C.byref(n)))
        return n.value

    def debug_gemm_tiled(self, min_tiles):
        self._check(self.lib.deer_debug_gemm_tiled(self.ctx, int(min_tiles)))

    def debug_force_commit(self, tokens):
        """Commits tokens[b] (a list per sequence, possibly empty) instead of running the acceptance rule."""
        n = np.array([len(t) for t in tokens], dtype=np.int32)
        stride = max(1, int(n.max()))
        buf = np.zeros((self.batch, stride), dtype=np.int32)
        for b, t in enumerate(tokens):
            buf[b, : len(t)] = t
        self._check(self.lib.deer_debug_force_commit(self.ctx, buf.ctypes.data, n.ctypes.data, stride))

    def debug_load_kv(self, model, layer, seq, first_slot, k_rows, v_rows):
        """k_rows, v_rows: contiguous device tensors [n][kv_head][head_dim], bfloat16 (or int16 bit patterns)."""
        assert k_rows.is_cuda and v_rows.is_cuda and k_rows.is_contiguous() and v_rows.is_contiguous()
        assert k_rows.shape == v_rows.shape and k_rows.element_size() == 2 and v_rows.element_size() == 2
        self._check(self.lib.deer_debug_load_kv(self.ctx, model, layer, seq, first_slot, k_rows.shape[0],
                                                k_rows.data_ptr(), v_rows.data_ptr()))

    def get_lengths(self):
        out = np.zeros(self.batch, dtype=np.int32)
        self._check(self.lib.deer_get_lengths(self.ctx, out.ctypes.data))
        return out

    def get_kv_layout(self, model):
        lay = KvLayout()
        self._check(self.lib.deer_get_kv_layout(self.ctx, model, C.byref(lay)))
        return lay

    def synchronize(self):
        self.torch.cuda.current_stream(self.device).synchronize()
