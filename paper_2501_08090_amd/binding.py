"""Thin ctypes binding of libchiron.so (include/chiron.h, include/chiron_ops.h).

Argument marshalling only: every function takes torch tensors that already live on the
GPU (torch supplies device memory and streams), checks dtype/contiguity, and passes raw
pointers through the C ABI.  No step of the decode path runs in Python, and there is no
fallback: if the library has not been built, loading raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CHIRON_LIB", os.path.join(_HERE, "libchiron.so"))

CHIRON_BF16 = 1
ERRORS = {0: "OK", -1: "INVALID_ARG", -2: "SHAPE", -3: "BATCH_TOO_LARGE", -4: "BLOCK_TABLE", -5: "OOM", -6: "HIP", -7: "TOKEN"}

# every symbol the headers declare (tests check that the library exports all of them)
SYMBOLS = [
    "chiron_model_create", "chiron_model_load_layer", "chiron_model_load_head", "chiron_model_destroy",
    "chiron_kv_block_bytes", "chiron_kv_pool_create", "chiron_kv_pool_destroy", "chiron_append_kv", "chiron_gather_kv",
    "chiron_kv_swap_out", "chiron_kv_swap_in",
    "chiron_decode_step", "chiron_decode_step_multi", "chiron_validate_step_inputs", "chiron_check_step_inputs_host",
    "chiron_validate_step_inputs_multi", "chiron_check_step_inputs_host_multi", "chiron_step_latency_profile",
    "chiron_last_error", "chiron_kernel_timing_begin", "chiron_kernel_timing_end", "chiron_local_autoscale_step",
    "chiron_op_rmsnorm", "chiron_linear_create", "chiron_linear_destroy", "chiron_op_linear", "chiron_linear_create_gate_up", "chiron_op_gate_up_swiglu", "chiron_op_swiglu_ffn",
    "chiron_op_rope", "chiron_op_rope_noalloc", "chiron_op_paged_attention", "chiron_set_tuning",
]


class ChironError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("chiron: %s (%d): %s" % (ERRORS.get(code, "?"), code, text))
        self.code = code


class ModelConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + [
        ("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32), ("max_batch", C.c_int32),
        ("max_blocks_per_seq", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class ProfilePoint(C.Structure):
    _fields_ = [("batch", C.c_int32), ("lat_ms_median", C.c_double), ("lat_ms_p99", C.c_double),
                ("lat_ms_mean", C.c_double), ("tokens_per_s", C.c_double)]


_lib = None


def load():
    """Load the built library; raises if it is missing (there is no other implementation)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libchiron.so is not built: run `python -m paper_2501_08090_amd.build` "
                              "(or __graft_entry__.build()); there is no fallback path")
        lib = C.CDLL(LIB_PATH)
        lib.chiron_last_error.restype = C.c_char_p
        lib.chiron_kv_block_bytes.restype = C.c_int64
        _lib = lib
    return _lib


def _check(rc):
    if rc != 0:
        raise ChironError(rc, load().chiron_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype=None):
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda:
        raise TypeError("expected a GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, t.dtype))
    if not t.is_contiguous():
        raise TypeError("expected a contiguous tensor")
    return C.c_void_p(t.data_ptr())


def make_config(m, max_batch, max_blocks_per_seq):
    return ModelConfig(m["n_layers"], m["hidden"], m["n_q_heads"], m["n_kv_heads"], m["head_dim"], m["ffn"], m["vocab"],
                       m["rope_base"], m["rms_eps"], CHIRON_BF16, int(max_batch), int(max_blocks_per_seq))


class Model:
    def __init__(self, m, max_batch, max_blocks_per_seq):
        self.cfg = make_config(m, max_batch, max_blocks_per_seq)
        self.shape = dict(m)
        self._h = C.c_void_p()
        _check(load().chiron_model_create(C.byref(self.cfg), C.byref(self._h)))

    def load_layer(self, layer, **w):
        lw = LayerWeights(*[_ptr(w[n], torch.bfloat16) for n, _ in LayerWeights._fields_])
        _check(load().chiron_model_load_layer(self._h, C.c_int32(layer), C.byref(lw), _stream()))

    def load_head(self, embed, final_norm, lm_head):
        _check(load().chiron_model_load_head(self._h, _ptr(embed, torch.bfloat16), _ptr(final_norm, torch.bfloat16),
                                             _ptr(lm_head, torch.bfloat16), _stream()))

    def load_weights(self, w):
        """w: dict as produced by inputs.make_weights (tensors on the GPU)."""
        for l in range(self.cfg.n_layers):
            self.load_layer(l, **{n: w[n][l] for n, _ in LayerWeights._fields_})
        self.load_head(w["embed"], w["final_norm"], w["lm_head"])

    def kv_block_bytes(self, block_size=16):
        return int(load().chiron_kv_block_bytes(self._h, C.c_int32(block_size)))

    def close(self):
        if self._h:
            torch.cuda.synchronize()
            load().chiron_model_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class KVPool:
    """Pool descriptor over a torch-allocated byte buffer (the caller owns the memory)."""

    def __init__(self, model, num_blocks=None, memory=None, block_size=16):
        self.model = model
        if memory is None:
            memory = torch.empty(int(num_blocks) * model.kv_block_bytes(block_size), dtype=torch.uint8, device="cuda")
        self.memory = memory
        self._h = C.c_void_p()
        nb = C.c_int32()
        _check(load().chiron_kv_pool_create(model._h, _ptr(memory), C.c_uint64(memory.numel() * memory.element_size()),
                                            C.c_int32(block_size), C.byref(self._h), C.byref(nb)))
        self.num_blocks = nb.value
        self.block_size = block_size

    def append(self, layer, k, v, block_table, seq_idx, pos):
        n = seq_idx.numel()
        _check(load().chiron_append_kv(self._h, C.c_int32(layer), _ptr(k, torch.bfloat16), _ptr(v, torch.bfloat16),
                                       _ptr(block_table, torch.int32), C.c_int32(block_table.shape[1]),
                                       _ptr(seq_idx, torch.int32), _ptr(pos, torch.int32), C.c_int64(n), _stream()))

    def gather(self, layer, block_table_row, length):
        cfg = self.model.cfg
        k = torch.empty((length, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
        v = torch.empty_like(k)
        _check(load().chiron_gather_kv(self._h, C.c_int32(layer), _ptr(block_table_row, torch.int32), C.c_int32(length),
                                       _ptr(k), _ptr(v), _stream()))
        return k, v

    def swap_out(self, block_table_row, n_pages, image):
        """image: uint8 tensor of n_pages*block_bytes, on the GPU or in pinned host memory"""
        _check(load().chiron_kv_swap_out(self._h, _ptr(block_table_row, torch.int32), C.c_int32(int(n_pages)),
                                         C.c_void_p(image.data_ptr()), _stream()))

    def swap_in(self, block_table_row, n_pages, image):
        _check(load().chiron_kv_swap_in(self._h, _ptr(block_table_row, torch.int32), C.c_int32(int(n_pages)),
                                        C.c_void_p(image.data_ptr()), _stream()))

    def close(self):
        if self._h:
            load().chiron_kv_pool_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _check_table(model, block_table, batch):
    """The library indexes the block table with the model's max_blocks_per_seq as row stride."""
    if block_table.dim() != 2 or block_table.shape[1] != model.cfg.max_blocks_per_seq:
        raise ValueError("block_table must be [rows, %d] (the model's max_blocks_per_seq), got %s" % (
            model.cfg.max_blocks_per_seq, tuple(block_table.shape)))
    if block_table.shape[0] < batch:
        raise ValueError("block_table has %d rows for a batch of %d" % (block_table.shape[0], batch))


def decode_step(model, pool, block_table, seq_lens, tokens, logits=None, batch=None):
    B = seq_lens.numel() if batch is None else int(batch)
    _check_table(model, block_table, B)
    if logits is None:
        logits = torch.empty((B, model.cfg.vocab), dtype=torch.float32, device="cuda")
    _check(load().chiron_decode_step(model._h, pool._h, _ptr(block_table, torch.int32), _ptr(seq_lens, torch.int32),
                                     _ptr(tokens, torch.int32), C.c_int32(B), _ptr(logits, torch.float32), _stream()))
    return logits


def decode_step_multi(model, pool, block_table, seq_lens, tokens, logits=None):
    """tokens [batch, q_len] int32 -> logits [batch, q_len, vocab]"""
    B, T = tokens.shape
    _check_table(model, block_table, B)
    if logits is None:
        logits = torch.empty((B, T, model.cfg.vocab), dtype=torch.float32, device="cuda")
    _check(load().chiron_decode_step_multi(model._h, pool._h, _ptr(block_table, torch.int32), _ptr(seq_lens, torch.int32),
                                           _ptr(tokens, torch.int32), C.c_int32(B), C.c_int32(T), _ptr(logits, torch.float32),
                                           _stream()))
    return logits


def validate_step_inputs(model, pool, block_table, seq_lens, tokens, batch=None):
    """tokens [batch] or, for the multi-token step, [batch, q_len]"""
    B = seq_lens.numel() if batch is None else int(batch)
    _check_table(model, block_table, B)
    if tokens.dim() == 2:
        _check(load().chiron_validate_step_inputs_multi(model._h, pool._h, _ptr(block_table, torch.int32), _ptr(seq_lens, torch.int32),
                                                        _ptr(tokens, torch.int32), C.c_int32(B), C.c_int32(tokens.shape[1]), _stream()))
        return
    _check(load().chiron_validate_step_inputs(model._h, pool._h, _ptr(block_table, torch.int32), _ptr(seq_lens, torch.int32),
                                              _ptr(tokens, torch.int32), C.c_int32(B), _stream()))


def check_step_inputs_host(cfg, num_blocks, block_table, seq_lens, tokens, block_size=16):
    """Host-only check of index arrays (numpy int32); tokens [batch] or [batch, q_len]."""
    import numpy as np
    bt = np.ascontiguousarray(block_table, np.int32)
    sl = np.ascontiguousarray(seq_lens, np.int32)
    tk = np.ascontiguousarray(tokens, np.int32)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    if tk.ndim == 2:
        return int(load().chiron_check_step_inputs_host_multi(C.byref(cfg), C.c_int32(num_blocks), C.c_int32(block_size), p(bt),
                                                              p(sl), p(tk), C.c_int32(sl.size), C.c_int32(tk.shape[1])))
    return int(load().chiron_check_step_inputs_host(C.byref(cfg), C.c_int32(num_blocks), C.c_int32(block_size), p(bt), p(sl),
                                                    p(tk), C.c_int32(sl.size)))


def last_error():
    return load().chiron_last_error().decode()


def step_latency_profile(model, pool, block_table, seq_lens, tokens, batch_sizes, warmup=2, iters=5, logits=None):
    n = len(batch_sizes)
    _check_table(model, block_table, max(batch_sizes))
    if logits is None:
        logits = torch.empty((max(batch_sizes), model.cfg.vocab), dtype=torch.float32, device="cuda")
    bs = (C.c_int32 * n)(*batch_sizes)
    out = (ProfilePoint * n)()
    _check(load().chiron_step_latency_profile(model._h, pool._h, _ptr(block_table, torch.int32), _ptr(seq_lens, torch.int32),
                                              _ptr(tokens, torch.int32), bs, C.c_int32(n), C.c_int32(warmup), C.c_int32(iters),
                                              _ptr(logits, torch.float32), _stream(), out))
    return [dict(batch=p.batch, lat_ms_median=p.lat_ms_median, lat_ms_p99=p.lat_ms_p99, lat_ms_mean=p.lat_ms_mean,
                 tokens_per_s=p.tokens_per_s) for p in out]


def local_autoscale_step(itl, itl_slo, tput_prev, tput_curr, max_batch, batch_limit, alpha=0.5):
    """One update of the maximum batch size (host arithmetic).  -> (new max batch, local backpressure)"""
    mb = C.c_int32(int(max_batch))
    lb = C.c_double()
    _check(load().chiron_local_autoscale_step(C.c_double(itl), C.c_double(itl_slo), C.c_double(tput_prev), C.c_double(tput_curr),
                                              C.c_double(alpha), C.c_int32(int(batch_limit)), C.byref(mb), C.byref(lb)))
    return mb.value, lb.value


KERNEL_CLASSES = ("qkv", "o", "gateup", "down", "lmhead", "attn", "attn_merge", "rmsnorm", "rope_append", "other")


class KernelTime(C.Structure):
    _fields_ = [("ms", C.c_double), ("launches", C.c_int64)]


def kernel_timing_begin(model):
    _check(load().chiron_kernel_timing_begin(model._h))


def kernel_timing_end(model):
    """-> {class: (total_ms, launches)}"""
    out = (KernelTime * len(KERNEL_CLASSES))()
    _check(load().chiron_kernel_timing_end(model._h, _stream(), out))
    return {n: (out[i].ms, int(out[i].launches)) for i, n in enumerate(KERNEL_CLASSES)}


# ---- single kernels -------------------------------------------------------------------------------

def op_rmsnorm(h, gain, eps):
    out = torch.empty_like(h)
    _check(load().chiron_op_rmsnorm(_ptr(h, torch.float32), _ptr(gain, torch.bfloat16), C.c_int32(h.shape[0]),
                                    C.c_int32(h.shape[1]), C.c_float(eps), _ptr(out), _stream()))
    return out


class Linear:
    def __init__(self, w):
        self.N, self.K = w.shape
        self._h = C.c_void_p()
        _check(load().chiron_linear_create(_ptr(w, torch.bfloat16), C.c_int32(self.N), C.c_int32(self.K), _stream(),
                                           C.byref(self._h)))

    def __call__(self, x, y=None, accumulate=False):
        M = x.shape[0]
        if y is None:
            y = torch.empty((M, self.N), dtype=torch.float32, device="cuda")
        _check(load().chiron_op_linear(self._h, _ptr(x, torch.float32), C.c_int32(M), _ptr(y, torch.float32),
                                       C.c_int32(1 if accumulate else 0), _stream()))
        return y

    def close(self):
        if self._h:
            torch.cuda.synchronize()
            load().chiron_linear_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class GateUp(Linear):
    """The fused gate/up matrix of a feed-forward block (w_gate, w_up [F, K] bf16)."""

    def __init__(self, w_gate, w_up):
        self.F, self.K = w_gate.shape
        if tuple(w_up.shape) != (self.F, self.K):
            raise ValueError("w_gate and w_up differ in shape")
        self.N = 2 * self.F
        self._h = C.c_void_p()
        _check(load().chiron_linear_create_gate_up(_ptr(w_gate, torch.bfloat16), _ptr(w_up, torch.bfloat16), C.c_int32(self.F),
                                                   C.c_int32(self.K), _stream(), C.byref(self._h)))

    def __call__(self, x, *a, **k):
        raise TypeError("a fused gate/up matrix has no plain product: use swiglu() or ffn()")

    def swiglu(self, x):
        """silu(x Wg^T) * (x Wu^T), fp32 [M, F]"""
        M = x.shape[0]
        act = torch.empty((M, self.F), dtype=torch.float32, device="cuda")
        _check(load().chiron_op_gate_up_swiglu(self._h, _ptr(x, torch.float32), C.c_int32(M), _ptr(act, torch.float32), _stream()))
        return act

    def ffn(self, down, x, y=None, accumulate=False):
        """y (+)= (silu(x Wg^T) * (x Wu^T)) Wd^T with down = Linear(Wd)"""
        M = x.shape[0]
        if y is None:
            y = torch.empty((M, down.N), dtype=torch.float32, device="cuda")
        _check(load().chiron_op_swiglu_ffn(self._h, down._h, _ptr(x, torch.float32), C.c_int32(M), _ptr(y, torch.float32),
                                           C.c_int32(1 if accumulate else 0), _stream()))
        return y


def set_tuning(key, value):
    _check(load().chiron_set_tuning(key.encode(), C.c_int32(int(value))))


def op_rope(x, pos, base):
    """x [rows, n_heads, d] fp32, rotated in place."""
    rows, nh, d = x.shape
    _check(load().chiron_op_rope(_ptr(x, torch.float32), C.c_int32(rows), C.c_int32(nh), C.c_int32(d), _ptr(pos, torch.int32),
                                 C.c_float(base), _stream()))
    return x


def op_rope_noalloc(x, pos, base):
    """op_rope through the entry point that allocates nothing (fixed table inside the library)."""
    rows, nh, d = x.shape
    _check(load().chiron_op_rope_noalloc(_ptr(x, torch.float32), C.c_int32(rows), C.c_int32(nh), C.c_int32(d),
                                         _ptr(pos, torch.int32), C.c_float(base), _stream()))
    return x


def op_paged_attention(model, pool, layer, q, block_table, ctx_lens):
    B = ctx_lens.numel()
    _check_table(model, block_table, B)
    out = torch.empty_like(q)
    _check(load().chiron_op_paged_attention(model._h, pool._h, C.c_int32(layer), _ptr(q, torch.float32),
                                            _ptr(block_table, torch.int32), _ptr(ctx_lens, torch.int32), C.c_int32(B),
                                            _ptr(out), _stream()))
    return out
