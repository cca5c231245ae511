"""ctypes front end of the CPU oracle (oracle/chiron_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU
baseline leg call this; the product package never does.  Arrays are numpy;
float tensors are float32, bf16 storage is uint16 bit patterns.
"""
import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "chiron_oracle.c")
_LIB = os.path.join(_HERE, "libchiron_oracle.so")

F32, BF16 = 0, 1


def build(force=False):
    """Compile the oracle with gcc (plain C + OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + [
        ("rope_base", C.c_float), ("rms_eps", C.c_float), ("block_size", C.c_int32), ("wdtype", C.c_int32),
        ("kvdtype", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + [
        (n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_slot.restype = C.c_int64
        _lib.orc_f32_to_bf16_bits.restype = C.c_uint16
        _lib.orc_f32_to_bf16_bits.argtypes = [C.c_float]
    return _lib


def _p(a):
    return C.c_void_p(a.ctypes.data)


def _dt(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("storage arrays must be float32 or uint16 (bf16 bits), got %s" % a.dtype)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def bf16_bits(x):
    """round-to-nearest-even float32 -> bf16 bit pattern, elementwise (scalar C routine)."""
    x = _f32(x)
    out = np.empty(x.shape, np.uint16)
    f = lib().orc_f32_to_bf16_bits
    xf, of = x.ravel(), out.ravel()
    for i in range(xf.size):
        of[i] = f(float(xf[i]))
    return out


def make_config(m, wdtype, kvdtype):
    """m: mapping with the model fields (see inputs.ModelShape)."""
    return Config(m["n_layers"], m["hidden"], m["n_q_heads"], m["n_kv_heads"], m["head_dim"], m["ffn"], m["vocab"],
                  m["rope_base"], m["rms_eps"], m["block_size"], wdtype, kvdtype)


def rmsnorm(h, g, eps):
    h = _f32(h)
    g = np.ascontiguousarray(g)
    out = np.empty_like(h)
    lib().orc_rmsnorm(_p(h), _p(g), _dt(g), C.c_int(h.size), C.c_float(eps), _p(out))
    return out


def linear(x, W):
    """x [rows,K] float32, W [N,K] storage -> [rows,N] float32."""
    x = _f32(x)
    W = np.ascontiguousarray(W)
    rows, K = x.shape
    N = W.shape[0]
    assert W.shape[1] == K
    y = np.empty((rows, N), np.float32)
    lib().orc_linear(_p(x), C.c_int(rows), _p(W), _dt(W), C.c_int(N), C.c_int(K), _p(y))
    return y


def rope(x, pos, base):
    """x [n_heads, d] float32 -> rotated copy."""
    x = _f32(x).copy()
    lib().orc_rope(_p(x), C.c_int(x.shape[0]), C.c_int(x.shape[1]), C.c_int(int(pos)), C.c_float(base))
    return x


def slot(block_table_row, pos, block_size):
    r = _i32(block_table_row)
    return int(lib().orc_slot(_p(r), C.c_int(int(pos)), C.c_int(block_size)))


def swiglu(g, u):
    g, u = _f32(g), _f32(u)
    out = np.empty_like(g)
    lib().orc_swiglu(_p(g), _p(u), C.c_int(g.size), _p(out))
    return out


class Pool:
    """The oracle's own KV pool: K and V as [n_layers, num_slots, n_kv, d] in fp32 or bf16 bits."""

    def __init__(self, cfg, num_blocks, dtype=np.float32):
        self.cfg = cfg
        self.num_blocks = int(num_blocks)
        self.num_slots = self.num_blocks * cfg.block_size
        shape = (cfg.n_layers, self.num_slots, cfg.n_kv_heads, cfg.head_dim)
        self.k = np.zeros(shape, dtype)
        self.v = np.zeros(shape, dtype)
        assert _dt(self.k) == cfg.kvdtype

    def copy(self):
        p = Pool.__new__(Pool)
        p.cfg, p.num_blocks, p.num_slots = self.cfg, self.num_blocks, self.num_slots
        p.k, p.v = self.k.copy(), self.v.copy()
        return p


def append_kv(pool, layer, k, v, block_table, seq_idx, pos):
    k, v = _f32(k), _f32(v)
    bt = _i32(block_table)
    si, ps = _i32(seq_idx), _i32(pos)
    n = si.size
    slots = np.empty(n, np.int64)
    lib().orc_append_kv(C.byref(pool.cfg), _p(pool.k), _p(pool.v), C.c_int64(pool.num_slots), C.c_int(layer), _p(k), _p(v),
                        _p(bt), C.c_int(bt.shape[1]), _p(si), _p(ps), C.c_int(n), _p(slots))
    return slots


def gather_kv(pool, layer, block_table_row, length):
    r = _i32(block_table_row)
    shape = (length, pool.cfg.n_kv_heads, pool.cfg.head_dim)
    k = np.empty(shape, pool.k.dtype)
    v = np.empty(shape, pool.v.dtype)
    lib().orc_gather_kv(C.byref(pool.cfg), _p(pool.k), _p(pool.v), C.c_int64(pool.num_slots), C.c_int(layer), _p(r),
                        C.c_int(length), _p(k), _p(v))
    return k, v


def swap(pool, block_table_row, n_pages, image=None):
    """image None: swap out and return the image (uint8 array); otherwise swap the image in."""
    r = _i32(block_table_row)
    cfg = pool.cfg
    es = 2 if cfg.kvdtype == BF16 else 4
    nbytes = cfg.n_layers * 2 * n_pages * cfg.block_size * cfg.n_kv_heads * cfg.head_dim * es
    out = image is None
    if out:
        image = np.zeros(nbytes, np.uint8)
    assert image.size == nbytes
    lib().orc_swap(C.byref(cfg), _p(pool.k), _p(pool.v), C.c_int64(pool.num_slots), _p(r), C.c_int(n_pages), _p(image),
                   C.c_int(1 if out else 0))
    return image


def paged_attention(pool, layer, block_table_row, length, q):
    r = _i32(block_table_row)
    q = _f32(q)
    out = np.empty_like(q)
    lib().orc_paged_attention(C.byref(pool.cfg), _p(pool.k), _p(pool.v), C.c_int64(pool.num_slots), C.c_int(layer), _p(r),
                              C.c_int(length), _p(q), _p(out))
    return out


def _weights_struct(w, n_layers):
    """w: dict name -> array (embed, final_norm, lm_head) or list of arrays per layer."""
    keep = []
    ws = Weights()
    for n in ("embed", "final_norm", "lm_head"):
        a = np.ascontiguousarray(w[n])
        keep.append(a)
        setattr(ws, n, a.ctypes.data)
    for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
        arrs = [np.ascontiguousarray(a) for a in w[n]]
        assert len(arrs) == n_layers
        keep.extend(arrs)
        ptrs = (C.c_void_p * n_layers)(*[a.ctypes.data for a in arrs])
        keep.append(ptrs)
        setattr(ws, n, C.cast(ptrs, C.POINTER(C.c_void_p)))
    return ws, keep


def decode_step(cfg, w, pool, block_table, seq_lens, tokens):
    """Runs the whole step; pool is updated in place.  Returns (logits [B,V] float32, slots [B] int64)."""
    ws, keep = _weights_struct(w, cfg.n_layers)
    for a in keep:
        if isinstance(a, np.ndarray) and a.dtype != np.int32:
            assert _dt(a) == cfg.wdtype, "weight dtype does not match config"
    bt = _i32(block_table)
    sl, tk = _i32(seq_lens), _i32(tokens)
    B = sl.size
    logits = np.empty((B, cfg.vocab), np.float32)
    slots = np.empty(B, np.int64)
    rc = lib().orc_decode_step(C.byref(cfg), C.byref(ws), _p(pool.k), _p(pool.v), C.c_int64(pool.num_slots), _p(bt),
                               C.c_int(bt.shape[1] if bt.ndim == 2 else 0), _p(sl), _p(tk), C.c_int(B), _p(logits), _p(slots))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return logits, slots


def decode_step_multi(cfg, w, pool, block_table, seq_lens, tokens):
    """tokens [B, T] -> logits [B, T, V]; pool is updated in place (T tokens per request appended)."""
    ws, keep = _weights_struct(w, cfg.n_layers)
    bt = _i32(block_table)
    sl, tk = _i32(seq_lens), _i32(tokens)
    B, T = tk.shape
    logits = np.empty((B, T, cfg.vocab), np.float32)
    rc = lib().orc_decode_step_multi(C.byref(cfg), C.byref(ws), _p(pool.k), _p(pool.v), C.c_int64(pool.num_slots), _p(bt),
                                     C.c_int(bt.shape[1]), _p(sl), _p(tk), C.c_int(B), C.c_int(T), _p(logits))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return logits


def autoscale_step(itl, itl_slo, thr_prev, thr_curr, alpha, limit, mbs):
    """-> (new max batch size, local backpressure or -1 if the tick was skipped)"""
    f = lib().orc_autoscale_step
    f.restype = C.c_int
    lb = C.c_double()
    r = f(C.c_double(itl), C.c_double(itl_slo), C.c_double(thr_prev), C.c_double(thr_curr), C.c_double(alpha),
          C.c_int(int(limit)), C.c_int(int(mbs)), C.byref(lb))
    return int(r), lb.value


def num_threads():
    return int(lib().orc_num_threads())
