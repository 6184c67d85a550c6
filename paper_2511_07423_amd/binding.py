"""ctypes binding with the same entry points as include/synera.h (marshalling only)."""
import ctypes as C
import os

import numpy as np
import torch

OK, EINVAL, ERANGE, ENOSPC, EUNSUP, EHIP, ENOMEM = 0, -1, -2, -3, -4, -5, -6
PAGE_SIZE = 16
MAX_CHUNK = 32
STAGES = {"none": 0, "qkv": 1, "attention": 2, "o": 3, "gate_up": 4, "down": 5, "lm_head": 6, "confidence": 7,
          "norm": 8, "rope_append": 9}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynera.so")


def lib_path():
    return _LIB_PATH


if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
        "There is no CPU fallback.")
_lib = C.CDLL(_LIB_PATH)

_i32p = C.POINTER(C.c_int32)
_vp = C.c_void_p


class _ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("rope_base", C.c_float), ("rms_eps", C.c_float)]


_LAYER_FIELDS = ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")


class _LayerWeights(C.Structure):
    _fields_ = [(n, _vp) for n in _LAYER_FIELDS]


class _Weights(C.Structure):
    _fields_ = [("embed", _vp), ("layers", C.POINTER(_LayerWeights)), ("final_norm", _vp), ("lm_head", _vp)]


_lib.synera_version.restype = C.c_int32
_lib.synera_strerror.restype = C.c_char_p
_lib.synera_strerror.argtypes = [C.c_int32]
_lib.synera_create.restype = C.c_int32
_lib.synera_create.argtypes = [C.POINTER(_vp), C.POINTER(_ModelDesc), C.POINTER(_Weights), C.c_int32, C.c_int32,
                               C.c_int32]
_lib.synera_destroy.restype = C.c_int32
_lib.synera_destroy.argtypes = [_vp]
_lib.synera_validate_batch.restype = C.c_int32
_lib.synera_validate_batch.argtypes = [C.c_int32, _i32p, _i32p, _i32p, _i32p, C.c_int32, C.c_int32, C.c_int32,
                                       C.c_int64, C.c_int32]
_lib.synera_verify.restype = C.c_int32
_lib.synera_verify.argtypes = [_vp, C.c_int32, _i32p, _i32p, _i32p, _vp, _vp, _i32p, C.c_int32, C.c_int32, _vp, _vp,
                               _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.synera_confidence.restype = C.c_int32
_lib.synera_confidence.argtypes = [_vp, C.c_int32, C.c_int64, C.c_int64, C.c_int64, _vp, _vp, _vp, _vp]
_lib.synera_confidence_topk.restype = C.c_int32
_lib.synera_confidence_topk.argtypes = [_vp, C.c_int32, C.c_int64, C.c_int64, C.c_int64, C.c_int32, _vp, _vp, _vp, _vp, _vp]
_lib.synera_nucleus.restype = C.c_int32
_lib.synera_nucleus.argtypes = [_vp, C.c_int32, C.c_int64, C.c_int64, C.c_int64, C.c_float, _vp, _vp, _vp, _vp]
_lib.synera_chunk_dispatch.restype = C.c_int32
_lib.synera_chunk_dispatch.argtypes = [_vp, _vp, C.c_int32, C.c_float, C.c_float, _vp, _vp, _vp]
_lib.synera_kv_append.restype = C.c_int32
_lib.synera_kv_append.argtypes = [_vp, C.c_int32, C.c_int32, _i32p, _i32p, _vp, _vp, _i32p, C.c_int32, C.c_int32,
                                  _vp, _vp, _vp]
_lib.synera_profile_begin.restype = C.c_int32
_lib.synera_profile_begin.argtypes = [_vp, C.c_int32]
_lib.synera_profile_end.restype = C.c_int32
_lib.synera_profile_end.argtypes = [_vp, C.POINTER(C.c_int32), C.POINTER(C.c_float)]
_lib.synera_gemm_pair.restype = C.c_int32
_lib.synera_gemm_pair.argtypes = [_vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, _vp]
_lib.synera_gemm_pair_static.restype = C.c_int32
_lib.synera_gemm_pair_static.argtypes = [_vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, _vp]
_lib.synera_debug_set_lo_off.restype = C.c_int32
_lib.synera_debug_set_lo_off.argtypes = [_vp, C.c_int32]
_lib.synera_debug_set_attention_plan.restype = C.c_int32
_lib.synera_debug_set_attention_plan.argtypes = [_vp, C.c_int32, C.c_float, C.c_float, C.c_float]
_lib.synera_debug_read_scratch.restype = C.c_int32
_lib.synera_debug_read_scratch.argtypes = [_vp, C.c_int32, _vp, C.c_int64, _vp]
_lib.synera_debug_set_gemm_tile.restype = C.c_int32
_lib.synera_debug_set_gemm_tile.argtypes = [C.c_int32]
_lib.synera_stochastic_accept.restype = C.c_int32
_lib.synera_stochastic_accept.argtypes = [_vp, _vp, C.c_int32, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.synera_topp_count.restype = C.c_int32
_lib.synera_topp_count.argtypes = [_vp, C.c_int64, C.c_int32, C.c_float, _vp, _vp, _vp]
_lib.synera_importance.restype = C.c_int32
_lib.synera_importance.argtypes = [_vp, C.c_int32, _vp, C.c_int64, _vp, C.c_float, C.c_float, _vp, _vp, _vp]
_lib.synera_debug_gemm_slices.restype = C.c_int32
_lib.synera_debug_gemm_slices.argtypes = [_vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32), _vp]
_lib.synera_measure_hbm_copy.restype = C.c_int32
_lib.synera_measure_hbm_copy.argtypes = [_vp, _vp, C.c_int64, _vp]
_lib.synera_measure_hbm_read.restype = C.c_int32
_lib.synera_measure_hbm_read.argtypes = [_vp, _vp, C.c_int64, _vp]
_lib.synera_measure_mfma_bf16.restype = C.c_int32
_lib.synera_measure_mfma_bf16.argtypes = [_vp, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int64), _vp]
_lib.synera_measure_mfma_f16.restype = C.c_int32
_lib.synera_measure_mfma_f16.argtypes = [_vp, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int64), _vp]
_lib.synera_debug_attention_plan.restype = C.c_int32
_lib.synera_debug_attention_plan.argtypes = [_vp, C.c_int32, C.c_int32, _i32p, _i32p, _i32p, _i32p, C.c_int32,
                                             _i32p, _i32p, C.c_int64, _i32p, C.c_int64, _i32p, C.c_int64, _i32p]
_lib.synera_debug_gemm_plan.restype = C.c_int32
_lib.synera_debug_gemm_plan.argtypes = [C.c_int32] * 5 + [C.POINTER(C.c_int32)] * 3
_lib.synera_debug_gemm_plan_bk.restype = C.c_int32
_lib.synera_debug_gemm_plan_bk.argtypes = [C.c_int32] * 5 + [C.POINTER(C.c_int32)]
_lib.synera_debug_gemm_paired.restype = C.c_int32
_lib.synera_debug_gemm_paired.argtypes = [_vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp]
_lib.synera_debug_gemm_epilogue.restype = C.c_int32
_lib.synera_debug_gemm_epilogue.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp]


class SyneraError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {_lib.synera_strerror(status).decode()} ({status})")


def _check(status, where):
    if status != OK:
        raise SyneraError(status, where)


def version():
    return _lib.synera_version()


def _host_i32(a):
    """contiguous int32 numpy array + its ctypes pointer (None passes NULL)."""
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(_i32p)


def _dev(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device tensors must be contiguous and on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def validate_batch(ctx_len, n_first, n_second, block_table, n_pages_in_pool, max_batch, max_tokens,
                   chunk_limit=MAX_CHUNK):
    """Host-only check of a batch description; returns the status code (no GPU needed)."""
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    _, p_ctx = _host_i32(ctx_len)
    _, p_a = _host_i32(n_first)
    keep = [_host_i32(x) for x in (ctx_len, n_first, n_second)]
    B = len(keep[0][0]) if keep[0][0] is not None else 0
    max_pages = bt.shape[1] if bt.ndim == 2 else 0
    return _lib.synera_validate_batch(B, keep[0][1], keep[1][1], keep[2][1], bt.ctypes.data_as(_i32p), max_pages,
                                      n_pages_in_pool, max_batch, max_tokens, chunk_limit)


def confidence(logits, want_prob=True, want_entropy=True):
    """Per row: (argmax id int32, top-1 probability f32, entropy f32) of a 2-D f32 or bf16 GPU tensor."""
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be 2-D with unit column stride")
    dt = {torch.float32: 0, torch.bfloat16: 1}[logits.dtype]
    rows, vocab = logits.shape
    dev = logits.device
    ids = torch.empty(rows, dtype=torch.int32, device=dev)
    p = torch.empty(rows, dtype=torch.float32, device=dev) if want_prob else None
    h = torch.empty(rows, dtype=torch.float32, device=dev) if want_entropy else None
    st = _lib.synera_confidence(logits.data_ptr(), dt, rows, vocab, logits.stride(0) if rows > 1 else vocab,
                                ids.data_ptr(), _dev(p), _dev(h), _stream())
    _check(st, "synera_confidence")
    return ids, p, h


def confidence_topk(logits, k, want_margin=True, want_entropy=True):
    """Per row of a 2-D f32 or bf16 GPU tensor: (top-k ids int32 [rows,k], their probabilities f32 [rows,k],
    margin p1 - p2 f32 [rows] or None, entropy f32 [rows] or None)."""
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be 2-D with unit column stride")
    dt = {torch.float32: 0, torch.bfloat16: 1}[logits.dtype]
    rows, vocab = logits.shape
    dev = logits.device
    ids = torch.empty((rows, k), dtype=torch.int32, device=dev)
    pr = torch.empty((rows, k), dtype=torch.float32, device=dev)
    mg = torch.empty(rows, dtype=torch.float32, device=dev) if want_margin else None
    h = torch.empty(rows, dtype=torch.float32, device=dev) if want_entropy else None
    st = _lib.synera_confidence_topk(logits.data_ptr(), dt, rows, vocab, logits.stride(0) if rows > 1 else vocab, k,
                                     ids.data_ptr(), pr.data_ptr(), _dev(mg), _dev(h), _stream())
    _check(st, "synera_confidence_topk")
    return ids, pr, mg, h


def nucleus(logits, top_p):
    """Full-vocabulary top-p per row of a 2-D f32 or bf16 GPU tensor -> (count i32 [rows], mass f32 [rows],
    cut logit f32 [rows])."""
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be 2-D with unit column stride")
    dt = {torch.float32: 0, torch.bfloat16: 1}[logits.dtype]
    rows, vocab = logits.shape
    dev = logits.device
    n = torch.empty(rows, dtype=torch.int32, device=dev)
    mass = torch.empty(rows, dtype=torch.float32, device=dev)
    cut = torch.empty(rows, dtype=torch.float32, device=dev)
    st = _lib.synera_nucleus(logits.data_ptr(), dt, rows, vocab, logits.stride(0) if rows > 1 else vocab, float(top_p),
                             n.data_ptr(), mass.data_ptr(), cut.data_ptr(), _stream())
    _check(st, "synera_nucleus")
    return n, mass, cut


def chunk_dispatch(top1_prob, cu_rows, c_th, k_slope=10.0):
    """(mean confidence f32 [B], P_conf f32 [B]) of the chunks cu_rows[b] .. cu_rows[b+1] of per-row top-1
    probabilities; both arguments GPU tensors (f32 [rows], int32 [B+1])."""
    B = cu_rows.numel() - 1
    mean = torch.empty(max(B, 0), dtype=torch.float32, device=top1_prob.device)
    pc = torch.empty_like(mean)
    st = _lib.synera_chunk_dispatch(_dev(top1_prob, torch.float32), _dev(cu_rows, torch.int32), B, float(c_th),
                                    float(k_slope), mean.data_ptr(), pc.data_ptr(), _stream())
    _check(st, "synera_chunk_dispatch")
    return mean, pc


LO_SITES = {"qkv_in": 1, "gate_up_in": 2, "down_in": 4, "o_in": 8, "lm_head_in": 16, "q": 32, "p": 64,
            "keep_lm_head": 128}      # the LM head runs on the high part alone unless keep_lm_head is set


def split_pair(x, scale=1.0):
    """The fp16 (hi, lo) pair of scale * x (float32 tensor): hi = fp16(v), lo = fp16(v - hi).  Test helper
    (plain torch ops on whatever device x is on); inside a verify the kernels produce the pairs."""
    v = x.float() * scale
    hi = v.to(torch.float16)
    return hi, (v - hi.float()).to(torch.float16)


def gemm_pair(a, a_lo, w, out=None):
    """C = (A + A_lo) W^T on the matrix cores; a, a_lo fp16 [M,K] (a_lo None: A alone), w bf16 [N,K] -> f32 [M,N]."""
    M, K = a.shape
    N = w.shape[0]
    c = torch.empty((M, N), dtype=torch.float32, device=a.device) if out is None else out
    st = _lib.synera_gemm_pair(_dev(a, torch.float16), _dev(a_lo, torch.float16), _dev(w, torch.bfloat16),
                               c.data_ptr(), M, N, K, _stream())
    _check(st, "synera_gemm_pair")
    return c


STATIC_GEMM_MAX_OUT = 524288


def gemm_pair_static(a, a_lo, w, out):
    """synera_gemm_pair for callers that cannot allocate: K slices go through the library's static device array.
    `out` (f32 [M,N]) is the caller's; nothing is allocated here or in the library."""
    M, K = a.shape
    N = w.shape[0]
    st = _lib.synera_gemm_pair_static(_dev(a, torch.float16), _dev(a_lo, torch.float16), _dev(w, torch.bfloat16),
                                      _dev(out, torch.float32), M, N, K, _stream())
    _check(st, "synera_gemm_pair_static")
    return out


def debug_gemm_epilogue(a, a_lo, w0, w1, c, c_lo, epilogue):
    """Test hook: one projection GEMM with epilogue 0 (store), 1 (add into c) or 2 (SwiGLU into the fp16 pair c, c_lo,
    which holds 8 x the value)."""
    M, K = a.shape
    N = w0.shape[0] * (2 if epilogue == 2 else 1)
    st = _lib.synera_debug_gemm_epilogue(_dev(a, torch.float16), _dev(a_lo, torch.float16), _dev(w0, torch.bfloat16),
                                         _dev(w1, torch.bfloat16), c.data_ptr(), c_lo.data_ptr() if c_lo is not None else None,
                                         M, N, K, epilogue, _stream())
    _check(st, "synera_debug_gemm_epilogue")


def debug_gemm_paired(a_pairs, w0, w1, c, epilogue):
    """Test hook: debug_gemm_epilogue with the activation pair as one array [M][K / 32][64] (32 high parts, then
    the 32 low parts of the same K block); epilogue 2 writes c in that form too ([M][N / 64][64])."""
    M = a_pairs.shape[0]
    K = a_pairs[0].numel() // 2
    N = w0.shape[0] * (2 if epilogue == 2 else 1)
    st = _lib.synera_debug_gemm_paired(_dev(a_pairs, torch.float16), _dev(w0, torch.bfloat16), _dev(w1, torch.bfloat16),
                                       c.data_ptr(), M, N, K, epilogue, _stream())
    _check(st, "synera_debug_gemm_paired")


def topp_count(topk_prob, top_p):
    """Nucleus size within each row's top-k window (probabilities most probable first) -> (count i32, mass f32)."""
    rows, k = topk_prob.shape
    n = torch.empty(rows, dtype=torch.int32, device=topk_prob.device)
    mass = torch.empty(rows, dtype=torch.float32, device=topk_prob.device)
    st = _lib.synera_topp_count(_dev(topk_prob, torch.float32), rows, k, float(top_p), _dev(n), _dev(mass), _stream())
    _check(st, "synera_topp_count")
    return n, mass


def debug_gemm_slices(a, a_lo, w):
    """Test hook: the store-form GEMM with K slices stored side by side; returns the f32 slices [n][M][N]."""
    M, K = a.shape
    N = w.shape[0]
    parts = torch.empty((8, M, N), dtype=torch.float32, device=a.device)
    n = C.c_int32(0)
    st = _lib.synera_debug_gemm_slices(_dev(a, torch.float16), _dev(a_lo, torch.float16), _dev(w, torch.bfloat16),
                                       parts.data_ptr(), M, N, K, C.byref(n), _stream())
    _check(st, "synera_debug_gemm_slices")
    return parts[:n.value]


def measure_hbm_copy(dst, src):
    """Measurement tool: one plain device copy dst <- src (same size, 16-byte multiple); HBM moves 2 x the bytes."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("measure_hbm_copy: sizes differ")
    st = _lib.synera_measure_hbm_copy(_dev(dst), _dev(src), nbytes, _stream())
    _check(st, "synera_measure_hbm_copy")
    return 2 * nbytes


MEASURE_READ_BLOCKS = 4096


def measure_hbm_read(out, src):
    """Measurement tool: read-only stream over src; out (int32, 4096 x 256) gets each lane's xor. Returns the bytes read."""
    nbytes = src.numel() * src.element_size()
    if out.numel() < MEASURE_READ_BLOCKS * 256:
        raise ValueError("measure_hbm_read: out needs 4096 x 256 words")
    st = _lib.synera_measure_hbm_read(_dev(out, torch.int32), _dev(src), nbytes, _stream())
    _check(st, "synera_measure_hbm_read")
    return nbytes


def measure_mfma_bf16(out, blocks, iters, random_operands=True):
    """Measurement tool: register-resident bf16 MFMA loop; returns the FLOPs of the launch."""
    if out.numel() < blocks * 256:
        raise ValueError("measure_mfma_bf16: out needs blocks x 256 floats")
    flops = C.c_int64(0)
    st = _lib.synera_measure_mfma_bf16(_dev(out, torch.float32), blocks, iters, 1 if random_operands else 0,
                                       C.byref(flops), _stream())
    _check(st, "synera_measure_mfma_bf16")
    return flops.value


def measure_mfma_f16(out, blocks, iters, random_operands=True):
    """Measurement tool: register-resident loop of the projection kernel's MFMA (16x16x32 fp16); returns the FLOPs
    of the launch."""
    if out.numel() < blocks * 256:
        raise ValueError("measure_mfma_f16: out needs blocks x 256 floats")
    flops = C.c_int64(0)
    st = _lib.synera_measure_mfma_f16(_dev(out, torch.float32), blocks, iters, 1 if random_operands else 0,
                                      C.byref(flops), _stream())
    _check(st, "synera_measure_mfma_f16")
    return flops.value


def debug_attention_plan(shape, attn_blocks, ctx_len, n_uncached, n_draft, block_table):
    """Test hook (host only): the chunk attention's work plan for one batch -> dict of int32 arrays
    shares [n][4], prog [n][4], units [n][8], cuts [n][8]."""
    desc = _ModelDesc(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                      shape.vocab, shape.rope_base, shape.rms_eps)
    ctx, unc, nd = (np.ascontiguousarray(a, dtype=np.int32) for a in (ctx_len, n_uncached, n_draft))
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    B, max_pages = bt.shape
    tiles = int(((ctx.astype(np.int64) + unc + nd + 31) // 32).sum())
    per_request = -(-MAX_CHUNK // max(1, 64 // (shape.n_q_heads // shape.n_kv_heads)))   # row groups of <= 64 rows
    groups = int(B * per_request)
    prog_cap = (tiles * per_request + 4 * groups) * shape.n_kv_heads + 8 * attn_blocks + 64
    unit_cap = groups * shape.n_kv_heads + attn_blocks + 8
    shares = np.zeros((attn_blocks, 4), np.int32)
    prog = np.zeros((prog_cap, 4), np.int32)
    units = np.zeros((unit_cap, 8), np.int32)
    cuts = np.zeros((2 * attn_blocks, 8), np.int32)
    counts = np.zeros(4, np.int32)
    p = lambda a: a.ctypes.data_as(_i32p)                                  # noqa: E731
    st = _lib.synera_debug_attention_plan(C.byref(desc), attn_blocks, B, p(ctx), p(unc), p(nd), p(bt), max_pages,
                                          p(shares), p(prog), prog_cap, p(units), unit_cap, p(cuts), len(cuts), p(counts))
    _check(st, "synera_debug_attention_plan")
    return {"shares": shares[:counts[0]], "prog": prog[:counts[1]], "units": units[:counts[2]], "cuts": cuts[:counts[3]]}


def debug_gemm_plan(M, N, K, epilogue=0, stored_slices=True):
    """Test hook (host only): (tile rows, tile columns, K slices) the planner gives this projection."""
    bm, bn, split = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    st = _lib.synera_debug_gemm_plan(M, N, K, epilogue, 1 if stored_slices else 0, C.byref(bm), C.byref(bn), C.byref(split))
    _check(st, "synera_debug_gemm_plan")
    return bm.value, bn.value, split.value


def debug_gemm_plan_bk(M, N, K, epilogue=0, stored_slices=True):
    """Test hook (host only): K extent of one LDS stage (32 or 64) of the plan debug_gemm_plan reports."""
    bk = C.c_int32(0)
    st = _lib.synera_debug_gemm_plan_bk(M, N, K, epilogue, 1 if stored_slices else 0, C.byref(bk))
    _check(st, "synera_debug_gemm_plan_bk")
    return bk.value


def debug_set_gemm_tile(variant):
    """Tuning hook: force a GEMM tile configuration (-1 = automatic)."""
    _lib.synera_debug_set_gemm_tile(variant)


class Verifier:
    """Owns a synera_ctx for one model.  `head` and `layers` are the bf16 GPU weight
    tensors (dict / list of dicts with the field names of synera_layer_weights);
    they are kept alive here because the context records their addresses."""

    def __init__(self, shape, head, layers, max_batch, max_tokens, max_pages):
        self.shape = shape
        self._keep = (head, layers)
        desc = _ModelDesc(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                          shape.d_ffn, shape.vocab, shape.rope_base, shape.rms_eps)
        arr = (_LayerWeights * shape.n_layers)()
        for l, lw in enumerate(layers):
            for n in _LAYER_FIELDS:
                setattr(arr[l], n, _dev(lw[n], torch.bfloat16))
        w = _Weights(_dev(head["embed"], torch.bfloat16), arr, _dev(head["final_norm"], torch.bfloat16),
                     _dev(head["lm_head"], torch.bfloat16))
        self._ctx = _vp()
        self.max_batch, self.max_tokens, self.max_pages = max_batch, max_tokens, max_pages
        _check(_lib.synera_create(C.byref(self._ctx), C.byref(desc), C.byref(w), max_batch, max_tokens, max_pages),
               "synera_create")

    def close(self):
        if self._ctx:
            _lib.synera_destroy(self._ctx)
            self._ctx = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def verify(self, ctx_len, n_uncached, n_draft, tokens, anchor, block_table, n_pages_in_pool, k_pool, v_pool,
               want_logits=True, want_prob=True, want_entropy=True):
        """One flattened ragged verify.  Host: ctx_len, n_uncached, n_draft, block_table (numpy int32).
        Device: tokens int32 [T], anchor int32 [B], pools bf16.  Returns a dict of GPU tensors."""
        a_ctx, p_ctx = _host_i32(ctx_len)
        a_u, p_u = _host_i32(n_uncached)
        a_k, p_k = _host_i32(n_draft)
        bt = np.ascontiguousarray(block_table, dtype=np.int32)
        B = len(a_ctx)
        R = int(a_k.sum())
        dev = tokens.device
        V = self.shape.vocab
        out = {
            "logits": torch.empty((R, V), dtype=torch.float32, device=dev) if want_logits else None,
            "argmax": torch.empty(R, dtype=torch.int32, device=dev),
            "top1_prob": torch.empty(R, dtype=torch.float32, device=dev) if want_prob else None,
            "entropy": torch.empty(R, dtype=torch.float32, device=dev) if want_entropy else None,
            "accept_len": torch.empty(B, dtype=torch.int32, device=dev),
            "correction": torch.empty(B, dtype=torch.int32, device=dev),
        }
        self.verify_into(a_ctx, a_u, a_k, tokens, anchor, bt, n_pages_in_pool, k_pool, v_pool, out)
        return out

    def verify_into(self, ctx_len, n_uncached, n_draft, tokens, anchor, block_table, n_pages_in_pool, k_pool, v_pool,
                    out):
        """Same call with caller-provided output tensors (int32 numpy metadata, no allocation here)."""
        st = _lib.synera_verify(
            self._ctx, len(ctx_len), ctx_len.ctypes.data_as(_i32p), n_uncached.ctypes.data_as(_i32p),
            n_draft.ctypes.data_as(_i32p), _dev(tokens, torch.int32), _dev(anchor, torch.int32),
            block_table.ctypes.data_as(_i32p), block_table.shape[1], n_pages_in_pool,
            _dev(k_pool, torch.bfloat16), _dev(v_pool, torch.bfloat16), _dev(out["logits"]), _dev(out["argmax"]),
            _dev(out["top1_prob"]), _dev(out["entropy"]), _dev(out["accept_len"]), _dev(out["correction"]),
            _stream())
        _check(st, "synera_verify")

    def importance(self, ctx_len, n_uncached, n_draft, n_pages_in_pool, k_pool, i_th=None, theta=-10.0):
        """Importance scores of the batch the last verify() forwarded (same ctx_len / n_uncached / n_draft):
        -> dict with "scores" (f32 [sum L_i + c_i], request-major), "offsets" (numpy prefix sums [B+1]),
        "mean" (f32 [B], mean over the draft positions) and, with i_th, "p_imp" (f32 [B])."""
        n = np.asarray(ctx_len, np.int64) + np.asarray(n_uncached, np.int64) + np.asarray(n_draft, np.int64)
        offsets = np.concatenate([[0], np.cumsum(n)])
        dev = k_pool.device
        out = {"scores": torch.empty(int(offsets[-1]), dtype=torch.float32, device=dev), "offsets": offsets,
               "mean": torch.empty(len(n), dtype=torch.float32, device=dev),
               "p_imp": torch.empty(len(n), dtype=torch.float32, device=dev) if i_th is not None else None}
        st = _lib.synera_importance(self._ctx, n_pages_in_pool, _dev(k_pool, torch.bfloat16), int(offsets[-1]),
                                    _dev(out["scores"]), float(i_th if i_th is not None else 0.0), float(theta),
                                    _dev(out["mean"]), _dev(out["p_imp"]), _stream())
        _check(st, "synera_importance")
        return out

    def stochastic_accept(self, tokens, p_id, p_prob, u_accept, u_sample):
        """Speculative sampling on the batch the last verify() forwarded -> (accept_len i32 [B], token i32 [B])."""
        R, k_list = p_id.shape
        B = u_sample.numel()
        acc = torch.empty(B, dtype=torch.int32, device=tokens.device)
        tok = torch.empty(B, dtype=torch.int32, device=tokens.device)
        st = _lib.synera_stochastic_accept(self._ctx, _dev(tokens, torch.int32), k_list, _dev(p_id, torch.int32),
                                           _dev(p_prob, torch.float32), _dev(u_accept, torch.float32),
                                           _dev(u_sample, torch.float32), _dev(acc), _dev(tok), _stream())
        _check(st, "synera_stochastic_accept")
        return acc, tok

    def debug_set_lo_off(self, sites):
        """Ablation hook: `sites` = names from LO_SITES (or the bit mask) whose low activation part is dropped."""
        mask = sites if isinstance(sites, int) else sum(LO_SITES[n] for n in sites)
        _check(_lib.synera_debug_set_lo_off(self._ctx, mask), "synera_debug_set_lo_off")

    def debug_set_attention_plan(self, attn_blocks=0, stream_cost=1.0, cut_slack=1.5, t_iter_ratio=3.4 / 1.85):
        _check(_lib.synera_debug_set_attention_plan(self._ctx, attn_blocks, stream_cost, cut_slack, t_iter_ratio),
               "synera_debug_set_attention_plan")

    def debug_read_scratch(self, which, out):
        """Test hook: copy an intermediate buffer of the last layer of the last verify into `out`."""
        _check(_lib.synera_debug_read_scratch(self._ctx, which, out.data_ptr(), out.numel() * out.element_size(),
                                              _stream()), "synera_debug_read_scratch")
        return out

    def profile_begin(self, stage):
        """Bracket every launch of `stage` (a STAGES value) in later verifies with HIP events."""
        _check(_lib.synera_profile_begin(self._ctx, stage), "synera_profile_begin")

    def profile_end(self):
        """-> (number of bracketed launches, their total duration in ms); switches the timing off."""
        n, ms = C.c_int32(0), C.c_float(0.0)
        _check(_lib.synera_profile_end(self._ctx, C.byref(n), C.byref(ms)), "synera_profile_end")
        return n.value, ms.value

    def kv_append(self, layer, ctx_len, n_new, k, v, block_table, n_pages_in_pool, k_pool, v_pool):
        """Scatter bf16 rows k, v [sum n_new, Hkv, hd] of one layer into the paged pools."""
        a_ctx, p_ctx = _host_i32(ctx_len)
        a_n, p_n = _host_i32(n_new)
        bt = np.ascontiguousarray(block_table, dtype=np.int32)
        st = _lib.synera_kv_append(self._ctx, layer, len(a_ctx), p_ctx, p_n, _dev(k, torch.bfloat16),
                                   _dev(v, torch.bfloat16), bt.ctypes.data_as(_i32p), bt.shape[1], n_pages_in_pool,
                                   _dev(k_pool, torch.bfloat16), _dev(v_pool, torch.bfloat16), _stream())
        _check(st, "synera_kv_append")


# ---------------------------------------------------------------------------------- scheduler (host only)
class _SchedStats(C.Structure):
    _fields_ = [("iterations_prefill", C.c_int64), ("iterations_verify", C.c_int64), ("iterations_idle", C.c_int64),
                ("engine_calls", C.c_int64), ("tokens_forwarded", C.c_int64), ("host_ns", C.c_int64),
                ("active_requests", C.c_int32), ("waiting_prefill", C.c_int32), ("waiting_verify", C.c_int32),
                ("free_pages", C.c_int32)]


_i32p, _i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
_lib.synera_sched_create.restype = C.c_int32
_lib.synera_sched_create.argtypes = [C.POINTER(_vp), C.c_int32, C.c_int32, C.c_int32, C.c_int32]
_lib.synera_sched_destroy.restype = C.c_int32
_lib.synera_sched_destroy.argtypes = [_vp]
_lib.synera_sched_submit_prefill.restype = C.c_int32
_lib.synera_sched_submit_prefill.argtypes = [_vp, C.c_int64, C.c_int32]
_lib.synera_sched_submit_verify.restype = C.c_int32
_lib.synera_sched_submit_verify.argtypes = [_vp, C.c_int64, C.c_int32, C.c_int32]
_lib.synera_sched_finish.restype = C.c_int32
_lib.synera_sched_finish.argtypes = [_vp, C.c_int64]
_lib.synera_sched_next.restype = C.c_int32
_lib.synera_sched_next.argtypes = [_vp, _i32p, _i32p, _i64p, _i32p, _i32p, _i32p, _i32p, _i32p, _i32p]
_lib.synera_sched_commit.restype = C.c_int32
_lib.synera_sched_commit.argtypes = [_vp, _i32p]
_lib.synera_sched_cached_len.restype = C.c_int64
_lib.synera_sched_cached_len.argtypes = [_vp, C.c_int64]
_lib.synera_sched_get_stats.restype = C.c_int32
_lib.synera_sched_get_stats.argtypes = [_vp, C.POINTER(_SchedStats)]

SCHED_IDLE, SCHED_PREFILL, SCHED_VERIFY = 0, 1, 2


class Scheduler:
    """Owns a synera_sched.  `next()` returns the host arrays of one engine call as numpy views that stay
    valid until the following `next()`; `commit(accept_len)` reports its result."""

    def __init__(self, n_pages_in_pool, max_pages, max_batch, max_tokens):
        import numpy as np
        self._h = _vp()
        _check(_lib.synera_sched_create(C.byref(self._h), n_pages_in_pool, max_pages, max_batch, max_tokens),
               "synera_sched_create")
        self.max_pages, self.max_batch = max_pages, max_batch
        self._ids = np.zeros(max_batch, dtype=np.int64)
        self._i32 = {n: np.zeros(max_batch, dtype=np.int32)
                     for n in ("ctx_len", "n_uncached", "n_draft", "token_begin", "final_verify")}
        self._bt = np.zeros((max_batch, max_pages), dtype=np.int32)

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.synera_sched_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:      # interpreter shutdown: the library handle may already be gone
            pass

    def submit_prefill(self, request_id, n_prompt):
        _check(_lib.synera_sched_submit_prefill(self._h, request_id, n_prompt), "synera_sched_submit_prefill")

    def submit_verify(self, request_id, n_uncached, n_draft):
        _check(_lib.synera_sched_submit_verify(self._h, request_id, n_uncached, n_draft), "synera_sched_submit_verify")

    def finish(self, request_id):
        _check(_lib.synera_sched_finish(self._h, request_id), "synera_sched_finish")

    def next(self):
        """-> (kind, dict of arrays cut to the call's B entries)"""
        kind, B = C.c_int32(0), C.c_int32(0)
        p = lambda a: a.ctypes.data_as(_i32p)
        _check(_lib.synera_sched_next(self._h, C.byref(kind), C.byref(B), self._ids.ctypes.data_as(_i64p),
                                      p(self._i32["ctx_len"]), p(self._i32["n_uncached"]), p(self._i32["n_draft"]),
                                      p(self._i32["token_begin"]), p(self._i32["final_verify"]), p(self._bt)),
               "synera_sched_next")
        b = B.value
        out = {n: a[:b] for n, a in self._i32.items()}
        out["request_id"] = self._ids[:b]
        out["block_table"] = self._bt[:b]
        return kind.value, out

    def commit(self, accept_len=None):
        import numpy as np
        ptr = None
        if accept_len is not None:
            self._acc = np.ascontiguousarray(accept_len, dtype=np.int32)
            ptr = self._acc.ctypes.data_as(_i32p)
        _check(_lib.synera_sched_commit(self._h, ptr), "synera_sched_commit")

    def cached_len(self, request_id):
        return _lib.synera_sched_cached_len(self._h, request_id)

    def stats(self):
        st = _SchedStats()
        _check(_lib.synera_sched_get_stats(self._h, C.byref(st)), "synera_sched_get_stats")
        return {n: getattr(st, n) for n, _ in _SchedStats._fields_}
