"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

numpy-facing wrapper around ``qmoe_oracle.c`` (plain C, fp64, one thread).
Only the tests, ``__graft_entry__.smoke()`` and the benchmark's CPU-baseline
leg may import this package; the product never does, and this package never
imports the product.

Paper passages followed: Section 4.3.2 (source model Eq. 2, Algorithm 1,
entry layout), Section 4.3.3 (decoding order, encoding by longest prefix
match over a trie), Section 2.1 (one expert per token).
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libqmoe_oracle.so")
_SRC = os.path.join(_HERE, "qmoe_oracle.c")

P0_DEFAULT = 0.885      # Section 4.3.2: "e.g. 0.885"
MAX_PAIRS_DEFAULT = 14  # Section 4.3.2: at most 14 pairs per sequence
N_ENTRIES_DEFAULT = 1 << 16


# ORACLE_SANITIZE=1: the same source built with AddressSanitizer and UndefinedBehaviorSanitizer
# (the process must then preload gcc's libasan; tests/test_sanitizers.py does that in a child)
_SANITIZE = os.environ.get("ORACLE_SANITIZE") == "1"
if _SANITIZE:
    _SO = os.path.join(_HERE, "libqmoe_oracle_san.so")


def build() -> str:
    flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] if _SANITIZE else ["-O2"]
    subprocess.check_call(["gcc", *flags, "-fPIC", "-shared", "-o", _SO, _SRC, "-lm"])
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        lib = ctypes.CDLL(_SO)
        c = ctypes
        vp, i64, u64, dbl, i32 = c.c_void_p, c.c_int64, c.c_uint64, c.c_double, c.c_int
        lib.orc_dict_build.argtypes = [dbl, i32, i32, vp, vp]
        lib.orc_dict_build.restype = i32
        lib.orc_dict_pack.argtypes = [vp, vp, i32, vp]
        lib.orc_dict_pack.restype = None
        lib.orc_encode.argtypes = [vp, vp, i32, vp, i64, i64, vp, u64, vp, vp]
        lib.orc_encode.restype = i32
        lib.orc_decode.argtypes = [vp, i32, vp, vp, i64, i64, vp]
        lib.orc_decode.restype = i32
        lib.orc_matvec.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp]
        lib.orc_matvec.restype = None
        lib.orc_ffn_token.argtypes = [vp, vp, vp, vp, vp, i64, i64, dbl, vp, vp, vp]
        lib.orc_ffn_token.restype = None
        lib.orc_matvec_asym.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp]
        lib.orc_matvec_asym.restype = None
        lib.orc_ffn_token_asym.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, dbl, vp, vp, vp]
        lib.orc_ffn_token_asym.restype = None
        lib.orc_slot_parallel_matvec.argtypes = [vp, i32, vp, vp, vp, vp, i64, i64, vp]
        lib.orc_slot_parallel_matvec.restype = i32
        lib.orc_dispatch.argtypes = [vp, i64, i64, vp, vp]
        lib.orc_dispatch.restype = None
        lib.orc_bf16_to_double.argtypes = [c.c_uint16]
        lib.orc_bf16_to_double.restype = dbl
        lib.orc_f16_to_double.argtypes = [c.c_uint16]
        lib.orc_f16_to_double.restype = dbl
        lib.orc_double_to_bf16.argtypes = [dbl]
        lib.orc_double_to_bf16.restype = c.c_uint16
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data


class Dictionary:
    """The static decoding dictionary of Section 4.3.2.

    syms   uint8 [n, 28]  ternary symbols 0/1/2, unused slots 0
    npairs uint8 [n]      pairs per entry
    words  uint32 [n, 2]  the packed 64-bit entries
    """

    def __init__(self, p0: float = P0_DEFAULT, max_pairs: int = MAX_PAIRS_DEFAULT,
                 n_entries: int = N_ENTRIES_DEFAULT):
        lib = _load()
        syms = np.zeros((n_entries, 28), dtype=np.uint8)
        npairs = np.zeros(n_entries, dtype=np.uint8)
        n = lib.orc_dict_build(p0, max_pairs, n_entries, _p(syms), _p(npairs))
        if n < 0:
            raise ValueError("bad dictionary parameters")
        self.p0, self.max_pairs = p0, max_pairs
        self.syms, self.npairs = syms[:n].copy(), npairs[:n].copy()
        self.n = n
        self.words = np.zeros((n, 2), dtype=np.uint32)
        lib.orc_dict_pack(_p(self.syms), _p(self.npairs), n, _p(self.words))

    def sequences(self):
        """Entries as tuples of symbols (for brute-force checks)."""
        return [tuple(int(v) for v in self.syms[k, : 2 * self.npairs[k]]) for k in range(self.n)]

    def expected_values_per_codeword(self, p: float) -> float:
        """Mean number of weights one codeword covers when an endless i.i.d.
        stream with zero probability p is parsed greedily.

        A phrase s is emitted when the stream continues with s and the pair t
        after it leads out of the dictionary (s.t not in D).  That pair t is not
        consumed: it opens the next phrase, so consecutive phrases are not
        independent -- the next phrase's first pair is drawn from the pairs that
        s could NOT be extended with.  The first pair of each phrase is a
        9-state Markov chain; with its stationary distribution pi,
        E[L] = sum_t0 pi(t0) * E[len | phrase starts with t0]
        (renewal-reward).  Valid because the dictionary is prefix-closed
        (checked by the tests).
        """
        q = (1.0 - p) / 2.0
        ps = [p, q, q]
        seqs = self.sequences()
        index = set(seqs)
        pairs = [(a, b) for a in range(3) for b in range(3)]
        pp = {t: ps[t[0]] * ps[t[1]] for t in pairs}
        trans = np.zeros((9, 9))
        mean_len = np.zeros(9)
        for s in seqs:
            t0 = pairs.index(s[:2])
            cond = math.prod(ps[v] for v in s) / pp[s[:2]]  # P(stream continues with s | first pair)
            for j, t in enumerate(pairs):
                if len(s) >= 2 * self.max_pairs or s + t not in index:
                    trans[t0, j] += cond * pp[t]
                    mean_len[t0] += cond * pp[t] * len(s)
        assert np.allclose(trans.sum(axis=1), 1.0, atol=1e-9)
        w, v = np.linalg.eig(trans.T)
        pi = np.real(v[:, np.argmin(np.abs(w - 1.0))])
        pi = pi / pi.sum()
        return float(pi @ mean_len)


def encode(d: Dictionary, tern: np.ndarray):
    """Longest-prefix encode of an int8 {-1,0,+1} matrix.

    Returns (codes uint16 [n_codes], row_off uint32 [rows+1])."""
    lib = _load()
    tern = np.ascontiguousarray(tern, dtype=np.int8)
    rows, cols = tern.shape
    row_off = np.zeros(rows + 1, dtype=np.uint32)
    n_codes = ctypes.c_uint64(0)
    cap = rows * (cols // 2) if cols % 2 == 0 else 0
    codes = np.zeros(max(cap, 1), dtype=np.uint16)
    rc = lib.orc_encode(_p(d.syms), _p(d.npairs), d.n, _p(tern), rows, cols, _p(codes), cap,
                        _p(row_off), ctypes.byref(n_codes))
    if rc:
        raise ValueError({1: "symbol outside {-1,0,+1}", 2: "odd number of columns",
                          3: "capacity", 4: "phrase not in dictionary"}.get(rc, f"error {rc}"))
    return codes[: n_codes.value].copy(), row_off


def decode(words: np.ndarray, codes: np.ndarray, row_off: np.ndarray, rows: int, cols: int) -> np.ndarray:
    lib = _load()
    words = np.ascontiguousarray(words, dtype=np.uint32)
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    row_off = np.ascontiguousarray(row_off, dtype=np.uint32)
    out = np.zeros((rows, cols), dtype=np.int8)
    rc = lib.orc_decode(_p(words), words.shape[0], _p(codes), _p(row_off), rows, cols, _p(out))
    if rc:
        raise ValueError({1: "row does not decode to exactly cols values", 2: "codeword out of range",
                          3: "symbol value 3", 4: "count nibbles differ"}.get(rc, f"error {rc}"))
    return out


def matvec(tern: np.ndarray, scale_f16: np.ndarray, x_bf16: np.ndarray, with_bound: bool = False,
           minmax_bf16: np.ndarray | None = None):
    """y[b, r] = s_r * sum_c T[r, c] x[b, c] in fp64.  x_bf16: uint16 [batch, cols].
    With minmax_bf16 (uint16 [rows, 2] = bfloat16 (w_min, w_max) per row; scale_f16 is not read
    then) the row's grid is {w_min, 0, w_max} (Section 4.1; "Ternary decoding" in Section 4.3.3):
    y = w_max * (sum of x under +1) + w_min * (sum of x under -1)."""
    lib = _load()
    tern = np.ascontiguousarray(tern, dtype=np.int8)
    rows, cols = tern.shape
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16).reshape(-1, cols)
    y = np.zeros((x.shape[0], rows), dtype=np.float64)
    bound = np.zeros_like(y) if with_bound else None
    if minmax_bf16 is None:
        s = np.ascontiguousarray(scale_f16, dtype=np.uint16)
        assert s.shape == (rows,)
        lib.orc_matvec(_p(tern), _p(s), _p(x), rows, cols, x.shape[0], _p(y),
                       _p(bound) if with_bound else None)
    else:
        mm = np.ascontiguousarray(minmax_bf16, dtype=np.uint16)
        assert mm.shape == (rows, 2)
        lib.orc_matvec_asym(_p(tern), _p(mm), _p(x), rows, cols, x.shape[0], _p(y),
                            _p(bound) if with_bound else None)
    return (y, bound) if with_bound else y


def slot_parallel_matvec(words: np.ndarray, codes: np.ndarray, row_off: np.ndarray, rows: int, cols: int,
                         w_min: np.ndarray, w_max: np.ndarray, x_bf16: np.ndarray) -> np.ndarray:
    """The product in its second formulation (Section 4.3.3 "Execution", Listing 1): 28 slot
    workers straight from (entry words, codewords, row offsets), no decoded matrix.
    w_min / w_max: float64 [rows]; x_bf16: uint16 [cols].  Returns y float64 [rows]."""
    lib = _load()
    words = np.ascontiguousarray(words, dtype=np.uint32)
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    row_off = np.ascontiguousarray(row_off, dtype=np.uint32)
    mm = np.ascontiguousarray(np.stack([w_min, w_max], axis=1), dtype=np.float64)
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    assert x.shape == (cols,) and mm.shape == (rows, 2) and row_off.shape == (rows + 1,)
    y = np.zeros(rows, dtype=np.float64)
    rc = lib.orc_slot_parallel_matvec(_p(words), words.shape[0], _p(codes), _p(row_off), _p(mm), _p(x), rows, cols,
                                      _p(y))
    if rc:
        raise ValueError({1: "a row's phrases run past its end", 2: "codeword out of range",
                          3: "symbol value 3"}.get(rc, f"error {rc}"))
    return y


def ffn_token(wi, wi_scale, wo, wo_scale, x_bf16, gate: float = 1.0, wi_minmax=None, wo_minmax=None):
    """One token through one expert: returns (y fp64 [d_model], h bf16 bits [d_ff], bound [d_model]).
    With wi_minmax and wo_minmax (both or neither) the matrices use the asymmetric grid."""
    lib = _load()
    wi = np.ascontiguousarray(wi, dtype=np.int8)
    wo = np.ascontiguousarray(wo, dtype=np.int8)
    d_ff, d_model = wi.shape
    assert wo.shape == (d_model, d_ff)
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    assert x.shape == (d_model,)
    assert (wi_minmax is None) == (wo_minmax is None)
    y = np.zeros(d_model, dtype=np.float64)
    h = np.zeros(d_ff, dtype=np.uint16)
    bound = np.zeros(d_model, dtype=np.float64)
    if wi_minmax is None:
        wis = np.ascontiguousarray(wi_scale, dtype=np.uint16)
        wos = np.ascontiguousarray(wo_scale, dtype=np.uint16)
        lib.orc_ffn_token(_p(wi), _p(wis), _p(wo), _p(wos), _p(x), d_model, d_ff, float(gate), _p(y), _p(h),
                          _p(bound))
    else:
        wim = np.ascontiguousarray(wi_minmax, dtype=np.uint16)
        wom = np.ascontiguousarray(wo_minmax, dtype=np.uint16)
        assert wim.shape == (d_ff, 2) and wom.shape == (d_model, 2)
        lib.orc_ffn_token_asym(_p(wi), None, _p(wim), _p(wo), None, _p(wom), _p(x), d_model, d_ff, float(gate),
                               _p(y), _p(h), _p(bound))
    return y, h, bound


def dispatch(expert_idx: np.ndarray, n_experts: int):
    """Stable grouping of tokens by expert: (tok_off int32 [E+1], perm int32 [n_valid])."""
    lib = _load()
    idx = np.ascontiguousarray(expert_idx, dtype=np.int32)
    tok_off = np.zeros(n_experts + 1, dtype=np.int32)
    perm = np.full(idx.size, -1, dtype=np.int32)
    lib.orc_dispatch(_p(idx), idx.size, n_experts, _p(tok_off), _p(perm))
    return tok_off, perm[: tok_off[-1]].copy()


def moe_layer(workload, expert_idx: np.ndarray, x_bf16: np.ndarray, gate=None, tokens=None, asym: bool = False):
    """y[t] = gate_t * Wo_e bf16(relu(Wi_e x_t)), e = expert_idx[t], for the tokens asked for.

    ``workload`` supplies wi_ternary(e), wo_ternary(e), wi_scale(e), wo_scale(e) and, for the
    asymmetric grid (asym), wi_minmax(e), wo_minmax(e).
    Returns dict token -> (y fp64, h bf16 bits, bound)."""
    out = {}
    toks = range(expert_idx.size) if tokens is None else tokens
    by_expert = {}
    for t in toks:
        by_expert.setdefault(int(expert_idx[t]), []).append(int(t))
    for e, ts in by_expert.items():
        wi, wo = workload.wi_ternary(e), workload.wo_ternary(e)
        wis, wos = workload.wi_scale(e), workload.wo_scale(e)
        wim = workload.wi_minmax(e) if asym else None
        wom = workload.wo_minmax(e) if asym else None
        for t in ts:
            g = 1.0 if gate is None else float(gate[t])
            out[t] = ffn_token(wi, wis, wo, wos, x_bf16[t], g, wim, wom)
    return out


def bits_per_param(n_codes: int, rows: int, cols: int, with_row_metadata: bool = False) -> float:
    """16 bits per codeword over rows*cols weights (Section 4.3.2, "Validation");
    row metadata = one 32-bit offset and one 16-bit scale per row."""
    bits = 16.0 * n_codes + (48.0 * rows if with_row_metadata else 0.0)
    return bits / (rows * cols)


def entropy_limit_ratio(p: float) -> float:
    """16 / H(p) for the ternary source of Eq. 2 (the paper's "theoretical compression limit")."""
    q = (1.0 - p) / 2.0
    h = -(p * math.log2(p) + 2.0 * q * math.log2(q))
    return 16.0 / h
