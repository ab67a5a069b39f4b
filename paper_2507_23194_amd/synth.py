"""Seeded synthetic workloads for the output-equivalence check.

These tensors stand in for the output tensors that the unit tests of the GEAK
benchmarks (TritonBench-revised, ROCm Triton Benchmark; paper section 3 and Table 1)
would hand to the evaluator: 2-D fp32/fp16 GEMM/softmax/layernorm-like outputs, a
flash-attention-forward-shaped bf16 tensor, a ragged batch of many test outputs of mixed
dtype, and one very large fp32 tensor.  The paper asks for consistently seeded random
tensors in its unit tests (section 3.1, third enhancement bullet); every generator below
takes explicit seeds.

This module only draws numbers and plants known perturbations.  It contains none of the
comparison rule's arithmetic and is the only code served to both the CPU oracle's tests
and the GPU path's tests.

Every generator returns a ``Workload``.  ``expect`` holds facts that follow from how the
data were planted (which candidates are exact copies, how many elements were pushed far
outside the tolerance and where the first one is), so that a checker can be tested
against something other than another checker.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

ELEM_SIZE = {"f32": 4, "f16": 2, "bf16": 2, "i32": 4, "i64": 8, "u8": 1, "i8": 1, "f64": 8, "f8e4m3": 1, "f8e5m2": 1}
TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i32": torch.int32,
               "i64": torch.int64, "u8": torch.uint8, "i8": torch.int8, "f64": torch.float64,
               "f8e4m3": torch.float8_e4m3fn, "f8e5m2": torch.float8_e5m2}

_CHUNK = 1 << 25  # elements generated per step, bounds temporary memory


@dataclass
class Workload:
    name: str
    atol: float
    rtol: float
    equal_nan: bool
    ref: torch.Tensor                      # dense: 1-D tensor of `dtype`; ragged: 1-D uint8 buffer
    cands: list                            # same kind as ref, one per candidate
    dtype: str | None = None               # dense only
    shape: tuple | None = None             # dense only (logical shape; storage is flat)
    segments: list | None = None           # ragged only: [(byte_offset, numel, dtype_name)]
    expect: dict = field(default_factory=dict)  # (seg, k) -> {"count": int, "first": int}

    @property
    def num_candidates(self) -> int:
        return len(self.cands)

    def algorithmic_bytes(self) -> int:
        """(K+1) x bytes of one tensor: every element of every tensor read once."""
        if self.segments is None:
            per = self.ref.numel() * ELEM_SIZE[self.dtype]
        else:
            per = sum(n * ELEM_SIZE[dt] for (_, n, dt) in self.segments)
        return (len(self.cands) + 1) * per


def to_numpy_raw(t: torch.Tensor) -> np.ndarray:
    """Host copy of a tensor's storage as a numpy array of its raw bits
    (f32 -> float32, f16/bf16 -> uint16 bit patterns, i32 -> int32, uint8 -> uint8)."""
    t = t.detach().contiguous().cpu()
    if t.dtype in (torch.float16, torch.bfloat16):
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _chunks(n: int):
    for lo in range(0, n, _CHUNK):
        yield lo, min(n, lo + _CHUNK)


def _first_true(mask: torch.Tensor, base: int) -> int:
    nz = torch.nonzero(mask.reshape(-1), as_tuple=False)
    return -1 if nz.numel() == 0 else base + int(nz[0, 0])


# --------------------------------------------------------------------------------------
# config 1: fp32 2-D tensor, small additive noise, 1 % far-off elements, two exact copies
# --------------------------------------------------------------------------------------
def config1(rows: int = 1024, cols: int = 1024, num_candidates: int = 8, device="cpu") -> Workload:
    n = rows * cols
    ref = torch.randn(n, generator=_gen(0, device), device=device, dtype=torch.float32)
    cands, expect = [], {}
    n_copies = 2 if num_candidates >= 3 else 0
    for k in range(num_candidates):
        if k >= num_candidates - n_copies:
            cands.append(ref.clone())
            expect[(0, k)] = {"count": 0, "first": -1}
            continue
        g = _gen(1000 * 1 + k, device)
        a = ref + 1e-7 * torch.randn(n, generator=g, device=device, dtype=torch.float32)
        mask = torch.rand(n, generator=g, device=device) < 0.01
        a = torch.where(mask, a + 1e-2, a)
        cands.append(a)
        expect[(0, k)] = {"count": int(mask.sum()), "first": _first_true(mask, 0)}
    return Workload("config1_fp32_2d", 1e-5, 1e-5, False, ref, cands, "f32", (rows, cols), None, expect)


# --------------------------------------------------------------------------------------
# config 2: fp16 heavy-tailed tensor with NaN / +-Inf planted in the reference
# --------------------------------------------------------------------------------------
def config2(rows: int = 8192, cols: int = 8192, num_candidates: int = 64, device="cpu",
            special_frac: float = 1e-4, perturb_frac: float = 1e-3) -> Workload:
    n = rows * cols
    g = _gen(1, device)
    pre = torch.empty(n, device=device, dtype=torch.float32)       # value before planting specials
    for lo, hi in _chunks(n):
        m = hi - lo
        z = torch.randn(m, generator=g, device=device)
        chi = torch.randn(3, m, generator=g, device=device).square_().sum(0)
        t3 = z / torch.sqrt(chi / 3.0)                              # Student-t, nu = 3
        pre[lo:hi] = (0.5 * t3).clamp_(-65504.0, 65504.0)
    pre = pre.to(torch.float16)
    special = torch.rand(n, generator=g, device=device) < special_frac
    sp_idx = torch.nonzero(special, as_tuple=False).reshape(-1)
    kinds = torch.arange(sp_idx.numel(), device=device) % 3         # 0 NaN, 1 +Inf, 2 -Inf
    sp_val = torch.where(kinds == 0, torch.full_like(kinds, float("nan"), dtype=torch.float32),
                         torch.where(kinds == 1, torch.full_like(kinds, float("inf"), dtype=torch.float32),
                                     torch.full_like(kinds, float("-inf"), dtype=torch.float32)))
    ref = pre.clone()
    ref[sp_idx] = sp_val.to(torch.float16)
    n_special = int(sp_idx.numel())

    cands, expect = [], {}
    half = num_candidates // 2
    eligible = (pre.float().abs() < 64.0) & ~special
    for k in range(num_candidates):
        gk = _gen(1000 * 2 + k, device)
        a = torch.empty(n, device=device, dtype=torch.float16)
        count, first = 0, -1
        for lo, hi in _chunks(n):
            m = hi - lo
            x = pre[lo:hi].float() + 1e-4 * torch.randn(m, generator=gk, device=device)
            pm = (torch.rand(m, generator=gk, device=device) < perturb_frac) & eligible[lo:hi]
            x = torch.where(pm, x + 1e-1, x)
            a[lo:hi] = x.to(torch.float16)
            c = int(pm.sum())
            if c and first < 0:
                first = _first_true(pm, lo)
            count += c
        if k < half:
            a[sp_idx] = ref[sp_idx]                 # shares the reference's NaN / Inf
        else:
            if k % 4 == 0:                          # opposite-signed infinity where the reference is infinite
                opp = torch.where(kinds == 1, torch.full_like(sp_val, float("-inf")),
                                  torch.where(kinds == 2, torch.full_like(sp_val, float("inf")),
                                              a[sp_idx].float()))
                a[sp_idx] = opp.to(torch.float16)
            count += n_special
            if n_special:
                f_sp = int(sp_idx[0])
                first = f_sp if first < 0 else min(first, f_sp)
        cands.append(a)
        expect[(0, k)] = {"count": count, "first": first}
    return Workload("config2_fp16_heavy_tail", 1e-3, 1e-3, True, ref, cands, "f16", (rows, cols), None, expect)


# --------------------------------------------------------------------------------------
# config 3: bf16 attention-output-shaped tensor
# --------------------------------------------------------------------------------------
def config3(shape=(16, 32, 4096, 128), num_candidates: int = 16, device="cpu", block: int = 4096) -> Workload:
    n = int(np.prod(shape))
    block = min(block, max(1, n // 4))
    g = _gen(2, device)
    ref = torch.empty(n, device=device, dtype=torch.bfloat16)
    for lo, hi in _chunks(n):
        ref[lo:hi] = torch.randn(hi - lo, generator=g, device=device).to(torch.bfloat16)
    cands, expect = [], {}
    half = num_candidates // 2
    for k in range(num_candidates):
        gk = _gen(1000 * 3 + k, device)
        if k < half:
            # one-ulp flips of the bit pattern on about half of the elements
            a = torch.empty_like(ref)
            for lo, hi in _chunks(n):
                m = hi - lo
                bits = ref[lo:hi].view(torch.int16).to(torch.int32) & 0xFFFF
                expo = bits & 0x7F80
                safe = (expo > 0) & (expo < 0x7F00)
                flip = (torch.rand(m, generator=gk, device=device) < 0.5) & safe
                step = torch.where(torch.rand(m, generator=gk, device=device) < 0.5, 1, -1).to(torch.int32)
                nb = torch.where(flip, bits + step, bits)
                nb = torch.where(nb >= 0x8000, nb - 0x10000, nb).to(torch.int16)
                a[lo:hi] = nb.view(torch.bfloat16)
            expect[(0, k)] = {"count": 0, "first": -1}
        else:
            a = ref.clone()
            off = int(torch.randint(0, n - block + 1, (1,), generator=gk, device=device))
            a[off:off + block] = (ref[off:off + block].float() + 1.0).to(torch.bfloat16)
            expect[(0, k)] = {"count": block, "first": off}
        cands.append(a)
    return Workload("config3_bf16_attention", 1e-2, 1.6e-2, False, ref, cands, "bf16", tuple(shape), None, expect)


# --------------------------------------------------------------------------------------
# config 4: ragged batch of many tensors of mixed dtype, packed with a segment table
# --------------------------------------------------------------------------------------
def config4(num_segments: int = 1024, log2_max: float = 20.0, num_candidates: int = 4, device="cpu",
            align: int = 16, seed: int = 3, dtypes=("f32", "f16", "bf16", "i32")) -> Workload:
    """align: byte alignment of every segment start (16 = the packed layout the benchmark uses;
    smaller values, down to the element size, exercise unaligned starts).  dtypes: the dtypes the
    segments are drawn from (the benchmark recipe is the default four; tests add "i64")."""
    rng = np.random.default_rng(seed)
    u = rng.random(num_segments)
    sizes = np.maximum(1, np.floor(2.0 ** (log2_max * u))).astype(np.int64)
    names = list(dtypes)
    dts = [names[i] for i in rng.integers(0, len(names), num_segments)]
    segments, off = [], 0
    for s in range(num_segments):
        w = ELEM_SIZE[dts[s]]
        a = max(align, w)
        if align < 16:                       # unaligned packing: random extra element-sized gap
            off += w * int(rng.integers(0, 4))
        off = (off + a - 1) // a * a
        segments.append((off, int(sizes[s]), dts[s]))
        off += int(sizes[s]) * w
    total = (off + 15) // 16 * 16
    ref = torch.zeros(total, device=device, dtype=torch.uint8)
    cands = [torch.zeros(total, device=device, dtype=torch.uint8) for _ in range(num_candidates)]
    expect = {}
    for s, (boff, n, dt) in enumerate(segments):
        w = ELEM_SIZE[dt]
        g = _gen(10_000 + s, device)
        if dt == "i32":
            b = torch.randint(-1000, 1001, (n,), generator=g, device=device, dtype=torch.int32)
        elif dt == "u8":
            b = torch.randint(0, 256, (n,), generator=g, device=device, dtype=torch.int32).to(torch.uint8)
        elif dt == "i8":
            b = torch.randint(-128, 128, (n,), generator=g, device=device, dtype=torch.int32).to(torch.int8)
        elif dt == "i64":
            b = torch.randint(-1000, 1001, (n,), generator=g, device=device, dtype=torch.int64)
            big = torch.rand(n, generator=g, device=device) < 0.05                # values beyond 2^53
            b = torch.where(big, b * (1 << 52) + 12345, b)
        elif dt == "f64":
            b = torch.randn(n, generator=g, device=device, dtype=torch.float64)
        else:
            b = torch.randn(n, generator=g, device=device).to(TORCH_DTYPE[dt])
        ref[boff:boff + n * w] = b.view(torch.uint8)
        for k in range(num_candidates):
            gk = _gen(1000 * 4 + 7919 * s + k, device)
            if dt in ("i32", "i64", "u8", "i8"):
                a = b.clone()
                if (s + k) % 2 == 1:
                    j = int(torch.randint(0, n, (1,), generator=gk, device=device))
                    a[j] += 1
                    expect[(s, k)] = {"count": 1, "first": j}
                else:
                    expect[(s, k)] = {"count": 0, "first": -1}
            else:
                wide = b if dt == "f64" else b.float()
                x = wide + 1e-6 * torch.randn(n, generator=gk, device=device, dtype=wide.dtype)
                om = torch.rand(n, generator=gk, device=device) < 0.005
                x = torch.where(om, wide + 0.5, x)
                a = x.to(TORCH_DTYPE[dt])
                expect[(s, k)] = {"count": int(om.sum()), "first": _first_true(om, 0)}
            cands[k][boff:boff + n * w] = a.view(torch.uint8)
    return Workload("config4_ragged_mixed", 1e-3, 1e-3, False, ref, cands, None, None, segments, expect)


# --------------------------------------------------------------------------------------
# config 5: one very large fp32 tensor with subnormals and signed zeros
# --------------------------------------------------------------------------------------
def config5(log2_n: int = 30, num_candidates: int = 32, device="cpu",
            special_frac: float = 0.01, mismatch_frac: float = 1e-6) -> Workload:
    n = 1 << log2_n
    g = _gen(4, device)
    ref = torch.empty(n, device=device, dtype=torch.float32)
    for lo, hi in _chunks(n):
        m = hi - lo
        b = (torch.rand(m, generator=g, device=device, dtype=torch.float32) * 2.0 - 1.0) * 1e3
        sp = torch.rand(m, generator=g, device=device) < special_frac
        kind = torch.randint(0, 3, (m,), generator=g, device=device)
        mant = torch.randint(1, 1 << 23, (m,), generator=g, device=device, dtype=torch.int32)
        sign = torch.randint(0, 2, (m,), generator=g, device=device, dtype=torch.int32) << 31
        denorm = (mant | sign).view(torch.float32)                  # +-m * 2^-149
        zero_p = torch.zeros(m, device=device)
        zero_n = torch.full((m,), -0.0, device=device)
        planted = torch.where(kind == 0, denorm, torch.where(kind == 1, zero_p, zero_n))
        ref[lo:hi] = torch.where(sp, planted, b)
    cands, expect = [], {}
    for k in range(num_candidates):
        gk = _gen(1000 * 5 + k, device)
        a = torch.empty(n, device=device, dtype=torch.float32)
        count, first = 0, -1
        for lo, hi in _chunks(n):
            m = hi - lo
            b = ref[lo:hi]
            x = b * (1.0 + 1e-7 * torch.randn(m, generator=gk, device=device, dtype=torch.float32))
            flip = (b == 0) & (torch.rand(m, generator=gk, device=device) < 0.5)
            x = torch.where(flip, -x, x)
            mm = torch.rand(m, generator=gk, device=device, dtype=torch.float64) < mismatch_frac
            x = torch.where(mm, b + 1.0, x)
            a[lo:hi] = x
            c = int(mm.sum())
            if c and first < 0:
                first = _first_true(mm, lo)
            count += c
        cands.append(a)
        expect[(0, k)] = {"count": count, "first": first}
    return Workload("config5_fp32_large", 1e-6, 1e-5, False, ref, cands, "f32", (n,), None, expect)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def dense_noise(dtype: str, log2_n: int, num_candidates: int, device="cpu") -> Workload:
    """A plain dense workload of any floating dtype, for measuring the dtypes the five configurations do not
    use (the 8-bit formats above all): standard normal reference, candidates = reference * (1 + 2 % noise),
    rounded to the dtype; finite values only."""
    n = 1 << log2_n
    g = _gen(77, device)
    ref32 = torch.randn(n, generator=g, device=device)
    ref = ref32.to(TORCH_DTYPE[dtype])
    cands = []
    for k in range(num_candidates):
        gk = _gen(7700 + k, device)
        cands.append((ref32 * (1.0 + 0.02 * torch.randn(n, generator=gk, device=device))).to(TORCH_DTYPE[dtype]))
    return Workload(f"dense_noise_{dtype}", 1e-2, 0.1, False, ref, cands, dtype, (n,), None, {})


def small(config_id: int, device="cpu") -> Workload:
    """Reduced-size version of a config with the same recipe, sized so the CPU oracle
    finishes in a second or so while the GPU path still sees several tiles and a ragged tail."""
    if config_id == 1:
        return config1(rows=257, cols=1031, num_candidates=8, device=device)
    if config_id == 2:
        return config2(rows=509, cols=1021, num_candidates=8, device=device, special_frac=1e-3)
    if config_id == 3:
        return config3(shape=(2, 3, 257, 128), num_candidates=6, device=device)
    if config_id == 4:
        return config4(num_segments=96, log2_max=16.0, num_candidates=4, device=device)
    if config_id == 5:
        return config5(log2_n=20, num_candidates=4, device=device, mismatch_frac=1e-4)
    raise ValueError(config_id)
