"""sage_quant_kv_static -- the entry point for callers that cannot allocate -- against sage_quant_kv, through
the C ABI: every output must be the same bits.  Two calls in a row share the library's built-in scratch, the
second with a smaller input (the scratch then still holds the first call's partial statistics); a problem
beyond the built-in scratch is refused with SAGE_ESCRATCH and enqueues nothing."""
import pytest
import torch

import paper_2505_21136_amd as sage
import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
NAMES = ("k_i8", "k_scale", "k_mean", "v_fp8", "v_scale")


def _bits(t):
    return t.contiguous().view(torch.uint8)


def _outputs(B, H, N, d):
    return (torch.full((B, H, N, d), 0x55, dtype=torch.int8, device=DEV),
            torch.full((B, H, -(-N // 64)), float("nan"), dtype=torch.float32, device=DEV),
            torch.full((B, H, d), float("nan"), dtype=torch.float32, device=DEV),
            torch.full((B, H, -(-N // 128), d, 128), 0x55, dtype=torch.uint8, device=DEV),
            torch.full((B, H, d), float("nan"), dtype=torch.float32, device=DEV))


def _run_static(k, v, v_r=4.5):
    """Direct ctypes call: inputs and preallocated outputs in, return code out -- what a caller that cannot
    allocate would do."""
    B, H, N, d = k.shape
    out = _outputs(B, H, N, d)
    torch.cuda.synchronize()
    rc = sage.lib().sage_quant_kv_static(k.data_ptr(), v.data_ptr(), *(t.data_ptr() for t in out), float(v_r),
                                         B, H, N, d, 1 if k.dtype == torch.bfloat16 else 0,
                                         torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return rc, out


def test_static_scratch_entry_point_equals_the_workspace_one_on_two_calls_in_a_row():
    big = wl.Workload("big", 5, 2, 6, 5000, 128, False, "bf16", "student_t3", 4)     # 5 chunks per head
    small = wl.Workload("small", 3, 1, 3, 333, 64, False, "bf16")                     # fewer heads, ragged, other d
    for i, cfg in enumerate((big, small)):
        print(f"[no-alloc] call {i}: B{cfg.B} H{cfg.H} N{cfg.N} d{cfg.d} {cfg.dtype}", flush=True)
        _, k, v = wl.generate(cfg, seed=wl.SEED0 + 40 + i)
        k, v = k.to(DEV), v.to(DEV)
        assert sage.quant_workspace_bytes(cfg.B, cfg.H, cfg.N, cfg.d) <= (8 << 20)
        want = sage.sage_quant_kv(k, v, 4.5)
        rc, got = _run_static(k, v)
        assert rc == 0, sage.lib().sage_strerror(rc)
        for name, a, b in zip(NAMES, got, want):
            assert torch.equal(_bits(a), _bits(b)), f"call {i}: {name} differs"


def test_static_scratch_refuses_a_problem_beyond_its_size():
    B, H, N, d = 1, 24, 262144, 128
    assert sage.quant_workspace_bytes(B, H, N, d) > (8 << 20)
    # nothing may be touched: tiny buffers would be overrun by any launch, so the call must return first
    k = torch.zeros(16, dtype=torch.bfloat16, device=DEV)
    o = torch.zeros(16, dtype=torch.float32, device=DEV)
    rc = sage.lib().sage_quant_kv_static(k.data_ptr(), k.data_ptr(), o.data_ptr(), o.data_ptr(), o.data_ptr(),
                                         o.data_ptr(), o.data_ptr(), 4.5, B, H, N, d, 1, 0)
    assert rc == -4
    assert b"static scratch" in sage.lib().sage_strerror(rc)
    torch.cuda.synchronize()


def test_python_wrapper_of_the_static_entry_point():
    cfg = wl.Workload("w", 1, 1, 2, 700, 128, False, "fp16")
    _, k, v = wl.generate(cfg, seed=wl.SEED0 + 44)
    k, v = k.to(DEV), v.to(DEV)
    got = sage.sage_quant_kv_static(k, v, 2.25)
    want = sage.sage_quant_kv(k, v, 2.25)
    torch.cuda.synchronize()
    for name, a, b in zip(NAMES, got, want):
        assert torch.equal(_bits(a), _bits(b)), name
