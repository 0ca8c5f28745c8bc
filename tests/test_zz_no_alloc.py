"""conf_kv_step_static (the confidence step with its partial sums in the library's own device
array) against conf_kv_step, through the C ABI: two calls in a row on one GPU, the second on a
smaller input, so the shared array still holds the first call's words."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _mk(lib, V, B):
    return lib.ConfKV(n_layers=3, batch=B, n_q_heads=4, n_kv_heads=1, head_dim=128, vocab=V, capacity=256,
                      fp16_window=16, protected_window=8, n_tight=[64, 48, 32], n_loose=[128, 96, 64])


def test_step_static_matches_step_on_two_calls_in_a_row(lib):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    rng = np.random.default_rng(5)
    shapes = [(128256, 8), (5003, 3)]                 # 32 chunks x 8 rows, then 2 chunks x 3 rows
    kvs = [_mk(lib, V, B) for V, B in shapes]
    for rnd, std in enumerate((6.0, 0.5, 6.0)):
        for (V, B), kv in zip(shapes, kvs):
            print(f"conf_kv_step_static round {rnd} V={V} B={B} std={std}", flush=True)
            x = torch.from_numpy((rng.standard_normal((B, V)) * std).astype(np.float32)).cuda()
            got_c = torch.full((B,), -1.0, dtype=torch.float32, device="cuda")
            got_s = torch.full((B,), 9, dtype=torch.uint8, device="cuda")
            ref_c = torch.full((B,), -2.0, dtype=torch.float32, device="cuda")
            ref_s = torch.full((B,), 7, dtype=torch.uint8, device="cuda")
            kv.step_static(x, got_c, got_s)
            budget_static = kv.state.clone()
            kv.step(x, ref_c, ref_s)
            torch.cuda.synchronize()
            # same kernel, same reduction order: bit-equal confidence, equal choice
            assert np.array_equal(got_c.cpu().numpy().view(np.uint32), ref_c.cpu().numpy().view(np.uint32))
            assert np.array_equal(got_s.cpu().numpy(), ref_s.cpu().numpy())
            assert set(np.unique(got_s.cpu().numpy())) <= {0, 1}
            # the per-layer budgets the two calls left in the cache state are the same bytes
            # (everything but the tight/loose step counters, which count both calls)
            a, b = budget_static.cpu().numpy(), kv.state.cpu().numpy()
            diff = np.flatnonzero(a != b)
            assert diff.size <= 16, diff[:32]         # two 8-byte counters at most
    for kv in kvs:
        st = kv.counters()
        assert st.device_errors == 0 and st.tight_steps + st.loose_steps == 2 * 3 * kv.cfg.batch
        kv.close()


def test_step_static_rejects_what_does_not_fit(lib):
    kv = _mk(lib, 152064, 512)                       # 38 chunks x 512 rows x 64 B > 1 MiB
    import torch
    x = torch.zeros((512, 152064), dtype=torch.float32, device="cuda")
    with pytest.raises(lib.ConfKVError) as e:
        kv.step_static(x)
    assert e.value.status == lib.binding.ERR_CAPACITY
    kv.step(x)                                        # the workspace form still serves it
    torch.cuda.synchronize()
    assert kv.counters().device_errors == 0
    kv.close()
