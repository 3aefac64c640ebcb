"""Seeded sweep over small random shapes: group sizes, head dims, pool types, chunk lengths, empty and
one-token sequences, shared-prefix groups and query stretches in random combination, each checked against
the oracle (GPU only).  The cases are valid inputs; this widens the combinations the targeted tests cover."""
import numpy as np
import pytest

import oracle
import workloads
from workloads import f32_to_bf16_bits
from tests.test_gpu_parity import check, check_fp8, device_workload, gpu_attend, gpu_attend_prefix, oracle_full, sd  # noqa: F401

pytestmark = pytest.mark.gpu

HEADS = [(1, 1), (2, 1), (3, 1), (4, 2), (6, 2), (7, 1), (8, 2), (8, 8), (16, 1), (12, 4), (28, 4), (32, 2),
         (17, 1), (32, 1), (40, 2), (64, 1), (48, 2)]   # the last five: more than 16 query heads per KV head


def draw_lens(rng, n, hi):
    lens = rng.integers(1, hi, size=n, endpoint=True)
    lens[rng.random(n) < 0.15] = 0                      # some empty sequences
    lens[rng.random(n) < 0.15] = rng.integers(1, 4)     # some very short ones
    edge = rng.random(n) < 0.3                          # some on page / tile / chunk edges
    lens[edge] = (lens[edge] // 128) * 128 + rng.choice([0, 1, 15, 16, 17, 31, 32, 33, 127], size=int(edge.sum()))
    return np.maximum(lens, 0)


@pytest.mark.parametrize("seed", range(24))
def test_decode_random_shapes(sd, seed):
    rng = np.random.default_rng(1000 + seed)
    Hq, Hkv = HEADS[int(rng.integers(len(HEADS)))]
    kv_dtype = "fp8" if rng.random() < 0.35 else "bf16"
    d = 128 if rng.random() < 0.6 else 64
    lens = draw_lens(rng, int(rng.integers(1, 24)), int(rng.choice([40, 300, 1500, 4000])))
    chunk = int(rng.choice([0, 128, 256, 384, 512, 1024, 4096]))
    wl = workloads.make_custom(lens, Hq, Hkv, d, kv_dtype, seed=2000 + seed)
    got = gpu_attend(wl, chunk_tokens=chunk)
    (check_fp8 if kv_dtype == "fp8" else check)(got, oracle_full(wl))


@pytest.mark.parametrize("seed", range(12))
def test_prefix_random_groups(sd, seed):
    rng = np.random.default_rng(3000 + seed)
    Hq, Hkv = HEADS[int(rng.integers(len(HEADS)))]
    kv_dtype = "fp8" if rng.random() < 0.3 else "bf16"
    d = 128 if rng.random() < 0.6 else 64
    chunk = int(rng.choice([128, 256, 512, 1024]))
    sizes = rng.integers(1, 20, size=int(rng.integers(1, 6)))
    prefix = rng.integers(0, 6 * chunk, size=len(sizes))
    if kv_dtype == "fp8":
        prefix = prefix // 16 * 16                        # fp8 prefix tails are not copied by the generator
    session_of, prefix_len = np.repeat(np.arange(len(sizes)), sizes), np.repeat(prefix, sizes)
    lens = prefix_len + rng.integers(0, 2 * chunk, size=len(session_of), endpoint=True)
    lens = np.maximum(lens, 1)
    prefix_len = np.minimum(prefix_len, lens)
    wl = workloads.make_custom(lens, Hq, Hkv, d, kv_dtype, seed=4000 + seed, session_of=session_of, prefix_len=prefix_len)
    got = gpu_attend_prefix(wl, chunk_tokens=chunk)
    (check_fp8 if kv_dtype == "fp8" else check)(got, oracle_full(wl))


@pytest.mark.parametrize("seed", range(12))
def test_prefill_random_stretches(sd, seed):
    import torch
    rng = np.random.default_rng(5000 + seed)
    Hq, Hkv = HEADS[int(rng.integers(len(HEADS)))]
    kv_dtype = "fp8" if rng.random() < 0.35 else "bf16"
    d = 128 if rng.random() < 0.6 else 64
    lens = draw_lens(rng, int(rng.integers(1, 10)), int(rng.choice([40, 300, 900])))
    nq = np.array([int(rng.integers(0, L + 3)) for L in lens])       # none .. more queries than tokens
    wl = workloads.make_custom(lens, Hq, Hkv, d, kv_dtype, seed=6000 + seed)
    q_start = np.concatenate([[0], np.cumsum(nq)]).astype(np.int32)
    rows = max(int(q_start[-1]), 1)
    q = f32_to_bf16_bits(rng.standard_normal((rows, Hq, d)).astype(np.float32))
    if q_start[-1] == 0:
        return                                                       # nothing to compute in this draw
    out = device_workload(wl).attend_prefill(q, q_start)
    torch.cuda.synchronize()
    ref = oracle.paged_prefill_attention(q, q_start, wl.k_pages, wl.v_pages, wl.block_table, wl.context_lens, wl.scale,
                                         wl.k_scales, wl.v_scales, wl.kv_dtype)
    if kv_dtype == "fp8":
        check_fp8(out.cpu().numpy(), ref, alarm_scale=2.0)
    else:
        check(out.cpu().numpy(), ref, alarm_scale=2.0)
