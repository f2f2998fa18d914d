"""Kernel-level parity (through the C ABI) against the oracle's definitions."""
import sys

import pytest
import torch

import workloads as WL
from oracle import swiftkv_oracle as O
from tests.helpers import cosine, rel_err

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _rand_bf16(seed, name, shape, std=1.0):
    return WL.seeded_normal_bf16(seed, name, shape, 0.0, std)


@pytest.mark.parametrize("variant,M,N,K", [
    (2, 128, 128, 64), (2, 300, 272, 200), (2, 1, 16, 8), (2, 517, 1040, 688),
    (1, 256, 256, 64), (1, 700, 528, 456), (1, 2304, 768, 1024),
    (3, 1, 16, 8), (3, 8, 1024, 256), (3, 16, 272, 688), (3, 17, 64, 96), (3, 65, 160, 1000),
    (3, 32, 96, 264), (3, 33, 192, 520), (3, 48, 80, 1000), (3, 49, 1056, 4096), (3, 64, 4096, 688), (3, 80, 144, 72),
    ("rows", 33, 192, 520), ("rows", 49, 1056, 4096), ("rows", 64, 4096, 1376), ("rows", 80, 1024, 4096), ("rows", 16, 1024, 4096),
    # the forms with the activation slice resident in LDS (K % 512 == 0).  Up to 32 rows (one slice per workgroup, at
    # least 1024 (column block, K slice) streams): one and several K slices, a ragged last workgroup, one and two
    # blocks per wave.  Beyond 32 rows (slices walked in sequence behind a producer wave): 3..5 row blocks, one and
    # several K ranges, 4 and 8 consumer waves with 1, 2 and 4 column blocks each, a ragged last column group
    ("rows", 1, 8192, 4096), ("rows", 7, 16384, 2048), ("rows", 8, 8208, 4096), ("rows", 17, 4096, 4096), ("rows", 16, 4096, 14336),
    ("rows", 40, 16384, 1024), ("rows", 64, 6144, 4096), ("rows", 64, 16384, 4096), ("rows", 80, 4096, 4096),
    ("rows", 64, 28672, 4096), ("rows", 48, 32064, 1024), ("rows", 33, 8208, 4096), ("rows", 72, 2048, 14336), ("rows", 64, 4096, 512),
    (0, 2500, 512, 256),
    (14, 256, 256, 64), (14, 700, 528, 448), (14, 2304, 768, 1024), (14, 1, 16, 128), (14, 1031, 1040, 320),
    (15, 256, 256, 64), (15, 700, 528, 448), (15, 2304, 768, 1024), (15, 517, 272, 192),
    ("packed", 1024, 256, 256), ("packed", 2304, 768, 1024), ("packed", 1031, 512, 256), ("packed", 3000, 1024, 2048),
])
def test_gemm_matches_definition(variant, M, N, K):
    """C = A W^T (Sec. 3.1 projections); fp32 accumulation of bf16 inputs."""
    from paper_2410_03960_amd import binding as B
    _say(f"gemm variant={variant} M={M} N={N} K={K}")
    A = _rand_bf16(1, f"A{M}{K}", (M, K))
    W = _rand_bf16(2, f"W{N}{K}", (N, K), 0.05)
    ref = A.double() @ W.double().T
    for out_f32 in ((False,) if variant == "packed" else (True, False)):
        if variant == "packed":
            got = B.op_gemm_packed(A.cuda(), W.cuda())
        elif variant == "rows":
            got = B.op_gemm_rows(A.cuda(), W.cuda(), out_f32=out_f32)
        else:
            got = B.op_gemm(A.cuda(), W.cuda(), out_f32=out_f32, variant=variant)
        torch.cuda.synchronize()
        tol = 1e-5 if out_f32 else 4e-3          # fp32 sum of exact products / one bf16 rounding
        assert rel_err(got.cpu(), ref) <= tol, (out_f32, rel_err(got.cpu(), ref))


def test_gemm_entry_points_reject_bad_arguments():
    from paper_2410_03960_amd import binding as B
    A = _rand_bf16(1, "A", (64, 256)).cuda()
    W = _rand_bf16(2, "W", (256, 256)).cuda()
    for variant in (4, 27, 29, -1):                    # no longer / never offered
        with pytest.raises(B.SwiftKVError):
            B.op_gemm(A, W, variant=variant)
    with pytest.raises(B.SwiftKVError):                # packed-weight loop needs M >= 1024
        B.op_gemm_packed(A, W)
    with pytest.raises(B.SwiftKVError):                # weight-streaming kernel: M <= 80
        B.op_gemm_rows(_rand_bf16(1, "A2", (81, 256)).cuda(), W)


@pytest.mark.parametrize("hd,Hq,Hkv,lens", [
    (64, 4, 2, [128]), (64, 4, 2, [1, 63, 64, 65, 200, 129]),
    (128, 8, 2, [300, 1, 127, 128, 513]), (128, 4, 4, [77]), (128, 8, 1, [1000]),
])
def test_prefill_attention_matches_bruteforce_softmax(hd, Hq, Hkv, lens):
    from paper_2410_03960_amd import binding as B
    _say(f"attention hd={hd} Hq={Hq} Hkv={Hkv} lens={lens}")
    T = sum(lens)
    q = _rand_bf16(3, "q", (T, Hq * hd))
    k = _rand_bf16(4, "k", (T, Hkv * hd))
    v = _rand_bf16(5, "v", (T, Hkv * hd))
    got = B.op_attention_prefill(q.cuda(), k.cuda(), v.cuda(), lens, Hq, Hkv, hd)
    torch.cuda.synchronize()
    got = got.cpu()
    off = 0
    for n in lens:
        ref = O.gqa_attention(q[off:off + n].double().view(n, Hq, hd), torch.arange(n),
                              k[off:off + n].double().view(n, Hkv, hd), v[off:off + n].double().view(n, Hkv, hd))
        g = got[off:off + n].view(n, Hq, hd)
        assert rel_err(g, ref) <= 1e-2 and cosine(g, ref) >= 0.9995, (n, rel_err(g, ref), cosine(g, ref))
        off += n


@pytest.mark.parametrize("hd,Hq,Hkv,mode,lens", [
    (128, 32, 8, "bf16", [4097, 1, 300]), (128, 32, 8, "fp8_head", [4097, 1, 300, 2048, 33]),
    (128, 32, 8, "fp8_token", [4097, 1, 300, 129]), (128, 8, 8, "fp8_head", [700, 5]), (128, 16, 2, "fp8_token", [1000, 17]),
    (64, 8, 4, "fp8_head", [1500, 64]), (64, 4, 4, "fp8_token", [90, 256]), (64, 8, 1, "fp8_head", [31, 2500]),
    (128, 8, 4, "fp8_head", [20000]),
])
def test_single_query_attention_over_paged_cache(hd, Hq, Hkv, mode, lens):
    """One query row per sequence over a paged cache with shuffled blocks (the decode / last-token
    attention), bf16 or e4m3 codes (per-head and per-slot scales; the e4m3 path feeds the codes to
    the matrix unit), against the oracle's attention over the values the cache decodes to."""
    from paper_2410_03960_amd import binding as B
    _say(f"single-query attention hd={hd} Hq={Hq} Hkv={Hkv} {mode} lens={lens}")
    n_rows = len(lens)
    need = [(n + 15) // 16 for n in lens]
    n_blocks = sum(need) + 3
    perm = torch.from_numpy(WL.seeded_permutation(7, f"blocks{n_blocks}", n_blocks))
    bt = torch.zeros((n_rows, max(need)), dtype=torch.int32)
    pos = 0
    for b, nb in enumerate(need):
        bt[b, :nb] = perm[pos:pos + nb].to(torch.int32)
        pos += nb
    q = _rand_bf16(21, f"q{mode}{hd}", (n_rows, Hq * hd))
    n_slots = n_blocks * 16
    if mode == "bf16":
        ck = _rand_bf16(22, f"k{hd}{n_slots}", (n_slots, Hkv, hd))
        cv = _rand_bf16(23, f"v{hd}{n_slots}", (n_slots, Hkv, hd))
        kf, vf = ck.double(), cv.double()
        sk = sv = None
    else:
        ck = WL.seeded_fp8_codes(24, f"k{hd}{n_slots}", (n_slots, Hkv, hd), mag_lo=0x20, mag_hi=0x7E)
        cv = WL.seeded_fp8_codes(25, f"v{hd}{n_slots}", (n_slots, Hkv, hd), mag_lo=0x01, mag_hi=0x7E)
        tab = O.fp8_e4m3fn_decode_table()
        if mode == "fp8_head":
            sk = (0.002 + 0.001 * torch.arange(Hkv)).float()
            sv = (0.004 + 0.0005 * torch.arange(Hkv)).float()
            kf, vf = tab[ck.long()] * sk.double()[None, :, None], tab[cv.long()] * sv.double()[None, :, None]
        else:     # per-slot scales spread over three binades
            sk = (0.001 * 2.0 ** (3 * WL.seeded_uniform01(26, "sk", n_slots))).astype("float32")
            sv = (0.0005 * 2.0 ** (3 * WL.seeded_uniform01(27, "sv", n_slots))).astype("float32")
            sk, sv = torch.from_numpy(sk), torch.from_numpy(sv)
            kf, vf = tab[ck.long()] * sk.double()[:, None, None], tab[cv.long()] * sv.double()[:, None, None]
    got = B.op_attention_decode(q.cuda(), lens, ck.cuda(), cv.cuda(), bt, Hq, Hkv, hd,
                                sk.cuda() if sk is not None else None, sv.cuda() if sv is not None else None,
                                per_token=(mode == "fp8_token")).cpu()
    for b, n in enumerate(lens):
        slots = bt[b].long()[torch.arange(n) // 16] * 16 + torch.arange(n) % 16
        ref = O.gqa_attention(q[b:b + 1].double().view(1, Hq, hd), torch.tensor([n - 1]), kf[slots], vf[slots])
        g = got[b].view(1, Hq, hd)
        r, cs = rel_err(g, ref), cosine(g, ref)
        assert r <= 1e-2 and cs >= 0.9995, (b, n, r, cs)


def test_fp8_quantiser_is_bit_exact():
    """Same fp32 inputs, same fp32 division: codes must agree bit for bit."""
    from paper_2410_03960_amd import binding as B
    _say("fp8 quantiser")
    g = torch.Generator().manual_seed(9)
    x = torch.cat([torch.randn(200000, generator=g) * 5, torch.randn(20000, generator=g) * 1e-3,
                   torch.tensor([0.0, -0.0, 1e9, -1e9, 448.0, 464.0, 2.0 ** -9, 2.0 ** -10, 1.5 * 2.0 ** -9])])
    tab = O.fp8_e4m3fn_decode_table()[:127].float()
    mids = (tab[:-1] + tab[1:]) / 2
    x = torch.cat([x, mids, -mids, torch.nextafter(mids, torch.tensor(0.0)), torch.nextafter(mids, torch.tensor(1e9))])
    for scale in (1.0, 0.0371, 3.3):
        want = O.fp8_quantize(x * scale, torch.tensor(scale))
        got = B.op_fp8_quantize((x * scale).cuda(), scale)
        torch.cuda.synchronize()
        assert torch.equal(got.cpu(), want), scale


def test_mfma_rate_measurement_runs():
    """The matrix-instruction rate probe returns a plausible figure (between a
    tenth of and the data-sheet peak) and rejects bad arguments."""
    from paper_2410_03960_amd import binding as B
    _say("mfma rate")
    ops = _rand_bf16(5, "ops", (16384,)).cuda()
    rate = B.op_mfma_rate(ops, 2000)
    assert 250.0 < rate < 2600.0, rate
    with pytest.raises(B.SwiftKVError):
        B.op_mfma_rate(ops, 0)
