"""The measurement aids behind bench.py's on-box ceilings do the work they are priced at: the read probe
touches every word once, the MFMA probe executes the products its flop count stands for."""
import numpy as np
import pytest
import torch

from paper_2410_09687_amd import moin

from . import gpu_common as gc

pytestmark = pytest.mark.gpu


def test_read_probe_reads_every_word_once():
    ctx = gc.ctx()
    g = torch.Generator(device="cuda").manual_seed(7)
    for n16 in (1, 1000, 8 * 262144 + 5, 3 * 2 ** 20 + 17):
        print(f"[gpu] read probe n16={n16}", flush=True)
        src = torch.randint(-2 ** 31, 2 ** 31 - 1, (n16 * 4,), dtype=torch.int32, device="cuda", generator=g)
        out = moin.moin_probe_read(ctx, src)
        ctx.check()
        assert int(out.to(torch.int64).sum().item()) % 2 ** 32 == int(src.to(torch.int64).sum().item()) % 2 ** 32


def test_mfma_probe_computes_the_products_it_counts():
    ctx = gc.ctx()
    g = torch.Generator(device="cuda").manual_seed(8)
    # small integers: every product and every partial sum is exact in fp32, in any order
    ops = torch.randint(-3, 4, (4096 * 8,), device="cuda", generator=g).to(torch.bfloat16)
    for iters in (1, 3):
        print(f"[gpu] mfma probe iters={iters}", flush=True)
        out, flops = moin.moin_probe_mfma_bf16(ctx, ops, iters)
        ctx.check()
        n_threads = out.numel()
        n_waves = n_threads // 64
        assert flops == n_waves * iters * 32 * 2.0 * 16 * 16 * 32
        # thread t holds operand pieces in[(8 t + j) mod n16], j < 4 for A, 4 <= j < 8 for B; a wave's MFMA with
        # pieces (ja, jb) multiplies the 16 x 32 matrices whose row l % 16, columns 8 (l / 16) .. + 8 is lane l's
        # piece.  The sum of all entries of A B^T is sum_k colsum_A[k] colsum_B[k].
        v = ops.view(-1, 8).double().cpu().numpy()
        n16 = v.shape[0]
        t = np.arange(n_threads)
        total = out.double().cpu().numpy().reshape(n_waves, 64).sum(axis=1)
        pieces = [v[(8 * t + j) % n16].reshape(n_waves, 4, 16, 8) for j in range(8)]   # [wave, k group, row, 8]
        colsum = [p.sum(axis=2).reshape(n_waves, 32) for p in pieces]                  # [wave, k]
        want = np.zeros(n_waves)
        for i in range(32):
            want += (colsum[i & 3] * colsum[4 + ((i >> 2) & 3)]).sum(axis=1)
        assert np.array_equal(total, iters * want)


def test_mxfp8_mfma_probe_computes_the_products_it_counts():
    ctx = gc.ctx()
    g = torch.Generator(device="cuda").manual_seed(9)
    # codes of 0, +-0.5, +-1, +-2: every product and partial sum exact in fp32
    table = torch.tensor([0x00, 0x30, 0xB0, 0x38, 0xB8, 0x40, 0xC0], dtype=torch.uint8, device="cuda")
    codes = table[torch.randint(0, 7, (2048 * 16,), device="cuda", generator=g)].contiguous()
    vals = codes.view(torch.float8_e4m3fn).double().cpu().numpy().reshape(-1, 16)
    n16 = vals.shape[0]
    for iters in (1, 2):
        print(f"[gpu] mxfp8 mfma probe iters={iters}", flush=True)
        out, flops = moin.moin_probe_mfma_mxfp8(ctx, codes, iters)
        ctx.check()
        n_threads = out.numel()
        n_waves = n_threads // 64
        assert flops == n_waves * iters * 8 * 2.0 * 32 * 32 * 64
        t = np.arange(n_threads)
        total = out.double().cpu().numpy().reshape(n_waves, 64).sum(axis=1)

        def kvec(first):
            # an operand of a wave: lane l holds bytes [16 h, 16 h + 16) of the first 32-step block (piece
            # `first`) and of the second (piece `first + 1`), h = l / 32; summed over the 32 rows
            halves = []
            for piece in (first, first + 1):
                p16 = vals[(8 * t + piece) % n16].reshape(n_waves, 2, 32, 16)
                halves.append(p16.sum(axis=2).reshape(n_waves, 32))
            return np.concatenate(halves, axis=1)            # [wave, 64 contraction steps]

        ka = [kvec(0), kvec(4)]
        kb = [kvec(2), kvec(6)]
        want = np.zeros(n_waves)
        for i in range(8):
            want += (ka[i & 1] * kb[(i >> 1) & 1]).sum(axis=1)
        assert np.array_equal(total, iters * want)


def test_probe_rejects_bad_sizes():
    ctx = gc.ctx()
    with pytest.raises(ValueError):
        moin.moin_probe_mfma_bf16(ctx, torch.zeros(12, dtype=torch.bfloat16, device="cuda"), 1)
    with pytest.raises(ValueError):
        moin.moin_probe_read(ctx, torch.zeros(3, dtype=torch.int32, device="cuda"))
