"""GPU parity on seeded random shapes: prefill (bf16 and fp32), decode and the gradients against the oracle, with
block sizes, windows, sinks, flags, head groupings, head_dims, batch sizes and lengths drawn at random inside what
the entry points accept (small enough for the dense float64 oracle); then the chunked, padded-batch and paged entry
points on random shapes through the checks of their own test files.  The hand-picked cases of the other files
name the situations they are meant to hit; this one looks for the ones nobody thought of.  Bars as there."""
import random

import pytest

from paper_2503_03588_amd import binding as pa
from gpu_util import check_prefill
from test_gpu_backward import run_backward
from test_gpu_decode import run_decode
from test_gpu_decode_paged import test_paged_matches_oracle_and_contiguous as check_paged
from test_gpu_prefill_chunk import test_chunks_equal_whole_prefill as check_chunks
from test_gpu_prefill_chunk_paged import test_paged_chunks_equal_whole_prefill as check_paged_chunks
from test_gpu_prefill_chunk_paged import test_batch_of_pieces_equals_each_piece_alone as check_batch_of_pieces
from test_gpu_prefill_varlen import test_padded_batch as check_padded_batch

pytestmark = pytest.mark.gpu


def draw_cases(seed, count):
    rng = random.Random(seed)
    cases = []
    for c in range(count):
        kind = rng.choice(["prefill_bf16", "prefill_bf16", "prefill_f32", "decode", "backward"])
        hkv = rng.choice([1, 1, 2, 3, 4])
        hq = hkv * rng.choice([1, 2, 3, 4, 5, 7, 8, 16])
        d = rng.choice([64, 128])
        W = rng.choice([0, 1, 2, 3, 4, 5, 8])
        S = rng.choice([0, 1, 1, 2])
        flags = rng.choice([pa.POWER, pa.POWER, pa.POWER, 0, pa.DENSE])
        if kind in ("decode", "backward"):
            flags &= ~pa.DENSE                     # these two take the pattern's own rows only
        if not (flags & (pa.POWER | pa.DENSE)) and W < 1:
            W = 1                                  # a sliding window needs at least the diagonal block
        if kind == "prefill_bf16":
            B = rng.choice([64, 64, 128, 128, 192, 256, 320, 512])
            n = rng.randint(1, 2600)
            batch = rng.choice([1, 1, 2])
            if hq * batch * n > 40000:             # keep the oracle's N x N matrices per head few
                hq, hkv = rng.choice([(4, 1), (4, 2), (6, 2), (7, 1)])
            cases.append((kind, dict(B=B, W=W, S=S, flags=flags, hq=hq, hkv=hkv, d=d, n=n, batch=batch, seed=1000 + c)))
        elif kind == "prefill_f32":
            B = rng.choice([16, 32, 48, 64, 80, 128, 256])
            hq, hkv = rng.choice([(2, 1), (2, 2), (4, 2), (3, 1)])
            cases.append((kind, dict(B=B, W=W, S=S, flags=flags, hq=hq, hkv=hkv, d=d, n=rng.randint(1, 900), batch=1,
                                     seed=2000 + c)))
        elif kind == "decode":
            B = rng.choice([64, 64, 128, 192, 256, 512])
            cap = rng.randint(1, 6000)
            lens = [cap] + [rng.randint(1, cap) for _ in range(rng.choice([0, 1, 2, 4]))]
            cases.append((kind, dict(B=B, W=W, S=S, flags=flags, hq=hq, hkv=hkv, d=d, cap=cap, lens=lens,
                                     calls=rng.choice([1, 2]), seed=3000 + c)))
        else:
            B = rng.choice([64, 128, 256])
            hq, hkv = rng.choice([(2, 1), (2, 2), (4, 2), (6, 2), (4, 1), (8, 1)])
            cases.append((kind, dict(B=B, W=W, S=S, flags=flags, hq=hq, hkv=hkv, d=d, n=rng.randint(1, 1100),
                                     seed=4000 + c)))
    return cases


CASES = draw_cases(20250303, 48)


@pytest.mark.parametrize("kind,c", CASES, ids=[f"{i}-{k}" for i, (k, _) in enumerate(CASES)])
def test_random_shape(kind, c):
    print(kind, c, flush=True)
    pat = pa.Pattern(c["B"], c["W"], c["S"], c["flags"])
    if kind == "prefill_bf16":
        check_prefill(pat, c["batch"], c["hq"], c["hkv"], c["n"], c["d"], "bf16", seed=c["seed"])
    elif kind == "prefill_f32":
        check_prefill(pat, c["batch"], c["hq"], c["hkv"], c["n"], c["d"], "f32", seed=c["seed"])
    elif kind == "decode":
        run_decode(pat, len(c["lens"]), c["hq"], c["hkv"], c["cap"], c["d"], c["lens"], seed=c["seed"], calls=c["calls"])
    else:
        run_backward(pat, 1, c["hq"], c["hkv"], c["n"], c["d"], seed=c["seed"])


def draw_serving_cases(seed, count):
    rng = random.Random(seed)
    cases = []
    for c in range(count):
        kind = rng.choice(["chunk", "varlen", "paged"])
        hkv = rng.choice([1, 2, 4])
        hq = hkv * rng.choice([1, 2, 4, 7])
        d = rng.choice([64, 128])
        W = rng.choice([0, 1, 2, 4, 5])
        S = rng.choice([0, 1, 2])
        B = rng.choice([64, 64, 128, 192, 256])
        if kind == "chunk":
            flags = rng.choice([pa.POWER, pa.POWER, 0, pa.DENSE])
            if not (flags & (pa.POWER | pa.DENSE)) and W < 1:
                W = 1
            nb = rng.randint(1, max(1, 2400 // B))
            n = nb * B - rng.randint(0, B - 1)
            cap = n + rng.randint(0, 300)
            inner = sorted(set(rng.randint(1, nb) * B for _ in range(rng.randint(0, 3))))
            cuts = [0] + [x for x in inner if x < n] + [n]          # chunks start at block boundaries
            batch = rng.choice([1, 2])
            if hq * batch * n > 30000:
                hq, hkv = 4, 2
            cases.append((kind, (n, B, W, S, hq, hkv, d, batch, cap, cuts, flags)))
        elif kind == "varlen":
            npad = rng.randint(1, 1500)
            lens = [rng.choice([0, npad, rng.randint(0, npad)]) for _ in range(rng.randint(1, 4))]
            if hq * len(lens) * npad > 30000:
                hq, hkv = 4, 2
            cases.append((kind, (B, W, S, pa.POWER, hq, hkv, d, npad, lens)))
        else:
            cap = rng.randint(1, max(1, 5000 // B)) * B             # whole pages
            lens = [cap] + [rng.randint(1, cap) for _ in range(rng.randint(0, 3))]
            cases.append((kind, (B, W, S, hq, hkv, d, cap, lens)))
    return cases


SERVING_CASES = draw_serving_cases(20250304, 24)


@pytest.mark.parametrize("kind,args", SERVING_CASES, ids=[f"{i}-{k}" for i, (k, _) in enumerate(SERVING_CASES)])
def test_random_serving_shape(kind, args):
    print(kind, args, flush=True)
    {"chunk": check_chunks, "varlen": check_padded_batch, "paged": check_paged}[kind](*args)


def draw_unaligned_chunk_cases(seed, count):
    """Chunks cut at any token, against a contiguous cache and against a paged one."""
    rng = random.Random(seed)
    cases = []
    for c in range(count):
        kind = rng.choice(["chunk", "chunk_paged", "chunk_paged"])
        hkv = rng.choice([1, 2, 4])
        hq = hkv * rng.choice([1, 2, 4, 7])
        d = rng.choice([64, 128])
        W = rng.choice([0, 1, 2, 4, 5])
        S = rng.choice([0, 1, 2])
        B = rng.choice([64, 64, 128, 192, 256])
        flags = rng.choice([pa.POWER, pa.POWER, 0]) if kind == "chunk_paged" else rng.choice([pa.POWER, 0, pa.DENSE])
        if not (flags & (pa.POWER | pa.DENSE)) and W < 1:
            W = 1
        n = rng.randint(1, 2400)
        cuts = [0] + sorted(set(rng.randint(1, n) for _ in range(rng.randint(0, 3))) - {n}) + [n]
        batch = rng.choice([1, 2])
        if hq * batch * n > 30000:
            hq, hkv = 4, 2
        if kind == "chunk":
            cases.append((kind, (n, B, W, S, hq, hkv, d, batch, n + rng.randint(0, 300), cuts, flags)))
        else:
            cases.append((kind, (n, B, W, S, hq, hkv, d, batch, cuts, flags)))
    return cases


UNALIGNED_CASES = draw_unaligned_chunk_cases(20250305, 16)


@pytest.mark.parametrize("kind,args", UNALIGNED_CASES, ids=[f"{i}-{k}" for i, (k, _) in enumerate(UNALIGNED_CASES)])
def test_random_unaligned_chunks(kind, args):
    print(kind, args, flush=True)
    {"chunk": check_chunks, "chunk_paged": check_paged_chunks}[kind](*args)


def draw_batch_cases(seed, count):
    """Pieces of several sequences in one launch against a paged cache."""
    rng = random.Random(seed)
    cases = []
    for c in range(count):
        hkv = rng.choice([1, 2, 4])
        hq = hkv * rng.choice([1, 2, 4, 7])
        d = rng.choice([64, 128])
        W = rng.choice([0, 1, 2, 4, 5])
        S = rng.choice([0, 1, 2])
        B = rng.choice([64, 64, 128, 192, 256])
        flags = rng.choice([pa.POWER, pa.POWER, 0])
        if not flags and W < 1:
            W = 1
        n = rng.randint(1, 2000)
        batch = rng.randint(1, 4)
        if hq * batch * n > 30000:
            hq, hkv = 4, 2
        pieces = []
        for _ in range(batch):
            a = rng.choice([0, rng.randint(0, n - 1)])
            pieces.append((a, rng.choice([0, 1, n - a, rng.randint(0, n - a)])))
        q_rows = max(1, max(ln for _, ln in pieces)) + rng.choice([0, 0, 5, 100])
        cases.append((n, B, W, S, hq, hkv, d, pieces, min(q_rows, ((n + B - 1) // B) * B), flags))
    return cases


BATCH_CASES = draw_batch_cases(20250306, 12)


@pytest.mark.parametrize("args", BATCH_CASES, ids=[str(i) for i in range(len(BATCH_CASES))])
def test_random_batches_of_pieces(args):
    print(args, flush=True)
    check_batch_of_pieces(*args)
