"""GPU test of oppo_chunk_step_noalloc, the entry point for callers that cannot allocate device
memory: called through the C ABI on two passes in a row (the second smaller than the first, on top
of what the first left in the cache), its outputs and the cache must equal those of oppo_chunk_step
given a caller-owned workspace of the same size as the built-in scratch buffer - bit for bit, since
the same number of partial slots gives the same plan - and agree with the float64 oracle within the
attention tolerance.  Both passes are thin (a few sequences on long contexts), so that key ranges
are split and the scratch buffer is really used; the second pass finds the first one's partial
results still in the buffer."""
import numpy as np
import pytest

from oracle import bf16_bits_to_f64, causal_attention

pytestmark = pytest.mark.gpu

MAX_ABS = 2e-2
MEAN_ABS = 2e-3


def _bf16_bits(rng, shape):
    x = rng.standard_normal(shape, dtype=np.float32).view(np.uint32)
    return (((x + 0x7FFF + ((x >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)


def test_noalloc_entry_point_equals_chunk_step_on_two_calls_in_a_row():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2509_25762_amd import binding as ob
    ob.load()
    dev = torch.device("cuda:0")
    Hq, Hkv, D = 32, 8, 128
    scale = 1.0 / np.sqrt(D)
    desc = ob.make_desc(Hq, Hkv, D, scale)
    rng = np.random.default_rng(20250926)
    kv0 = np.array([2900, 700, 130], dtype=np.int64)          # tokens cached before the first pass
    passes = [np.array([256, 256, 40]), np.array([100, 0, 7])]   # new rows per sequence: second pass smaller
    total = kv0 + sum(passes)
    slot_begin = np.concatenate([[0], np.cumsum(total + 3)])
    B = len(kv0)
    q_all = [_bf16_bits(rng, (int(total[i]), Hq, D)) for i in range(B)]
    k_all = [_bf16_bits(rng, (int(total[i]), Hkv, D)) for i in range(B)]
    v_all = [_bf16_bits(rng, (int(total[i]), Hkv, D)) for i in range(B)]
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev)

    def fresh_cache():
        ck = torch.full((int(slot_begin[-1]), Hkv, D), -1, dtype=torch.int16, device=dev)
        cv = torch.full_like(ck, -1)
        for i in range(B):
            b, n = int(slot_begin[i]), int(kv0[i])
            ck[b:b + n] = to_dev(k_all[i][:n])
            cv[b:b + n] = to_dev(v_all[i][:n])
        return ob.KVCache(ck, cv, slot_begin, kv0.astype(np.int32))

    ws = torch.empty(ob.oppo_static_scratch_bytes(), dtype=torch.uint8, device=dev)
    caches = {"step": fresh_cache(), "noalloc": fresh_cache()}
    done = kv0.copy()
    for t, ql in enumerate(passes):
        cu = np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)
        rows = lambda arrs: np.concatenate([arrs[i][done[i]:done[i] + ql[i]] for i in range(B)])
        q, k, v = to_dev(rows(q_all)), to_dev(rows(k_all)), to_dev(rows(v_all))
        out_a = torch.zeros_like(q)
        out_b = torch.zeros_like(q)
        ob.oppo_chunk_step(desc, caches["step"], cu, q, k, v, out_a, ws)
        ob.oppo_chunk_step_noalloc(desc, caches["noalloc"], cu, q, k, v, out_b)
        torch.cuda.synchronize()
        a = out_a.cpu().numpy().view(np.uint16)
        b = out_b.cpu().numpy().view(np.uint16)
        assert np.array_equal(a, b), f"pass {t}: outputs differ from oppo_chunk_step's"
        for name in ("k", "v"):
            ca = getattr(caches["step"], name).cpu().numpy()
            cb = getattr(caches["noalloc"], name).cpu().numpy()
            assert np.array_equal(ca, cb), f"pass {t}: cache {name} differs"
        assert caches["step"].kv_len.tolist() == caches["noalloc"].kv_len.tolist() == (done + ql).tolist()
        # and against the definition, for the rows of this pass
        got = bf16_bits_to_f64(b)
        errs = []
        for i in range(B):
            if ql[i] == 0:
                continue
            n = int(done[i] + ql[i])
            ref = causal_attention(bf16_bits_to_f64(q_all[i][done[i]:n]), bf16_bits_to_f64(k_all[i][:n]),
                                   bf16_bits_to_f64(v_all[i][:n]), int(done[i]) + np.arange(int(ql[i])), scale)
            errs.append(np.abs(got[cu[i]:cu[i + 1]] - ref).ravel())
        err = np.concatenate(errs)
        assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, f"pass {t}: max {err.max():.3e} mean {err.mean():.3e}"
        done += ql
    # the cache holds exactly the tokens so far, everything else untouched
    ck = caches["noalloc"].k.cpu().numpy().view(np.uint16)
    for i in range(B):
        b, n = int(slot_begin[i]), int(done[i])
        assert np.array_equal(ck[b:b + n], k_all[i][:n])
        assert np.all(ck[b + n:int(slot_begin[i + 1])] == 0xFFFF)
