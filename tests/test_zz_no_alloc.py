"""The allocation-free entry point, ivftq_encode_only_noalloc, through the C ABI: its outputs equal
ivftq_encode_only's bit for bit, on two calls in a row (the second smaller, so the static scratch still
holds the first call's leftovers), it requests no device memory, and it refuses sizes beyond its limit."""
import numpy as np
import pytest

import gpu_cases

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

DEV = "cuda:0"
LIMIT = 65536


def _pkg():
    import paper_2605_17415_amd as pkg
    return pkg


class Ledger:
    """Allocator callbacks that count requests (memory from PyTorch's caching allocator)."""

    def __init__(self):
        pkg = _pkg()
        self.requests = 0
        self.alloc_cb = pkg.ALLOC_FN(self._alloc)
        self.free_cb = pkg.FREE_FN(lambda p, ctx: torch.cuda.caching_allocator_delete(p))

    def _alloc(self, nbytes, ctx):
        self.requests += 1
        return torch.cuda.caching_allocator_alloc(int(nbytes))


@pytest.mark.parametrize("name", ["d96_b4", "d200"])
def test_noalloc_encode_equals_encode_only_twice_in_a_row(name):
    pkg = _pkg()
    cs = gpu_cases.get_case(name)
    led = Ledger()
    ix = pkg.Index(cs.d, cs.b_stage1, cs.nlist, sign_bit=cs.sign_bit, allocator=(led.alloc_cb, led.free_cb))
    ix.set_coarse(cs.cent)
    ix.set_rotation(cs.Pi)
    x = torch.from_numpy(cs.X).to(DEV)
    for n in (len(cs.X), 1_733):                     # the second call is smaller than the first
        xs = x[:n].contiguous()
        print(f"[noalloc {name}] n={n}", flush=True)
        a_ref, c_ref, g_ref = ix.encode_only(xs)
        a = torch.full((n,), -7, dtype=torch.int32, device=DEV)
        c = torch.full((n, cs.d), 255, dtype=torch.uint8, device=DEV)
        g = torch.full((n,), -1.0, dtype=torch.float16, device=DEV)
        before = led.requests
        ix.encode_only_noalloc(xs, a, c, g)
        torch.cuda.synchronize()
        assert led.requests == before                # nothing was requested from the allocator
        assert torch.equal(a, a_ref) and torch.equal(c, c_ref)
        assert torch.equal(g.view(torch.int16), g_ref.view(torch.int16))
        # outputs are optional: codes and norms without the cell numbers
        c2 = torch.empty_like(c)
        g2 = torch.empty_like(g)
        ix.encode_only_noalloc(xs, None, c2, g2)
        torch.cuda.synchronize()
        assert torch.equal(c2, c_ref) and torch.equal(g2.view(torch.int16), g_ref.view(torch.int16))
    ix.close()


def test_noalloc_encode_rejects_what_does_not_fit():
    pkg = _pkg()
    cs = gpu_cases.get_case("d8_b1")
    ix = pkg.Index(cs.d, cs.b_stage1, cs.nlist)
    x = torch.zeros((LIMIT + 1, cs.d), dtype=torch.float32, device=DEV) + 1.0
    a = torch.full((LIMIT + 1,), -7, dtype=torch.int32, device=DEV)
    with pytest.raises(pkg.IvftqError) as e:
        ix.encode_only_noalloc(x, a, None, None)             # no centroids yet
    assert e.value.status == pkg.binding.UNSUPPORTED or e.value.status == pkg.binding.BAD_STATE
    ix.set_coarse(cs.cent)
    ix.set_rotation(cs.Pi)
    with pytest.raises(pkg.IvftqError) as e:
        ix.encode_only_noalloc(x, a, None, None)
    assert e.value.status == pkg.binding.UNSUPPORTED and "65536" in str(e.value)
    torch.cuda.synchronize()
    assert (a == -7).all()                                   # nothing ran
    ix.encode_only_noalloc(x[:LIMIT], a[:LIMIT], None, None)  # the limit itself is fine
    ref, _, _ = ix.encode_only(x[:LIMIT], want_codes=False)
    torch.cuda.synchronize()
    assert torch.equal(a[:LIMIT], ref)
    ix.close()
