"""The allocator callbacks of ivftq_create on the GPU: every byte of index storage and workspace comes
through them, goes back through them, and a callback that returns NULL turns into IVFTQ_OOM with the
stored vectors unchanged."""
import ctypes

import numpy as np
import pytest

import gpu_cases

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _pkg():
    import paper_2605_17415_amd as pkg
    return pkg


class CountingAllocator:
    """ivftq_alloc_fn / ivftq_free_fn on PyTorch's caching allocator, with a ledger and a switch that
    makes every further request fail."""

    def __init__(self):
        pkg = _pkg()
        self.live = {}
        self.requests = 0
        self.refuse = False
        self.refused = 0
        self.alloc_cb = pkg.ALLOC_FN(self._alloc)
        self.free_cb = pkg.FREE_FN(self._free)

    def _alloc(self, nbytes, ctx):
        self.requests += 1
        if self.refuse:
            self.refused += 1
            return None
        p = torch.cuda.caching_allocator_alloc(int(nbytes))
        self.live[p] = int(nbytes)
        return p

    def _free(self, p, ctx):
        del self.live[p]                      # KeyError (reported by ctypes) if the library frees what it never got
        torch.cuda.caching_allocator_delete(p)

    def pair(self):
        return (self.alloc_cb, self.free_cb)


def test_all_memory_goes_through_the_callbacks_and_comes_back():
    pkg = _pkg()
    cs = gpu_cases.get_case("d96_b3")
    al = CountingAllocator()
    torch.cuda.synchronize()
    base = torch.cuda.memory_allocated()
    ix = pkg.Index(cs.d, cs.b_stage1, cs.nlist, sign_bit=cs.sign_bit, allocator=al.pair())
    ix.set_coarse(cs.cent)
    ix.set_rotation(cs.Pi)
    x = torch.from_numpy(cs.X).to(DEV)
    q = torch.from_numpy(cs.Q).to(DEV)
    held_by_test = torch.cuda.memory_allocated() - base - sum(al.live.values())
    ix.encode_add(x)
    s, i = ix.search(q, cs.nprobe, cs.k)
    torch.cuda.synchronize()
    ledger = sum(al.live.values())
    assert ledger >= ix.index_bytes() > 0
    # PyTorch's own count moved by what the ledger says (its blocks are rounded up, never down)
    assert torch.cuda.memory_allocated() - base - held_by_test - s.numel() * 4 - i.numel() * 8 >= ledger
    n_req = al.requests
    s2, i2 = ix.search(q, cs.nprobe, cs.k)            # same shape again: nothing new is requested
    torch.cuda.synchronize()
    assert al.requests == n_req and torch.equal(i, i2)
    ix.close()
    assert al.live == {}


def test_refusing_callback_gives_oom_and_leaves_the_index_unchanged():
    pkg = _pkg()
    cs = gpu_cases.get_case("d96_b3")
    al = CountingAllocator()
    ix = pkg.Index(cs.d, cs.b_stage1, cs.nlist, sign_bit=cs.sign_bit, allocator=al.pair())
    ix.set_coarse(cs.cent)
    ix.set_rotation(cs.Pi)
    ix.set_search_mode(2)          # the batched scan (its candidate buffers grow with k) although the case has few queries
    x = torch.from_numpy(cs.X).to(DEV)
    q = torch.from_numpy(cs.Q).to(DEV)
    half = len(cs.X) // 2
    ix.encode_add(x[:half])
    s0, i0 = ix.search(q, cs.nprobe, cs.k)
    torch.cuda.synchronize()
    sizes = [ix.list_size(l) for l in range(cs.nlist)]
    lists = [ix.export_list(l) for l in (0, cs.nlist // 2, cs.nlist - 1)]
    al.refuse = True
    with pytest.raises(pkg.IvftqError) as e:
        ix.encode_add(x[half:])                       # the lists would have to grow
    assert e.value.status == pkg.binding.OOM and al.refused >= 1
    assert ix.ntotal() == half and [ix.list_size(l) for l in range(cs.nlist)] == sizes
    for before, l in zip(lists, (0, cs.nlist // 2, cs.nlist - 1)):
        for u, v in zip(before, ix.export_list(l)):
            np.testing.assert_array_equal(u.view(np.uint16) if u.dtype == np.float16 else u,
                                          v.view(np.uint16) if v.dtype == np.float16 else v)
    with pytest.raises(pkg.IvftqError) as e:
        ix.search(q, cs.nprobe, 5 * cs.k + 300)       # a larger k needs larger work buffers
    assert e.value.status == pkg.binding.OOM
    al.refuse = False
    s1, i1 = ix.search(q, cs.nprobe, cs.k)
    torch.cuda.synchronize()
    assert torch.equal(i0, i1) and torch.equal(s0, s1)
    ix.encode_add(x[half:])                           # and the append goes through once memory is there
    ref = pkg.Index(cs.d, cs.b_stage1, cs.nlist, sign_bit=cs.sign_bit, allocator="hip")
    ref.set_coarse(cs.cent)
    ref.set_rotation(cs.Pi)
    ref.set_search_mode(2)
    ref.encode_add(x)
    s2, i2 = ix.search(q, cs.nprobe, cs.k)
    s3, i3 = ref.search(q, cs.nprobe, cs.k)
    torch.cuda.synchronize()
    assert torch.equal(i2, i3) and torch.equal(s2, s3)
    ix.close()
    ref.close()
    assert al.live == {}


def test_create_with_a_refusing_callback():
    pkg = _pkg()
    al = CountingAllocator()
    al.refuse = True
    with pytest.raises(pkg.IvftqError) as e:
        pkg.Index(64, 4, 16, allocator=al.pair())
    assert e.value.status == pkg.binding.OOM and al.live == {}
