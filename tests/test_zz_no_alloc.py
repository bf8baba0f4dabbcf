"""unique_decode_step_static (the entry point for callers that cannot allocate or bring a workspace) against
unique_decode_step: same kernels on the library's built-in scratch, so every output has to be the same bits. Two
calls in a row on one GPU, the second with a smaller input, so that whatever the first left in the shared
scratch is there when the second runs."""
import pytest
import torch

from paper_2605_27740_amd import binding
from paper_2605_27740_amd import workloads as W
from paper_2605_27740_amd.session import DecodeSession

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _both(wl, stats_dtype):
    ref = DecodeSession(wl, stats_dtype=stats_dtype)
    ref.update_page_stats()
    ref.decode_step(refresh_tail=True)
    torch.cuda.synchronize()
    got = DecodeSession(wl, stats_dtype=stats_dtype)
    got.update_page_stats()
    got.workspace = None                       # nothing of the caller's is used as scratch
    got.decode_step_static(refresh_tail=True)
    torch.cuda.synchronize()
    for name in ("page_stats", "sel_pages", "sel_count", "lse"):
        assert torch.equal(getattr(ref, name), getattr(got, name)), name
    assert torch.equal(ref.out.view(torch.uint8), got.out.view(torch.uint8)), "out"
    assert int(ref.sel_count.min()) > 0 and bool(torch.isfinite(got.out.float()).all())


@pytest.mark.parametrize("stats_dtype", [torch.float32, torch.bfloat16])
def test_static_scratch_step_matches_the_workspace_step_twice_in_a_row(gpu_lib, stats_dtype):
    print("no-alloc step: B=3 x 20000 tokens (many chunks per row), then B=2 x 700 tokens", flush=True)
    big = W.config3(batch=3, context=20000 + 5, top_k=300).to(DEV)
    _both(big, stats_dtype)
    small = W.build("small", 17, dtype=torch.float32, B=2, H=8, Hkv=2, D=64, S=8, seq_lens=[700, 33], top_k=5,
                    key_mode="shift", plant_mode="one_percent", permute=True).to(DEV)
    _both(small, stats_dtype)


def test_static_scratch_step_rejects_what_does_not_fit(gpu_lib):
    """A step whose score rows exceed the built-in scratch is refused on the host, before any launch."""
    wl = W.config3(batch=2, context=4096, top_k=16).to(DEV)
    sess = DecodeSession(wl)
    need = gpu_lib.workspace_bytes(sess.desc, sess.top_k)
    assert need <= binding.STATIC_SCRATCH_BYTES
    wide = torch.zeros((wl.B, 2 ** 21), dtype=torch.int32, device=DEV)        # 2 x 8 rows x 2M pages x 4 B = 128 MiB of scores
    wide[:, :wl.max_pages] = wl.page_table
    import dataclasses
    wl2 = dataclasses.replace(wl, page_table=wide)
    s2 = DecodeSession(wl2, max_seq_len_hint=0, want_scores=False)
    with pytest.raises(binding.UniqueError) as e:
        s2.decode_step_static()
    assert e.value.code == binding.ERR_WORKSPACE and "built-in scratch" in str(e.value)
