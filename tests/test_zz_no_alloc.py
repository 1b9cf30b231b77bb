"""pcc_decode_static (the decoder whose mailbox is a static device array: no allocation inside the call)
against pcc_decode, through the C ABI.  Needs an MI355X."""
import ctypes as C

import numpy as np
import pytest

from paper_2212_01185_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _log(msg):
    print(msg, flush=True)


def test_decode_static_equals_decode_on_two_calls_in_a_row(blob):
    """Two calls in a row on one context, the second with a smaller image (the array still holds the first
    call's tagged pixels where the second does not clear): each must return what pcc_decode returns for the same
    stream, which is the image.  A job beyond the array's size is refused before anything runs."""
    from paper_2212_01185_amd import binding
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    lib = binding.load()
    codec = binding.Codec(blob, 0)
    try:
        st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        big = np.stack([synth.make_image(60 + s, synth.ImageSpec(200, 90, 6, 4.0, 20.0)) for s in range(3)])
        small = synth.make_image(70, synth.ImageSpec(75, 37, 4, 3.0, 12.0))[None]
        rng = np.random.default_rng(71)
        tiny = rng.integers(0, 256, (1, 1, 1, 3), dtype=np.uint8)
        for name, imgs in (("3 x 200x90", big), ("1 x 75x37", small), ("1 x 1x1", tiny), ("3 x 200x90 again", big)):
            n, h, w, _ = imgs.shape
            d = torch.from_numpy(imgs).cuda()
            stream = codec.pcc_encode(d)
            want = codec.pcc_decode(stream, n, h, w)
            torch.cuda.synchronize()
            assert lib.pcc_decode_static_scratch_bytes(n, h, w) <= (8 << 20)
            out = torch.full_like(d, 77)
            _log("pcc_decode_static %s" % name)
            rc = lib.pcc_decode_static(codec._h, stream.data_ptr(), stream.numel(), n, h, w, out.data_ptr(), st)
            assert rc == 0, binding.pcc_strerror(rc)
            torch.cuda.synchronize()
            assert torch.equal(out, want) and torch.equal(out, d), name
        # too large for the static array: refused, nothing launched, the context still works
        n, h, w = 64, 1024, 1024
        assert lib.pcc_decode_static_scratch_bytes(n, h, w) > (8 << 20)
        rc = lib.pcc_decode_static(codec._h, stream.data_ptr(), stream.numel(), n, h, w, out.data_ptr(), st)
        assert rc == binding.PCC_E_SCRATCH and "scratch" in binding.pcc_strerror(rc)
        n, h, w, _ = small.shape
        d = torch.from_numpy(small).cuda()
        out = codec.pcc_decode_static(codec.pcc_encode(d), n, h, w, out=torch.empty_like(d))
        torch.cuda.synchronize()
        assert torch.equal(out, d)
        # a damaged stream is reported, not hung on, as by pcc_decode
        stream = codec.pcc_encode(d)
        with pytest.raises(binding.PccError) as e:
            codec.pcc_decode_static(stream[:-4].clone(), n, h, w, out=torch.empty_like(d))
        assert e.value.code == binding.PCC_E_STREAM
    finally:
        codec.close()
