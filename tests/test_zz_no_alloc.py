"""The GEMM entry point that allocates nothing (sts_op_gemm_noalloc: caller's device buffers, split-K
partial sums and cut-last-wave partial tiles in the library's fixed device array) against the
allocating entry point it is a variant of (sts_op_gemm, fp32 store), on two calls in a row, the
second with a smaller input, so that whatever the first call left in the shared array is there when
the second runs. Same kernels, same order of summation: the results are compared to the fp32
accumulator tolerance of 1e-3 (max-abs-rel) and are in fact expected to be equal."""
import ctypes as C

import numpy as np
import pytest

from paper_2504_19516_amd import synth

pytestmark = pytest.mark.gpu
TOL_ACC = 1e-3


class Hip:
    """Plain device memory for the test's inputs and outputs (the HIP runtime the library links)."""

    def __init__(self):
        self.rt = C.CDLL("libamdhip64.so")
        self.bufs = []

    def ck(self, rc, what):
        assert rc == 0, f"{what}: hip error {rc}"

    def malloc(self, nbytes):
        p = C.c_void_p()
        self.ck(self.rt.hipMalloc(C.byref(p), C.c_size_t(nbytes)), "hipMalloc")
        self.bufs.append(p)
        return p.value

    def upload(self, arr):
        arr = np.ascontiguousarray(arr)
        p = self.malloc(arr.nbytes)
        self.ck(self.rt.hipMemcpy(C.c_void_p(p), arr.ctypes.data_as(C.c_void_p), C.c_size_t(arr.nbytes), 1), "hipMemcpy H2D")
        return p

    def download(self, p, shape, dtype):
        out = np.empty(shape, dtype)
        self.ck(self.rt.hipMemcpy(out.ctypes.data_as(C.c_void_p), C.c_void_p(p), C.c_size_t(out.nbytes), 2), "hipMemcpy D2H")
        return out

    def sync(self):
        self.ck(self.rt.hipDeviceSynchronize(), "hipDeviceSynchronize")

    def free_all(self):
        for p in self.bufs:
            self.rt.hipFree(p)
        self.bufs = []


def rel(a, b):
    return float(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64)).max() / np.abs(b).max())


# (m, n, k, tile, split_k, tail_slots): split-K partial sums, then the cut last wave, each first at a
# larger then at a smaller size; ragged m (not a multiple of the tile height) in every case
CASES = [
    [(150, 1024, 2048, "64x128", 4, 0), (37, 512, 1024, "64x128", 3, 0)],
    [(300, 1024, 1024, "128x128", 1, 20), (130, 512, 512, "128x128", 1, 6)],
    [(520, 1024, 1024, "256x256", 1, 10), (64, 256, 512, "64x128", 8, 0)],
]


@pytest.mark.parametrize("pair", CASES)
def test_noalloc_gemm_equals_the_allocating_entry_point(pair):
    from paper_2504_19516_amd import sts
    sts.lib()
    hip = Hip()
    try:
        for seed, (m, n, k, tile, split_k, tail_slots) in enumerate(pair):
            a = synth.normal_bf16(100 + seed, (m, k))
            w = synth.normal_bf16(200 + seed, (n, k), 0.05)
            want = sts.op_gemm(a, w, tile, epilogue=1, split_k=split_k, tail_slots=tail_slots)
            a_dev, w_dev = hip.upload(synth.bf16_bits(a)), hip.upload(synth.bf16_bits(w))
            c_dev = hip.upload(np.full((m, n), np.nan, np.float32))          # every element must be written
            sts.op_gemm_noalloc(a_dev, w_dev, c_dev, m, n, k, tile, split_k, tail_slots)
            hip.sync()
            got = hip.download(c_dev, (m, n), np.float32)
            assert np.isfinite(got).all()
            assert rel(got, want) <= TOL_ACC, (m, n, k, tile, split_k, tail_slots)
            assert np.array_equal(got, want)                                 # same kernels, same summation order
    finally:
        hip.free_all()


def test_noalloc_gemm_rejects_what_does_not_fit_its_scratch():
    from paper_2504_19516_amd import sts
    sts.lib()
    hip = Hip()
    try:
        buf = hip.malloc(1 << 20)
        with pytest.raises(sts.StsError) as e:                               # 8 x 2048 x 1024 floats = 64 MiB of partial sums
            sts.op_gemm_noalloc(buf, buf, buf, 2048, 1024, 512, "64x128", 8, 0)
        assert e.value.code == sts.EINVAL
        with pytest.raises(sts.StsError) as e:                               # 256 partial tiles of 256 x 256 floats = 64 MiB
            sts.op_gemm_noalloc(buf, buf, buf, 512, 1024, 512, "256x256", 1, 256)
        assert e.value.code == sts.EINVAL
        with pytest.raises(sts.StsError) as e:
            sts.op_gemm_noalloc(buf, buf, buf, 64, 128, 100, "64x128", 1, 0)  # k not a multiple of 64
        assert e.value.code == sts.EINVAL
        with pytest.raises(sts.StsError) as e:
            sts.op_gemm_noalloc(0, buf, buf, 64, 128, 128, "64x128", 1, 0)    # null input
        assert e.value.code == sts.EINVAL
    finally:
        hip.free_all()
